"""Pins for the CPU checker's elementwise / per-row steps (logits, SoftTopk, quantise, gates,
dispatch) against things other than itself: the paper's quoted numbers, library routines,
closed forms and brute-force loops."""
import os

import numpy as np
import pytest
import scipy.special

import oracle
from workloads import bf16_bits, bf16_from_bits, bf16_round, make_inputs, make_logits, CONFIGS, capacity

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _table(path):
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    return np.array(rows, dtype=np.float64)


# ---- workloads ----------------------------------------------------------------------------------

def test_bf16_roundtrip_and_rounding():
    a = np.array([1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.1415927], dtype=np.float32)
    r = bf16_round(a)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: even mantissa (1.0) wins; 1 + 3*2^-8 ties upward to even
    assert r[0] == 1.0 and r[2] == 1.0 and r[3] == np.float32(1.0 + 2 ** -6)
    assert np.all(bf16_from_bits(bf16_bits(r)) == r)
    assert np.all(np.abs(r - a) <= np.abs(a) * 2.0 ** -8)


def test_config_capacities_match_formula():
    # c' = c_f * k*n/e (Section 2.3)
    for name, f in [("cfg1", 1.0), ("cfg2", 1.0), ("cfg3", 1.0), ("cfg4a", 1.25), ("cfg5", 1.0)]:
        c = CONFIGS[name]
        assert c["C"] == capacity(c["T"], c["E"], c["k"], f)


def test_inputs_are_seeded_and_bf16_exact():
    a = make_inputs("cfg2", seed=3, T=128)
    b = make_inputs("cfg2", seed=3, T=128)
    c = make_inputs("cfg2", seed=4, T=128)
    assert np.array_equal(a.x_bits, b.x_bits) and np.array_equal(a.W_bits, b.W_bits)
    assert not np.array_equal(a.x_bits, c.x_bits)
    assert np.array_equal(bf16_from_bits(a.x_bits), a.x)
    d = make_inputs("cfg4b_exact", T=256)
    uniq = np.unique(d.x_bits, axis=0).shape[0]
    assert uniq == 256 - 64 + 1


# ---- a1 logits ----------------------------------------------------------------------------------

def test_logits_against_explicit_loops():
    r = make_inputs("cfg1")
    L = oracle.router_logits(r.x, r.W, None)
    ref = np.zeros((r.T, r.E))
    for i in range(0, r.T, 7):
        for j in range(r.E):
            ref[i, j] = sum(float(r.x[i, m]) * float(r.W[m, j]) for m in range(r.d))
    assert np.allclose(L[::7], ref[::7], rtol=1e-12, atol=1e-12)
    b = np.arange(r.E, dtype=np.float32)
    assert np.allclose(oracle.router_logits(r.x, r.W, b) - L, b[None, :], atol=1e-12)


# ---- a2 SoftTopk --------------------------------------------------------------------------------

def test_softtopk_paper_numbers():
    tab = _table(os.path.join(GOLD, "softtopk_example.txt"))
    p = tab[:, 0]
    L = np.log(p)[None, :] + 3.0          # any shift: softmax(L) == p
    assert np.allclose(oracle.softmax_rows(L)[0], p, atol=1e-15)
    assert np.allclose(oracle.soft_topk(L, 2, 4.0)[0], tab[:, 1], atol=1e-12)
    assert np.allclose(oracle.soft_topk(L, 3, 4.0)[0], tab[:, 2], atol=1e-12)


def test_softtopk_reduces_to_softmax():
    L = make_logits("cfg3", T=64).astype(np.float64)
    ref = scipy.special.softmax(L, axis=1)
    assert np.allclose(oracle.soft_topk(L, 8, 0.0), ref, rtol=1e-13, atol=0)   # t -> 0
    assert np.allclose(oracle.soft_topk(L, 1, 3.0), ref, rtol=1e-13, atol=0)   # k = 1


def test_softtopk_closed_form_and_row_sum():
    L = make_logits("cfg5", T=50).astype(np.float64)
    for k, t in [(2, 1.0), (8, 1.0), (8, 4.0), (5, 0.3)]:
        A = oracle.soft_topk(L, k, t)
        p = scipy.special.softmax(L, axis=1)
        # brute-force rank: number of entries that beat entry j (ties: lower index wins)
        E = L.shape[1]
        idx = np.arange(E)
        beats = (L[:, None, :] > L[:, :, None]) | ((L[:, None, :] == L[:, :, None]) & (idx[None, None, :] < idx[None, :, None]))
        rank = 1 + beats.sum(axis=2)
        assert np.allclose(A, p * (1 + t * (np.minimum(rank, k) - 1)), rtol=1e-13)
        ps = -np.sort(-p, axis=1)
        tail = sum(1.0 - ps[:, :m].sum(axis=1) for m in range(1, k))
        assert np.allclose(A.sum(axis=1), 1.0 + t * tail, rtol=1e-12)
        assert (A < max(1.0, t) + 1e-12).all()


def test_softtopk_tie_order_and_overtaking():
    p = np.array([[0.5, 0.2, 0.2, 0.1]])
    A = oracle.soft_topk(np.log(p), 3, 1.0)[0]
    assert np.allclose(A, [0.5, 0.4, 0.6, 0.3])          # equal entries: lower index ranks first
    p = np.array([[0.4, 0.35, 0.25]])
    A = oracle.soft_topk(np.log(p), 2, 4.0)[0]
    assert np.allclose(A, [0.4, 1.75, 1.25])             # runner-up may overtake the leader


# ---- a2, the other readings of Eq. 6 -------------------------------------------------------------

def _brute_rank(L):
    E = L.shape[1]
    idx = np.arange(E)
    beats = (L[:, None, :] > L[:, :, None]) | ((L[:, None, :] == L[:, :, None]) & (idx[None, None, :] < idx[None, :, None]))
    return 1 + beats.sum(axis=2)


def test_softtopk_readings_limits():
    """Every reading is Softmax at t = 0; A, B and C are Softmax at k = 1 (no level is added), A1 is not (its first
    level already lifts everything but the largest entry); reading "A" is soft_topk itself."""
    L = make_logits("cfg3", T=40).astype(np.float64)
    ref = scipy.special.softmax(L, axis=1)
    for rd in ("A", "A1", "B", "C"):
        assert np.allclose(oracle.soft_topk_reading(L, 8, 0.0, rd), ref, rtol=1e-13, atol=0)
    for rd in ("A", "B", "C"):
        assert np.allclose(oracle.soft_topk_reading(L, 1, 3.0, rd), ref, rtol=1e-13, atol=0)
    rank = _brute_rank(L)
    assert np.allclose(oracle.soft_topk_reading(L, 1, 3.0, "A1"), ref * np.where(rank == 1, 1.0, 4.0), rtol=1e-13)
    assert np.array_equal(oracle.soft_topk_reading(L, 5, 2.0, "A"), oracle.soft_topk(L, 5, 2.0))


def test_softtopk_readings_closed_forms_and_row_sums():
    """Closed forms with ranks counted by brute force, and what every row must sum to: A1 adds t times the mass
    outside the m largest entries at level m = 1..k; B adds t times the mass outside the k largest, k - 1 times;
    C adds exactly t per level (a distribution scaled by t)."""
    L = make_logits("cfg5", T=30).astype(np.float64)
    p = scipy.special.softmax(L, axis=1)
    rank = _brute_rank(L)
    ps = -np.sort(-p, axis=1)
    for k, t in [(2, 1.0), (8, 1.0), (8, 4.0), (5, 0.3)]:
        A1 = oracle.soft_topk_reading(L, k, t, "A1")
        assert np.allclose(A1, p * (1 + t * np.minimum(rank - 1, k)), rtol=1e-13)
        assert np.allclose(A1.sum(axis=1), 1 + t * sum(1.0 - ps[:, :m].sum(axis=1) for m in range(1, k + 1)), rtol=1e-12)
        B = oracle.soft_topk_reading(L, k, t, "B")
        assert np.allclose(B, p * np.where(rank <= k, 1.0, 1 + t * (k - 1)), rtol=1e-13)
        assert np.allclose(B.sum(axis=1), 1 + t * (k - 1) * (1.0 - ps[:, :k].sum(axis=1)), rtol=1e-12)
        C = oracle.soft_topk_reading(L, k, t, "C")
        assert np.allclose(C.sum(axis=1), 1 + t * (k - 1), rtol=1e-12)
        w = np.zeros_like(p)                       # sum over the levels m = 2..min(rank, k) of 1 / (mass outside the m-1 largest)
        for m in range(2, k + 1):
            w += np.where(rank >= m, 1.0 / (1.0 - ps[:, :m - 1].sum(axis=1, keepdims=True)), 0.0)
        assert np.allclose(C, p * (1 + t * w), rtol=1e-10)


def test_softtopk_readings_hand_example():
    """p = (0.8, 0.05, 0.05, 0.04, 0.03, 0.03), k = 2, t = 4 (the 0.8 / 0.05 pair of Section 3.1), worked by hand:
    A lifts everything but the leader 5 times; A1 lifts the runner-up 5 times and the rest 9 times; B leaves the two
    largest alone and lifts the rest 5 times; C gives the leader nothing and the others 1 + 4 / 0.2 = 21 times."""
    p = np.array([[0.8, 0.05, 0.05, 0.04, 0.03, 0.03]])
    L = np.log(p)
    assert np.allclose(oracle.soft_topk_reading(L, 2, 4.0, "A")[0], [0.8, 0.25, 0.25, 0.2, 0.15, 0.15])
    assert np.allclose(oracle.soft_topk_reading(L, 2, 4.0, "A1")[0], [0.8, 0.25, 0.45, 0.36, 0.27, 0.27])
    assert np.allclose(oracle.soft_topk_reading(L, 2, 4.0, "B")[0], [0.8, 0.05, 0.25, 0.2, 0.15, 0.15])
    assert np.allclose(oracle.soft_topk_reading(L, 2, 4.0, "C")[0], [0.8, 1.05, 1.05, 0.84, 0.63, 0.63])


# ---- a3 quantise --------------------------------------------------------------------------------

def test_quantise_half_even_and_scale():
    s = 2.0 ** -20
    A = np.array([[0.0, 0.5 * s, 1.5 * s, 2.5 * s, 1.0, 0.75, 3 * s + 0.49 * s]])
    assert oracle.quantise(A).tolist() == [[0, 0, 2, 2, 1 << 20, 3 << 18, 3]]
    assert oracle.quantise(np.array([[0.3]]), shift=4).tolist() == [[5]]


# ---- a5 gates -----------------------------------------------------------------------------------

def test_gates_pick_assigned_affinities():
    A = np.arange(12, dtype=np.float64).reshape(3, 4) / 10
    assign = np.array([[3, 0], [1, -1], [-1, -1]])
    g = oracle.gates(A, assign)
    assert g.tolist() == [[0.3, 0.0], [0.5, 0.0], [0.0, 0.0]]


# ---- a6 dispatch --------------------------------------------------------------------------------

def test_dispatch_against_loops():
    rng = np.random.default_rng(5)
    T, E, k = 37, 5, 3
    assign = np.full((T, k), -1)
    for i in range(T):
        n = rng.integers(0, k + 1)
        assign[i, :n] = rng.permutation(E)[:n]
        rng.shuffle(assign[i])
    gate = rng.random((T, k))
    d = oracle.dispatch(assign, gate, E)
    toks, gts, offs = [], [], [0]
    pos = np.full((T, k), -1)
    for j in range(E):
        n = 0
        for i in range(T):
            for s in range(k):
                if assign[i, s] == j:
                    toks.append(i); gts.append(gate[i, s]); pos[i, s] = n; n += 1
        offs.append(offs[-1] + n)
    assert d["expert_offsets"].tolist() == offs
    assert d["disp_token"].tolist() == toks
    assert d["disp_gate"].tolist() == gts
    assert np.array_equal(d["token_pos"], pos)


def test_route_end_to_end_small():
    r = make_inputs("cfg1")
    out = oracle.route(r.x, r.W, r.bias, r.k, r.C, r.t)
    ok, why = oracle.check_feasible(out["P"], r.k, r.C)
    assert ok, why
    assert (out["P"].sum(axis=0) == r.C).all()          # tight config: every expert exactly full
    assert np.allclose(out["scores"], scipy.special.softmax(out["logits"], axis=1))   # t = 0
    assert out["expert_offsets"][-1] == r.T * r.k
    assert out["total"] == int(out["q"][out["P"].astype(bool)].sum())
