"""GPU parity of the exact assignment with one k per token (the vector k of Eq. 7) through the C ABI: every
token ends with exactly its k_i distinct experts, the total is bit-equal to the CPU checker's optimum, and
the returned prices certify the optimum (every token holds its k_i best experts by net value, up to 1 unit of
the scaled rewards; experts with room have price 0)."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, make_logits

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ms():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2508_12801_amd as m
    m.load_library()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_rows(a, kvec, E):
    """Row i: kvec[i] distinct experts first, then -1."""
    T, k = a.shape
    slot = np.arange(k)[None, :]
    assert ((a >= 0) == (slot < kvec[:, None])).all()
    assert (a < E).all()
    return oracle.assignment_matrix(a, E)


def check_prices(q, P, out, caps):
    """eps = 1 complementary slackness in the solver's scaled units."""
    S = out["price_scale"]
    p = out["prices"].cpu().numpy()
    net = q.astype(np.int64) * S - p[None, :]
    big = np.int64(1) << 60
    held = P.astype(bool)
    assert (np.where(held, net, big).min(axis=1) + 1 >= np.where(held, -big, net).max(axis=1)).all()
    load = P.sum(axis=0)
    assert (p >= 0).all() and (p[load < caps] == 0).all()


@pytest.mark.parametrize("T,E,kmax,slack,mode", [
    (300, 8, 2, 0, "mixed"), (300, 8, 3, 40, "mixed"), (2000, 16, 4, 0, "zeros"), (4099, 64, 8, 0, "mixed"),
    (4099, 64, 8, 333, "mixed"), (5000, 128, 8, 0, "mixed"), (1500, 300, 6, 9, "mixed"),
    (700, 8, 8, 0, "full"),             # some tokens take every expert (k_i = E)
    (3000, 32, 16, 0, "mixed"), (1000, 128, 64, 5, "mixed"), (513, 16, 2, 0, "ones"),
])
def test_per_token_k_matches_the_checker(ms, T, E, kmax, slack, mode):
    print(f"kvec T={T} E={E} kmax={kmax} slack={slack} {mode}", flush=True)
    rng = np.random.default_rng(T + E + kmax + slack)
    q = (rng.integers(0, 1 << 20, (T, E)) + rng.integers(0, 1 << 19, E)[None, :]).astype(np.int32)
    if mode == "ones":
        kvec = rng.integers(0, 2, T)
    else:
        kvec = rng.integers(0 if mode != "full" else 1, kmax + 1, T)
    if mode == "zeros":
        kvec[rng.random(T) < 0.5] = 0
    kvec = kvec.astype(np.int32)
    demand = int(kvec.sum())
    C = -(-(demand + slack) // E)
    if slack == 0 and demand % E:                   # make the instance tight: no spare place at all
        extra = E - demand % E
        idx = np.nonzero(kvec < kmax)[0][:extra]
        kvec[idx] += 1
        demand = int(kvec.sum())
        C = demand // E
        assert demand == E * C
    C = max(C, int((kvec == E).sum()), 1)           # an expert must be able to take every token that takes all experts
    out = ms.assign_kvec_i32(dev(q), kmax, dev(kvec), C)
    a = out["assign"].cpu().numpy()
    P = check_rows(a, kvec, E)
    assert (P.sum(axis=0) <= C).all()
    assert out["stats"]["flow_value"] == demand
    ref = oracle.max_score_assignment_kvec(q.astype(np.int64), kvec, C)
    assert ref["flow"] == demand
    assert out["stats"]["total_score_q"] == ref["total"] == int(q.astype(np.int64)[P.astype(bool)].sum())
    check_prices(q, P, out, np.full(E, min(C, T)))


def test_per_token_k_with_a_capacity_vector(ms):
    print("kvec + caps", flush=True)
    rng = np.random.default_rng(77)
    T, E, kmax = 2500, 32, 4
    q = rng.integers(0, 1 << 20, (T, E)).astype(np.int32)
    kvec = rng.integers(0, kmax + 1, T).astype(np.int32)
    w = rng.random(E) + 0.5
    caps = np.ceil(w / w.sum() * kvec.sum() * 1.02).astype(np.int64) + 1
    out = ms.assign_kvec_i32(dev(q), kmax, dev(kvec), caps=caps)
    P = check_rows(out["assign"].cpu().numpy(), kvec, E)
    assert (P.sum(axis=0) <= caps).all()
    ref = oracle.max_score_assignment_kvec(q.astype(np.int64), kvec, caps)
    assert ref["flow"] == int(kvec.sum()) == out["stats"]["flow_value"]
    assert out["stats"]["total_score_q"] == ref["total"]
    check_prices(q, P, out, np.minimum(caps, T))


def test_uniform_vector_equals_the_scalar_entry_point_and_feeds_gates_and_dispatch(ms):
    print("kvec uniform / downstream", flush=True)
    c = CONFIGS["cfg3"]
    A = oracle.soft_topk(make_logits("cfg3", 5), c["k"], c["t"])
    q = oracle.quantise(A).astype(np.int32)
    T, E, k = q.shape[0], c["E"], c["k"]
    a = ms.assign_i32(dev(q), k, c["C"])
    b = ms.assign_kvec_i32(dev(q), k, dev(np.full(T, k, dtype=np.int32)), c["C"])
    assert a["stats"]["total_score_q"] == b["stats"]["total_score_q"]
    # a skewed k vector on the same rewards: gates and dispatch take the result with its -1 slots as it is
    rng = np.random.default_rng(5)
    kvec = rng.integers(0, k + 1, T).astype(np.int32)
    out = ms.assign_kvec_i32(dev(q), k, dev(kvec), c["C"])
    assign = out["assign"].cpu().numpy()
    P = check_rows(assign, kvec, E)
    cert = oracle.verify_optimal(q.astype(np.int64), P, kvec, c["C"])
    assert cert["optimal"] and cert["total"] == out["stats"]["total_score_q"]
    scores = dev(A.astype(np.float32))
    g = ms.gates(scores, out["assign"])
    ref_g = oracle.gates(A.astype(np.float32).astype(np.float64), assign)
    assert np.array_equal(g.cpu().numpy() == 0, assign < 0)
    assert np.allclose(g.cpu().numpy(), ref_g, rtol=1e-6, atol=0)
    d = ms.dispatch(out["assign"], g, E, c["C"])
    ref_d = oracle.dispatch(assign, g.cpu().numpy(), E)
    assert np.array_equal(d["expert_offsets"].cpu().numpy(), ref_d["expert_offsets"])
    n = int(kvec.sum())
    assert np.array_equal(d["disp_token"].cpu().numpy()[:n], ref_d["disp_token"][:n])


def test_headline_shape_with_a_skewed_k_vector_is_certified(ms):
    print("kvec cfg5", flush=True)
    c = CONFIGS["cfg5"]
    T, E, k, C = c["T"], c["E"], c["k"], c["C"]
    q = oracle.quantise(oracle.soft_topk(make_logits("cfg5", 3), k, c["t"])).astype(np.int32)
    rng = np.random.default_rng(11)
    kvec = np.clip(rng.poisson(5.0, T), 0, k).astype(np.int32)       # about 5 experts per token on average
    out = ms.assign_kvec_i32(dev(q), k, dev(kvec), C)
    P = check_rows(out["assign"].cpu().numpy(), kvec, E)
    assert (P.sum(axis=0) <= C).all() and out["stats"]["flow_value"] == int(kvec.sum())
    assert out["stats"]["total_score_q"] == int(q.astype(np.int64)[P.astype(bool)].sum())
    check_prices(q, P, out, np.full(E, C))
    cert = oracle.verify_optimal(q.astype(np.int64), P, kvec, C)
    assert cert["optimal"]


def test_per_token_k_errors(ms):
    print("kvec errors", flush=True)
    q = dev(np.zeros((100, 4), dtype=np.int32))
    bad = np.full(100, 2, dtype=np.int32)
    bad[7] = 3
    with pytest.raises(ms.MaxScoreError):
        ms.assign_kvec_i32(q, 2, dev(bad), 50)                        # an entry above k
    bad[7] = -1
    with pytest.raises(ms.MaxScoreError):
        ms.assign_kvec_i32(q, 2, dev(bad), 50)
    with pytest.raises(ms.MaxScoreError):
        ms.assign_kvec_i32(q, 2, dev(np.full(100, 2, dtype=np.int32)), 49)    # 196 places for 200 pairs
    out = ms.assign_kvec_i32(q, 2, dev(np.zeros(100, dtype=np.int32)), 1)     # nobody wants anything
    assert (out["assign"].cpu().numpy() == -1).all() and out["stats"]["flow_value"] == 0
