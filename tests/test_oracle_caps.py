"""Pins of the CPU checker's assignment with one capacity per expert and of the top-1-then-residual split of
Algorithm 1: enumeration of every feasible matrix on tiny inputs, scipy's linear assignment on replicated
columns for k = 1, the uniform case, and the two C solvers against each other."""
import itertools

import numpy as np
import pytest
from scipy.optimize import linear_sum_assignment

import oracle


def enumerate_best(q, k, caps):
    """(max flow, max total at that flow) over all binary P with row sums <= k and column sums <= caps."""
    T, E = q.shape
    best = (-1, -1)
    rows = [c for r in range(k + 1) for c in itertools.combinations(range(E), r)]
    for choice in itertools.product(rows, repeat=T):
        load = np.zeros(E, dtype=int)
        tot = 0
        for i, c in enumerate(choice):
            for j in c:
                load[j] += 1
                tot += q[i, j]
        if (load <= caps).all():
            best = max(best, (sum(len(c) for c in choice), tot))
    return best


@pytest.mark.parametrize("seed", range(8))
def test_against_enumeration(seed):
    rng = np.random.default_rng(seed)
    T, E = int(rng.integers(2, 5)), int(rng.integers(2, 4))
    k = int(rng.integers(1, E + 1))
    caps = rng.integers(0, T + 1, E)
    q = rng.integers(0, 20, (T, E))
    r = oracle.max_score_assignment_caps(q, k, caps)
    assert (r["flow"], r["total"]) == enumerate_best(q, k, caps)
    P = r["P"].astype(int)
    assert (P.sum(axis=0) <= caps).all() and (P.sum(axis=1) <= k).all()


@pytest.mark.parametrize("seed", range(4))
def test_k1_is_linear_assignment_on_replicated_columns(seed):
    rng = np.random.default_rng(50 + seed)
    T, E = 40, 6
    caps = rng.integers(0, 14, E)
    caps[rng.integers(E)] += max(0, T - caps.sum())           # enough room for every token
    q = rng.integers(0, 1000, (T, E))
    cols = np.repeat(np.arange(E), caps)
    r, c = linear_sum_assignment(q[:, cols], maximize=True)
    got = oracle.max_score_assignment_caps(q, 1, caps)
    assert got["flow"] == T and got["total"] == int(q[:, cols][r, c].sum())


def test_uniform_caps_equal_the_scalar_solver_and_both_graphs_agree():
    rng = np.random.default_rng(7)
    q = rng.integers(0, 10 ** 6, (60, 7))
    a = oracle.max_score_assignment(q, 2, 20)
    b = oracle.max_score_assignment_caps(q, 2, np.full(7, 20))
    assert a["total"] == b["total"] and a["flow"] == b["flow"]
    caps = np.array([30, 0, 25, 5, 40, 11, 9])
    c = oracle.max_score_assignment_caps(q, 2, caps)           # contracted (120 <= 120)
    import ctypes
    from oracle import reference as ref
    P = np.zeros(q.shape, dtype=np.uint8)
    flow, total, arcs = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    qq = np.ascontiguousarray(q, dtype=np.int64)
    cc = np.ascontiguousarray(caps, dtype=np.int32)
    rc = ref._load().mcmf_literal_caps(qq.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), 60, 7, 2,
                                       cc.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                       P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), ctypes.byref(flow),
                                       ctypes.byref(total), ctypes.byref(arcs))
    assert rc == 0 and flow.value == c["flow"] == 120 and total.value == c["total"]
    assert c["P"][:, 1].sum() == 0                             # an expert without capacity holds nobody


def test_top1_then_residual_by_hand_and_bounds():
    # 4 tokens, 3 experts, C = 2.  top-1: tokens 0,1,2 -> expert 0 (load 3 > C), token 3 -> expert 2.
    # residual capacities (0, 2, 1); residual rewards have the top-1 entries zeroed.
    q = np.array([[9, 5, 1], [8, 2, 6], [7, 3, 4], [1, 2, 9]])
    r = oracle.top1_then_residual(q, 2)
    assert r["assign"][:, 0].tolist() == [0, 0, 0, 2] and r["caps"].tolist() == [0, 2, 1]
    # best second choices under (0,2,1): tokens {0: e1 (5), 1: e2 (6), 2: e1 (3)} and token 3 needs a place:
    # only 3 places exist for 4 tokens -> flow 3; dropping token 3 (best remaining 2) is optimal: 5 + 6 + 3 = 14
    assert r["residual_flow"] == 3 and r["residual_total"] == 14
    assert r["total"] == 9 + 8 + 7 + 9 + 14
    rng = np.random.default_rng(3)
    q = rng.integers(0, 1 << 20, (200, 8))
    r = oracle.top1_then_residual(q, 50)                       # c = 2n/e
    exact = oracle.max_score_assignment(q, 2, 50)
    load1 = np.bincount(r["assign"][:, 0], minlength=8)
    if load1.max() <= 50 and r["residual_flow"] == 200 and r["repeat"] == 0:
        assert r["total"] <= exact["total"]                    # feasible for the full problem, so bounded by its optimum
    second = r["assign"][:, 1]
    assert (np.bincount(second[second >= 0], minlength=8) <= r["caps"]).all()


def test_certificate_accepts_the_optimum_and_rejects_a_worse_matrix_with_a_capacity_vector():
    rng = np.random.default_rng(21)
    T, E, k = 80, 6, 2
    caps = np.array([40, 0, 35, 30, 25, 40])
    q = rng.integers(0, 10 ** 5, (T, E))
    best = oracle.max_score_assignment_caps(q, k, caps)
    cert = oracle.verify_optimal(q, best["P"], k, caps)
    assert cert["optimal"] and cert["total"] == best["total"]
    # swap one token's expert for a worse free one: still feasible, no longer optimal
    P = best["P"].copy()
    load = P.sum(axis=0)
    done = False
    for i in range(T):
        for j in np.nonzero(P[i])[0]:
            for j2 in range(E):
                if not P[i, j2] and load[j2] < caps[j2] and q[i, j2] < q[i, j]:
                    P[i, j], P[i, j2] = 0, 1
                    done = True
                    break
            if done:
                break
        if done:
            break
    assert done and not oracle.verify_optimal(q, P, k, caps)["optimal"]
