"""Pins of the CPU checker's assignment with one k per token (the vector k of Eq. 7): enumeration of every
feasible matrix on tiny inputs, the LP relaxation solved by scipy (the constraint matrix is totally unimodular,
so its optimum is the integer optimum), scipy's linear assignment for k_i in {0, 1}, the uniform case, rows with
k_i = 0 removed, the two C solvers against each other, and the optimality certificate."""
import itertools

import numpy as np
import pytest
from scipy.optimize import linear_sum_assignment, linprog

import oracle


def enumerate_best(q, kvec, caps):
    """(max flow, max total at that flow) over all binary P with row sums <= kvec and column sums <= caps."""
    T, E = q.shape
    best = (-1, -1)
    per_row = [[c for r in range(int(kvec[i]) + 1) for c in itertools.combinations(range(E), r)] for i in range(T)]
    for choice in itertools.product(*per_row):
        load = np.zeros(E, dtype=int)
        tot = 0
        for i, c in enumerate(choice):
            for j in c:
                load[j] += 1
                tot += q[i, j]
        if (load <= caps).all():
            best = max(best, (sum(len(c) for c in choice), tot))
    return best


@pytest.mark.parametrize("seed", range(12))
def test_against_enumeration(seed):
    rng = np.random.default_rng(seed)
    T, E = int(rng.integers(2, 6)), int(rng.integers(2, 4))
    kvec = rng.integers(0, E + 1, T)
    caps = rng.integers(0, T + 1, E) if seed % 2 else np.full(E, int(rng.integers(1, T + 1)))
    q = rng.integers(0, 6 if seed % 3 == 0 else 50, (T, E))          # every third case is tie-heavy
    want = enumerate_best(q, kvec, caps)
    for solver in ("auto", "literal"):
        r = oracle.max_score_assignment_kvec(q, kvec, caps, solver=solver)
        assert (r["flow"], r["total"]) == want, solver
        P = r["P"].astype(int)
        assert (P.sum(axis=0) <= caps).all() and (P.sum(axis=1) <= kvec).all()
        assert int(q[P.astype(bool)].sum()) == r["total"]


@pytest.mark.parametrize("seed", range(4))
def test_lp_relaxation_has_the_same_optimum(seed):
    # every token ships all its units (sum k_i <= E*C, k_i <= E), so "flow first" is the equality P 1 = k
    rng = np.random.default_rng(100 + seed)
    T, E, C = 30, 5, 14
    kvec = rng.integers(0, 4, T)
    while kvec.sum() > E * C:
        kvec[rng.integers(T)] = 0
    q = rng.integers(0, 1000, (T, E))
    A_eq = np.zeros((T, T * E))
    for i in range(T):
        A_eq[i, i * E:(i + 1) * E] = 1
    A_ub = np.zeros((E, T * E))
    for j in range(E):
        A_ub[j, j::E] = 1
    res = linprog(-q.reshape(-1).astype(float), A_ub=A_ub, b_ub=np.full(E, C), A_eq=A_eq, b_eq=kvec,
                  bounds=(0, 1), method="highs")
    assert res.status == 0
    got = oracle.max_score_assignment_kvec(q, kvec, C)
    assert got["flow"] == int(kvec.sum())
    assert got["total"] == int(round(-res.fun))
    assert (got["P"].sum(axis=1) == kvec).all()


@pytest.mark.parametrize("seed", range(3))
def test_zero_one_k_is_linear_assignment_of_the_active_tokens(seed):
    rng = np.random.default_rng(200 + seed)
    T, E, C = 60, 6, 8
    kvec = (rng.random(T) < 0.7).astype(int)
    while kvec.sum() > E * C:
        kvec[np.nonzero(kvec)[0][0]] = 0
    q = rng.integers(0, 1000, (T, E))
    act = np.nonzero(kvec)[0]
    cols = np.repeat(np.arange(E), C)
    r, c = linear_sum_assignment(q[act][:, cols], maximize=True)
    got = oracle.max_score_assignment_kvec(q, kvec, C)
    assert got["flow"] == act.size and got["total"] == int(q[act][:, cols][r, c].sum())
    assert got["P"][kvec == 0].sum() == 0


def test_uniform_k_equals_the_scalar_solver_and_idle_rows_can_be_removed():
    rng = np.random.default_rng(9)
    q = rng.integers(0, 10 ** 6, (64, 8))
    a = oracle.max_score_assignment(q, 2, 16)
    b = oracle.max_score_assignment_kvec(q, np.full(64, 2), 16)
    assert (a["flow"], a["total"]) == (b["flow"], b["total"])
    kvec = rng.integers(0, 5, 64)
    kvec[::4] = 0
    full = oracle.max_score_assignment_kvec(q, kvec, 16)
    keep = kvec > 0
    sub = oracle.max_score_assignment_kvec(q[keep], kvec[keep], 16)
    assert (full["flow"], full["total"]) == (sub["flow"], sub["total"])
    assert full["flow"] == int(kvec.sum()) and (full["P"].sum(axis=1) == kvec).all()


def test_both_graphs_agree_and_the_certificate_accepts_only_the_optimum():
    rng = np.random.default_rng(31)
    T, E, C = 90, 7, 50
    kvec = rng.integers(0, E + 1, T)                         # up to k_i = E
    assert kvec.sum() <= E * C
    q = rng.integers(0, 10 ** 5, (T, E))
    c = oracle.max_score_assignment_kvec(q, kvec, C, solver="contracted")
    l = oracle.max_score_assignment_kvec(q, kvec, C, solver="literal")
    assert (c["flow"], c["total"]) == (l["flow"], l["total"]) and c["flow"] == int(kvec.sum())
    cert = oracle.verify_optimal(q, c["P"], kvec, C)
    assert cert["optimal"] and cert["total"] == c["total"]
    # prices of the contracted solver: every token holds its k_i best experts by q - p
    net = q - c["prices"][None, :]
    P = c["P"].astype(bool)
    big = np.int64(1) << 60
    assert (np.where(P, net, big).min(axis=1) >= np.where(P, -big, net).max(axis=1)).all()
    # move one unit to a worse free expert: feasible, same flow, no longer optimal
    P2 = c["P"].copy()
    load = P2.sum(axis=0)
    done = False
    for i in range(T):
        for j in np.nonzero(P2[i])[0]:
            for j2 in range(E):
                if not P2[i, j2] and load[j2] < C and q[i, j2] < q[i, j]:
                    P2[i, j], P2[i, j2] = 0, 1
                    done = True
                    break
            if done:
                break
        if done:
            break
    assert done and not oracle.verify_optimal(q, P2, kvec, C)["optimal"]
    # a token given one expert more than its k_i is rejected as well
    P3 = c["P"].copy()
    i = int(np.nonzero(kvec < E)[0][0])
    P3[i, np.nonzero(P3[i] == 0)[0][0]] = 1
    assert not oracle.verify_optimal(q, P3, kvec, C)["optimal"]
