"""Pins for the CPU checker's exact assignment (Eq. 7-8, Table 1): enumeration of every binary
matrix on tiny instances, LP duality via a library LP solver, a library min-cost-flow on the
literal graph, a library linear-assignment routine for k = 1, closed-form special cases and
invariants.  A plausible mistake in either solver (a dropped arc, a wrong sign, stopping when the
path cost turns positive, a stale contracted arc) fails at least one of these."""
import itertools
import os

import numpy as np
import pytest
import scipy.optimize
import scipy.sparse

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def brute_force(q, k, C):
    """Enumerate every P in {0,1}^{T x E}: maximum number of ones first, then maximum score."""
    q = np.asarray(q)
    T, E = q.shape
    n = T * E
    codes = np.arange(1 << n, dtype=np.int64)
    bits = ((codes[:, None] >> np.arange(n)[None, :]) & 1).astype(np.int8).reshape(-1, T, E)
    ok = (bits.sum(axis=2) <= k).all(axis=1) & (bits.sum(axis=1) <= C).all(axis=1)
    flow = bits.sum(axis=(1, 2))
    score = (bits * q[None]).sum(axis=(1, 2))
    fmax = flow[ok].max()
    best = score[ok & (flow == fmax)].max()
    return int(fmax), int(best)


def rand_q(rng, T, E, kind):
    if kind == "uniform":
        return rng.integers(0, 1 << 20, (T, E))
    if kind == "ties":
        return rng.integers(0, 4, (T, E))
    if kind == "rows_equal":
        return np.tile(rng.integers(0, 50, (1, E)), (T, 1))
    if kind == "signed":
        return rng.integers(-20, 20, (T, E))
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["uniform", "ties", "rows_equal", "signed"])
def test_enumeration_tiny(kind):
    rng = np.random.default_rng(11)
    shapes = [(6, 3), (5, 3), (4, 3), (6, 2), (3, 3), (4, 4)]
    for T, E in shapes:
        for k in range(1, E + 1):
            for C in range(1, T + 2):
                q = rand_q(rng, T, E, kind)
                fmax, best = brute_force(q, k, C)
                lit = oracle.assign_literal_graph(q, k, C)
                assert (lit["flow"], lit["total"]) == (fmax, best), (T, E, k, C, q.tolist())
                assert lit["flow"] == oracle.max_flow_value(T, E, k, C)
                assert oracle.check_feasible(lit["P"], k, C)[0]
                if T * k <= E * min(C, T):
                    con = oracle.assign_contracted(q, k, C)
                    assert (con["flow"], con["total"]) == (fmax, best), (T, E, k, C, q.tolist())
                    assert oracle.check_feasible(con["P"], k, C)[0]


def test_flow_first_fixture():
    q = np.loadtxt(os.path.join(GOLD, "flow_first_example.txt"), comments="#", dtype=np.int64)
    fmax, best = brute_force(q, 2, 2)
    assert (fmax, best) == (6, 312)
    # the best 5-edge matrix scores more, and must not be returned
    n = 9
    codes = np.arange(1 << n)
    bits = ((codes[:, None] >> np.arange(n)[None, :]) & 1).reshape(-1, 3, 3)
    ok = (bits.sum(axis=2) <= 2).all(axis=1) & (bits.sum(axis=1) <= 2).all(axis=1)
    assert (bits * q[None]).sum(axis=(1, 2))[ok].max() == 410
    for sol in (oracle.assign_literal_graph(q, 2, 2), oracle.assign_contracted(q, 2, 2)):
        assert (sol["flow"], sol["total"]) == (6, 312)


def test_table1_arc_count():
    # Table 1: n source arcs, e sink arcs, n*e token-expert arcs
    q = np.zeros((7, 4), dtype=np.int64)
    assert oracle.assign_literal_graph(q, 2, 3)["arcs"] == 7 + 4 + 7 * 4


def lp_optimum(q, k, C):
    """LP relaxation of Eq. 7-8 with rows forced to k (valid when T*k <= E*C): the constraint
    matrix is totally unimodular, so the LP optimum equals the integer optimum."""
    T, E = q.shape
    n = T * E
    rows = scipy.sparse.kron(scipy.sparse.identity(T), np.ones((1, E)))      # row sums
    cols = scipy.sparse.kron(np.ones((1, T)), scipy.sparse.identity(E))      # column sums
    res = scipy.optimize.linprog(-q.reshape(-1).astype(np.float64), A_ub=cols, b_ub=np.full(E, C),
                                 A_eq=rows, b_eq=np.full(T, k), bounds=(0, 1), method="highs")
    assert res.status == 0
    return -res.fun


@pytest.mark.parametrize("T,E,k,C,kind", [(120, 8, 2, 30, "uniform"), (96, 12, 3, 24, "uniform"),
                                           (100, 8, 2, 32, "uniform"), (64, 16, 4, 16, "ties"),
                                           (90, 6, 2, 30, "signed")])
def test_lp_duality(T, E, k, C, kind):
    rng = np.random.default_rng(T + E)
    q = rand_q(rng, T, E, kind)
    con = oracle.assign_contracted(q, k, C)
    lp = lp_optimum(q, k, C)
    assert abs(lp - con["total"]) <= 1e-6 * max(1.0, abs(lp))
    assert oracle.assign_literal_graph(q, k, C)["total"] == con["total"]
    # dual objective from the solver's own prices: sum_i (sum of k best q_ij - p_j) + C * sum_j p_j
    p = con["prices"]
    net = np.sort(q - p[None, :], axis=1)[:, ::-1][:, :k]
    assert int(net.sum() + min(C, T) * p.sum()) == con["total"]
    assert (p >= 0).all() and (p[con["P"].sum(axis=0) < min(C, T)] == 0).all()


def test_networkx_literal_graph():
    nx = pytest.importorskip("networkx")
    rng = np.random.default_rng(2)
    for (T, E, k, C) in [(12, 4, 2, 6), (10, 5, 3, 5), (9, 3, 2, 4), (8, 4, 2, 10)]:
        q = rng.integers(0, 1000, (T, E))
        G = nx.DiGraph()
        for i in range(T):
            G.add_edge("S", ("t", i), capacity=k, weight=0)
            for j in range(E):
                G.add_edge(("t", i), ("e", j), capacity=1, weight=-int(q[i, j]))
        for j in range(E):
            G.add_edge(("e", j), "Z", capacity=C, weight=0)
        flow = nx.max_flow_min_cost(G, "S", "Z")
        total = sum(int(q[i, j]) for i in range(T) for j in range(E) if flow[("t", i)][("e", j)])
        fval = sum(flow["S"][("t", i)] for i in range(T))
        sol = oracle.max_score_assignment(q, k, C)
        assert (sol["flow"], sol["total"]) == (fval, total)
        lit = oracle.assign_literal_graph(q, k, C)
        assert (lit["flow"], lit["total"]) == (fval, total)


def test_k1_matches_linear_assignment():
    # k = 1 only: each expert replicated C times is a plain assignment problem.  (For k > 1 the
    # replication would let one pair match twice, the flaw Section 3.1 describes for OT.)
    rng = np.random.default_rng(3)
    for (T, E, C) in [(40, 5, 8), (30, 4, 9), (25, 5, 5)]:
        q = rng.integers(0, 10000, (T, E))
        big = np.repeat(q, C, axis=1)
        r, c = scipy.optimize.linear_sum_assignment(big, maximize=True)
        assert oracle.assign_contracted(q, 1, C)["total"] == int(big[r, c].sum())


def test_no_capacity_is_rowwise_topk_and_k_equals_E():
    rng = np.random.default_rng(4)
    q = rng.integers(0, 1 << 20, (50, 9))
    sol = oracle.assign_contracted(q, 3, 50)
    assert sol["total"] == int(np.sort(q, axis=1)[:, -3:].sum())
    assert (sol["prices"] == 0).all()
    sol = oracle.assign_contracted(q, 9, 60)          # C > T is clamped to T
    assert sol["P"].all() and sol["total"] == int(q.sum())


def test_identical_rows_tight():
    q = np.tile(np.array([[5, 9, 1, 7]]), (8, 1))
    sol = oracle.assign_contracted(q, 2, 4)
    assert sol["total"] == 4 * int(q[0].sum())
    assert (sol["P"].sum(axis=0) == 4).all()


@pytest.mark.parametrize("seed", range(6))
def test_literal_vs_contracted_midsize(seed):
    rng = np.random.default_rng(100 + seed)
    T = int(rng.integers(40, 160)); E = int(rng.integers(3, 17)); k = int(rng.integers(1, min(E, 5) + 1))
    Cmin = -(-T * k // E)
    C = int(Cmin + rng.integers(0, 4) * (seed % 2))          # tight on even seeds, slack on odd
    kind = ["uniform", "ties", "signed"][seed % 3]
    q = rand_q(rng, T, E, kind)
    a = oracle.assign_literal_graph(q, k, C)
    b = oracle.assign_contracted(q, k, C)
    assert (a["flow"], a["total"]) == (b["flow"], b["total"])
    for sol in (a, b):
        v = oracle.verify_optimal(q, sol["P"], k, C)
        assert v["optimal"] and v["total"] == a["total"]
    if T * k == E * C:
        assert (b["P"].sum(axis=0) == C).all()                # every expert exactly full (ratio 1)


def test_verify_optimal_rejects_suboptimal_and_bounds():
    rng = np.random.default_rng(9)
    T, E, k, C = 60, 6, 2, 20
    q = rng.integers(0, 1 << 20, (T, E))
    sol = oracle.assign_contracted(q, k, C)
    assert oracle.verify_optimal(q, sol["P"], k, C)["optimal"]
    # a feasible but different assignment: round-robin
    P = np.zeros((T, E), dtype=np.uint8)
    for i in range(T):
        for r in range(k):
            P[i, (i * k + r) % E] = 1
    assert oracle.check_feasible(P, k, C)[0]
    v = oracle.verify_optimal(q, P, k, C)
    assert not v["optimal"] and v["total"] < sol["total"]
    # optimum <= unconstrained row-wise top-k and <= column-wise top-C
    assert sol["total"] <= int(np.sort(q, axis=1)[:, -k:].sum())
    assert sol["total"] <= int(np.sort(q, axis=0)[-C:, :].sum())


def test_monotone_in_capacity_and_row_shift():
    rng = np.random.default_rng(10)
    T, E, k = 48, 6, 2
    q = rng.integers(0, 5000, (T, E))
    totals = [oracle.assign_contracted(q, k, C)["total"] for C in (16, 17, 20, 48)]
    assert totals == sorted(totals)
    shift = rng.integers(0, 1000, (T, 1))
    a = oracle.assign_contracted(q, k, 16)
    b = oracle.assign_contracted(q + shift, k, 16)
    assert b["total"] == a["total"] + k * int(shift.sum())
    perm = rng.permutation(E)
    assert oracle.assign_contracted(q[:, perm], k, 16)["total"] == a["total"]
