"""Pins of the CPU checker's iterative rerouting (Section 2.3) against things other than itself:
a hand-worked example, a literal pair-by-pair walk of the stated orders, the cases where the
heuristic must coincide with plain top-k, and the exact solver as an upper bound."""
import numpy as np
import pytest

import oracle


def walk(q, k, C):
    """The stated reading, pair by pair with Python loops and no sorting primitives."""
    T, E = q.shape
    assign = [[-1] * k for _ in range(T)]
    load = [0] * E

    def best(i, allowed):
        bj = -1
        for j in range(E):
            if allowed(j) and (bj < 0 or q[i, j] > q[i, bj]):
                bj = j
        return bj

    choice = []
    for i in range(T):
        taken = []
        for _ in range(k):
            taken.append(best(i, lambda j: j not in taken))
        choice.append(taken)
    for s in range(k):
        for i in range(T):
            j = choice[i][s]
            if load[j] < C:
                assign[i][s] = j
                load[j] += 1
    stage1 = [row[:] for row in assign]
    rounds = 0
    while True:
        room = [C - l for l in load]
        proposals = []
        for i in range(T):
            used = [j for j in assign[i] if j >= 0]
            for s in range(k):
                if assign[i][s] < 0:
                    j = best(i, lambda j: room[j] > 0 and j not in used)
                    if j >= 0:
                        used.append(j)
                        proposals.append((s, i, j))
        if not proposals:
            break
        rounds += 1
        for s, i, j in sorted(proposals):
            if load[j] < C:
                assign[i][s] = j
                load[j] += 1
    return np.array(assign), np.array(stage1), np.array(load), rounds


def test_hand_worked_example():
    # 4 tokens, 3 experts, k = 1, C = 2.  Everybody prefers expert 0; tokens 0 and 1 get it.
    # Round 1: tokens 2 and 3 propose their next best: token 2 -> expert 1, token 3 -> expert 2.
    q = np.array([[9, 1, 0], [8, 2, 1], [7, 5, 3], [6, 2, 4]])
    r = oracle.iter_reroute(q, 1, 2)
    assert r["stage1"].ravel().tolist() == [0, 0, -1, -1]
    assert r["assign"].ravel().tolist() == [0, 0, 1, 2]
    assert r["total"] == 9 + 8 + 5 + 4 and r["flow"] == 4 and r["rounds"] == 1
    # k = 2, C = 3 (8 pairs, 9 places).  First choices: expert 0 takes tokens 0, 1, 2; token 3 is dropped.
    # Second choices 1, 1, 1, 2 all fit.  Round 1: token 3 holds expert 2 and expert 0 is full -> expert 1 (full
    # after tokens 0..2 took it) has no room, so the only experts with room are 2 (held) -> no proposal possible.
    r = oracle.iter_reroute(q, 2, 3)
    assert r["stage1"].tolist() == [[0, 1], [0, 1], [0, 1], [-1, 2]]
    assert r["assign"].tolist() == [[0, 1], [0, 1], [0, 1], [-1, 2]]
    assert r["flow"] == 7 and r["rounds"] == 0 and r["load"].tolist() == [3, 3, 1]


def test_second_round_is_needed_when_a_proposal_is_refused():
    # k = 1, C = 1: token 0 takes expert 0.  Round 1: tokens 1 and 2 both propose expert 1, token 1 wins;
    # round 2: token 2 proposes expert 2.
    q = np.array([[9, 0, 0], [8, 7, 1], [8, 7, 1]])
    r = oracle.iter_reroute(q, 1, 1)
    assert r["assign"].ravel().tolist() == [0, 1, 2] and r["rounds"] == 2


@pytest.mark.parametrize("T,E,k,C,seed", [(40, 5, 2, 16, 0), (64, 8, 3, 24, 1), (33, 7, 5, 24, 2), (50, 6, 2, 17, 3),
                                           (30, 4, 1, 8, 4), (25, 9, 4, 12, 5), (48, 6, 3, 20, 6)])
def test_matches_the_pair_by_pair_walk(T, E, k, C, seed):
    rng = np.random.default_rng(seed)
    q = rng.integers(0, 50, (T, E))                    # narrow range: many ties
    bias = rng.integers(0, 40, E)                      # skewed popularity so that stage 1 drops pairs
    q = q + bias[None, :]
    r = oracle.iter_reroute(q, k, C)
    a, s1, load, rounds = walk(q, k, C)
    assert np.array_equal(r["stage1"], s1)
    assert np.array_equal(r["assign"], a)
    assert np.array_equal(r["load"], load)
    assert r["rounds"] == rounds
    assert (r["stage1"] < 0).any()                     # the case does exercise rerouting


def test_equals_plain_topk_when_nothing_overflows():
    rng = np.random.default_rng(11)
    q = rng.integers(0, 10 ** 6, (60, 8))
    r = oracle.iter_reroute(q, 3, 60)                  # C >= T: no expert can overflow
    top = np.argsort(-q, axis=1, kind="stable")[:, :3]
    assert np.array_equal(r["assign"], top) and r["rounds"] == 0
    exact = oracle.max_score_assignment(q, 3, 60)
    assert r["total"] == exact["total"]


@pytest.mark.parametrize("seed", range(6))
def test_feasible_and_bounded_by_the_exact_optimum(seed):
    rng = np.random.default_rng(100 + seed)
    T, E, k = 96, 8, 2
    C = T * k // E + (seed % 3)                        # tight and slightly slack capacities
    q = rng.integers(0, 1 << 20, (T, E)) + (rng.integers(0, 1 << 19, E))[None, :]
    r = oracle.iter_reroute(q, k, C)
    P = oracle.assignment_matrix(r["assign"], E)       # raises on a repeated expert
    assert P.sum(axis=0).max() <= C and np.array_equal(P.sum(axis=0), r["load"])
    exact = oracle.max_score_assignment(q, k, C)
    s1 = r["stage1"]
    stage1_total = int(q[np.nonzero(s1 >= 0)[0], s1[s1 >= 0]].sum())
    assert stage1_total <= r["total"]
    if r["flow"] == exact["flow"]:
        assert r["total"] <= exact["total"]
    else:
        assert r["flow"] < exact["flow"]
    # stage 1 keeps exactly the first C pairs per expert in (rank, token) order: nobody dropped from an expert
    # that still had room at the end of stage 1
    top = np.argsort(-q, axis=1, kind="stable")[:, :k]
    load1 = np.bincount(s1[s1 >= 0], minlength=E)
    dropped = top[s1 < 0]
    assert (load1[dropped] == C).all()


def test_round_limit_stops_early():
    q = np.array([[9, 0, 0], [8, 7, 1], [8, 7, 1]])
    r = oracle.iter_reroute(q, 1, 1, max_rounds=1)
    assert r["assign"].ravel().tolist() == [0, 1, -1] and r["rounds"] == 1
