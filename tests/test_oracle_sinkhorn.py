"""Pins of the CPU checker's Sinkhorn step (Algorithm 1, step 9): the marginals it must converge to, the
plain top-2 special case, and the low-temperature limit, where the rounded plan must be the exact solution of
the residual problem (the correspondence the paper invokes)."""
import numpy as np
import pytest

import oracle


def test_zero_iterations_is_the_second_best_expert():
    rng = np.random.default_rng(0)
    A = rng.random((50, 6))
    r = oracle.top1_then_sinkhorn(A, 100, tau=0.1, n_iter=0)
    order = np.argsort(-A, axis=1, kind="stable")
    assert np.array_equal(r["assign"][:, 0], order[:, 0])
    assert np.array_equal(r["assign"][:, 1], order[:, 1])


def test_marginals_after_convergence():
    rng = np.random.default_rng(1)
    T, E = 120, 5
    a = rng.random((T, E))
    caps = np.array([40, 0, 35, 30, 25])               # sums to 130 > T: targets are scaled to total T
    r = oracle.sinkhorn_plan(a, caps, tau=0.2, n_iter=300)
    assert np.allclose(r["plan"].sum(axis=0), caps * T / caps.sum(), rtol=1e-12)      # exact after the v update
    assert np.allclose(r["plan"].sum(axis=1), 1.0, rtol=1e-9)                          # converged
    assert (r["plan"][:, 1] == 0).all() and (r["second"] != 1).all()                   # a closed expert gets nothing
    assert (r["plan"] >= 0).all()


def test_row_shift_does_not_change_the_plan():
    rng = np.random.default_rng(2)
    a = rng.random((30, 4))
    caps = np.array([10, 8, 7, 5])
    p1 = oracle.sinkhorn_plan(a, caps, 0.3, 25)["plan"]
    p2 = oracle.sinkhorn_plan(a + rng.normal(size=(30, 1)), caps, 0.3, 25)["plan"]
    assert np.allclose(p1, p2, rtol=1e-10)


@pytest.mark.parametrize("seed", range(5))
def test_low_temperature_limit_is_the_exact_residual_assignment(seed):
    rng = np.random.default_rng(10 + seed)
    T, E = 24, 4
    caps = np.array([6, 6, 6, 6])
    # rewards on a coarse grid: a unique optimum has a margin of at least one grid step
    q = rng.permutation(T * E).reshape(T, E) * 7
    exact = oracle.max_score_assignment_caps(q, 1, caps)
    a = q / q.max()
    r = oracle.sinkhorn_plan(a, caps, tau=2e-3, n_iter=4000)
    second = r["second"]
    assert (np.bincount(second, minlength=E) == caps).all()
    assert int(q[np.arange(T), second].sum()) == exact["total"]


def test_whole_algorithm_1_keeps_top1_and_rounds_within_the_plan():
    rng = np.random.default_rng(4)
    A = oracle.soft_topk(rng.normal(size=(400, 8)) + rng.normal(size=(1, 8)), 2, 1.0)
    r = oracle.top1_then_sinkhorn(A, 100, tau=0.05, n_iter=50)
    assert np.array_equal(r["assign"][:, 0], A.argmax(axis=1))
    assert np.array_equal(r["caps"], np.maximum(0, 100 - np.bincount(A.argmax(axis=1), minlength=8)))
    rows = np.arange(400)
    assert np.allclose(r["plan"][rows, r["assign"][:, 1]], r["plan"].max(axis=1))
    # balancing: the second choices are spread more evenly than the plain second-best experts
    plain = oracle.top1_then_sinkhorn(A, 100, tau=0.05, n_iter=0)
    over = lambda res: np.maximum(0, res["load2"] - res["caps"]).sum()
    assert over(r) <= over(plain)
