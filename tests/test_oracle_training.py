"""Pins of the CPU checker's training-side by-products: the load-balance loss (Eq. 9) against closed forms and
a double loop, and the derivative of the gates against central finite differences of the forward pass."""
import numpy as np
import pytest

import oracle


def routed(seed, T=40, E=6, k=2, C=None, t=1.0):
    rng = np.random.default_rng(seed)
    L = rng.normal(size=(T, E)) + rng.normal(size=(1, E))
    A = oracle.soft_topk(L, k, t)
    C = C if C is not None else -(-T * k // E) + 1
    P = oracle.max_score_assignment(oracle.quantise(A), k, C)["P"]
    assign = np.full((T, k), -1, dtype=np.int64)
    for i in range(T):
        held = np.nonzero(P[i])[0]
        assign[i, :held.size] = held
    return L, A, assign, rng


def test_aux_loss_closed_forms():
    T, E, k, lam = 24, 6, 2, 0.01
    A = np.full((T, E), 1.0 / E)
    assign = np.array([[(2 * i) % E, (2 * i + 1) % E] for i in range(T)])       # perfectly balanced
    r = oracle.aux_loss(A, assign, lam)
    assert np.allclose(r["mean_P"], k / E)
    assert np.isclose(r["loss"], lam * (1.0 / E) * E * (1.0 / E) * (k / E))     # = lam*k/e^2
    # all tokens on expert 0 with all the score mass there: lam/e * 1 * 1
    A = np.zeros((T, E)); A[:, 0] = 1.0
    assign = np.zeros((T, 1), dtype=np.int64)
    assert np.isclose(oracle.aux_loss(A, assign, lam)["loss"], lam / E)


def test_aux_loss_double_loop_and_gradient():
    L, A, assign, rng = routed(3)
    T, E = A.shape
    lam = 0.37
    acc = 0.0
    for j in range(E):
        sa = sum(A[i, j] for i in range(T)) / T
        sp = sum(1 for i in range(T) for s in range(assign.shape[1]) if assign[i, s] == j) / T
        acc += sa * sp
    r = oracle.aux_loss(A, assign, lam)
    assert np.isclose(r["loss"], lam * acc / E, rtol=1e-13)
    # the loss is linear in A: the directional derivative along any D equals <dA, D> exactly
    D = rng.normal(size=A.shape)
    r2 = oracle.aux_loss(A + D, assign, lam)
    assert np.isclose(r2["loss"] - r["loss"], (r["dA"][None, :] * D).sum(), rtol=1e-10)


@pytest.mark.parametrize("seed,k,t", [(0, 2, 1.0), (1, 3, 0.5), (2, 1, 1.0), (3, 2, 0.0), (4, 4, 2.0)])
def test_gates_backward_matches_finite_differences(seed, k, t):
    L, A, assign, rng = routed(seed, T=12, E=6, k=k, t=t)
    T, E = L.shape
    dgate = rng.normal(size=assign.shape)
    dA_all = rng.normal(size=E)

    def loss(Lx):                                       # any scalar whose gradients are (dgate, dA_all)
        Ax = oracle.soft_topk(Lx, k, t)
        return (oracle.gates(Ax, assign) * dgate).sum() + (Ax * dA_all[None, :]).sum()

    g = oracle.gates_backward(L, k, t, assign, dgate, dA_all)
    h = 1e-6                                            # far below the gaps between the logits of a row
    gaps = np.diff(np.sort(L, axis=1), axis=1).min()
    assert gaps > 100 * h
    num = np.zeros_like(L)
    for i in range(T):
        for l in range(E):
            Lp, Lm = L.copy(), L.copy()
            Lp[i, l] += h
            Lm[i, l] -= h
            num[i, l] = (loss(Lp) - loss(Lm)) / (2 * h)
    assert np.allclose(g, num, rtol=1e-6, atol=1e-8)


def test_gates_backward_special_cases():
    L, A, assign, rng = routed(7, T=10, E=5, k=2, t=1.0)
    dgate = rng.normal(size=assign.shape)
    g = oracle.gates_backward(L, 2, 1.0, assign, dgate)
    assert np.allclose(g.sum(axis=1), 0.0, atol=1e-14)  # softmax is shift invariant: the row gradients sum to 0
    # t = 0, k = 1: the gate is the softmax probability of the chosen expert
    a1 = assign[:, :1]
    g1 = oracle.gates_backward(L, 1, 0.0, a1, np.ones((10, 1)))
    p = oracle.softmax_rows(L)
    expect = -p * p[np.arange(10), a1[:, 0]][:, None]
    expect[np.arange(10), a1[:, 0]] += p[np.arange(10), a1[:, 0]]
    assert np.allclose(g1, expect, rtol=1e-13)
    # empty slots contribute nothing
    a2 = assign.copy(); a2[:, 1] = -1
    d2 = dgate.copy(); d2[:, 1] = 123.0
    assert np.allclose(oracle.gates_backward(L, 2, 1.0, a2, d2), oracle.gates_backward(L, 2, 1.0, assign[:, :1], dgate[:, :1]))
