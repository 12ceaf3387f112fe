"""Pins of the CPU checker's other Table 2 operators: library routines at the levels where they reduce to one,
row-sum identities, hand-computed two-expert values and symmetry."""
import numpy as np
import pytest
from scipy.special import expit, softmax

import oracle


def logits(seed, T=30, E=7):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(T, E)) * 1.5


def test_sigmoid_is_scipy_expit():
    L = logits(0)
    assert np.allclose(oracle.sigmoid_scores(L), expit(L), rtol=1e-14)


@pytest.mark.parametrize("op", [oracle.softkmax, oracle.itertopk])
def test_level_one_is_softmax_and_rows_sum_to_k(op):
    L = logits(1)
    assert np.allclose(op(L, 1), softmax(L, axis=1), rtol=1e-13)
    for k in (2, 3, 5):
        assert np.allclose(op(L, k).sum(axis=1), k, rtol=1e-12)       # every level adds a distribution


@pytest.mark.parametrize("op", [oracle.softkmax, oracle.itertopk])
def test_uniform_logits_and_permutations(op):
    assert np.allclose(op(np.full((3, 8), 0.7), 3), 3 / 8)
    L = logits(2)
    perm = np.random.default_rng(3).permutation(L.shape[1])
    assert np.allclose(op(L[:, perm], 3), op(L, 3)[:, perm], rtol=1e-12)


def test_itertopk_two_expert_value_by_hand():
    # p = (0.9, 0.1): level 2 weights w = (0.1, 0.9); w*p = (0.09, 0.09) -> g = (0.5, 0.5); y = (1.4, 0.6)
    L = np.log(np.array([[0.9, 0.1]]))
    assert np.allclose(oracle.itertopk(L, 2), [[1.4, 0.6]], rtol=1e-13)
    # level 3: w = (-0.4, 0.4); w*p = (-0.36, 0.04) -> g = (1.125, -0.125); y = (2.525, 0.475)
    assert np.allclose(oracle.itertopk(L, 3), [[2.525, 0.475]], rtol=1e-12)


def test_softkmax_two_expert_value_by_hand():
    # x = (ln 3, 0): y1 = (0.75, 0.25); g = (0.25 ln 3, 0.75 * 0) = (0.25 ln 3, 0)
    # softmax(g) = (3^0.25, 1) / (3^0.25 + 1)
    L = np.array([[np.log(3.0), 0.0]])
    a = 3.0 ** 0.25
    assert np.allclose(oracle.softkmax(L, 2), [[0.75 + a / (a + 1), 0.25 + 1 / (a + 1)]], rtol=1e-13)


def test_itertopk_is_shift_invariant_and_softkmax_is_not():
    L = logits(4)
    assert np.allclose(oracle.itertopk(L + 3.0, 3), oracle.itertopk(L, 3), rtol=1e-12)
    assert not np.allclose(oracle.softkmax(L + 3.0, 3), oracle.softkmax(L, 3), rtol=1e-6)   # g multiplies x


def test_gradtopk_level_one_row_sums_and_the_level_two_closed_form():
    L = logits(5, T=40, E=9)
    p = softmax(L, axis=1)
    assert np.allclose(oracle.gradtopk(L, 1), p, rtol=1e-13)
    for k in (2, 3, 4):
        y = oracle.gradtopk(L, k)
        assert np.isfinite(y).all() and np.allclose(y.sum(axis=1), k, rtol=1e-12)
    # level 2 by hand: e^{g2} = e^x (S - e^x), so y2 = 2 p (1 - p) / sum p (1 - p)
    w = p * (1 - p)
    assert np.allclose(oracle.gradtopk(L, 2), 2 * w / w.sum(axis=1, keepdims=True), rtol=1e-12)
    assert np.allclose(oracle.gradtopk(np.full((2, 8), -0.3), 3), 3 / 8)
    # p = (0.6, 0.3, 0.1): p(1-p) = (0.24, 0.21, 0.09), sum 0.54 -> y2 = (8/9, 7/9, 1/3)
    L3 = np.log(np.array([[0.6, 0.3, 0.1]]))
    assert np.allclose(oracle.gradtopk(L3, 2), [[8 / 9, 7 / 9, 1 / 3]], rtol=1e-13)


def test_gradtopk_leaves_its_domain_for_two_equal_experts():
    y2 = oracle.gradtopk(np.zeros((1, 2)), 2)
    assert np.allclose(y2, 1.0)                          # both values reach 1 ...
    assert not np.isfinite(oracle.gradtopk(np.zeros((1, 2)), 3)).any()   # ... and level 3 takes log(0)
