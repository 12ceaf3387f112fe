"""Pins of the CPU checker's activation movement (expert input buffers, Eq. 1 combine) against what the
definitions fix: closed forms, a brute-force double loop and the round trip through identity experts."""
import numpy as np

import oracle


def small_case(seed=0, T=37, E=5, k=3, C=None, d=12):
    rng = np.random.default_rng(seed)
    q = rng.integers(0, 1000, (T, E))
    C = C if C is not None else -(-T * k // E) + 2
    res = oracle.max_score_assignment(q, k, C)
    assign = np.full((T, k), -1, dtype=np.int64)
    for i in range(T):
        held = np.nonzero(res["P"][i])[0]
        assign[i, :held.size] = held
    gate = rng.random((T, k))
    disp = oracle.dispatch(assign, gate, E)
    x = rng.normal(size=(T, d))
    return x, assign, gate, disp, E, C


def test_dispatch_tokens_matches_a_double_loop_and_pads_with_zeros():
    x, assign, gate, disp, E, C = small_case()
    buf = oracle.dispatch_tokens(x, disp["expert_offsets"], disp["disp_token"], E, C)
    assert buf.shape == (E, C, x.shape[1])
    ref = np.zeros_like(buf)
    fill = np.zeros(E, dtype=int)
    for i in range(assign.shape[0]):                 # token-major, so ascending token id inside an expert
        for s in range(assign.shape[1]):
            j = assign[i, s]
            if j >= 0:
                ref[j, fill[j]] = x[i]
                fill[j] += 1
    assert np.array_equal(buf, ref)
    for j in range(E):
        assert not buf[j, fill[j]:].any()
    # the slot of pair (i, s) is token_pos[i, s]
    for i in range(assign.shape[0]):
        for s in range(assign.shape[1]):
            if assign[i, s] >= 0:
                assert np.array_equal(buf[assign[i, s], disp["token_pos"][i, s]], x[i])


def test_combine_through_identity_experts_is_the_gate_sum_times_x():
    x, assign, gate, disp, E, C = small_case(seed=3)
    buf = oracle.dispatch_tokens(x, disp["expert_offsets"], disp["disp_token"], E, C)
    y = oracle.combine(buf, assign, disp["token_pos"], gate)
    gsum = np.where(assign >= 0, gate, 0.0).sum(axis=1)
    assert np.allclose(y, gsum[:, None] * x, rtol=1e-12, atol=1e-12)


def test_combine_is_the_sum_of_eq_1_term_by_term():
    x, assign, gate, disp, E, C = small_case(seed=5, T=20, E=4, k=2, d=7)
    rng = np.random.default_rng(9)
    out = rng.normal(size=(E, C, 7))                  # arbitrary expert outputs
    y = oracle.combine(out, assign, disp["token_pos"], gate)
    for i in range(assign.shape[0]):
        acc = np.zeros(7)
        for s in range(assign.shape[1]):
            if assign[i, s] >= 0:
                acc += gate[i, s] * out[assign[i, s], disp["token_pos"][i, s]]
        assert np.allclose(y[i], acc, rtol=1e-13, atol=1e-13)
    # linear in the gates and in the expert outputs
    assert np.allclose(oracle.combine(2 * out, assign, disp["token_pos"], gate), 2 * y)
    assert np.allclose(oracle.combine(out, assign, disp["token_pos"], 3 * gate), 3 * y)


def test_empty_slots_contribute_nothing():
    x, assign, gate, disp, E, C = small_case(seed=7, T=9, E=3, k=2, C=2)     # over-subscribed: some slots stay -1
    assert (assign < 0).any()
    buf = oracle.dispatch_tokens(x, disp["expert_offsets"], disp["disp_token"], E, C)
    y = oracle.combine(buf, assign, disp["token_pos"], gate)
    gsum = np.where(assign >= 0, gate, 0.0).sum(axis=1)
    assert np.allclose(y, gsum[:, None] * x)
