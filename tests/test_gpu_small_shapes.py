"""Degenerate and tiny shapes of the entry points beside the main path (one token, one expert, k = E, a batch
smaller than a wavefront, sizes rejected by validation), through the C ABI against the CPU checker."""
import numpy as np
import pytest

import oracle

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


SHAPES = [(1, 1, 1, 1), (1, 5, 3, 1), (2, 2, 2, 2), (7, 3, 3, 7), (63, 9, 2, 14), (65, 64, 1, 2), (5, 1024, 64, 1),
          (129, 65, 5, 10)]


@pytest.mark.parametrize("T,E,k,C", SHAPES)
def test_iterative_rerouting_small(ms, T, E, k, C):
    print(f"small iter T={T} E={E} k={k} C={C}", flush=True)
    rng = np.random.default_rng(T * 7 + E)
    q = rng.integers(-50, 50, (T, E))
    ref = oracle.iter_reroute(q, k, C)
    out = ms.assign_iter_i32(dev(q.astype(np.int32)), k, C)
    assert np.array_equal(out["assign"].cpu().numpy(), ref["assign"])
    assert (out["total"], out["flow"], out["rounds"]) == (ref["total"], ref["flow"], ref["rounds"])


@pytest.mark.parametrize("T,E,k,C", SHAPES)
def test_capacity_vector_small(ms, T, E, k, C):
    print(f"small caps T={T} E={E} k={k}", flush=True)
    rng = np.random.default_rng(T * 11 + E)
    q = rng.integers(0, 1000, (T, E))
    need = T * k
    caps = np.zeros(E, dtype=np.int64)
    order = rng.permutation(E)
    i = 0
    while caps.sum() < need:                          # fill experts one by one up to T each
        caps[order[i % E]] = min(T, caps[order[i % E]] + 1 + int(rng.integers(0, T)))
        i += 1
    if k == E:
        caps[:] = T
    out = ms.assign_caps_i32(dev(q.astype(np.int32)), k, caps)
    P = oracle.assignment_matrix(out["assign"].cpu().numpy(), E)
    assert (P.sum(axis=1) == k).all() and (P.sum(axis=0) <= caps).all()
    assert out["stats"]["total_score_q"] == oracle.max_score_assignment_caps(q, k, caps)["total"]


@pytest.mark.parametrize("T,E", [(1, 2), (3, 2), (64, 4), (100, 1024)])
def test_top1_then_residual_small(ms, T, E):
    print(f"small algorithm 1 T={T} E={E}", flush=True)
    rng = np.random.default_rng(T + E)
    q = rng.integers(1, 1000, (T, E))
    C = -(-2 * T // E)
    ref = oracle.top1_then_residual(q, C)
    out = ms.assign_top1_residual_i32(dev(q.astype(np.int32)), C)
    assert np.array_equal(out["assign"].cpu().numpy()[:, 0], ref["assign"][:, 0])
    assert out["caps"] == ref["caps"].tolist() and out["total"] == ref["total"]
    assert out["stats"]["total_score_q"] == ref["residual_total"]


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (1, 7, 3), (3, 1024, 64), (65, 2, 2), (200, 96, 5)])
def test_operators_and_training_small(ms, T, E, k):
    print(f"small operators T={T} E={E} k={k}", flush=True)
    rng = np.random.default_rng(T + E + k)
    L = rng.normal(size=(T, E)).astype(np.float32)
    for op, ref in (("sigmoid", oracle.sigmoid_scores(L.astype(np.float64))),
                    ("softkmax", oracle.softkmax(L.astype(np.float64), min(k, 3))),
                    ("itertopk", oracle.itertopk(L.astype(np.float64), min(k, 2)))):
        levels = {"sigmoid": 1, "softkmax": min(k, 3), "itertopk": min(k, 2)}[op]
        sc, _ = ms.scores_op(dev(L), levels, op)
        assert np.allclose(sc.cpu().numpy(), ref, rtol=1e-5, atol=1e-7)
    C = -(-T * k // E) + 1
    out = ms.route_logits(dev(L), k, C, t=1.0)
    aux = ms.aux_loss(out["scores"], out["expert_offsets"], 0.5)
    ref = oracle.aux_loss(out["scores"].cpu().numpy().astype(np.float64), out["assign"].cpu().numpy(), 0.5)
    assert np.isclose(aux["loss"].item(), ref["loss"], rtol=1e-5)
    dg = rng.normal(size=(T, k)).astype(np.float32)
    got = ms.gates_backward(dev(L), out["scores"], out["assign"], dev(dg), aux["dscores_col"]).cpu().numpy()
    want = oracle.gates_backward(L.astype(np.float64), k, 1.0, out["assign"].cpu().numpy(), dg.astype(np.float64),
                                 aux["dscores_col"].cpu().numpy().astype(np.float64))
    assert np.allclose(got, want, rtol=0, atol=2e-5 * max(1e-30, np.abs(want).max()))


def test_rejected_sizes(ms):
    print("small rejected", flush=True)
    q = dev(np.zeros((4, 4), dtype=np.int32))
    with pytest.raises(ms.MaxScoreError):
        ms.assign_iter_i32(q, 5, 2)                   # k > E
    with pytest.raises(ms.MaxScoreError):
        ms.assign_iter_i32(q, 2, 0)                   # C < 1
    with pytest.raises(ms.MaxScoreError):
        ms.assign_top1_residual_i32(dev(np.zeros((4, 1), dtype=np.int32)), 8)   # top-2 needs two experts
    with pytest.raises(KeyError):
        ms.scores_op(dev(np.zeros((4, 4), dtype=np.float32)), 2, "no such operator")
