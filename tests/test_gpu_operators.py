"""GPU parity of the other Table 2 operators through the C ABI against the fp64 checker on the same fp32 logits."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, make_logits

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

REF = {"sigmoid": lambda L, k: oracle.sigmoid_scores(L), "softkmax": oracle.softkmax, "itertopk": oracle.itertopk,
       "gradtopk": oracle.gradtopk}


@pytest.fixture(scope="module")
def ms():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2508_12801_amd as m
    m.load_library()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("op", ["sigmoid", "softkmax", "itertopk", "gradtopk"])
@pytest.mark.parametrize("T,E,k", [(300, 8, 2), (1000, 16, 4), (4099, 64, 2), (257, 7, 3), (2048, 128, 8),
                                   (700, 300, 6), (130, 1024, 2), (65, 5, 1), (65536, 128, 8)])
def test_scores_match_the_checker(ms, op, T, E, k):
    print(f"operator {op} T={T} E={E} k={k}", flush=True)
    rng = np.random.default_rng(T + E + k)
    L = (rng.normal(size=(T, E)) + 1.0 * rng.normal(size=(1, E))).astype(np.float32)
    kk = min(k, 2) if op in ("itertopk", "gradtopk") else k   # levels 1-2 stay inside the domain on peaked rows
    sc, q = ms.scores_op(dev(L), kk, op)
    ref = REF[op](L.astype(np.float64), kk)
    got = sc.cpu().numpy()
    assert np.allclose(got, ref, rtol=1e-5, atol=1e-7)
    # the integer is decided in the kernel's own precision
    assert np.array_equal(q.cpu().numpy(), np.rint(got.astype(np.float32) * np.float32(1 << 20)).astype(np.int64))
    assert np.abs(q.cpu().numpy() - oracle.quantise(ref)).max() <= max(2, 2e-5 * oracle.quantise(ref).max())


def test_gradtopk_deeper_levels_and_the_edge_of_its_domain(ms):
    print("gradtopk k=4", flush=True)
    rng = np.random.default_rng(13)
    L = (0.3 * rng.normal(size=(2000, 64))).astype(np.float32)     # flat rows: every level stays below 1
    sc, _ = ms.scores_op(dev(L), 4, "gradtopk")
    ref = oracle.gradtopk(L.astype(np.float64), 4)
    assert np.isfinite(ref).all()
    assert np.allclose(sc.cpu().numpy(), ref, rtol=1e-5, atol=1e-7)
    # the edge of the domain that the size checks (k <= E) leave reachable: two equally likely experts reach
    # exactly 1 at level 2
    L2 = np.zeros((4, 2), dtype=np.float32)
    assert np.allclose(ms.scores_op(dev(L2), 2, "gradtopk")[0].cpu().numpy(), 1.0)
    assert np.allclose(oracle.gradtopk(L2.astype(np.float64), 2), 1.0)


def test_itertopk_deeper_levels_away_from_the_pole(ms):
    print("itertopk k=4", flush=True)
    rng = np.random.default_rng(12)
    L = (0.3 * rng.normal(size=(2000, 64))).astype(np.float32)     # flat rows: 1 - y stays positive for k << E
    sc, _ = ms.scores_op(dev(L), 4, "itertopk")
    ref = oracle.itertopk(L.astype(np.float64), 4)
    assert (ref < 1).all()
    assert np.allclose(sc.cpu().numpy(), ref, rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("op", ["sigmoid", "softkmax"])
def test_operator_scores_route_through_the_exact_solver(ms, op):
    print(f"route with {op}", flush=True)
    c = CONFIGS["cfg2"]
    L = make_logits("cfg2", 0)
    sc, q = ms.scores_op(dev(L), c["k"], op)
    out = ms.assign_i32(q, c["k"], c["C"])
    ref = oracle.max_score_assignment(q.cpu().numpy().astype(np.int64), c["k"], c["C"])
    assert out["stats"]["total_score_q"] == ref["total"]
    g = ms.gates(sc, out["assign"])
    assert np.allclose(g.cpu().numpy(), oracle.gates(sc.cpu().numpy().astype(np.float64), out["assign"].cpu().numpy()),
                       rtol=1e-6)
