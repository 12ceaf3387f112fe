"""GPU parity of Algorithm 1 with Sinkhorn on the residual problem through the C ABI: the fp32 plan against the
fp64 checker, and the rounded choice checked for validity (it must be a maximiser of the checker's plan row up
to the plan's tolerance; where the maximiser is clear it must be the same expert)."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, make_logits

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


def compare(ms, A32, C, tau, n_iter, rtol):
    out = ms.assign_top1_sinkhorn(dev(A32), C, tau, n_iter, want_plan=True)
    ref = oracle.top1_then_sinkhorn(A32.astype(np.float64), C, tau, n_iter)
    a = out["assign"].cpu().numpy()
    plan = out["plan"].cpu().numpy().astype(np.float64)
    assert np.array_equal(a[:, 0], ref["assign"][:, 0])
    assert out["caps"] == ref["caps"].tolist()
    scale = ref["plan"].max(axis=1, keepdims=True)
    assert (np.abs(plan - ref["plan"]) <= rtol * scale + 1e-30).all()
    rows = np.arange(a.shape[0])
    chosen = ref["plan"][rows, np.maximum(a[:, 1], 0)]
    assert ((a[:, 1] >= 0) == (ref["assign"][:, 1] >= 0)).all()
    ok = a[:, 1] >= 0
    assert (chosen[ok] >= (1 - 2 * rtol) * scale[ok, 0]).all()             # a maximiser up to the tolerance
    srt = np.sort(ref["plan"], axis=1)
    clear = ok & (srt[:, -2] < (1 - 4 * rtol) * srt[:, -1])
    assert np.array_equal(a[clear, 1], ref["assign"][clear, 1])            # and the same one when it is clear
    assert clear.mean() > 0.9
    return out, ref


@pytest.mark.parametrize("T,E,C,tau,n_iter", [
    (300, 8, 75, 0.1, 0), (300, 8, 75, 0.1, 10), (1000, 16, 125, 0.05, 30), (4099, 64, 129, 0.05, 20),
    (257, 7, 74, 0.2, 5), (2048, 128, 32, 0.05, 15), (700, 300, 5, 0.1, 8), (513, 1024, 2, 0.1, 3),
])
def test_plan_and_choice_match_the_checker(ms, T, E, C, tau, n_iter):
    print(f"sinkhorn T={T} E={E} C={C} tau={tau} n={n_iter}", flush=True)
    rng = np.random.default_rng(T + E)
    L = rng.normal(size=(T, E)) + 0.5 * rng.normal(size=(1, E))
    A32 = oracle.soft_topk(L, 2, 1.0).astype(np.float32)
    compare(ms, A32, C, tau, n_iter, rtol=2e-4)


def test_cfg2_balances_the_second_choices(ms):
    print("sinkhorn cfg2", flush=True)
    c = CONFIGS["cfg2"]
    A32 = oracle.soft_topk(make_logits("cfg2", 0), 2, 1.0).astype(np.float32)
    out, ref = compare(ms, A32, c["C"], 0.05, 50, rtol=5e-4)
    a = out["assign"].cpu().numpy()
    caps = np.array(out["caps"])
    load2 = np.bincount(a[:, 1][a[:, 1] >= 0], minlength=c["E"])
    plain = ms.assign_top1_sinkhorn(dev(A32), c["C"], 0.05, 0)["assign"].cpu().numpy()
    load2_plain = np.bincount(plain[:, 1], minlength=c["E"])
    assert np.maximum(0, load2 - caps).sum() < np.maximum(0, load2_plain - caps).sum()


def test_repeatable_and_validated(ms):
    print("sinkhorn repeat", flush=True)
    rng = np.random.default_rng(2)
    A32 = oracle.soft_topk(rng.normal(size=(3000, 32)), 2, 1.0).astype(np.float32)
    a = ms.assign_top1_sinkhorn(dev(A32), 200, 0.05, 25, want_plan=True)
    b = ms.assign_top1_sinkhorn(dev(A32), 200, 0.05, 25, want_plan=True)
    assert torch.equal(a["plan"], b["plan"]) and torch.equal(a["assign"], b["assign"])
    with pytest.raises(ms.MaxScoreError):
        ms.assign_top1_sinkhorn(dev(A32), 200, 0.0, 5)
    with pytest.raises(ms.MaxScoreError):
        ms.assign_top1_sinkhorn(dev(A32), 200, 0.1, -1)
