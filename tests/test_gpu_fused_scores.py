"""GPU parity of a1 + a2 + a3 computed in one kernel (the SoftTopk scores of Eq. 6 and the integer rewards come out of
the projection's accumulators, Eq. 2): bit-equal to the projection kernel followed by the score kernel, and within
the path's bars of the CPU checker."""
import numpy as np
import pytest

import oracle
from workloads import make_inputs

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


def bf16_inputs(rng, T, d, E):
    x = rng.standard_normal((T, d)).astype(np.float32)
    W = (rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32)
    xb = torch.from_numpy(x).to(torch.bfloat16)
    Wb = torch.from_numpy(W).to(torch.bfloat16)
    return xb, Wb, xb.to(torch.float32).numpy().astype(np.float64), Wb.to(torch.float32).numpy().astype(np.float64)


@pytest.mark.parametrize("T,d,E,k,t,with_bias", [(128, 64, 32, 2, 1.0, False), (1000, 256, 64, 8, 1.0, True),
                                                  (129, 128, 128, 8, 4.0, True), (4097, 512, 128, 8, 1.0, False),
                                                  (31, 64, 128, 1, 1.0, True), (300, 192, 64, 64, 0.5, True),
                                                  (257, 2048, 128, 8, 0.0, True)])
def test_fused_equals_two_kernels_and_checker(ms, T, d, E, k, t, with_bias):
    print(f"fused scores T={T} d={d} E={E} k={k} t={t}", flush=True)
    rng = np.random.default_rng(T + d + E)
    xb, Wb, x64, W64 = bf16_inputs(rng, T, d, E)
    bias = rng.standard_normal(E).astype(np.float32) if with_bias else None
    xd, Wd = xb.cuda(), Wb.cuda()
    bd = dev(bias) if with_bias else None
    fused = ms.router_softtopk(xd, Wd, bd, k, t)
    nolog = ms.router_softtopk(xd, Wd, bd, k, t, want_logits=False)
    logits = ms.router_logits(xd, Wd, bd)
    scores, q = ms.softtopk(logits, k, t)
    # the same values from the same instructions: bit-equal, with and without the logits being written
    assert torch.equal(fused["logits"], logits)
    assert torch.equal(fused["scores"], scores) and torch.equal(fused["q"], q)
    assert nolog["logits"] is None
    assert torch.equal(nolog["scores"], scores) and torch.equal(nolog["q"], q)
    # against the checker: logits within the projection's bar, scores from the kernel's own logits within 1e-5
    ref = oracle.router_logits(x64, W64, bias)
    L = logits.cpu().numpy()
    assert (np.abs(L - ref) / np.maximum(np.abs(ref), 1.0)).max() <= 2e-2
    A = oracle.soft_topk(L.astype(np.float64), k, t)
    S = fused["scores"].cpu().numpy()
    assert np.all(np.abs(S - A) <= 1e-5 * np.abs(A) + 1e-12)
    assert np.array_equal(fused["q"].cpu().numpy(), np.rint(S.astype(np.float64) * 2.0 ** 20).astype(np.int64))


def test_shapes_the_fused_kernel_does_not_take(ms):
    """E = 16 (cfg2) and fp32 inputs go through the two kernels: logits required, results as before."""
    print("fused scores fallback", flush=True)
    rng = np.random.default_rng(3)
    xb, Wb, _, _ = bf16_inputs(rng, 200, 128, 16)
    out = ms.router_softtopk(xb.cuda(), Wb.cuda(), None, 2, 1.0)
    logits = ms.router_logits(xb.cuda(), Wb.cuda(), None)
    scores, q = ms.softtopk(logits, 2, 1.0)
    assert torch.equal(out["logits"], logits) and torch.equal(out["scores"], scores) and torch.equal(out["q"], q)
    with pytest.raises(ms.MaxScoreError) as e:
        ms.router_softtopk(xb.cuda(), Wb.cuda(), None, 2, 1.0, want_logits=False)
    assert e.value.code == -1
    x32 = rng.standard_normal((64, 64)).astype(np.float32)
    W32 = rng.standard_normal((64, 32)).astype(np.float32)
    out = ms.router_softtopk(dev(x32), dev(W32), None, 2, 1.0)
    s2, q2 = ms.softtopk(ms.router_logits(dev(x32), dev(W32), None), 2, 1.0)
    assert torch.equal(out["scores"], s2) and torch.equal(out["q"], q2)


def test_route_xw_without_logits_at_the_headline_size(ms):
    """The whole path at the benchmark's shapes without a logits buffer: scores, rewards, assignment total and
    dispatch lists equal to the call that also writes the logits."""
    print("route_xw no logits cfg5", flush=True)
    r = make_inputs("cfg5")
    xd = dev(r.x_bits.view(np.int16)).view(torch.bfloat16)
    Wd = dev(r.W_bits.view(np.int16)).view(torch.bfloat16)
    bd = dev(r.bias)
    a = ms.route_xw(xd, Wd, bd, r.k, r.C, t=r.t)
    b = ms.route_xw(xd, Wd, bd, r.k, r.C, t=r.t, want_logits=False)
    assert b["logits"] is None
    assert torch.equal(a["scores"], b["scores"]) and torch.equal(a["q"], b["q"])
    assert a["stats"]["total_score_q"] == b["stats"]["total_score_q"]
    assert torch.equal(a["assign"], b["assign"]) and torch.equal(a["disp_token"], b["disp_token"])
    # and the two-kernel form gives the same scores
    logits = ms.router_logits(xd, Wd, bd)
    assert torch.equal(logits, a["logits"])
    s2, q2 = ms.softtopk(logits, r.k, r.t)
    assert torch.equal(s2, a["scores"]) and torch.equal(q2, a["q"])
