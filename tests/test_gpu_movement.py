"""GPU parity of the activation movement around the experts (expert input buffers, Eq. 1 combine) through
the C ABI: the dispatch is a byte copy (bit-exact), the combine is checked against the fp64 checker."""
import numpy as np
import pytest

import oracle
from workloads import bf16_bits, bf16_from_bits

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


def routed_case(ms, T, E, k, C, seed):
    """A feasible assignment with gates from the GPU path itself (its parity is tested elsewhere)."""
    rng = np.random.default_rng(seed)
    L = rng.normal(size=(T, E)).astype(np.float32) + (2.0 * rng.normal(size=(1, E))).astype(np.float32)
    out = ms.route_logits(dev(L), k, C, t=1.0)
    return out, rng


@pytest.mark.parametrize("T,d,E,k,C,dtype", [
    (300, 64, 8, 2, 80, "fp32"), (1000, 256, 16, 4, 260, "bf16"), (4099, 2048, 64, 8, 520, "bf16"),
    (257, 100, 7, 3, 120, "bf16"),      # 200-byte rows: not a whole number of 16-byte vectors
    (513, 33, 5, 2, 300, "fp32"),       # odd row length, slack capacity (zero padding)
    (64, 4096, 128, 8, 4, "bf16"),      # rows longer than one pass of the combine kernel
])
def test_dispatch_tokens_and_combine(ms, T, d, E, k, C, dtype):
    print(f"movement T={T} d={d} E={E} k={k} C={C} {dtype}", flush=True)
    out, rng = routed_case(ms, T, E, k, C, seed=T + d)
    assign = out["assign"].cpu().numpy()
    pos = out["token_pos"].cpu().numpy()
    gates = out["gates"].cpu().numpy()
    off = out["expert_offsets"].cpu().numpy()
    tok = out["disp_token"].cpu().numpy()
    x = rng.normal(size=(T, d)).astype(np.float32)
    if dtype == "bf16":
        xb = bf16_bits(x)
        x_ref = bf16_from_bits(xb).astype(np.float64)
        x_dev = dev(xb.view(np.int16)).view(torch.bfloat16)
    else:
        x_ref = x.astype(np.float64)
        x_dev = dev(x)
    buf = ms.dispatch_tokens(x_dev, out["expert_offsets"], out["disp_token"], E, C)
    ref_buf = oracle.dispatch_tokens(x_ref, off, tok, E, C)
    got = buf.float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref_buf)                               # a copy: exact, padding included

    # expert outputs = arbitrary function of the inputs (here: scaled and shifted per expert)
    scale = rng.normal(size=(E, 1, 1)).astype(np.float32)
    eo = (got * scale + 0.25).astype(np.float32)
    if dtype == "bf16":
        eob = bf16_bits(eo)
        eo_ref = bf16_from_bits(eob).astype(np.float64)
        eo_dev = dev(eob.view(np.int16)).view(torch.bfloat16)
    else:
        eo_ref = eo.astype(np.float64)
        eo_dev = dev(eo)
    y = ms.combine(eo_dev, out["assign"], out["token_pos"], out["gates"]).cpu().numpy()
    y_ref = oracle.combine(eo_ref, assign, pos, gates.astype(np.float64))
    # k fused multiply-adds in fp32 against fp64: a few ulp of the largest term
    bound = 1e-6 * (np.abs(gates.astype(np.float64))[:, :, None] * np.abs(eo_ref[assign, pos])).sum(axis=1) + 1e-30
    assert (np.abs(y - y_ref) <= bound).all()


def test_identity_experts_return_gate_sum_times_x(ms):
    print("movement identity", flush=True)
    T, d, E, k, C = 2048, 512, 32, 4, 256
    out, rng = routed_case(ms, T, E, k, C, seed=5)
    x = rng.normal(size=(T, d)).astype(np.float32)
    buf = ms.dispatch_tokens(dev(x), out["expert_offsets"], out["disp_token"], E, C)
    y = ms.combine(buf, out["assign"], out["token_pos"], out["gates"]).cpu().numpy()
    gsum = out["gates"].cpu().numpy().astype(np.float64).sum(axis=1)
    assert np.allclose(y, gsum[:, None] * x, rtol=2e-6, atol=1e-7)


def test_movement_at_the_headline_size(ms):
    """T=65536, d=2048, E=128, k=8, C=4096, bf16 (the shapes the benchmark times): the expert input buffers of
    sampled experts and the combined rows of sampled tokens against the checker, which gets the sub-problem of
    exactly those experts / tokens; plus two properties over all rows (every filled slot is a bit copy of its
    token's row; identity experts return the gate sum times x)."""
    print("movement headline size", flush=True)
    T, d, E, k, C = 65536, 2048, 128, 8, 4096
    out, rng = routed_case(ms, T, E, k, C, seed=11)
    off = out["expert_offsets"].cpu().numpy()
    tok = out["disp_token"].cpu().numpy()
    xb = bf16_bits(rng.standard_normal((T, d), dtype=np.float32))
    x_dev = dev(xb.view(np.int16)).view(torch.bfloat16)
    buf = ms.dispatch_tokens(x_dev, out["expert_offsets"], out["disp_token"], E, C)
    assert tuple(buf.shape) == (E, C, d)
    # sampled experts: the checker on the sub-problem made of their segments of the dispatch list
    es = np.array([0, 1, 37, 64, 126, 127])
    seg = [tok[off[e]:off[e + 1]] for e in es]
    off_sub = np.concatenate([[0], np.cumsum([len(s) for s in seg])]).astype(off.dtype)
    ref = oracle.dispatch_tokens(bf16_from_bits(xb).astype(np.float64), off_sub, np.concatenate(seg), len(es), C)
    got = buf[torch.from_numpy(es).cuda()].float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)
    # all experts: filled slots are bit copies, the rest is zero
    bits = buf.view(torch.int16)
    for e in range(E):
        n = int(off[e + 1] - off[e])
        rows = torch.from_numpy(tok[off[e]:off[e + 1]].astype(np.int64)).cuda()
        assert torch.equal(bits[e, :n], x_dev.view(torch.int16)[rows])
        assert not bits[e, n:].any()

    # expert outputs: a different scale per expert (exact in bf16: powers of two), applied on the device
    scale = torch.from_numpy((2.0 ** rng.integers(-2, 3, E)).astype(np.float32)).cuda()
    eo = (buf.float() * scale[:, None, None]).to(torch.bfloat16)
    y = ms.combine(eo, out["assign"], out["token_pos"], out["gates"])
    rows = np.concatenate([np.random.default_rng(12).choice(T, 512, replace=False), [0, 1, T - 2, T - 1]])
    ri = torch.from_numpy(rows).cuda()
    a_s, p_s = out["assign"][ri].long(), out["token_pos"][ri].long()
    eo_sub = eo[a_s, p_s].float().cpu().numpy().astype(np.float64)          # [n, k, d]: one "expert" per sampled token
    g_s = out["gates"][ri].cpu().numpy().astype(np.float64)
    n = len(rows)
    y_ref = oracle.combine(eo_sub, np.repeat(np.arange(n)[:, None], k, axis=1), np.tile(np.arange(k), (n, 1)), g_s)
    bound = 1e-6 * (np.abs(g_s)[:, :, None] * np.abs(eo_sub)).sum(axis=1) + 1e-30
    assert (np.abs(y[ri].cpu().numpy() - y_ref) <= bound).all()
    # all rows: with identity experts the combine returns (sum of the gates) * x
    y1 = ms.combine(buf, out["assign"], out["token_pos"], out["gates"])
    want = out["gates"].double().sum(dim=1, keepdim=True) * x_dev.double()
    assert torch.allclose(y1.double(), want, rtol=2e-6, atol=1e-7)


def test_movement_argument_errors(ms):
    x = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    off = torch.zeros(3, dtype=torch.int32, device="cuda")
    tok = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(ms.MaxScoreError):
        ms.dispatch_tokens(x, off, tok, 2000, 4)            # more experts than supported
    with pytest.raises(TypeError):
        ms.dispatch_tokens(x.double(), off, tok, 2, 4)      # unsupported element type
