"""GPU parity of the training-side by-products through the C ABI: the Eq. 9 load-balance loss and the
derivative of the gates with respect to the logits, against the fp64 checker on the same fp32 inputs."""
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


def routed(ms, L, k, C, t):
    out = ms.route_logits(dev(L), k, C, t=t)
    return out


CASES = [(300, 8, 2, 80, 1.0), (1000, 16, 4, 260, 0.5), (4099, 64, 8, 520, 1.0), (257, 7, 3, 120, 2.0),
         (2048, 128, 8, 130, 1.0), (1500, 300, 6, 31, 1.0), (700, 1024, 64, 44, 1.0), (65, 5, 5, 65, 0.0)]


@pytest.mark.parametrize("T,E,k,C,t", CASES)
def test_aux_loss(ms, T, E, k, C, t):
    print(f"aux loss T={T} E={E} k={k} C={C}", flush=True)
    rng = np.random.default_rng(T + E)
    L = (rng.normal(size=(T, E)) + 1.5 * rng.normal(size=(1, E))).astype(np.float32)
    out = routed(ms, L, k, C, t)
    lam = 0.01
    got = ms.aux_loss(out["scores"], out["expert_offsets"], lam)
    ref = oracle.aux_loss(out["scores"].cpu().numpy().astype(np.float64), out["assign"].cpu().numpy(), lam)
    assert np.isclose(got["loss"].item(), ref["loss"], rtol=1e-5, atol=0)
    assert np.allclose(got["mean_scores"].cpu().numpy(), ref["mean_A"], rtol=1e-5, atol=1e-12)
    assert np.allclose(got["dscores_col"].cpu().numpy(), ref["dA"], rtol=1e-6, atol=0)
    again = ms.aux_loss(out["scores"], out["expert_offsets"], lam)
    assert again["loss"].item() == got["loss"].item()                  # fixed summation order


@pytest.mark.parametrize("T,E,k,C,t", CASES)
def test_gates_backward(ms, T, E, k, C, t):
    print(f"gates backward T={T} E={E} k={k} C={C} t={t}", flush=True)
    rng = np.random.default_rng(7 * T + E)
    L = (rng.normal(size=(T, E)) + 1.5 * rng.normal(size=(1, E))).astype(np.float32)
    out = routed(ms, L, k, C, t)
    assign = out["assign"].cpu().numpy()
    dgate = rng.normal(size=(T, k)).astype(np.float32)
    dcol = (rng.normal(size=E) * 0.1).astype(np.float32)
    for col in (None, dcol):
        got = ms.gates_backward(dev(L), out["scores"], out["assign"], dev(dgate),
                                dev(col) if col is not None else None).cpu().numpy()
        ref = oracle.gates_backward(L.astype(np.float64), k, t, assign, dgate.astype(np.float64),
                                    col.astype(np.float64) if col is not None else None)
        # per-row scale of the terms that are added: sum_j |gA_ij * A_ij|
        A = oracle.soft_topk(L.astype(np.float64), k, t)
        gA = np.zeros((T, E))
        for s in range(k):
            ok = assign[:, s] >= 0
            np.add.at(gA, (np.nonzero(ok)[0], assign[ok, s]), dgate[ok, s].astype(np.float64))
        if col is not None:
            gA += col.astype(np.float64)[None, :]
        scale = np.abs(gA * A).sum(axis=1, keepdims=True)
        assert (np.abs(got - ref) <= 1e-5 * scale + 1e-30).all()


def test_backward_with_holes_and_full_size(ms):
    print("gates backward cfg5 sample", flush=True)
    c = CONFIGS["cfg5"]
    L = make_logits("cfg5", 0)
    out = routed(ms, L, c["k"], c["C"], c["t"])
    a = out["assign"].clone()
    a[::3, 1] = -1                                                      # empty slots contribute nothing
    rng = np.random.default_rng(1)
    dgate = rng.normal(size=(c["T"], c["k"])).astype(np.float32)
    aux = ms.aux_loss(out["scores"], out["expert_offsets"], 0.01)
    got = ms.gates_backward(dev(L), out["scores"], a, dev(dgate), aux["dscores_col"]).cpu().numpy()
    rows = rng.choice(c["T"], 512, replace=False)
    ref = oracle.gates_backward(L[rows].astype(np.float64), c["k"], c["t"], a.cpu().numpy()[rows],
                                dgate[rows].astype(np.float64), aux["dscores_col"].cpu().numpy().astype(np.float64))
    assert np.allclose(got[rows], ref, rtol=0, atol=1e-5 * np.abs(ref).max())
    ref_loss = oracle.aux_loss(out["scores"].cpu().numpy().astype(np.float64), out["assign"].cpu().numpy(), 0.01)
    assert np.isclose(aux["loss"].item(), ref_loss["loss"], rtol=1e-5)
