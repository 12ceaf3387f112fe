"""GPU parity: every step of the HIP path against the CPU checker, through the C ABI binding."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, capacity, make_inputs, make_logits

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ms():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2508_12801_amd as m
    m.load_library()
    return m


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def cfg_case(name, T=None):
    cfg = CONFIGS[name]
    L = make_logits(name, T=T)
    T = L.shape[0]
    E, k = cfg["E"], cfg["k"]
    C = cfg["C"] if T == cfg["T"] else capacity(T, E, k, cfg["C"] * E / (cfg["T"] * k))
    return L, E, k, C, cfg["t"]


# ---- a2 + a3 ------------------------------------------------------------------------------------

@pytest.mark.parametrize("T,E,k,t", [(64, 8, 2, 0.0), (300, 16, 2, 1.0), (257, 64, 8, 1.0), (1000, 128, 8, 1.0),
                                      (130, 128, 8, 4.0), (77, 5, 3, 1.0), (50, 100, 7, 0.5), (33, 200, 16, 1.0),
                                      (9, 1000, 64, 1.0), (40, 12, 12, 2.0), (1, 8, 1, 1.0), (65536, 128, 8, 1.0)])
def test_softtopk(ms, T, E, k, t):
    print(f"softtopk T={T} E={E} k={k} t={t}", flush=True)
    rng = np.random.default_rng(T * 1000 + E)
    L = (rng.standard_normal((T, E)) * 1.5).astype(np.float32)
    if T > 8:
        L[3] = L[2]                      # duplicated row
        L[5, : E // 2] = L[5, 0]         # ties inside a row: lower index must rank first
    scores, q = ms.softtopk(dev(L), k, t)
    scores, q = scores.cpu().numpy(), q.cpu().numpy()
    ref = oracle.soft_topk(L.astype(np.float64), k, t)
    assert np.all(np.abs(scores - ref) <= 1e-5 * np.abs(ref) + 1e-12)
    # the integer decision is taken in the kernel's own precision: exact round-half-even of its fp32 score
    assert np.array_equal(q, np.rint(scores.astype(np.float64) * 2.0 ** 20).astype(np.int64))
    qo = oracle.quantise(ref)
    assert np.all(np.abs(q - qo) <= np.maximum(2, 2e-5 * qo))       # element by element


@pytest.mark.parametrize("reading", ["A", "A1", "B", "C"])
@pytest.mark.parametrize("T,E,k,t", [(300, 16, 2, 1.0), (257, 64, 8, 1.0), (1000, 128, 8, 4.0), (77, 5, 3, 1.0),
                                      (50, 100, 7, 0.5), (33, 200, 16, 1.0), (40, 12, 12, 2.0), (9, 8, 1, 1.0)])
def test_softtopk_other_readings(ms, reading, T, E, k, t):
    """The other readings of Eq. 6 (maxscore_softtopk_reading) against the checker's recursions, same bars as the
    reading the path uses; reading A through this entry is bit-equal to maxscore_softtopk."""
    print(f"softtopk reading {reading} T={T} E={E} k={k} t={t}", flush=True)
    rng = np.random.default_rng(T * 1000 + E)
    L = (rng.standard_normal((T, E)) * 1.5).astype(np.float32)
    L[3] = L[2]
    L[5, : E // 2] = L[5, 0]
    scores, q = ms.softtopk(dev(L), k, t, reading=reading)
    scores, q = scores.cpu().numpy(), q.cpu().numpy()
    ref = oracle.soft_topk_reading(L.astype(np.float64), k, t, reading)
    assert np.all(np.abs(scores - ref) <= 1e-5 * np.abs(ref) + 1e-12)
    assert np.array_equal(q, np.rint(scores.astype(np.float64) * 2.0 ** 20).astype(np.int64))
    qo = oracle.quantise(ref)
    assert np.all(np.abs(q - qo) <= np.maximum(2, 2e-5 * qo))
    if reading == "A":
        s0, q0 = ms.softtopk(dev(L), k, t)
        assert np.array_equal(s0.cpu().numpy(), scores) and np.array_equal(q0.cpu().numpy(), q)


# ---- a4 -----------------------------------------------------------------------------------------

def check_assignment(ms, q64, k, C, ref_total=None, **kw):
    T, E = q64.shape
    out = ms.assign_i32(dev(q64.astype(np.int32)), k, C, **kw)
    a = out["assign"].cpu().numpy()
    P = oracle.assignment_matrix(a, E)
    ok, why = oracle.check_feasible(P, k, C)
    assert ok, why
    total = int(q64[P.astype(bool)].sum())
    st = out["stats"]
    assert st["total_score_q"] == total and st["flow_value"] == int(P.sum()) and st["status"] == 0
    if ref_total is None:
        ref_total = oracle.max_score_assignment(q64, k, C)["total"]
    assert total == ref_total, (total, ref_total, st)
    # dual side: scaled prices, eps = 1 complementary slackness, unfilled experts at price 0
    S = out["price_scale"]
    p = out["prices"].cpu().numpy()
    assert S > E and (p >= 0).all()
    load = P.sum(axis=0)
    assert (p[load < min(C, T)] == 0).all()
    net = q64 * S - p[None, :]
    big = np.int64(1) << 60
    held_min = np.where(P.astype(bool), net, big).min(axis=1)
    unheld_max = np.where(P.astype(bool), -big, net).max(axis=1)
    assert (held_min >= unheld_max - 1).all()
    return out


@pytest.mark.parametrize("T,E,k,C,kind", [
    (6, 3, 2, 4, "uniform"), (100, 5, 2, 40, "uniform"), (257, 7, 3, 111, "ties"), (64, 8, 8, 64, "uniform"),
    (50, 9, 3, 50, "uniform"), (333, 16, 2, 42, "rows_equal"), (1, 4, 2, 1, "uniform"), (200, 1, 1, 200, "uniform"),
    (513, 33, 5, 78, "signed"), (1000, 130, 9, 70, "uniform"), (96, 12, 3, 24, "ties"), (400, 300, 17, 23, "uniform"),
])
def test_assign_small(ms, T, E, k, C, kind):
    print(f"assign_small T={T} E={E} k={k} C={C} {kind}", flush=True)
    rng = np.random.default_rng(T + 7 * E)
    if kind == "uniform":
        q = rng.integers(0, 1 << 20, (T, E))
    elif kind == "ties":
        q = rng.integers(0, 4, (T, E))
    elif kind == "rows_equal":
        q = np.tile(rng.integers(0, 1 << 20, (1, E)), (T, 1))
    else:
        q = rng.integers(-(1 << 19), 1 << 19, (T, E))
    check_assignment(ms, q.astype(np.int64), k, C)


def test_flow_first_fixture(ms):
    """Section 3.2 / Table 1: the maximum flow comes before the maximum score.  The fixture is tight
    (T*k = E*C = 6): the best matrix with 5 ones scores 410, the answer is the best one with 6 ones, 312."""
    import os
    q = np.loadtxt(os.path.join(os.path.dirname(__file__), "golden", "flow_first_example.txt"), comments="#",
                   dtype=np.int64)
    out = check_assignment(ms, q, 2, 2, ref_total=312)
    assert out["stats"]["flow_value"] == 6 and out["stats"]["total_score_q"] == 312


@pytest.mark.parametrize("name,T", [("cfg1", None), ("cfg2", None), ("cfg3", 2048), ("cfg4a", 2048),
                                     ("cfg4b_exact", 2048), ("cfg4b_near", 2048), ("cfg5", 4096)])
def test_assign_configs_reduced(ms, name, T):
    print(f"assign_cfg {name} T={T}", flush=True)
    L, E, k, C, t = cfg_case(name, T)
    q = oracle.quantise(oracle.soft_topk(L, k, t))
    out = check_assignment(ms, q, k, C)
    if L.shape[0] * k == E * C:
        a = out["assign"].cpu().numpy()
        assert (np.bincount(a.reshape(-1), minlength=E) == C).all()      # every expert exactly full


@pytest.mark.parametrize("name", ["cfg3", "cfg4a", "cfg4b_exact", "cfg4b_near", "cfg5"])
def test_assign_configs_full(ms, name):
    print(f"assign_full {name}", flush=True)
    L, E, k, C, t = cfg_case(name)
    q = oracle.quantise(oracle.soft_topk(L, k, t))
    out = check_assignment(ms, q, k, C)
    print(name, out["stats"], flush=True)
    v = oracle.verify_optimal(q, oracle.assignment_matrix(out["assign"].cpu().numpy(), E), k, C)
    assert v["optimal"]


# ---- a5, a6 -------------------------------------------------------------------------------------

@pytest.mark.parametrize("T,E,k", [(37, 5, 3), (1000, 16, 2), (4099, 64, 8), (70000, 128, 8), (3, 1000, 64)])
def test_gates_and_dispatch(ms, T, E, k):
    print(f"dispatch T={T} E={E} k={k}", flush=True)
    rng = np.random.default_rng(T)
    assign = np.full((T, k), -1, dtype=np.int32)
    for i in range(T):
        n = k if i % 7 else rng.integers(0, k + 1)
        assign[i, :n] = rng.permutation(E)[:n]
        rng.shuffle(assign[i])
    scores = rng.random((T, E)).astype(np.float32)
    g = ms.gates(dev(scores), dev(assign)).cpu().numpy()
    gref = oracle.gates(scores.astype(np.float64), assign)
    assert np.array_equal(g.astype(np.float64), gref)
    d = ms.dispatch(dev(assign), dev(g), E)
    ref = oracle.dispatch(assign, g, E)
    n = int(ref["expert_offsets"][-1])
    assert np.array_equal(d["expert_offsets"].cpu().numpy(), ref["expert_offsets"])
    assert np.array_equal(d["disp_token"].cpu().numpy()[:n], ref["disp_token"])
    assert np.array_equal(d["disp_gate"].cpu().numpy()[:n], ref["disp_gate"].astype(np.float32))
    assert np.array_equal(d["token_pos"].cpu().numpy(), ref["token_pos"])


# ---- a1 -----------------------------------------------------------------------------------------

@pytest.mark.parametrize("T,d,E,dtype", [(64, 64, 8, "fp32"), (300, 1024, 16, "bf16"), (257, 2048, 64, "bf16"),
                                         (1000, 2048, 128, "bf16"), (129, 200, 100, "bf16"), (70, 67, 9, "bf16"),
                                         (130, 512, 300, "bf16")])
def test_router_logits(ms, T, d, E, dtype):
    print(f"gemm T={T} d={d} E={E} {dtype}", flush=True)
    rng = np.random.default_rng(d + E)
    x = rng.standard_normal((T, d)).astype(np.float32)
    W = (rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32)
    b = rng.standard_normal(E).astype(np.float32)
    if dtype == "bf16":
        from workloads import bf16_bits, bf16_from_bits
        xb, Wb = bf16_bits(x), bf16_bits(W)
        x, W = bf16_from_bits(xb), bf16_from_bits(Wb)
        xd = dev(xb.view(np.int16)).view(torch.bfloat16)
        Wd = dev(Wb.view(np.int16)).view(torch.bfloat16)
    else:
        xd, Wd = dev(x), dev(W)
    out = ms.router_logits(xd, Wd, dev(b)).cpu().numpy()
    ref = oracle.router_logits(x, W, b)
    err = np.abs(out - ref) / np.maximum(np.abs(ref), 1.0)
    assert err.max() <= 2e-2, err.max()
    assert err.max() <= 1e-4          # fp32 accumulation of exact bf16 products is far tighter than the bar
    out2 = ms.router_logits(xd, Wd, None).cpu().numpy()
    assert np.allclose(out2 + b[None, :], out, atol=1e-5)


# ---- whole path ---------------------------------------------------------------------------------

@pytest.mark.parametrize("name,T", [("cfg1", None), ("cfg2", None), ("cfg3", 3000), ("cfg4b_near", 1500)])
def test_route_xw_end_to_end(ms, name, T):
    print(f"route_xw {name} T={T}", flush=True)
    r = make_inputs(name, T=T)
    if r.dtype == "bf16":
        xd = dev(r.x_bits.view(np.int16)).view(torch.bfloat16)
        Wd = dev(r.W_bits.view(np.int16)).view(torch.bfloat16)
    else:
        xd, Wd = dev(r.x), dev(r.W)
    bd = dev(r.bias) if r.bias is not None else None
    out = ms.route_xw(xd, Wd, bd, r.k, r.C, t=r.t)
    logits = out["logits"].cpu().numpy()
    refL = oracle.router_logits(r.x, r.W, r.bias)
    assert (np.abs(logits - refL) / np.maximum(np.abs(refL), 1.0)).max() <= 2e-2
    # from here on the checker follows the GPU's own fp32 logits (the gate bar is on a2..a6)
    A = oracle.soft_topk(logits.astype(np.float64), r.k, r.t)
    scores = out["scores"].cpu().numpy()
    assert np.all(np.abs(scores - A) <= 1e-5 * np.abs(A) + 1e-12)
    q = out["q"].cpu().numpy().astype(np.int64)
    assign = out["assign"].cpu().numpy()
    P = oracle.assignment_matrix(assign, r.E)
    ok, why = oracle.check_feasible(P, r.k, r.C)
    assert ok, why
    # second half of the two-matrix protocol: the GPU's own integer rewards, solved by the checker
    ref = oracle.max_score_assignment(q, r.k, r.C)
    assert int(q[P.astype(bool)].sum()) == ref["total"] == out["stats"]["total_score_q"]
    g = out["gates"].cpu().numpy()
    gref = oracle.gates(A, assign)
    assert np.all(np.abs(g - gref) <= 1e-5 * np.abs(gref) + 1e-12)
    d = oracle.dispatch(assign, g, r.E)
    assert np.array_equal(out["expert_offsets"].cpu().numpy(), d["expert_offsets"])
    assert np.array_equal(out["disp_token"].cpu().numpy(), d["disp_token"])
    assert np.array_equal(out["disp_gate"].cpu().numpy(), d["disp_gate"].astype(np.float32))
    assert np.array_equal(out["token_pos"].cpu().numpy(), d["token_pos"])


@pytest.mark.parametrize("name,T", [("cfg2", None), ("cfg3", 3000), ("cfg4a", 2000)])
def test_route_scores_end_to_end(ms, name, T):
    """The entry that starts from given affinities (a3..a6): rewards are the rounding of the given scores, the
    assignment is the checker's optimum on them, gates are the given scores at the assigned experts."""
    print(f"route_scores {name} T={T}", flush=True)
    L, E, k, C, t = cfg_case(name, T)
    A32 = oracle.soft_topk(L.astype(np.float64), k, t).astype(np.float32)
    out = ms.route_scores(dev(A32), k, C)
    q = out["q"].cpu().numpy().astype(np.int64)
    assert np.array_equal(q, oracle.quantise(A32))
    assign = out["assign"].cpu().numpy()
    P = oracle.assignment_matrix(assign, E)
    ok, why = oracle.check_feasible(P, k, C)
    assert ok, why
    ref = oracle.max_score_assignment(q, k, C)
    assert int(P.sum()) == ref["flow"] == out["stats"]["flow_value"]
    assert int(q[P.astype(bool)].sum()) == ref["total"] == out["stats"]["total_score_q"]
    g = out["gates"].cpu().numpy()
    assert np.array_equal(g.astype(np.float64), oracle.gates(A32.astype(np.float64), assign))
    d = oracle.dispatch(assign, g, E)
    assert np.array_equal(out["expert_offsets"].cpu().numpy(), d["expert_offsets"])
    assert np.array_equal(out["disp_token"].cpu().numpy(), d["disp_token"])
    assert np.array_equal(out["disp_gate"].cpu().numpy(), d["disp_gate"].astype(np.float32))
    assert np.array_equal(out["token_pos"].cpu().numpy(), d["token_pos"])


def test_route_scores_with_256_experts(ms):
    """a3..a6 with E = 256, k = 8 (the fine-grained shape): the solve ends in the cycle-cancelling finisher and the
    gates and dispatch lists are built from its key blocks; everything equal to the checker's."""
    print("route_scores E=256", flush=True)
    rng = np.random.default_rng(77)
    T, E, k = 3072, 256, 8
    L = (rng.standard_normal((T, E)) + 1.2 * rng.standard_normal((1, E))).astype(np.float32)
    C = T * k // E
    A32 = oracle.soft_topk(L.astype(np.float64), k, 1.0).astype(np.float32)
    out = ms.route_scores(dev(A32), k, C)
    q = out["q"].cpu().numpy().astype(np.int64)
    assert np.array_equal(q, oracle.quantise(A32))
    assign = out["assign"].cpu().numpy()
    P = oracle.assignment_matrix(assign, E)
    ok, why = oracle.check_feasible(P, k, C)
    assert ok, why
    ref = oracle.max_score_assignment(q, k, C)
    assert int(P.sum()) == ref["flow"] == out["stats"]["flow_value"]
    assert int(q[P.astype(bool)].sum()) == ref["total"] == out["stats"]["total_score_q"]
    assert out["stats"]["finish_passes"] >= 1, out["stats"]
    g = out["gates"].cpu().numpy()
    assert np.array_equal(g.astype(np.float64), oracle.gates(A32.astype(np.float64), assign))
    d = oracle.dispatch(assign, g, E)
    assert np.array_equal(out["expert_offsets"].cpu().numpy(), d["expert_offsets"])
    assert np.array_equal(out["disp_token"].cpu().numpy(), d["disp_token"])
    assert np.array_equal(out["disp_gate"].cpu().numpy(), d["disp_gate"].astype(np.float32))
    assert np.array_equal(out["token_pos"].cpu().numpy(), d["token_pos"])


def test_route_with_token_dropping_when_capacity_is_short(ms):
    """T*k > E*C: iterative rerouting routes with holes (Section 2.3, Figure 1(b)/(c)) and matches the checker
    element by element (the exact solver's answer to the same case is in test_gpu_oversubscribed.py)."""
    print("route iter oversubscribed", flush=True)
    L, E, k, _, t = cfg_case("cfg3", 2000)
    C = 200                                           # 2000*8 = 16000 > 64*200 = 12800
    out = ms.route_logits(dev(L), k, C, t=t, assignment="iter")
    q = out["q"].cpu().numpy().astype(np.int64)
    ref = oracle.iter_reroute(q, k, C)
    a = out["assign"].cpu().numpy()
    assert np.array_equal(a, ref["assign"])
    assert out["stats"]["flow_value"] == ref["flow"] <= E * C
    assert np.bincount(a[a >= 0], minlength=E).max() <= C
    pos = out["token_pos"].cpu().numpy()
    assert pos[a >= 0].max() < C


def route_xw_full_size(ms, name):
    """The whole path at a configuration's full size, in the launch shape `bench.py` times: logits, scores,
    rewards and gates against the checker on sampled rows, the assignment by the certificate of optimality on
    the path's own rewards (second half of the two-matrix protocol), the dispatch lists against the checker in
    full."""
    r = make_inputs(name)
    if r.dtype == "bf16":
        xd = dev(r.x_bits.view(np.int16)).view(torch.bfloat16)
        Wd = dev(r.W_bits.view(np.int16)).view(torch.bfloat16)
    else:
        xd, Wd = dev(r.x), dev(r.W)
    bd = dev(r.bias) if r.bias is not None else None
    out = ms.route_xw(xd, Wd, bd, r.k, r.C, t=r.t)
    del xd
    print(name, out["stats"], flush=True)
    n_s = min(1024, r.T)
    rows = np.random.default_rng(5).choice(r.T, n_s, replace=False)
    rows = np.unique(np.concatenate([rows, [0, 1, min(63, r.T - 1), min(64, r.T - 1), max(r.T - 65, 0), r.T - 1]]))
    logits = out["logits"].cpu().numpy()
    refL = oracle.router_logits(r.x[rows], r.W, r.bias)
    assert (np.abs(logits[rows] - refL) / np.maximum(np.abs(refL), 1.0)).max() <= 2e-2
    # from here on the checker follows the path's own fp32 logits
    A = oracle.soft_topk(logits[rows].astype(np.float64), r.k, r.t)
    scores = out["scores"].cpu().numpy()
    assert np.all(np.abs(scores[rows] - A) <= 1e-5 * np.abs(A) + 1e-12)
    q = out["q"].cpu().numpy().astype(np.int64)
    # the rewards are the rounding of the path's own fp32 scores (same precision on both sides)
    assert np.array_equal(q, oracle.quantise(scores))
    assign = out["assign"].cpu().numpy()
    P = oracle.assignment_matrix(assign, r.E)
    ok, why = oracle.check_feasible(P, r.k, r.C)
    assert ok, why
    assert int(P.sum()) == out["stats"]["flow_value"] == min(r.T * r.k, r.E * min(r.C, r.T))
    assert int(q[P.astype(bool)].sum()) == out["stats"]["total_score_q"]
    assert oracle.verify_optimal(q, P, r.k, r.C)["optimal"]
    g = out["gates"].cpu().numpy()
    gref = oracle.gates(A, assign[rows])
    assert np.all(np.abs(g[rows] - gref) <= 1e-5 * np.abs(gref) + 1e-12)
    # all gates are the path's own scores at the assigned experts, bit for bit
    assert np.array_equal(g, np.take_along_axis(scores, assign.astype(np.int64), axis=1))
    d = oracle.dispatch(assign, g, r.E)
    assert np.array_equal(out["expert_offsets"].cpu().numpy(), d["expert_offsets"])
    assert np.array_equal(out["disp_token"].cpu().numpy(), d["disp_token"])
    assert np.array_equal(out["disp_gate"].cpu().numpy(), d["disp_gate"].astype(np.float32))
    assert np.array_equal(out["token_pos"].cpu().numpy(), d["token_pos"])
    return out


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4a", "cfg4b_exact", "cfg4b_near"])
def test_route_xw_full_size(ms, name):
    print(f"route_xw {name} full size", flush=True)
    route_xw_full_size(ms, name)


def test_route_xw_headline_size(ms):
    """The benchmark's configuration (T=65536, d=2048, E=128, k=8, C=4096, bf16)."""
    print("route_xw cfg5 full size", flush=True)
    route_xw_full_size(ms, "cfg5")
