"""GPU parity of the iterative rerouting entry point (Section 2.3) through the C ABI: every decision is an
integer comparison, so the assignment, the total, the flow and the number of rounds must equal the CPU
checker's element by element."""
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


def check(ms, q, k, C, max_rounds=-1):
    ref = oracle.iter_reroute(q, k, C, max_rounds=max_rounds if max_rounds >= 0 else None)
    out = ms.assign_iter_i32(dev(q.astype(np.int32)), k, C, max_rounds=max_rounds, allow_not_converged=True)
    got = out["assign"].cpu().numpy()
    assert np.array_equal(got, ref["assign"])
    assert out["total"] == ref["total"] and out["flow"] == ref["flow"] and out["rounds"] == ref["rounds"]
    return ref, out


def skewed(rng, T, E, hi, bias_hi):
    return rng.integers(0, hi, (T, E)) + rng.integers(0, bias_hi, E)[None, :]


@pytest.mark.parametrize("T,E,k,C,hi", [
    (64, 8, 2, 16, 1 << 20), (1000, 16, 4, 250, 50), (4099, 64, 8, 513, 1 << 20), (257, 7, 3, 120, 9),
    (3000, 5, 5, 3000, 100),          # k = E: everybody takes every expert
    (2048, 128, 8, 128, 1 << 18),     # two experts per lane
    (1500, 300, 6, 30, 1 << 16),      # expert count that is no power of two
    (700, 1024, 64, 44, 1 << 12),     # the largest expert and slot counts
    (5000, 32, 2, 1, 1000),           # capacity 1: almost everything stays a hole
    (513, 33, 4, 80, 3),              # nearly all rewards tie
])
def test_matches_the_checker(ms, T, E, k, C, hi):
    print(f"iter T={T} E={E} k={k} C={C} hi={hi}", flush=True)
    rng = np.random.default_rng(T + E)
    q = skewed(rng, T, E, hi, hi // 2 + 1)
    ref, out = check(ms, q, k, C)
    P = oracle.assignment_matrix(out["assign"].cpu().numpy(), E)
    assert P.sum(axis=0).max() <= C


def test_negative_rewards_and_ties_to_the_lower_expert(ms):
    print("iter negative rewards", flush=True)
    rng = np.random.default_rng(5)
    q = rng.integers(-1000, 1000, (900, 24))
    q[:, 3] = q[:, 11]                                  # exact ties between two columns
    check(ms, q, 3, 100)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4a", "cfg4b_exact", "cfg5"])
def test_configs(ms, name):
    print(f"iter {name}", flush=True)
    c = CONFIGS[name]
    A = oracle.soft_topk(make_logits(name, 1), c["k"], c["t"])
    q = oracle.quantise(A)
    ref, out = check(ms, q, c["k"], c["C"])
    assert out["flow"] <= c["T"] * c["k"] and out["flow"] >= 0.999 * c["T"] * c["k"]


def test_score_is_bounded_by_the_exact_solver(ms):
    print("iter vs exact", flush=True)
    c = CONFIGS["cfg3"]
    q = oracle.quantise(oracle.soft_topk(make_logits("cfg3", 2), c["k"], c["t"])).astype(np.int32)
    it = ms.assign_iter_i32(dev(q), c["k"], c["C"])
    ex = ms.assign_i32(dev(q), c["k"], c["C"])
    best = ex["stats"]["total_score_q"]
    if it["flow"] == c["T"] * c["k"]:                   # same flow value: the exact optimum bounds the heuristic
        assert it["total"] <= best
    assert 0.98 * best < it["total"] < 1.0001 * best


def test_round_limit(ms):
    print("iter round limit", flush=True)
    rng = np.random.default_rng(8)
    q = skewed(rng, 3000, 16, 1 << 16, 1 << 16)
    full, _ = check(ms, q, 2, 375)
    assert full["rounds"] >= 3
    ref, out = check(ms, q, 2, 375, max_rounds=2)
    assert out["rc"] != 0 and ref["rounds"] == 2        # proposals were still pending
    ref, out = check(ms, q, 2, 375, max_rounds=full["rounds"] + 1)
    assert out["rc"] == 0
    # no rerouting at all: plain top-k with capacity, the dropped pairs stay holes
    ref, out = check(ms, q, 2, 375, max_rounds=0)
    assert out["rc"] == 0 and out["rounds"] == 0 and np.array_equal(out["assign"].cpu().numpy(), full["stage1"])
    assert out["flow"] < 2 * 3000


def test_gates_and_dispatch_accept_the_result(ms):
    print("iter downstream", flush=True)
    rng = np.random.default_rng(9)
    T, E, k, C = 2000, 16, 2, 200                       # over-subscribed: holes remain
    L = (rng.normal(size=(T, E)) + 2.0 * rng.normal(size=(1, E))).astype(np.float32)
    st = ms.softtopk(dev(L), k, 1.0)
    out = ms.assign_iter_i32(st[1], k, C)
    assert out["flow"] == E * C and out["flow"] < T * k
    g = ms.gates(st[0], out["assign"])
    d = ms.dispatch(out["assign"], g, E, C)
    a = out["assign"].cpu().numpy()
    ref_g = oracle.gates(st[0].cpu().numpy().astype(np.float64), a)
    assert np.allclose(g.cpu().numpy(), ref_g, rtol=1e-6, atol=0)
    ref_d = oracle.dispatch(a, ref_g, E)
    assert np.array_equal(d["expert_offsets"].cpu().numpy(), ref_d["expert_offsets"])
    assert np.array_equal(d["disp_token"].cpu().numpy()[: out["flow"]], ref_d["disp_token"])
    assert np.array_equal(d["token_pos"].cpu().numpy(), ref_d["token_pos"])


def test_whole_path_with_iterative_rerouting(ms):
    print("iter whole path", flush=True)
    c = CONFIGS["cfg3"]
    L = make_logits("cfg3", 3)
    out = ms.route_logits(dev(L), c["k"], c["C"], t=c["t"], assignment="iter")
    q = out["q"].cpu().numpy().astype(np.int64)
    ref = oracle.iter_reroute(q, c["k"], c["C"])
    a = out["assign"].cpu().numpy()
    assert np.array_equal(a, ref["assign"])
    st = out["stats"]
    assert st["total_score_q"] == ref["total"] and st["flow_value"] == ref["flow"] and st["rounds"] == ref["rounds"]
    sc = out["scores"].cpu().numpy().astype(np.float64)
    ref_g = oracle.gates(sc, a)
    assert np.allclose(out["gates"].cpu().numpy(), ref_g, rtol=1e-6, atol=0)
    ref_d = oracle.dispatch(a, ref_g, c["E"])
    assert np.array_equal(out["expert_offsets"].cpu().numpy(), ref_d["expert_offsets"])
    assert np.array_equal(out["token_pos"].cpu().numpy(), ref_d["token_pos"])
    assert np.array_equal(out["disp_token"].cpu().numpy()[: ref["flow"]], ref_d["disp_token"])
