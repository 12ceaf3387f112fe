"""GPU parity of the assignment step (a4) on the solver's different code paths: 32-bit quick checks and
64-bit full evaluation, with and without the tail pass, zero slack and slack capacity, several seeds,
and the error statuses.  Every optimum is compared bit for bit with the CPU checker's."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, capacity, make_logits

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


def solve_and_check(ms, q64, k, C, **kw):
    T, E = q64.shape
    out = ms.assign_i32(dev(q64.astype(np.int32)), k, C, **kw)
    a = out["assign"].cpu().numpy()
    P = oracle.assignment_matrix(a, E)
    ok, why = oracle.check_feasible(P, k, C)
    assert ok, why
    total = int(q64[P.astype(bool)].sum())
    ref = oracle.max_score_assignment(q64, k, C)
    assert out["stats"]["status"] == 0 and out["stats"]["total_score_q"] == total
    assert int(P.sum()) == ref["flow"] and total == ref["total"], (total, ref["total"], out["stats"])
    return out


def skewed_rewards(rng, T, E, hi_bits):
    """Softmax-like rows with popular experts, scaled to integers below 2^hi_bits."""
    L = rng.normal(size=(T, E)) + 2.0 * rng.normal(size=(1, E))
    p = np.exp(L - L.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    return np.rint(p * ((1 << hi_bits) - 1)).astype(np.int64)


# reward range below / at / above the point where S * range stops fitting the 32-bit value path
# (S = 128 for E = 64: 2^28 / S = 2^21), zero slack (T*k = E*C) and slack capacity
@pytest.mark.parametrize("hi_bits", [12, 20, 21, 22, 27])
@pytest.mark.parametrize("slack", [False, True])
def test_value_width_paths(ms, hi_bits, slack):
    print(f"value_width hi_bits={hi_bits} slack={slack}", flush=True)
    T, E, k = 2048, 64, 4
    C = T * k // E + (7 if slack else 0)
    q = skewed_rewards(np.random.default_rng(hi_bits + 100 * slack), T, E, hi_bits)
    solve_and_check(ms, q, k, C)


@pytest.mark.parametrize("E,k,T", [(512, 4, 4096), (320, 6, 1280), (1024, 2, 2048), (128, 64, 512),
                                   (1024, 64, 256), (64, 64, 300), (640, 5, 1536)])
def test_many_experts_and_many_slots(ms, E, k, T):
    """Expert counts in every size class of the tail pass and the finisher (up to 256, 512 and 1024 experts) and k up
    to 64, with both accelerators and with the dense rounds alone."""
    print(f"many_experts E={E} k={k} T={T}", flush=True)
    C = T * k // E
    q = skewed_rewards(np.random.default_rng(E + k), T, E, 18)
    solve_and_check(ms, q, k, C)
    solve_and_check(ms, q, k, C, tail_pass=False, finisher=False)


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("name,T", [("cfg5", 8192), ("cfg3", 4096)])
def test_config_seeds(ms, name, T, seed):
    print(f"config_seeds {name} T={T} seed={seed}", flush=True)
    cfg = CONFIGS[name]
    L = make_logits(name, seed=seed, T=T)
    E, k = cfg["E"], cfg["k"]
    C = capacity(T, E, k, cfg["C"] * E / (cfg["T"] * k))
    q = oracle.quantise(oracle.soft_topk(L, k, cfg["t"]))
    solve_and_check(ms, q, k, C)


def test_same_input_same_output(ms):
    print("determinism", flush=True)
    q = skewed_rewards(np.random.default_rng(5), 4096, 128, 20)
    qd = dev(q.astype(np.int32))
    a = ms.assign_i32(qd, 8, 256)
    b = ms.assign_i32(qd, 8, 256)
    assert torch.equal(a["assign"], b["assign"]) and torch.equal(a["prices"], b["prices"])
    assert a["stats"]["rounds"] == b["stats"]["rounds"]


@pytest.mark.parametrize("eps_div", [2, 5, 64])
def test_eps_schedule_does_not_change_the_optimum(ms, eps_div):
    print(f"eps_div {eps_div}", flush=True)
    q = skewed_rewards(np.random.default_rng(9), 1024, 32, 20)
    solve_and_check(ms, q, 4, 128, eps_div=eps_div)


def test_round_cap_reports_not_converged(ms):
    """At the round cap the call reports it and still returns a feasible (incomplete) assignment: at most C tokens
    per expert, distinct experts per token, empty slots where the solver still had to move somebody."""
    print("round_cap", flush=True)
    T, E, k, C = 4096, 64, 8, 512
    q = skewed_rewards(np.random.default_rng(11), T, E, 20)
    for cap_rounds in (1, 2, 3, 7):
        out = ms.assign_i32(dev(q.astype(np.int32)), k, C, max_rounds=cap_rounds, allow_not_converged=True)
        assert out["rc"] == -8 and out["stats"]["status"] == -8 and out["stats"]["rounds"] <= cap_rounds
        a = out["assign"].cpu().numpy()
        P = oracle.assignment_matrix(a, E)
        assert P.max() <= 1 and P.sum(axis=1).max() <= k and P.sum(axis=0).max() <= C, cap_rounds
        assert int(P.sum()) == out["stats"]["flow_value"] == int((a >= 0).sum())     # distinct experts per token
        assert int(P.sum()) < T * k                                                  # incomplete, as reported
        assert out["stats"]["total_score_q"] == int(q[P.astype(bool)].sum())
    with pytest.raises(ms.MaxScoreError):
        ms.assign_i32(dev(q.astype(np.int32)), k, C, max_rounds=3)
    # through the routing entry: every position lies inside its expert's buffer of C places
    L = np.random.default_rng(12).standard_normal((T, E)).astype(np.float32) * 2
    r = ms.route_logits(dev(L), k, C, max_rounds=2, allow_not_converged=True)
    assert r["rc"] == -8
    a = r["assign"].cpu().numpy()
    pos = r["token_pos"].cpu().numpy()
    assert pos[a >= 0].max() < C and (pos[a < 0] == -1).all()
    d = oracle.dispatch(a, r["gates"].cpu().numpy(), E)
    assert np.array_equal(r["expert_offsets"].cpu().numpy(), d["expert_offsets"])
    assert np.diff(d["expert_offsets"]).max() <= C
    n = int(d["expert_offsets"][-1])
    assert np.array_equal(r["disp_token"].cpu().numpy()[:n], d["disp_token"])
    assert np.array_equal(pos, d["token_pos"])


def test_reward_range_too_wide_is_an_error(ms):
    print("range_error", flush=True)
    q = np.zeros((64, 1000), dtype=np.int64)          # S = 1024: range * S reaches 2^38 at 2^28
    q[0, 0] = 1 << 29
    with pytest.raises(ms.MaxScoreError) as e:
        ms.assign_i32(dev(q.astype(np.int32)), 2, 64)
    assert e.value.code == -7
    # through a routing entry the gates and dispatch kernels are already queued behind the solve when the error is
    # known: they must stay inside their buffers on a state that holds no keys at all, and the call reports the error
    # (the second call finds the workspace as another shape's solve left it)
    scores = np.full((64, 1000), 1e-3, dtype=np.float32)
    scores[0, 0] = 600.0                              # 600 * 2^20 > 2^29
    for _ in range(2):
        with pytest.raises(ms.MaxScoreError) as e:
            ms.route_scores(dev(scores), 2, 64)
        assert e.value.code == -7
        solve_and_check(ms, skewed_rewards(np.random.default_rng(3), 64, 1000, 16), 2, 64)


def test_tail_pass_switch_gives_the_same_optimum(ms):
    """Switching the tail pass off (MAXSCORE_FLAG_NO_TAIL_PASS) must not change the total (different, equally
    optimal assignments are allowed)."""
    print("tail_switch", flush=True)
    q = skewed_rewards(np.random.default_rng(13), 4096, 64, 20)
    qd = dev(q.astype(np.int32))
    with_tail = ms.assign_i32(qd, 8, 512)
    without = ms.assign_i32(qd, 8, 512, tail_pass=False)
    assert with_tail["stats"]["total_score_q"] == without["stats"]["total_score_q"]
    assert without["stats"]["rounds"] > with_tail["stats"]["rounds"]       # the switch did switch something
    ref = oracle.max_score_assignment(q, 8, 512)["total"]
    assert with_tail["stats"]["total_score_q"] == ref


def certified(q64, out, k, C):
    """eps = 1 complementary slackness of the returned prices, price 0 on unfilled experts."""
    T, E = q64.shape
    P = oracle.assignment_matrix(out["assign"].cpu().numpy(), E).astype(bool)
    p, S = out["prices"].cpu().numpy(), out["price_scale"]
    load = P.sum(axis=0)
    if not ((p >= 0).all() and (p[load < min(C, T)] == 0).all()):
        return False
    net = q64 * S - p[None, :]
    big = np.int64(1) << 60
    return bool((np.where(P, net, big).min(axis=1) >= np.where(P, -big, net).max(axis=1) - 1).all())


@pytest.mark.parametrize("name,T,seed", [("cfg5", 8192, 0), ("cfg5", 16384, 1), ("cfg3", 4096, 2), ("cfg4a", 4096, 0),
                                         ("cfg4b_exact", 4096, 0), ("cfg4b_near", 4096, 1), ("cfg2", None, 3)])
def test_finisher_and_auction_reach_the_same_optimum(ms, name, T, seed):
    """The last phases of the eps ladder are replaced by cancelling negative cycles (the default) or run by the
    auction itself (MAXSCORE_FLAG_NO_FINISHER): same total as the checker either way, prices that certify it, and
    fewer auction rounds with the finisher."""
    print(f"finisher {name} T={T} seed={seed}", flush=True)
    cfg = CONFIGS[name]
    L = make_logits(name, seed=seed, T=T)
    T = L.shape[0]
    E, k = cfg["E"], cfg["k"]
    C = capacity(T, E, k, cfg["C"] * E / (cfg["T"] * k))
    q = oracle.quantise(oracle.soft_topk(L, k, cfg["t"]))
    fin = solve_and_check(ms, q, k, C)
    auc = solve_and_check(ms, q, k, C, finisher=False)
    assert certified(q, fin, k, C) and certified(q, auc, k, C)
    assert fin["stats"]["rounds"] <= auc["stats"]["rounds"]
    again = ms.assign_i32(dev(q.astype(np.int32)), k, C)
    assert again["stats"]["total_score_q"] == fin["stats"]["total_score_q"]
    if name != "cfg4b_exact":        # (among thousands of identical rows the auction's own tie order varies from run to run)
        assert torch.equal(again["assign"], fin["assign"]) and torch.equal(again["prices"], fin["prices"])


@pytest.mark.parametrize("name,seed", [("cfg5", 0), ("cfg5", 1), ("cfg3", 1), ("cfg2", 0), ("cfg2", 3)])
def test_finisher_certifies_in_one_pass_at_full_size(ms, name, seed):
    """At the benchmark's sizes the first finisher pass holds every arc under its bound and keeps that list complete
    while it moves tokens (the arcs of a moved token are replaced on the spot), so it cancels all cycles and
    certifies without a second pass.  Same total as the auction alone, prices that certify it."""
    print(f"finisher one pass {name} seed={seed}", flush=True)
    cfg = CONFIGS[name]
    E, k, C = cfg["E"], cfg["k"], cfg["C"]
    q = oracle.quantise(oracle.soft_topk(make_logits(name, seed=seed), k, cfg["t"]))
    qd = dev(q.astype(np.int32))
    fin = ms.assign_i32(qd, k, C)
    auc = ms.assign_i32(qd, k, C, finisher=False)
    assert fin["stats"]["status"] == 0 and fin["stats"]["total_score_q"] == auc["stats"]["total_score_q"]
    assert certified(q, fin, k, C)
    assert fin["stats"]["finish_passes"] == 1, fin["stats"]
    assert fin["stats"]["finish_cycles"] > 0 or name == "cfg2", fin["stats"]     # (the small batch may leave no cycle)
    a = fin["assign"].cpu().numpy()
    P = oracle.assignment_matrix(a, E)
    ok, why = oracle.check_feasible(P, k, C)
    assert ok, why
    assert int(q[P.astype(bool)].sum()) == fin["stats"]["total_score_q"]


@pytest.mark.parametrize("T,E,k,spread,seed", [(16384, 128, 2, 2.0, 0), (8192, 32, 4, 2.0, 1), (4096, 64, 8, 2.0, 2)])
def test_finisher_that_cannot_take_over_at_its_first_rung(ms, T, E, k, spread, seed):
    """Strongly skewed expert popularity: at the rung the finisher is first tried on, more arcs lie under its bound
    than it can hold (or it runs out of room for moved tokens), so it hands back; the auction goes one rung down,
    with phases that now run to quiescence, and the finisher tries again there.  The result is the checker's optimum
    with prices that certify it, as on every other path."""
    print(f"finisher retry T={T} E={E} k={k}", flush=True)
    rng = np.random.default_rng(seed)
    L = rng.normal(size=(T, E)) + spread * rng.normal(size=(1, E))
    p = np.exp(L - L.max(axis=1, keepdims=True))
    q = np.rint(p / p.sum(axis=1, keepdims=True) * ((1 << 20) - 1)).astype(np.int64)
    C = -(-T * k // E)
    out = solve_and_check(ms, q, k, C)
    assert certified(q, out, k, C)
    print("  ", out["stats"], flush=True)
    auc = ms.assign_i32(dev(q.astype(np.int32)), k, C, finisher=False)
    assert auc["stats"]["total_score_q"] == out["stats"]["total_score_q"]


@pytest.mark.parametrize("T,E,k,slack", [(4096, 160, 5, 0), (3072, 200, 8, 3), (4096, 256, 4, 0), (2048, 256, 8, 0),
                                        (3072, 384, 6, 0), (4096, 512, 4, 2), (2048, 512, 8, 0), (2560, 640, 5, 0),
                                        (4096, 1024, 4, 0), (2048, 1000, 8, 1)])
def test_finisher_beyond_128_experts(ms, T, E, k, slack):
    """At every supported expert count the finisher takes over from the auction (four, eight or sixteen experts per
    lane in its arc kernels; up to 256 experts with the arc matrix of E*E entries as a fallback, beyond that with the
    complete arc list only): the checker's optimum, prices that certify it, and the finisher did run."""
    print(f"finisher E={E} T={T} k={k} slack={slack}", flush=True)
    C = -(-T * k // E) + slack
    q = skewed_rewards(np.random.default_rng(E + 7 * k), T, E, 20)
    out = solve_and_check(ms, q, k, C)
    assert certified(q, out, k, C)
    assert out["stats"]["finish_passes"] >= 1, out["stats"]
    auc = solve_and_check(ms, q, k, C, finisher=False)
    assert auc["stats"]["finish_passes"] == 0
    # (a finisher that has to hand back can cost a few rounds more than it saves: the round counts are only shown)
    print("   rounds", out["stats"]["rounds"], "with the finisher,", auc["stats"]["rounds"], "without", flush=True)


@pytest.mark.parametrize("T,E,k", [(65536, 256, 8), (32768, 512, 8), (16384, 1024, 8)])
def test_finisher_with_many_experts_full_batch(ms, T, E, k):
    """Large batches with 256, 512 and 1024 experts (tight capacity, Zipf-biased experts): the finisher certifies; the
    total equals the auction's own and the returned prices certify it."""
    print(f"finisher E={E} full batch", flush=True)
    rng = np.random.default_rng(5)
    z = np.arange(1, E + 1, dtype=np.float64) ** -1.2
    z = (z - z.min()) / (z.max() - z.min()) * 2.0
    rng.shuffle(z)
    L = (rng.standard_normal((T, E)) + z[None, :]).astype(np.float32)
    q = oracle.quantise(oracle.soft_topk(L, k, 1.0))
    C = T * k // E
    qd = dev(q.astype(np.int32))
    fin = ms.assign_i32(qd, k, C)
    auc = ms.assign_i32(qd, k, C, finisher=False)
    print("  ", fin["stats"], flush=True)
    assert fin["stats"]["status"] == 0 and fin["stats"]["total_score_q"] == auc["stats"]["total_score_q"]
    assert certified(q, fin, k, C)
    assert fin["stats"]["finish_passes"] >= 1 and fin["stats"]["rounds"] < auc["stats"]["rounds"]
    P = oracle.assignment_matrix(fin["assign"].cpu().numpy(), E)
    ok, why = oracle.check_feasible(P, k, C)
    assert ok, why
    assert int(q[P.astype(bool)].sum()) == fin["stats"]["total_score_q"]


@pytest.mark.parametrize("T,E,k,cap_lo,cap_hi", [(3000, 48, 6, 200, 500), (3000, 192, 6, 50, 125), (2500, 257, 6, 31, 80),
                                                 (2000, 513, 4, 9, 24), (1500, 1024, 8, 7, 18)])
def test_finisher_with_k_vector_and_capacity_vector(ms, T, E, k, cap_lo, cap_hi):
    """Per-token k (with zeros) and unequal capacities through the finisher: checker's optimum, valid rows."""
    print(f"finisher kvec+caps E={E}", flush=True)
    rng = np.random.default_rng(31)
    q = skewed_rewards(rng, T, E, 20)
    kvec = rng.integers(0, k + 1, T).astype(np.int32)
    caps = rng.integers(cap_lo, cap_hi, E).astype(np.int32)
    caps[3] = 0
    assert caps.sum() >= kvec.sum()
    out = ms.assign_kvec_i32(dev(q.astype(np.int32)), k, dev(kvec), caps=list(caps))
    a = out["assign"].cpu().numpy()
    ref = oracle.max_score_assignment_kvec(q, kvec, caps)
    P = oracle.assignment_matrix(a, E)
    assert (P.sum(axis=1) == kvec).all() and (P.sum(axis=0) <= caps).all()
    assert int(q[P.astype(bool)].sum()) == ref["total"] == out["stats"]["total_score_q"]


@pytest.mark.parametrize("name,T,slack", [("cfg5", 8192, False), ("cfg3", 4096, False), ("cfg4a", 4096, True)])
def test_starting_prices_do_not_change_the_optimum(ms, name, T, slack):
    """Starting prices (the prices another batch of the same router ended with, or arbitrary ones) only change the
    number of rounds: totals equal the checker's optimum, and the returned prices certify it."""
    print(f"starting_prices {name} T={T}", flush=True)
    cfg = CONFIGS[name]
    E, k = cfg["E"], cfg["k"]
    C = capacity(T, E, k, cfg["C"] * E / (cfg["T"] * k))
    qs = [oracle.quantise(oracle.soft_topk(make_logits(name, T=T, batch=b), k, cfg["t"])) for b in (0, 1)]
    other = ms.assign_i32(dev(qs[1].astype(np.int32)), k, C)          # another batch of the same router
    cold = solve_and_check(ms, qs[0], k, C)
    rng = np.random.default_rng(3)
    S = other["price_scale"]
    starts = [("other batch", other["prices"], 0), ("other batch, eps 1", other["prices"], 1),
              ("other batch, large eps", other["prices"], 1 << 40),
              ("own prices", cold["prices"], 1),
              ("random", dev(rng.integers(0, (1 << 20) * S, E).astype(np.int64)), 0),
              ("random, eps 1", dev(rng.integers(0, (1 << 16) * S, E).astype(np.int64)), 1),
              ("zeros", dev(np.zeros(E, dtype=np.int64)), 0)]
    for label, p_in, eps_start in starts:
        out = solve_and_check(ms, qs[0], k, C, prices_in=p_in, eps_start=eps_start)
        print(f"  {label}: rounds {out['stats']['rounds']} (cold {cold['stats']['rounds']}), phases "
              f"{out['stats']['phases']}", flush=True)
        # eps = 1 complementary slackness of the returned prices, price 0 on unfilled experts
        a = out["assign"].cpu().numpy()
        P = oracle.assignment_matrix(a, E).astype(bool)
        p = out["prices"].cpu().numpy()
        load = P.sum(axis=0)
        assert (p >= 0).all() and (p[load < min(C, T)] == 0).all()
        net = qs[0] * S - p[None, :]
        big = np.int64(1) << 60
        assert (np.where(P, net, big).min(axis=1) >= np.where(P, -big, net).max(axis=1) - 1).all()
    own = solve_and_check(ms, qs[0], k, C, prices_in=cold["prices"], eps_start=1)
    assert own["stats"]["rounds"] < cold["stats"]["rounds"]        # its own final prices: little left to do


def test_large_batch_certified_by_its_prices(ms):
    """T = 2^18 tokens: too many for the CPU flow solver in a test, so optimality is certified by the dual
    side alone: with rewards scaled by S > E, complementary slackness within 1 and price 0 on every
    unfilled expert leave no improving cycle (a cycle gains a multiple of S but visits at most E experts)."""
    print("large_batch", flush=True)
    T, E, k = 1 << 18, 64, 2
    C = T * k // E + 3                                  # a little slack: some experts stay unfilled
    rng = np.random.default_rng(21)
    q = skewed_rewards(rng, T, E, 20)
    out = ms.assign_i32(dev(q.astype(np.int32)), k, C)
    a = out["assign"].cpu().numpy()
    assert a.min() >= 0 and (np.sort(a, axis=1)[:, 1:] != np.sort(a, axis=1)[:, :-1]).all()   # k distinct experts
    load = np.bincount(a.reshape(-1), minlength=E)
    assert load.max() <= C and load.sum() == T * k == out["stats"]["flow_value"]
    S, p = out["price_scale"], out["prices"].cpu().numpy()
    assert S > E and (p >= 0).all() and (p[load < C] == 0).all()
    net = q * S - p[None, :]
    held = np.zeros((T, E), dtype=bool)
    held[np.arange(T)[:, None], a] = True
    big = np.int64(1) << 60
    assert (np.where(held, net, big).min(axis=1) >= np.where(held, -big, net).max(axis=1) - 1).all()
    assert out["stats"]["total_score_q"] == int(q[held].sum())
