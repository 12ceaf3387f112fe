"""GPU parity of the exact assignment on a seeded random sweep of shapes: expert counts around the powers of two
and beyond the tail pass's limit, token counts around the workgroup sizes, tight, slack and unconstrained
capacity, uniform, tie-heavy, skewed and signed rewards, with and without a k of its own per token.  Every result
must be feasible, report the total it has, and be proved optimal by the checker's certificate (no improving cycle
in the contracted residual graph) or, on the small cases, equal the checker's optimum."""
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


def one_case(ms, rng, case):
    E = int(rng.choice([2, 3, 5, 8, 16, 17, 31, 32, 33, 64, 65, 100, 128, 129, 200, 256, 257, 300]))
    k = int(rng.integers(1, min(E, 16) + 1))
    T = int(rng.choice([1, 7, 63, 64, 65, 500, 1000, 4097, 8191, 20000]))
    kind = rng.choice(["tight", "slack", "big"])
    base = -(-T * k // E)
    C = base if kind == "tight" else base + int(rng.integers(1, max(2, base // 3 + 2))) if kind == "slack" else T
    C = max(C, 1)
    dist = rng.choice(["uniform", "ties", "skew", "signed"])
    if dist == "uniform":
        q = rng.integers(0, 1 << 20, (T, E))
    elif dist == "ties":
        q = rng.integers(0, 5, (T, E))
    elif dist == "skew":
        q = rng.integers(0, 1 << 20, (T, E)) + (rng.integers(0, 1 << 21, E) * (rng.random(E) < 0.2))[None, :]
    else:
        q = rng.integers(-(1 << 19), 1 << 19, (T, E))
    q = q.astype(np.int32)
    use_kvec = rng.random() < 0.3
    print(f"sweep case {case}: T={T} E={E} k={k} C={C} {kind} {dist} kvec={use_kvec}", flush=True)
    dq = torch.from_numpy(q).cuda()
    if use_kvec:
        kk = rng.integers(0, k + 1, T).astype(np.int32)
        if int(kk.sum()) > E * min(C, T):
            C = -(-int(kk.sum()) // E)
        out = ms.assign_kvec_i32(dq, k, torch.from_numpy(kk).cuda(), C)
    else:
        kk = np.full(T, k)
        out = ms.assign_i32(dq, k, C)
    P = oracle.assignment_matrix(out["assign"].cpu().numpy(), E)
    assert (P.sum(axis=1) == kk).all() and (P.sum(axis=0) <= min(C, T)).all()
    total = int(q.astype(np.int64)[P.astype(bool)].sum())
    assert total == out["stats"]["total_score_q"] and out["stats"]["flow_value"] == int(kk.sum())
    if T * E <= 3_000_000:
        assert oracle.verify_optimal(q.astype(np.int64), P, kk, C)["optimal"]
    if T * E <= 40000:
        assert oracle.max_score_assignment_kvec(q.astype(np.int64), kk, C)["total"] == total


@pytest.mark.parametrize("seed", [1, 2])
def test_random_shapes_are_feasible_and_certified_optimal(ms, seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        one_case(ms, rng, case)
