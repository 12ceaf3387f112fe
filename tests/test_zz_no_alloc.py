"""The dispatch entry point that uses the library's built-in scratch must give exactly what maxscore_dispatch
gives, on two calls in a row (the second on a smaller input, so stale contents of the shared scratch would show),
and must reject sizes beyond its scratch."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ms():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2508_12801_amd as m
    m.load_library()
    return m


def random_assignment(rng, T, E, k):
    a = np.full((T, k), -1, dtype=np.int32)
    for i in range(T):
        n = k if i % 5 else int(rng.integers(0, k + 1))
        a[i, :n] = rng.permutation(E)[:n]
        rng.shuffle(a[i])
    return a


def test_static_dispatch_matches_workspace_dispatch(ms):
    rng = np.random.default_rng(77)
    for T, E, k in ((20000, 128, 8), (3001, 64, 4)):          # the second call is smaller than the first
        print(f"dispatch_static T={T} E={E} k={k}", flush=True)
        a = torch.from_numpy(random_assignment(rng, T, E, k)).cuda()
        g = torch.from_numpy(rng.random((T, k)).astype(np.float32)).cuda()
        ref = ms.dispatch(a, g, E)
        got = ms.dispatch_static(a, g, E)
        torch.cuda.synchronize()
        n = int(ref["expert_offsets"][-1].item())
        assert torch.equal(got["expert_offsets"], ref["expert_offsets"])
        assert torch.equal(got["disp_token"][:n], ref["disp_token"][:n])
        assert torch.equal(got["disp_gate"][:n], ref["disp_gate"][:n])
        assert torch.equal(got["token_pos"], ref["token_pos"])


def test_static_dispatch_rejects_sizes_beyond_its_scratch(ms):
    lib = ms.load_library()
    one = ctypes.c_void_p(256)          # never dereferenced: the size check comes first
    # ceil(T*k/1024)*E + 1024 > 262144
    assert lib.maxscore_dispatch_static(one, None, 1 << 20, 1024, 8, one, one, None, one, None) == -3
    assert lib.maxscore_dispatch_static(None, None, 64, 8, 2, one, one, None, one, None) == -1
