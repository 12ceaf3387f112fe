"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2508_12801_amd as ms
from paper_2508_12801_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ms.lib_path()):
        from paper_2508_12801_amd.build import build
        build()
    return ms.load_library()


def header_functions():
    text = open(os.path.join(ROOT, "include", "maxscore.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(maxscore_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert len(names) >= 11
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(ms.exported_symbols()) == names          # the binding covers the whole header


def test_workspace_query(lib):
    # room for one bid key per (token, slot), the per-workgroup counts and the transposed weight copy
    assert ms.workspace_bytes(65536, 2048, 128, 8, 4096) > 65536 * 8 * 8 + 2048 * 128 * 2
    assert ms.workspace_bytes(65536, 2048, 128, 8, 4096) < 64 << 20
    assert ms.workspace_bytes(64, 64, 8, 2, 16) % 256 == 0
    assert ms.workspace_bytes(64, 64, 8, 9, 16) == 0          # k > E
    assert ms.workspace_bytes(0, 64, 8, 2, 16) == 0
    assert ms.workspace_bytes(64, 64, 2000, 2, 16) == 0        # E beyond the supported maximum
    assert ms.workspace_bytes(64, 64, 128, 65, 16) == 0        # k beyond the supported maximum


def test_argument_errors_are_found_on_the_host(lib):
    one = ctypes.c_void_p(256)       # never dereferenced: every call below fails validation first
    null = None
    # NULL pointers
    assert lib.maxscore_assign_i32(null, 4, 4, 2, 2, null, one, null, null, null, one, 1 << 20, null) == -1
    assert lib.maxscore_softtopk(null, 4, 4, 2, 1.0, 20, one, one, null) == -1
    assert lib.maxscore_router_logits(one, null, null, 0, 4, 4, 4, one, null, 0, null) == -1
    assert lib.maxscore_gates(one, null, 4, 4, 2, one, null) == -1
    # shapes
    assert lib.maxscore_assign_i32(one, 4, 4, 5, 2, null, one, null, null, null, one, 1 << 20, null) == -2   # k > E
    assert lib.maxscore_assign_i32(one, 4, 4, 2, 0, null, one, null, null, null, one, 1 << 20, null) == -2   # C < 1
    assert lib.maxscore_softtopk(one, 4, 4, 2, -1.0, 20, one, one, null) == -2                                  # t < 0
    assert lib.maxscore_softtopk(one, 4, 4, 2, 1.0, 40, one, one, null) == -2                                   # shift
    # capacity too small for every token to get k experts is solved with k padding experts; refused when E + k of them
    # do not fit, and with the workspace of the plain problem
    assert lib.maxscore_assign_i32(one, 40, 1000, 30, 1, null, one, null, null, null, one, 1 << 30, null) == -6
    plain = lib.maxscore_workspace_bytes(10, 0, 4, 2, 5)
    assert lib.maxscore_workspace_bytes(10, 0, 4, 2, 4) > plain
    assert lib.maxscore_assign_i32(one, 10, 4, 2, 4, null, one, null, null, null, one, plain, null) == -3
    # workspace: missing, misaligned, too small
    assert lib.maxscore_assign_i32(one, 8, 4, 2, 4, null, one, null, null, null, null, 1 << 20, null) == -3
    assert lib.maxscore_assign_i32(one, 8, 4, 2, 4, null, one, null, null, null, ctypes.c_void_p(260), 1 << 20, null) == -3
    assert lib.maxscore_assign_i32(one, 8, 4, 2, 4, null, one, null, null, null, one, 16, null) == -3
    # per-token k: missing vector, k > E, capacity < 1 without a capacity vector, missing workspace
    assert lib.maxscore_assign_kvec_i32(one, 8, 4, 2, null, 4, null, null, one, null, null, null, one, 1 << 20, null) == -1
    assert lib.maxscore_assign_kvec_i32(one, 8, 4, 5, one, 4, null, null, one, null, null, null, one, 1 << 20, null) == -2
    assert lib.maxscore_assign_kvec_i32(one, 8, 4, 2, one, 0, null, null, one, null, null, null, one, 1 << 20, null) == -2
    assert lib.maxscore_assign_kvec_i32(one, 8, 4, 2, one, 4, null, null, one, null, null, null, null, 1 << 20, null) == -3
    # dtype
    assert lib.maxscore_router_logits(one, one, null, 7, 4, 4, 4, one, null, 0, null) == -4
    assert lib.maxscore_copy_bytes(one, one, 10, null) == -2
    for code in range(-8, 1):
        assert len(lib.maxscore_status_string(code)) > 1


def test_compute_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(binding.MaxScoreError):
        ms.softtopk(torch.zeros(4, 4), 2, 1.0)
