"""ctypes binding with the same names as include/maxscore.h (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

OK = 0
ERR_NOT_CONVERGED = -8
DTYPE_BF16, DTYPE_FP32 = 0, 1


class MaxScoreError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


class _Opts(ctypes.Structure):
    _fields_ = [("t", ctypes.c_float), ("quant_shift", ctypes.c_int32), ("max_rounds", ctypes.c_int32),
                ("eps_div", ctypes.c_int32), ("assignment", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("prices_in", ctypes.c_void_p), ("eps_start", ctypes.c_int64)]


class Stats(ctypes.Structure):
    _fields_ = [("total_score_q", ctypes.c_int64), ("flow_value", ctypes.c_int32), ("rounds", ctypes.c_int32),
                ("phases", ctypes.c_int32), ("status", ctypes.c_int32), ("solver_ms", ctypes.c_float),
                ("bid_ms", ctypes.c_float), ("bid_launches", ctypes.c_int32), ("select_ms", ctypes.c_float),
                ("gates_dispatch_ms", ctypes.c_float), ("finish_passes", ctypes.c_int32),
                ("finish_cycles", ctypes.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


def lib_path() -> str:
    return os.path.join(_HERE, "libmaxscore.so")


_SIGS = {
    "maxscore_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int32] * 5),
    "maxscore_router_logits": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                                ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_assign_iter_i32": (ctypes.c_int32, [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p] * 5 +
                                 [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_aux_loss": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_gates_backward": (ctypes.c_int32, [ctypes.c_void_p] * 5 + [ctypes.c_int32] * 3 +
                                [ctypes.c_void_p, ctypes.c_void_p]),
    "maxscore_scores_op": (ctypes.c_int32, [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p] * 3),
    "maxscore_assign_caps_i32": (ctypes.c_int32, [ctypes.c_void_p] + [ctypes.c_int32] * 3 + [ctypes.c_void_p] * 7 +
                                 [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_assign_kvec_i32": (ctypes.c_int32, [ctypes.c_void_p] + [ctypes.c_int32] * 3 + [ctypes.c_void_p,
                                 ctypes.c_int32] + [ctypes.c_void_p] * 7 + [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_assign_top1_residual_i32": (ctypes.c_int32, [ctypes.c_void_p] + [ctypes.c_int32] * 3 +
                                          [ctypes.c_void_p] * 8 + [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_assign_top1_sinkhorn": (ctypes.c_int32, [ctypes.c_void_p] + [ctypes.c_int32] * 3 + [ctypes.c_float,
                                      ctypes.c_int32] + [ctypes.c_void_p] * 4 + [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_softtopk": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_float, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p]),
    "maxscore_softtopk_reading": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                   ctypes.c_float, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                                   ctypes.c_void_p, ctypes.c_void_p]),
    "maxscore_assign_i32": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                             ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                             ctypes.c_void_p]),
    "maxscore_gates": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]),
    "maxscore_dispatch": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_dispatch_static": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_void_p]),
    "maxscore_dispatch_tokens": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_void_p, ctypes.c_void_p]),
    "maxscore_combine": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]),
    "maxscore_route_logits": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                               ctypes.c_int32, ctypes.c_void_p] + [ctypes.c_void_p] * 11 +
                              [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_route_scores": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                               ctypes.c_int32, ctypes.c_void_p] + [ctypes.c_void_p] * 10 +
                              [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_route_xw": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_void_p] + [ctypes.c_void_p] * 12 +
                          [ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_router_softtopk": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                                  ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_float, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_set_kernel_timing": (None, [ctypes.c_int32]),
    "maxscore_copy_bytes": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "maxscore_status_string": (ctypes.c_char_p, [ctypes.c_int32]),
}


def exported_symbols():
    return sorted(_SIGS)


def load_library():
    """Load libmaxscore.so built in-tree; raises if it has not been built."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise MaxScoreError(-5, f"{path} is missing: run `python -m paper_2508_12801_amd.build` first")
        # torch first: it brings its own copy of the HIP runtime, and the library must bind to that copy (the device
        # memory and the streams it is handed come from there).  Loaded the other way round, the process holds two
        # runtimes and every launch on torch's memory fails with a HIP error.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(path)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB


def status_string(code: int) -> str:
    try:
        return load_library().maxscore_status_string(code).decode()
    except Exception:
        return "status %d" % code


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise MaxScoreError(-5, "no GPU visible: the MaxScore kernels have no CPU fallback")
    return torch


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str, allow=()):
    if rc != OK and rc not in allow:
        raise MaxScoreError(rc, where)


_WS = {}


def workspace_bytes(T: int, d: int, E: int, k: int, C: int) -> int:
    return int(load_library().maxscore_workspace_bytes(T, d, E, k, C))


def _workspace(T, E, k, C, device, d=0):
    torch = _torch()
    need = workspace_bytes(T, d, E, k, C)
    if need == 0:
        raise MaxScoreError(-2, "workspace_bytes")
    # one buffer per device and stream: calls on different streams may overlap and must not share scratch
    key = (str(device), torch.cuda.current_stream(device).cuda_stream)
    buf = _WS.get(key)
    if buf is None or buf.numel() < need:
        buf = torch.empty(need, dtype=torch.uint8, device=device)
        _WS[key] = buf
    return buf, need


ASSIGNMENTS = {"exact": 0, "iter": 1}


FLAG_NO_TAIL_PASS = 1
FLAG_NO_FINISHER = 2


def _opts(t=1.0, quant_shift=20, max_rounds=200000, eps_div=12, assignment="exact", tail_pass=True, prices_in=None,
          eps_start=0, finisher=True):
    flags = (0 if tail_pass else FLAG_NO_TAIL_PASS) | (0 if finisher else FLAG_NO_FINISHER)
    return _Opts(float(t), int(quant_shift), int(max_rounds), int(eps_div), ASSIGNMENTS[assignment], flags,
                 prices_in.data_ptr() if prices_in is not None else None, int(eps_start))


def set_kernel_timing(on: bool) -> None:
    load_library().maxscore_set_kernel_timing(1 if on else 0)


def copy_bytes(src, dst) -> None:
    nbytes = src.numel() * src.element_size()
    _check(load_library().maxscore_copy_bytes(_ptr(src), _ptr(dst), nbytes, _stream()), "maxscore_copy_bytes")


def _in_dtype(x):
    torch = _torch()
    if x.dtype == torch.float32:
        return DTYPE_FP32
    if x.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        return DTYPE_BF16
    raise MaxScoreError(-4, "input dtype")


def router_logits(x, W, bias=None, use_workspace=True):
    """a1: logits[T,E] fp32 = x[T,d] . W[d,E] + bias.  x, W: bf16 (or int16 bit patterns) or fp32."""
    torch = _torch()
    T, d = x.shape
    E = W.shape[1]
    assert W.shape[0] == d and x.is_contiguous() and W.is_contiguous() and x.dtype == W.dtype
    out = torch.empty((T, E), dtype=torch.float32, device=x.device)
    ws, need = (None, 0)
    if use_workspace:
        need = 2 * d * E
        key = ("wt", str(x.device), torch.cuda.current_stream(x.device).cuda_stream)
        ws = _WS.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
            _WS[key] = ws
    rc = load_library().maxscore_router_logits(_ptr(x), _ptr(W), _ptr(bias), _in_dtype(x), T, d, E, _ptr(out),
                                               _ptr(ws), need, _stream())
    _check(rc, "maxscore_router_logits")
    return out


def router_softtopk(x, W, bias, k: int, t: float, quant_shift: int = 20, want_logits: bool = True):
    """a1 + a2 + a3: dict(logits or None, scores fp32 [T,E], q int32 [T,E]) from x and W_g; one kernel where the
    library can fuse them (then the logits are optional), else the projection and the score kernel."""
    torch = _torch()
    T, d = x.shape
    E = W.shape[1]
    assert W.shape[0] == d and x.is_contiguous() and W.is_contiguous() and x.dtype == W.dtype
    logits = torch.empty((T, E), dtype=torch.float32, device=x.device) if want_logits else None
    scores = torch.empty((T, E), dtype=torch.float32, device=x.device)
    q = torch.empty((T, E), dtype=torch.int32, device=x.device)
    need = 2 * d * E
    key = ("wt", str(x.device), torch.cuda.current_stream(x.device).cuda_stream)
    ws = _WS.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
        _WS[key] = ws
    rc = load_library().maxscore_router_softtopk(_ptr(x), _ptr(W), _ptr(bias), _in_dtype(x), T, d, E, k, float(t),
                                                 quant_shift, _ptr(logits), _ptr(scores), _ptr(q), _ptr(ws), need,
                                                 _stream())
    _check(rc, "maxscore_router_softtopk")
    return dict(logits=logits, scores=scores, q=q)


READINGS = {"A": 0, "A1": 1, "B": 2, "C": 3}


def softtopk(logits, k: int, t: float, quant_shift: int = 20, reading: str = None):
    """a2 + a3: (scores fp32 [T,E], q int32 [T,E]).  reading: None (maxscore_softtopk) or one of READINGS
    (maxscore_softtopk_reading: the other readings of Eq. 6)."""
    torch = _torch()
    T, E = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    scores = torch.empty_like(logits)
    q = torch.empty((T, E), dtype=torch.int32, device=logits.device)
    if reading is None:
        rc = load_library().maxscore_softtopk(_ptr(logits), T, E, k, float(t), quant_shift, _ptr(scores), _ptr(q),
                                              _stream())
        _check(rc, "maxscore_softtopk")
    else:
        rc = load_library().maxscore_softtopk_reading(_ptr(logits), T, E, k, float(t), quant_shift, READINGS[reading],
                                                      _ptr(scores), _ptr(q), _stream())
        _check(rc, "maxscore_softtopk_reading")
    return scores, q


OPS = {"sigmoid": 1, "softkmax": 2, "itertopk": 3, "gradtopk": 4}


def scores_op(logits, k: int, op: str, quant_shift: int = 20):
    """Another operator of Table 2 in place of SoftTopk: (scores fp32 [T,E], q int32 [T,E])."""
    torch = _torch()
    T, E = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    scores = torch.empty_like(logits)
    q = torch.empty((T, E), dtype=torch.int32, device=logits.device)
    rc = load_library().maxscore_scores_op(_ptr(logits), T, E, k, OPS[op], quant_shift, _ptr(scores), _ptr(q),
                                           _stream())
    _check(rc, "maxscore_scores_op")
    return scores, q


def assign_i32(q, k: int, C: int, max_rounds: int = 200000, eps_div: int = 12, allow_not_converged=False,
               tail_pass: bool = True, prices_in=None, eps_start: int = 0, finisher: bool = True):
    """a4: exact assignment on int32 rewards.  Returns dict(assign, prices, price_scale, stats).  prices_in: int64
    device tensor of E starting prices (the `prices` of an earlier call), eps_start: first-phase eps with them."""
    torch = _torch()
    T, E = q.shape
    assert q.dtype == torch.int32 and q.is_contiguous()
    if prices_in is not None:
        assert prices_in.dtype == torch.int64 and prices_in.numel() == E and prices_in.device == q.device
    assign = torch.empty((T, k), dtype=torch.int32, device=q.device)
    prices = torch.empty(E, dtype=torch.int64, device=q.device)
    scale = torch.empty(1, dtype=torch.int64, device=q.device)
    stats = Stats()
    ws, need = _workspace(T, E, k, C, q.device)
    o = _opts(max_rounds=max_rounds, eps_div=eps_div, tail_pass=tail_pass, prices_in=prices_in, eps_start=eps_start,
              finisher=finisher)
    rc = load_library().maxscore_assign_i32(_ptr(q), T, E, k, C, ctypes.byref(o), _ptr(assign), _ptr(prices),
                                            _ptr(scale), ctypes.byref(stats), _ptr(ws), need, _stream())
    _check(rc, "maxscore_assign_i32", allow=(ERR_NOT_CONVERGED,) if allow_not_converged else ())
    return dict(assign=assign, prices=prices, price_scale=int(scale.item()), stats=stats.as_dict(), rc=rc)


def assign_iter_i32(q, k: int, C: int, max_rounds: int = -1, allow_not_converged=False):
    """Iterative rerouting on int32 rewards (Section 2.3); max_rounds=0 stops after the top-k-with-capacity stage
    (plain token dropping), a negative value means the default limit.  Returns dict(assign, total, flow, rounds, rc)."""
    torch = _torch()
    T, E = q.shape
    assert q.dtype == torch.int32 and q.is_contiguous()
    assign = torch.empty((T, k), dtype=torch.int32, device=q.device)
    total, flow, rounds = ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32()
    ws, need = _workspace(T, E, k, C, q.device)
    rc = load_library().maxscore_assign_iter_i32(_ptr(q), T, E, k, C, max_rounds, _ptr(assign),
                                                 ctypes.addressof(total), ctypes.addressof(flow),
                                                 ctypes.addressof(rounds), _ptr(ws), need, _stream())
    _check(rc, "maxscore_assign_iter_i32", allow=(ERR_NOT_CONVERGED,) if allow_not_converged else ())
    return dict(assign=assign, total=total.value, flow=flow.value, rounds=rounds.value, rc=rc)


def aux_loss(scores, expert_offsets, lam: float):
    """Eq. 9.  Returns dict(loss[1], mean_scores[E], dscores_col[E]) as device tensors."""
    torch = _torch()
    T, E = scores.shape
    assert scores.dtype == torch.float32 and scores.is_contiguous()
    assert expert_offsets.dtype == torch.int32 and expert_offsets.numel() == E + 1
    dev = scores.device
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    mean_scores = torch.empty(E, dtype=torch.float32, device=dev)
    dcol = torch.empty(E, dtype=torch.float32, device=dev)
    ws, need = _workspace(T, E, 1, 1, dev)
    rc = load_library().maxscore_aux_loss(_ptr(scores), _ptr(expert_offsets), T, E, float(lam), _ptr(loss),
                                          _ptr(mean_scores), _ptr(dcol), _ptr(ws), need, _stream())
    _check(rc, "maxscore_aux_loss")
    return dict(loss=loss, mean_scores=mean_scores, dscores_col=dcol)


def gates_backward(logits, scores, assign, dgates, dscores_col=None):
    """d loss / d logits [T, E] from d loss / d gates [T, k] (and, optionally, a per-column score gradient)."""
    torch = _torch()
    T, E = logits.shape
    k = assign.shape[1]
    for a in (logits, scores, dgates):
        assert a.dtype == torch.float32 and a.is_contiguous()
    assert assign.dtype == torch.int32 and assign.is_contiguous() and dgates.shape == assign.shape
    out = torch.empty_like(logits)
    rc = load_library().maxscore_gates_backward(_ptr(logits), _ptr(scores), _ptr(assign), _ptr(dgates),
                                                _ptr(dscores_col), T, E, k, _ptr(out), _stream())
    _check(rc, "maxscore_gates_backward")
    return out


def assign_caps_i32(q, k: int, caps, max_rounds: int = 200000, eps_div: int = 12, allow_not_converged=False):
    """a4 with one capacity per expert (host sequence of E ints).  Returns dict(assign, prices, price_scale, stats)."""
    torch = _torch()
    T, E = q.shape
    assert q.dtype == torch.int32 and q.is_contiguous()
    caps_arr = (ctypes.c_int32 * E)(*[int(c) for c in caps])
    assign = torch.empty((T, k), dtype=torch.int32, device=q.device)
    prices = torch.empty(E, dtype=torch.int64, device=q.device)
    scale = torch.empty(1, dtype=torch.int64, device=q.device)
    stats = Stats()
    ws, need = _workspace(T, E, k, 1, q.device)
    o = _opts(max_rounds=max_rounds, eps_div=eps_div)
    rc = load_library().maxscore_assign_caps_i32(_ptr(q), T, E, k, ctypes.addressof(caps_arr), ctypes.byref(o),
                                                 _ptr(assign), _ptr(prices), _ptr(scale), ctypes.byref(stats),
                                                 _ptr(ws), need, _stream())
    _check(rc, "maxscore_assign_caps_i32", allow=(ERR_NOT_CONVERGED,) if allow_not_converged else ())
    return dict(assign=assign, prices=prices, price_scale=int(scale.item()), stats=stats.as_dict(), rc=rc)


def assign_kvec_i32(q, k: int, kvec, C: int = 0, caps=None, max_rounds: int = 200000, eps_div: int = 12,
                    allow_not_converged=False):
    """a4 with one k per token: kvec is an int32 device tensor of T values in 0..k, k the row width of the result;
    capacities are C for all experts or the host sequence caps.  Returns dict(assign, prices, price_scale, stats)."""
    torch = _torch()
    T, E = q.shape
    assert q.dtype == torch.int32 and q.is_contiguous()
    assert kvec.dtype == torch.int32 and kvec.is_contiguous() and kvec.numel() == T and kvec.device == q.device
    caps_arr = (ctypes.c_int32 * E)(*[int(c) for c in caps]) if caps is not None else None
    assign = torch.empty((T, k), dtype=torch.int32, device=q.device)
    prices = torch.empty(E, dtype=torch.int64, device=q.device)
    scale = torch.empty(1, dtype=torch.int64, device=q.device)
    stats = Stats()
    ws, need = _workspace(T, E, k, 1, q.device)
    o = _opts(max_rounds=max_rounds, eps_div=eps_div)
    rc = load_library().maxscore_assign_kvec_i32(_ptr(q), T, E, k, _ptr(kvec), int(C),
                                                 ctypes.addressof(caps_arr) if caps_arr is not None else None,
                                                 ctypes.byref(o), _ptr(assign), _ptr(prices), _ptr(scale),
                                                 ctypes.byref(stats), _ptr(ws), need, _stream())
    _check(rc, "maxscore_assign_kvec_i32", allow=(ERR_NOT_CONVERGED,) if allow_not_converged else ())
    return dict(assign=assign, prices=prices, price_scale=int(scale.item()), stats=stats.as_dict(), rc=rc)


def assign_top1_residual_i32(q, C: int, max_rounds: int = 200000, eps_div: int = 12):
    """Algorithm 1 with the residual problem solved exactly.  Returns dict(assign[T,2], q_residual, caps, total,
    flow, stats)."""
    torch = _torch()
    T, E = q.shape
    assert q.dtype == torch.int32 and q.is_contiguous()
    q2 = torch.empty_like(q)
    assign = torch.empty((T, 2), dtype=torch.int32, device=q.device)
    caps = (ctypes.c_int32 * E)()
    total, flow = ctypes.c_int64(), ctypes.c_int32()
    stats = Stats()
    ws, need = _workspace(T, E, 2, C, q.device)
    o = _opts(max_rounds=max_rounds, eps_div=eps_div)
    rc = load_library().maxscore_assign_top1_residual_i32(_ptr(q), T, E, C, ctypes.byref(o), _ptr(q2), _ptr(assign),
                                                          ctypes.addressof(caps), ctypes.addressof(total),
                                                          ctypes.addressof(flow), ctypes.byref(stats), _ptr(ws),
                                                          need, _stream())
    _check(rc, "maxscore_assign_top1_residual_i32")
    return dict(assign=assign, q_residual=q2, caps=list(caps), total=total.value, flow=flow.value,
                stats=stats.as_dict(), rc=rc)


def assign_top1_sinkhorn(scores, C: int, tau: float, n_iter: int, want_plan: bool = False):
    """Algorithm 1 with Sinkhorn on the residual problem.  Returns dict(assign[T,2], plan or None, caps)."""
    torch = _torch()
    T, E = scores.shape
    assert scores.dtype == torch.float32 and scores.is_contiguous()
    assign = torch.empty((T, 2), dtype=torch.int32, device=scores.device)
    plan = torch.empty_like(scores) if want_plan else None
    caps = (ctypes.c_int32 * E)()
    ws, need = _workspace(T, E, 2, C, scores.device)
    rc = load_library().maxscore_assign_top1_sinkhorn(_ptr(scores), T, E, C, float(tau), int(n_iter), _ptr(assign),
                                                      _ptr(plan), ctypes.addressof(caps), _ptr(ws), need,
                                                      _stream())
    _check(rc, "maxscore_assign_top1_sinkhorn")
    return dict(assign=assign, plan=plan, caps=list(caps))


def gates(scores, assign):
    """a5: gates[T,k] = scores[i, assign[i,s]]."""
    torch = _torch()
    T, E = scores.shape
    k = assign.shape[1]
    out = torch.empty((T, k), dtype=torch.float32, device=scores.device)
    _check(load_library().maxscore_gates(_ptr(scores), _ptr(assign), T, E, k, _ptr(out), _stream()),
           "maxscore_gates")
    return out


def dispatch(assign, gate, E: int, C: int = 1):
    """a6: dict(expert_offsets[E+1], disp_token[T*k], disp_gate[T*k], token_pos[T,k])."""
    torch = _torch()
    T, k = assign.shape
    dev = assign.device
    offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
    disp_token = torch.full((T * k,), -1, dtype=torch.int32, device=dev)
    disp_gate = torch.zeros(T * k, dtype=torch.float32, device=dev) if gate is not None else None
    token_pos = torch.empty((T, k), dtype=torch.int32, device=dev)
    ws, need = _workspace(T, E, k, max(C, 1), dev)
    rc = load_library().maxscore_dispatch(_ptr(assign), _ptr(gate), T, E, k, _ptr(offsets), _ptr(disp_token),
                                          _ptr(disp_gate), _ptr(token_pos), _ptr(ws), need, _stream())
    _check(rc, "maxscore_dispatch")
    return dict(expert_offsets=offsets, disp_token=disp_token, disp_gate=disp_gate, token_pos=token_pos)


def dispatch_static(assign, gate, E: int, out: Optional[dict] = None):
    """a6 through the entry point that uses the library's built-in scratch (no workspace, nothing allocated by the
    call itself: pass `out` to reuse output tensors)."""
    torch = _torch()
    T, k = assign.shape
    dev = assign.device
    if out is None:
        out = dict(expert_offsets=torch.empty(E + 1, dtype=torch.int32, device=dev),
                   disp_token=torch.full((T * k,), -1, dtype=torch.int32, device=dev),
                   disp_gate=torch.zeros(T * k, dtype=torch.float32, device=dev) if gate is not None else None,
                   token_pos=torch.empty((T, k), dtype=torch.int32, device=dev))
    rc = load_library().maxscore_dispatch_static(_ptr(assign), _ptr(gate), T, E, k, _ptr(out["expert_offsets"]),
                                                 _ptr(out["disp_token"]), _ptr(out["disp_gate"]),
                                                 _ptr(out["token_pos"]), _stream())
    _check(rc, "maxscore_dispatch_static")
    return out


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return 0
    if t.dtype == torch.float32:
        return 1
    raise TypeError("bf16 or fp32 expected")


def dispatch_tokens(x, expert_offsets, disp_token, E: int, C: int, out=None):
    """Expert input buffers [E, C, d] (dtype of x): rows of x in dispatch order, zero padding."""
    torch = _torch()
    T, d = x.shape
    assert x.is_contiguous()
    if out is None:
        out = torch.empty((E, C, d), dtype=x.dtype, device=x.device)
    rc = load_library().maxscore_dispatch_tokens(_ptr(x), _dtype_code(x), _ptr(expert_offsets), _ptr(disp_token),
                                                 T, d, E, C, _ptr(out), _stream())
    _check(rc, "maxscore_dispatch_tokens")
    return out


def combine(expert_out, assign, token_pos, gate, out=None):
    """y[T, d] fp32 = sum_s gate[i, s] * expert_out[assign[i, s], token_pos[i, s], :] (Eq. 1)."""
    torch = _torch()
    E, C, d = expert_out.shape
    T, k = assign.shape
    assert expert_out.is_contiguous()
    if out is None:
        out = torch.empty((T, d), dtype=torch.float32, device=expert_out.device)
    rc = load_library().maxscore_combine(_ptr(expert_out), _dtype_code(expert_out), _ptr(assign), _ptr(token_pos),
                                         _ptr(gate), T, d, E, k, C, _ptr(out), _stream())
    _check(rc, "maxscore_combine")
    return out


def _route_outputs(T, E, k, dev):
    torch = _torch()
    return dict(scores=torch.empty((T, E), dtype=torch.float32, device=dev),
                q=torch.empty((T, E), dtype=torch.int32, device=dev),
                assign=torch.empty((T, k), dtype=torch.int32, device=dev),
                gates=torch.empty((T, k), dtype=torch.float32, device=dev),
                expert_offsets=torch.empty(E + 1, dtype=torch.int32, device=dev),
                disp_token=torch.empty(T * k, dtype=torch.int32, device=dev),
                disp_gate=torch.empty(T * k, dtype=torch.float32, device=dev),
                token_pos=torch.empty((T, k), dtype=torch.int32, device=dev),
                prices=torch.empty(E, dtype=torch.int64, device=dev))


def route_logits(logits, k: int, C: int, t: float = 1.0, quant_shift: int = 20, max_rounds: int = 200000,
                 eps_div: int = 12, out: Optional[dict] = None, assignment: str = "exact",
                 allow_not_converged: bool = False):
    """a2..a6 from logits; assignment = "exact" (the solver) or "iter" (iterative rerouting)."""
    torch = _torch()
    T, E = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    o = out if out is not None else _route_outputs(T, E, k, logits.device)
    ws, need = _workspace(T, E, k, C, logits.device)
    stats = Stats()
    opts = _opts(t, quant_shift, max_rounds, eps_div, assignment)
    rc = load_library().maxscore_route_logits(
        _ptr(logits), T, E, k, C, ctypes.byref(opts), _ptr(o["scores"]), _ptr(o["q"]), _ptr(o["assign"]),
        _ptr(o["gates"]), _ptr(o["expert_offsets"]), _ptr(o["disp_token"]), _ptr(o["disp_gate"]),
        _ptr(o["token_pos"]), _ptr(o["prices"]), ctypes.byref(stats), _ptr(ws), need, _stream())
    _check(rc, "maxscore_route_logits", allow=(ERR_NOT_CONVERGED,) if allow_not_converged else ())
    o = dict(o)
    o["stats"] = stats.as_dict()
    o["rc"] = rc
    return o


def route_scores(scores, k: int, C: int, quant_shift: int = 20, max_rounds: int = 200000, eps_div: int = 12,
                 out: Optional[dict] = None, assignment: str = "exact", allow_not_converged: bool = False):
    """a3..a6 from given fp32 scores [T, E]."""
    torch = _torch()
    T, E = scores.shape
    assert scores.dtype == torch.float32 and scores.is_contiguous()
    o = out if out is not None else _route_outputs(T, E, k, scores.device)
    ws, need = _workspace(T, E, k, C, scores.device)
    stats = Stats()
    opts = _opts(1.0, quant_shift, max_rounds, eps_div, assignment)
    rc = load_library().maxscore_route_scores(
        _ptr(scores), T, E, k, C, ctypes.byref(opts), _ptr(o["q"]), _ptr(o["assign"]), _ptr(o["gates"]),
        _ptr(o["expert_offsets"]), _ptr(o["disp_token"]), _ptr(o["disp_gate"]), _ptr(o["token_pos"]),
        _ptr(o["prices"]), ctypes.byref(stats), _ptr(ws), need, _stream())
    _check(rc, "maxscore_route_scores", allow=(ERR_NOT_CONVERGED,) if allow_not_converged else ())
    o = dict(o)
    o["scores"] = scores
    o["stats"] = stats.as_dict()
    o["rc"] = rc
    return o


def route_xw(x, W, bias, k: int, C: int, t: float = 1.0, quant_shift: int = 20, max_rounds: int = 200000,
             eps_div: int = 12, out: Optional[dict] = None, assignment: str = "exact", want_logits: bool = True):
    """a1..a6 from x and W_g.  want_logits=False passes no logits buffer (accepted where the library computes the
    scores inside the projection kernel; MaxScoreError -1 otherwise)."""
    torch = _torch()
    T, d = x.shape
    E = W.shape[1]
    assert W.shape[0] == d and x.is_contiguous() and W.is_contiguous() and x.dtype == W.dtype
    o = out if out is not None else _route_outputs(T, E, k, x.device)
    if "logits" not in o:
        o["logits"] = torch.empty((T, E), dtype=torch.float32, device=x.device) if want_logits else None
    ws, need = _workspace(T, E, k, C, x.device, d)
    stats = Stats()
    opts = _opts(t, quant_shift, max_rounds, eps_div, assignment)
    rc = load_library().maxscore_route_xw(
        _ptr(x), _ptr(W), _ptr(bias), _in_dtype(x), T, d, E, k, C, ctypes.byref(opts), _ptr(o["logits"]),
        _ptr(o["scores"]), _ptr(o["q"]), _ptr(o["assign"]), _ptr(o["gates"]), _ptr(o["expert_offsets"]),
        _ptr(o["disp_token"]), _ptr(o["disp_gate"]), _ptr(o["token_pos"]), _ptr(o["prices"]),
        ctypes.byref(stats), _ptr(ws), need, _stream())
    _check(rc, "maxscore_route_xw")
    o = dict(o)
    o["stats"] = stats.as_dict()
    return o
