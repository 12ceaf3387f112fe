"""Slow, plain CPU implementation of the MaxScore routing path (TEST INFRASTRUCTURE).

Only tests, the smoke check and the benchmark's cpu_baseline leg may call this package; the
product library never does, and this package imports nothing from the product.

Everything is fp64 / int64 and written to be checked against the paper by eye:

  router_logits      Eq. 2 / Algorithm 1 step 2:  L = x . W_g (+ optional per-expert bias)
  softmax_rows       Table 2 row 1
  soft_topk          Eq. 6 (reading stated in the function)
  quantise           integer rewards round(A * 2^shift)
  max_score_assignment   Eq. 7-8 / Table 1, successive cheapest augmenting paths (mcmf.c)
  gates              Eq. 2: the affinity of each selected (token, expert) pair, not renormalised
  dispatch           per-expert buffers (Section 2.3 capacity layout): stable sort by expert
  verify_optimal     independent optimality proof for any assignment (no negative residual cycle)
  sigmoid_scores, softkmax, itertopk, gradtopk   other operators of Table 2 (base cases are a stated reading)
  aux_loss           Eq. 9 load-balance loss and its derivative with respect to the scores
  gates_backward     derivative of the selected scores (and of Eq. 9) with respect to the logits
  max_score_assignment_caps   the exact assignment with one capacity per expert
  max_score_assignment_kvec   the exact assignment with one k per token (and one capacity per expert)
  top1_then_residual Algorithm 1 steps 4-8 with the residual problem solved exactly
  sinkhorn_plan, top1_then_sinkhorn   Algorithm 1 with Sinkhorn on the residual problem (a stated reading)
  iter_reroute       Section 2.3 iterative rerouting: top-k with capacity, then greedy re-proposal rounds
                     (a heuristic; the processing orders are a stated reading, parity with the
                     authors' code is unpinned)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmcmf_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile mcmf.c with gcc into libmcmf_oracle.so next to this file."""
    src = os.path.join(_HERE, "mcmf.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
        i64p = ctypes.POINTER(ctypes.c_int64)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        _lib.mcmf_literal.argtypes = [i64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      u8p, i64p, i64p, i64p]
        _lib.mcmf_literal.restype = ctypes.c_int
        _lib.mcmf_contracted.argtypes = [i64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         u8p, i64p, i64p, i64p, i64p, i64p]
        _lib.mcmf_contracted.restype = ctypes.c_int
        i32p = ctypes.POINTER(ctypes.c_int)
        _lib.mcmf_literal_caps.argtypes = [i64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p, u8p, i64p, i64p, i64p]
        _lib.mcmf_literal_caps.restype = ctypes.c_int
        _lib.mcmf_contracted_caps.argtypes = [i64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p,
                                              u8p, i64p, i64p, i64p, i64p, i64p]
        _lib.mcmf_contracted_caps.restype = ctypes.c_int
        _lib.mcmf_literal_kc.argtypes = [i64p, ctypes.c_int, ctypes.c_int, i32p, i32p, u8p, i64p, i64p, i64p]
        _lib.mcmf_literal_kc.restype = ctypes.c_int
        _lib.mcmf_contracted_kc.argtypes = [i64p, ctypes.c_int, ctypes.c_int, i32p, i32p,
                                            u8p, i64p, i64p, i64p, i64p, i64p]
        _lib.mcmf_contracted_kc.restype = ctypes.c_int
    return _lib


# ------------------------------------------------------------------------------------------------
# a1  router projection

def router_logits(x: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. 2 / Algorithm 1 step 2: logits = x . W_g in fp64 over the given stored values.
    `bias` (per expert) is a workload device of the synthetic configs, added to the logits."""
    L = np.asarray(x, dtype=np.float64) @ np.asarray(W, dtype=np.float64)
    if bias is not None:
        L = L + np.asarray(bias, dtype=np.float64)[None, :]
    return L


# ------------------------------------------------------------------------------------------------
# a2  SoftTopk

def softmax_rows(L: np.ndarray) -> np.ndarray:
    """Table 2, row 1: y = e^x / sum_j e^x_j per token row (max-subtracted, fp64)."""
    L = np.asarray(L, dtype=np.float64)
    z = np.exp(L - L.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


def descending_rank(L: np.ndarray) -> np.ndarray:
    """1-based rank of each entry within its row, largest first, ties to the lower index."""
    L = np.asarray(L)
    order = np.argsort(-L, axis=1, kind="stable")
    rank = np.empty_like(order)
    rows = np.arange(L.shape[0])[:, None]
    rank[rows, order] = np.arange(1, L.shape[1] + 1)[None, :]
    return rank


def soft_topk(L: np.ndarray, k: int, t: float) -> np.ndarray:
    """Eq. 6, taken level by level.

    Reading: level 1 is Softmax(a); level m (2..k) adds SE^(m), which is t*Softmax(a)_i on the
    entries not among the m-1 largest of a and 0 on those m-1 entries.  The loop below is that
    recursion written out; its closed form is p_i * (1 + t*(min(rank_i, k) - 1)).
    """
    L = np.asarray(L, dtype=np.float64)
    p = softmax_rows(L)
    rank = descending_rank(L)
    A = p.copy()                                   # SoftTopk^(1)
    for m in range(2, k + 1):
        SE = np.where(rank <= m - 1, 0.0, t * p)   # entries already in Top(m-1) get nothing
        A = A + SE                                 # SoftTopk^(m) = SoftTopk^(m-1) + SE
    return A


def soft_topk_reading(L: np.ndarray, k: int, t: float, reading: str) -> np.ndarray:
    """Eq. 6 under the other readings its print admits (it gives no base case, and its SE term does not depend
    on the recursion level as printed).  Each is the recursion SoftTopk^(m) = SoftTopk^(m-1) + SE written out:

    "A"   the reading of soft_topk(): level 1 is Softmax(a), level m = 2..k masks the m-1 largest entries;
    "A1"  level 0 is Softmax(a), level m = 1..k masks the m largest entries (one level more, masks shifted by one);
    "B"   the mask as printed, the k largest entries at every level: level 1 is Softmax(a), levels 2..k each add
          t*Softmax(a) outside the top k and nothing inside it;
    "C"   as "A", with SE renormalised over the entries it is added to (t * p_i / sum of the unmasked p), in the
          manner of the iterated operators of Table 2: every level adds a distribution scaled by t.
    Ranks as in soft_topk (equal logits: lower index first)."""
    L = np.asarray(L, dtype=np.float64)
    p = softmax_rows(L)
    rank = descending_rank(L)
    A = p.copy()
    if reading == "A":
        return soft_topk(L, k, t)
    if reading == "A1":
        for m in range(1, k + 1):
            A = A + np.where(rank <= m, 0.0, t * p)
        return A
    if reading == "B":
        for m in range(2, k + 1):
            A = A + np.where(rank <= k, 0.0, t * p)
        return A
    if reading == "C":
        for m in range(2, k + 1):
            free = rank > m - 1
            mass = np.where(free, p, 0.0).sum(axis=1, keepdims=True)
            A = A + np.where(free, t * p / mass, 0.0)
        return A
    raise ValueError(reading)


# ------------------------------------------------------------------------------------------------
# a3  integer rewards

def quantise(A: np.ndarray, shift: int = 20) -> np.ndarray:
    """q = round-half-even(A * 2^shift) as int64."""
    return np.rint(np.asarray(A, dtype=np.float64) * float(1 << shift)).astype(np.int64)


# ------------------------------------------------------------------------------------------------
# a4  assignment

def _as_q(q) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int64)
    assert q.ndim == 2
    return q


def assign_literal_graph(q, k: int, C: int) -> dict:
    """Successive cheapest paths on the literal graph of Table 1.  Any sizes; small inputs only."""
    q = _as_q(q)
    T, E = q.shape
    P = np.zeros((T, E), dtype=np.uint8)
    flow, total, arcs = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = _load().mcmf_literal(q.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), T, E, k, C,
                              P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                              ctypes.byref(flow), ctypes.byref(total), ctypes.byref(arcs))
    if rc:
        raise ValueError(f"mcmf_literal failed rc={rc}")
    return dict(P=P, flow=flow.value, total=total.value, arcs=arcs.value)


def assign_contracted(q, k: int, C: int) -> dict:
    """Same optimum with the token layer contracted (needs T*k <= E*min(C,T))."""
    q = _as_q(q)
    T, E = q.shape
    P = np.zeros((T, E), dtype=np.uint8)
    prices = np.zeros(E, dtype=np.int64)
    flow, total, paths, hops = (ctypes.c_int64() for _ in range(4))
    rc = _load().mcmf_contracted(q.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), T, E, k, C,
                                 P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                 prices.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                 ctypes.byref(flow), ctypes.byref(total), ctypes.byref(paths),
                                 ctypes.byref(hops))
    if rc:
        raise ValueError(f"mcmf_contracted failed rc={rc}")
    return dict(P=P, prices=prices, flow=flow.value, total=total.value, paths=paths.value,
                hops=hops.value)


def max_score_assignment(q, k: int, C: int) -> dict:
    """Exact maximum-flow-then-maximum-score assignment; picks the solver by the precondition."""
    q = _as_q(q)
    T, E = q.shape
    if T * k <= E * min(C, T):
        return assign_contracted(q, k, C)
    return assign_literal_graph(q, k, C)


def max_score_assignment_caps(q, k: int, caps) -> dict:
    """The same optimum with a capacity of its own for every expert (the vector c of Eq. 7; Table 1's
    Expert_j -> Sink arc gets capacity caps[j]).  Contracted solver when T*k <= sum_j min(caps_j, T),
    literal graph otherwise."""
    q = _as_q(q)
    T, E = q.shape
    caps = np.ascontiguousarray(caps, dtype=np.int32)
    assert caps.shape == (E,) and (caps >= 0).all()
    P = np.zeros((T, E), dtype=np.uint8)
    cp = caps.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
    qp = q.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    Pp = P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    if T * k <= int(np.minimum(caps, T).sum()):
        prices = np.zeros(E, dtype=np.int64)
        flow, total, paths, hops = (ctypes.c_int64() for _ in range(4))
        rc = _load().mcmf_contracted_caps(qp, T, E, k, cp, Pp, prices.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                          ctypes.byref(flow), ctypes.byref(total), ctypes.byref(paths),
                                          ctypes.byref(hops))
        if rc:
            raise ValueError(f"mcmf_contracted_caps failed rc={rc}")
        return dict(P=P, prices=prices, flow=flow.value, total=total.value)
    flow, total, arcs = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = _load().mcmf_literal_caps(qp, T, E, k, cp, Pp, ctypes.byref(flow), ctypes.byref(total), ctypes.byref(arcs))
    if rc:
        raise ValueError(f"mcmf_literal_caps failed rc={rc}")
    return dict(P=P, flow=flow.value, total=total.value)


def max_score_assignment_kvec(q, kvec, C, solver: str = "auto") -> dict:
    """The same optimum with a k of its own for every token (the vector k of Eq. 7; Table 1's Source -> Token_i
    arc gets capacity kvec[i]) and C either one capacity for all experts or one per expert.  Contracted solver
    when every kvec[i] <= E and sum_i kvec[i] <= sum_j min(C_j, T) (with one capacity for all experts every
    token then ships all its units: a deficient expert set J would need more than C tokens with more than
    E - |J| units each, i.e. more than E*C units in total; with unequal capacities the contracted solver can
    report that a token cannot ship all its units, and the literal graph takes over); literal graph otherwise.  `solver` = "literal" or
    "contracted" forces one of them."""
    q = _as_q(q)
    T, E = q.shape
    kvec = np.ascontiguousarray(kvec, dtype=np.int32)
    caps = np.ascontiguousarray(np.broadcast_to(np.asarray(C, dtype=np.int32), (E,)))
    assert kvec.shape == (T,) and (kvec >= 0).all() and (caps >= 0).all()
    P = np.zeros((T, E), dtype=np.uint8)
    i32p, i64p = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int64)
    qp, kp, cp = q.ctypes.data_as(i64p), kvec.ctypes.data_as(i32p), caps.ctypes.data_as(i32p)
    Pp = P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    fits = int(kvec.max(initial=0)) <= E and int(kvec.sum()) <= int(np.minimum(caps, T).sum())
    if solver == "contracted" or (solver == "auto" and fits):
        prices = np.zeros(E, dtype=np.int64)
        flow, total, paths, hops = (ctypes.c_int64() for _ in range(4))
        rc = _load().mcmf_contracted_kc(qp, T, E, kp, cp, Pp, prices.ctypes.data_as(i64p), ctypes.byref(flow),
                                        ctypes.byref(total), ctypes.byref(paths), ctypes.byref(hops))
        if rc == 0:
            return dict(P=P, prices=prices, flow=flow.value, total=total.value)
        if rc != 4 or solver == "contracted":
            raise ValueError(f"mcmf_contracted_kc failed rc={rc}")
        P[:] = 0          # some token cannot ship all its units: the literal graph decides who ships what
    flow, total, arcs = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = _load().mcmf_literal_kc(qp, T, E, kp, cp, Pp, ctypes.byref(flow), ctypes.byref(total), ctypes.byref(arcs))
    if rc:
        raise ValueError(f"mcmf_literal_kc failed rc={rc}")
    return dict(P=P, flow=flow.value, total=total.value)


def max_flow_value(T: int, E: int, k: int, C: int) -> int:
    """Flow value of the complete bipartite network of Table 1 when k <= E."""
    return min(T * k, E * min(C, T))


def assignment_matrix(assign: np.ndarray, E: int) -> np.ndarray:
    """[T, k] expert ids (-1 = empty slot) -> P in {0,1}^{T x E}; rejects repeated experts."""
    assign = np.asarray(assign)
    T = assign.shape[0]
    P = np.zeros((T, E), dtype=np.int64)
    rows, cols = np.nonzero(assign >= 0)
    np.add.at(P, (rows, assign[rows, cols]), 1)
    if P.max(initial=0) > 1:
        raise ValueError("a token holds the same expert twice")
    return P.astype(np.uint8)


def check_feasible(P: np.ndarray, k: int, C: int) -> Tuple[bool, str]:
    """Row sums <= k, column sums <= C, flow value = min(T*k, E*min(C,T)) (Eq. 7 read as <=)."""
    P = np.asarray(P).astype(np.int64)
    T, E = P.shape
    if P.min(initial=0) < 0 or P.max(initial=0) > 1:
        return False, "P not binary"
    if P.sum(axis=1).max(initial=0) > k:
        return False, "a token exceeds k experts"
    if P.sum(axis=0).max(initial=0) > C:
        return False, "an expert exceeds capacity"
    if int(P.sum()) != max_flow_value(T, E, k, C):
        return False, f"flow {int(P.sum())} != {max_flow_value(T, E, k, C)}"
    return True, ""


def verify_optimal(q, P, k, C) -> dict:
    """C is one capacity for all experts or an array with one capacity per expert; k is one number for all
    tokens or an array with one k per token.
    Proof of optimality for a feasible maximum-flow P when T*k <= E*min(C,T), independent of
    how P was found: the residual network, with tokens contracted, has experts and the sink as
    nodes; arc j->j' costs min over tokens on j and not on j' of q_uj - q_uj'; j->sink costs 0
    if j has spare capacity; sink->j costs 0 if j holds a token.  P is optimal iff no negative
    cycle exists (Bellman-Ford from a virtual root).  The resulting potentials give expert
    prices p >= 0 (0 on unfilled experts) under which every token holds its k best q_ij - p_j:
    complementary slackness of the LP dual of Eq. 7-8."""
    q = _as_q(q)
    P = np.asarray(P).astype(bool)
    T, E = q.shape
    Ce = np.minimum(np.broadcast_to(np.asarray(C, dtype=np.int64), (E,)), T)
    kv = np.broadcast_to(np.asarray(k, dtype=np.int64), (T,))
    assert int(kv.sum()) <= int(Ce.sum())
    load = P.sum(axis=0)
    INF = np.int64(1) << 60
    Lm = np.full((E + 1, E + 1), INF, dtype=np.int64)      # node E = sink
    for j in range(E):
        rows = np.nonzero(P[:, j])[0]
        if rows.size:
            diff = q[rows, j][:, None] - q[rows, :]          # cost of moving u from j to j'
            diff = np.where(P[rows, :], INF, diff)
            Lm[j, :E] = diff.min(axis=0)
            Lm[E, j] = 0
        Lm[j, j] = INF
        if load[j] < Ce[j]:
            Lm[j, E] = 0
    dist = np.zeros(E + 1, dtype=np.int64)
    changed = True
    for _ in range(E + 2):
        cand = (dist[:, None] + np.minimum(Lm, INF // 2)).min(axis=0)
        new = np.minimum(dist, cand)
        changed = bool((new != dist).any())
        dist = new
        if not changed:
            break
    optimal = not changed
    prices = dist[E] - dist[:E]                               # p_j = phi_sink - phi_j
    prices = np.where(load == 0, np.maximum(prices, 0), prices)  # nobody holds j: any p_j >= 0 above it works
    ok_cs = False
    if optimal:
        net = q - prices[None, :]
        held_min = np.where(P, net, INF).min(axis=1)
        unheld_max = np.where(P, -INF, net).max(axis=1)
        ok_cs = bool((held_min >= unheld_max).all() and (prices >= 0).all()
                     and (prices[load < Ce] == 0).all() and (P.sum(axis=1) == kv).all())
    return dict(optimal=optimal and ok_cs, prices=prices, total=int(q[P].sum()))


# ------------------------------------------------------------------------------------------------
# a5  gates

def gates(A: np.ndarray, assign: np.ndarray) -> np.ndarray:
    """Eq. 2: R(x) keeps the affinity A_ij of every selected pair (no renormalisation);
    empty slots (-1) get 0."""
    A = np.asarray(A, dtype=np.float64)
    assign = np.asarray(assign)
    rows = np.arange(A.shape[0])[:, None]
    g = A[rows, np.maximum(assign, 0)]
    return np.where(assign >= 0, g, 0.0)


# ------------------------------------------------------------------------------------------------
# a6  dispatch

def dispatch(assign: np.ndarray, gate: np.ndarray, E: int) -> dict:
    """Per-expert buffers in compact form: all (expert, token) pairs sorted by expert, then by
    token id (stable sort); offsets = exclusive prefix sum of the per-expert counts.
    token_pos[i, s] is the position of pair (i, assign[i, s]) inside its expert's buffer."""
    assign = np.asarray(assign)
    gate = np.asarray(gate)
    T, k = assign.shape
    tok, slot = np.nonzero(assign >= 0)                  # row-major: token ascending
    exp = assign[tok, slot]
    order = np.argsort(exp, kind="stable")
    tok_s, slot_s, exp_s = tok[order], slot[order], exp[order]
    counts = np.bincount(exp, minlength=E).astype(np.int64)
    offsets = np.zeros(E + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts)
    token_pos = np.full((T, k), -1, dtype=np.int64)
    token_pos[tok_s, slot_s] = np.arange(exp_s.size) - offsets[exp_s]
    return dict(expert_offsets=offsets, disp_token=tok_s.astype(np.int64),
                disp_gate=gate[tok_s, slot_s], token_pos=token_pos)


# ------------------------------------------------------------------------------------------------
# activation movement around the experts (Eq. 1; capacity buffers of Section 2.3)

def dispatch_tokens(x, expert_offsets, disp_token, E: int, C: int) -> np.ndarray:
    """Expert input buffers [E, C, d]: slot s of expert j holds the activation row of the s-th token
    dispatched to j (ascending token id); the slots past the expert's count are zero."""
    x = np.asarray(x)
    off = np.asarray(expert_offsets)
    tok = np.asarray(disp_token)
    buf = np.zeros((E, C, x.shape[1]), dtype=x.dtype)
    for j in range(E):
        n = int(off[j + 1] - off[j])
        if n > C:
            raise ValueError("an expert holds more tokens than its capacity")
        buf[j, :n] = x[tok[off[j]:off[j + 1]]]
    return buf


def combine(expert_out, assign, token_pos, gate) -> np.ndarray:
    """Eq. 1: y_i = sum over the selected experts of gate * expert output, read back from the
    expert output buffers [E, C, d] at the slot the token was dispatched to (fp64)."""
    buf = np.asarray(expert_out, dtype=np.float64)
    assign = np.asarray(assign)
    pos = np.asarray(token_pos)
    g = np.asarray(gate, dtype=np.float64)
    T, k = assign.shape
    y = np.zeros((T, buf.shape[2]), dtype=np.float64)
    for s in range(k):
        ok = assign[:, s] >= 0
        rows = buf[assign[ok, s], pos[ok, s]]
        y[ok] += g[ok, s, None] * rows
    return y


# ------------------------------------------------------------------------------------------------
# whole path

def route(x, W, bias, k: int, C: int, t: float, shift: int = 20) -> dict:
    """x, W -> logits -> SoftTopk -> integer rewards -> exact assignment -> gates -> dispatch."""
    L = router_logits(x, W, bias)
    return route_from_logits(L, k, C, t, shift)


def route_from_logits(L, k: int, C: int, t: float, shift: int = 20) -> dict:
    L = np.asarray(L, dtype=np.float64)
    A = soft_topk(L, k, t)
    q = quantise(A, shift)
    sol = max_score_assignment(q, k, C)
    P = sol["P"].astype(bool)
    T, E = P.shape
    assign = np.full((T, k), -1, dtype=np.int64)
    for i in range(T):
        js = np.nonzero(P[i])[0]
        assign[i, : js.size] = js
    g = gates(A, assign)
    out = dict(logits=L, scores=A, q=q, P=sol["P"], assign=assign, gates=g, total=sol["total"],
               flow=sol["flow"], prices=sol.get("prices"))
    out.update(dispatch(assign, g, E))
    return out


# ------------------------------------------------------------------------------------------------
# iterative rerouting (Section 2.3; the assignment step of the "-I" variants of Section 4)

def _accept_in_order(e_sorted_by_priority: np.ndarray, room: np.ndarray) -> np.ndarray:
    """For a list of expert ids in priority order, mark the entries an expert still has room for:
    expert j takes its first room[j] entries."""
    e = np.asarray(e_sorted_by_priority)
    order = np.argsort(e, kind="stable")
    es = e[order]
    within = np.arange(es.size) - np.searchsorted(es, es, side="left")
    ok = np.zeros(e.size, dtype=bool)
    ok[order] = within < room[es]
    return ok


def iter_reroute(q, k: int, C: int, max_rounds: Optional[int] = None) -> dict:
    """Two-stage greedy assignment on integer rewards.  The paper gives the two stages in one
    sentence; the orders below are this build's reading of it.

    Stage 1 (top-k with capacity): every token lists its k highest-reward experts (ties to the
    lower expert id).  The pairs are taken in the order (choice rank, token id): all first choices
    before all second choices, tokens in sequence order inside a rank.  An expert keeps the first
    C pairs that name it; the others are dropped and leave a hole in slot `rank` of the token.

    Stage 2 (rerouting), in synchronous rounds: at the start of a round the experts with room left
    are fixed.  Every token fills its holes in slot order with proposals: the highest-reward expert
    that has room, that the token does not hold and has not proposed in this round.  The
    proposals are then taken in the order (slot, token id) and an expert accepts while it has room.
    Rounds repeat until nobody can propose.

    Returns assign [T, k] (-1 = hole left), the stage-1 assignment, per-expert load, total reward,
    flow and the number of stage-2 rounds that had proposals."""
    q = _as_q(q)
    T, E = q.shape
    assert 1 <= k <= E
    choice = np.argsort(-q, axis=1, kind="stable")[:, :k]
    assign = np.full((T, k), -1, dtype=np.int64)
    load = np.zeros(E, dtype=np.int64)
    for s in range(k):                                   # stage 1, one choice rank at a time
        e = choice[:, s]
        ok = _accept_in_order(e, C - load)               # tokens already in id order
        assign[ok, s] = e[ok]
        load += np.bincount(e[ok], minlength=E)
    stage1 = assign.copy()
    rounds = 0
    NEG = -(np.int64(1) << 62)                       # below any reward; its negation still fits
    while max_rounds is None or rounds < max_rounds:
        holes = assign < 0
        rows = np.nonzero(holes.any(axis=1))[0]
        room = C - load
        if rows.size == 0 or not (room > 0).any():
            break
        sub = assign[rows]
        held = np.zeros((rows.size, E), dtype=bool)
        r_idx, s_idx = np.nonzero(sub >= 0)
        held[r_idx, sub[r_idx, s_idx]] = True
        cand = (room > 0)[None, :] & ~held
        pref = np.argsort(-np.where(cand, q[rows], NEG), axis=1, kind="stable")   # best candidate first
        ncand = cand.sum(axis=1)
        nth_hole = np.cumsum(holes[rows], axis=1) - 1                              # per slot: index among the token's holes
        prop = np.full((T, k), -1, dtype=np.int64)
        r_idx, s_idx = np.nonzero(holes[rows])
        h = nth_hole[r_idx, s_idx]
        can = h < ncand[r_idx]
        prop[rows[r_idx[can]], s_idx[can]] = pref[r_idx[can], h[can]]
        if not (prop >= 0).any():
            break
        rounds += 1
        s_list, i_list = np.nonzero(prop.T >= 0)          # (slot, token) order
        e_list = prop[i_list, s_list]
        ok = _accept_in_order(e_list, room)
        assign[i_list[ok], s_list[ok]] = e_list[ok]
        load += np.bincount(e_list[ok], minlength=E)
    got = assign >= 0
    total = int(q[np.nonzero(got)[0], assign[got]].sum())
    return dict(assign=assign, stage1=stage1, load=load, total=total, flow=int(got.sum()), rounds=rounds)


# ------------------------------------------------------------------------------------------------
# training-side by-products: load-balance loss (Eq. 9) and the derivative of the gates

def aux_loss(A, assign, lam: float) -> dict:
    """Eq. 9: lambda * (1/e) * sum_j mean_i(A_ij) * mean_i(P_ij), P the binary assignment.
    Also returns the two column means and dL/dA_ij = lambda/(e*n) * mean_i(P_ij) (P is a constant)."""
    A = np.asarray(A, dtype=np.float64)
    T, E = A.shape
    P = assignment_matrix(assign, E).astype(np.float64)
    mean_A = A.sum(axis=0) / T
    mean_P = P.sum(axis=0) / T
    loss = lam * (mean_A * mean_P).sum() / E
    return dict(loss=float(loss), mean_A=mean_A, mean_P=mean_P, dA=lam / (E * T) * mean_P)


def gates_backward(L, k: int, t: float, assign, dgate, dA_all=None) -> np.ndarray:
    """d(loss)/d(logits) through the gates of Eq. 2 with SoftTopk scores (Eq. 6) whose rank
    multipliers are constants (they are piecewise constant in the logits, so this is the derivative
    wherever no two logits of a row tie): A_ij = m_ij * p_ij, p = Softmax(L_i), hence
    dA_ij/dL_il = A_ij * (delta_jl - p_il).  The upstream gradient is dgate[i, s] on the selected
    pairs plus, optionally, dA_all[j] on every entry of column j (the Eq. 9 term)."""
    L = np.asarray(L, dtype=np.float64)
    T, E = L.shape
    p = softmax_rows(L)
    A = soft_topk(L, k, t)
    gA = np.zeros((T, E), dtype=np.float64)
    assign = np.asarray(assign)
    dgate = np.asarray(dgate, dtype=np.float64)
    for s in range(assign.shape[1]):
        ok = assign[:, s] >= 0
        np.add.at(gA, (np.nonzero(ok)[0], assign[ok, s]), dgate[ok, s])
    if dA_all is not None:
        gA = gA + np.asarray(dA_all, dtype=np.float64)[None, :]
    w = gA * A
    return w - p * w.sum(axis=1, keepdims=True)


# ------------------------------------------------------------------------------------------------
# Algorithm 1 (top-2): top-1 first, then the residual problem

def top1_then_residual(q, C: int) -> dict:
    """Algorithm 1, steps 4-8, with the residual problem of step 9 solved exactly instead of by
    Sinkhorn (the paper does not give Sinkhorn's iteration count, regulariser or rounding):
    every token takes its highest-reward expert (ties to the lower id) whatever the load;
    that entry of the reward matrix is set to 0; the capacities become max(0, C - load_j); each
    token then gets one more expert (k_i = 1) by the exact assignment on the residual problem.
    Returns assign [T, 2] = (top-1 expert, second expert), the residual capacities, the total of the
    original rewards over both choices, and `repeat`: tokens whose second expert is their top-1
    expert again (possible because step 5 zeroes the entry instead of forbidding it)."""
    q = _as_q(q)
    T, E = q.shape
    top1 = np.argmax(q, axis=1)                       # first maximum = lower expert id
    load = np.bincount(top1, minlength=E)
    caps = np.maximum(0, C - load)
    q2 = q.copy()
    q2[np.arange(T), top1] = 0
    sol = max_score_assignment_caps(q2, 1, caps)
    P2 = sol["P"].astype(bool)
    second = np.where(P2.any(axis=1), P2.argmax(axis=1), -1)
    assign = np.stack([top1, second], axis=1).astype(np.int64)
    got = second >= 0
    total = int(q[np.arange(T), top1].sum() + q[np.nonzero(got)[0], second[got]].sum())
    return dict(assign=assign, caps=caps, q_residual=q2, residual_total=sol["total"], residual_flow=sol["flow"],
                total=total, repeat=int((second == top1).sum()))


# ------------------------------------------------------------------------------------------------
# other routing operators of Table 2 (alternatives to SoftTopk for the affinity scores)

def sigmoid_scores(L: np.ndarray) -> np.ndarray:
    """Table 2, row 2: y = 1 / (1 + e^-x), element-wise."""
    return 1.0 / (1.0 + np.exp(-np.asarray(L, dtype=np.float64)))


def softkmax(L: np.ndarray, k: int) -> np.ndarray:
    """Table 2, SoftKmax: y^(m) = y^(m-1) + Softmax(g^(m-1)), g^(m-1) = (1 - y^(m-1)) (x) x.
    The table gives no base case; reading: y^(0) = 0, so that level 1 is Softmax(x)."""
    x = np.asarray(L, dtype=np.float64)
    y = np.zeros_like(x)
    for _ in range(k):
        g = (1.0 - y) * x
        y = y + softmax_rows(g)
    return y


def itertopk(L: np.ndarray, k: int) -> np.ndarray:
    """Table 2, IterTopk: y^(m) = y^(m-1) + g(x; 1 - y^(m-1)), g(x; w) = w e^x / sum_j w_j e^x_j.
    Base case as above: y^(0) = 0.  The weights 1 - y may turn negative from level 3 on; the
    expression is evaluated as printed."""
    x = np.asarray(L, dtype=np.float64)
    ex = np.exp(x - x.max(axis=1, keepdims=True))      # a common factor of e^x cancels in g
    y = np.zeros_like(x)
    for _ in range(k):
        w = 1.0 - y
        y = y + w * ex / (w * ex).sum(axis=1, keepdims=True)
    return y


# ------------------------------------------------------------------------------------------------
# Algorithm 1, step 9 as the paper does it: Sinkhorn on the residual problem

def sinkhorn_plan(a_res, caps, tau: float, n_iter: int) -> dict:
    """Matrix scaling for the residual problem of Algorithm 1 (row sums k_i = 1, column sums
    proportional to the residual capacities).  The paper names the algorithm only; the regulariser,
    the iteration count and the rounding are this build's reading:

      K_ij = exp(a_ij / tau) on experts with caps_j > 0, else 0   (rows are max-shifted first,
                                                                   which the row scaling absorbs)
      m_j  = caps_j * T / sum(caps)                                (column targets, total T)
      v = 1;  n_iter times:  u_i = 1 / sum_j K_ij v_j ;  v_j = m_j / sum_i K_ij u_i
      plan_ij = u_i K_ij v_j   (u = 1 when n_iter = 0)
      second_i = argmax_j plan_ij (ties to the lower expert id), -1 if the row is all zero."""
    a = np.asarray(a_res, dtype=np.float64)
    T, E = a.shape
    caps = np.asarray(caps, dtype=np.float64)
    live = caps > 0
    K = np.exp((a - a.max(axis=1, keepdims=True)) / tau) * live[None, :]
    m = caps * (T / caps.sum()) if caps.sum() > 0 else caps
    u = np.ones(T)
    v = np.ones(E)
    for _ in range(n_iter):
        u = 1.0 / (K @ v)
        v = np.where(live, m / np.maximum(K.T @ u, 1e-300), 0.0)
    plan = u[:, None] * K * v[None, :]
    second = np.where(plan.max(axis=1) > 0, plan.argmax(axis=1), -1)
    return dict(plan=plan, second=second, u=u, v=v, targets=m)


def top1_then_sinkhorn(A, C: int, tau: float, n_iter: int) -> dict:
    """Algorithm 1 on the affinity scores A: steps 4-8 as in top1_then_residual (on the scores
    themselves), step 9 by sinkhorn_plan.  Returns assign [T, 2], the residual capacities, the plan
    and the per-expert load of the second choices."""
    A = np.asarray(A, dtype=np.float64)
    T, E = A.shape
    top1 = np.argmax(A, axis=1)
    load = np.bincount(top1, minlength=E)
    caps = np.maximum(0, C - load)
    a_res = A.copy()
    a_res[np.arange(T), top1] = 0.0
    sk = sinkhorn_plan(a_res, caps, tau, n_iter)
    second = sk["second"]
    assign = np.stack([top1, second], axis=1).astype(np.int64)
    load2 = np.bincount(second[second >= 0], minlength=E)
    return dict(assign=assign, caps=caps, plan=sk["plan"], load2=load2, a_res=a_res, v=sk["v"], u=sk["u"])


def gradtopk(L: np.ndarray, k: int) -> np.ndarray:
    """Table 2, GradTopk, level by level as printed:
        g^(m) = x + log(e^{z^(m-1)} - e^{g^(m-1)}),  z^(m) = log sum_j e^{g^(m)_j} - log m,  y^(m) = e^{g^(m) - z^(m)}.
    The table gives no base case; reading: e^{z^(0)} - e^{g^(0)} = 1, i.e. g^(1) = x, so that level 1 is
    Softmax(x).  Where a level-(m-1) value reaches 1 the logarithm has no real value: NaN, as printed."""
    x = np.asarray(L, dtype=np.float64)
    g = x.copy()
    with np.errstate(invalid="ignore", divide="ignore"):
        for m in range(1, k + 1):
            if m > 1:
                g = x + np.log(np.exp(z) - np.exp(g))
            gm = np.where(np.isnan(g), -np.inf, g).max(axis=1, keepdims=True)
            z = gm + np.log(np.exp(g - gm).sum(axis=1, keepdims=True)) - np.log(m)
        return np.exp(g - z)
