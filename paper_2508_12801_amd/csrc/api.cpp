// Host side of the C ABI: argument validation, workspace carving, stream enqueue.
#include <cstring>

#include "common.h"

namespace maxscore {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

WorkspaceLayout workspace_layout(int T, int E, int k, int d)
{
    WorkspaceLayout L;
    size_t off = 0;
    L.state_off = off; off = align_up(off + 2 * sizeof(SolverState), 256);
    L.theta_off = off; off = align_up(off + sizeof(long long) * 2 * kMaxE, 256);
    L.gcount_off = off; off = align_up(off + sizeof(int) * (2 * kMaxE + 4), 256);
    // bid keys: one block of rows*k keys per bid workgroup, rows*k <= 1024, at most T + rows - 1 rows in all
    L.klist_off = off; off = align_up(off + sizeof(long long) * (((size_t)T + 1024) * k + 1024), 256);
    L.max_wg = (T + 3) / 4 < 1 ? 1 : (T + 3) / 4;   // a bid workgroup covers at least 4 token rows
    L.wcnt_off = off; off = align_up(off + sizeof(int) * (size_t)E * L.max_wg, 256);
    L.wmoves_off = off; off = align_up(off + sizeof(int) * (size_t)L.max_wg, 256);
    L.cand_off = off; off = align_up(off + sizeof(long long) * (size_t)kMaxE * (kCand + 2), 256);
    L.n_tiles = (int)(((size_t)T * k + kDispTile - 1) / kDispTile);
    L.tiles_off = off; off = align_up(off + sizeof(int) * ((size_t)L.n_tiles * E + kMaxE), 256);
    L.cap_off = off; off = align_up(off + sizeof(int) * (size_t)kMaxE, 256);     // per-expert capacities
    L.aux_off = off; off = align_up(off + sizeof(int) * 2 * (size_t)T, 256);     // two token-long lists
    L.dbase_off = off; off = align_up(off + sizeof(int) * ((size_t)E * L.max_wg + kMaxE), 256);   // dispatch from key blocks
    // finisher scratch: a bit per token, the moved-token list, loads and potentials (same layout as fin_area())
    L.fin_off = off; off = align_up(off + sizeof(unsigned) * (((size_t)T + 31) / 32 + 1) + 16 + sizeof(int) * (4 + kFinMovedCap + kFinMaxE) + 16 + sizeof(long long) * (kFinMaxE + 2), 256);
    // finisher arc matrix: smallest loss (and its token) per expert pair
    L.finm_off = off; off = align_up(off + sizeof(unsigned long long) * (size_t)kFinMatrixMaxE * kFinMatrixMaxE, 256);
    // finisher arc lists: one segment per key block (fin_seg_cap(rows, k) arcs of 12 bytes each) and a count per block
    L.tri_off = off; off = align_up(off + 12 * fin_tri_entries(T, k, L.max_wg) + sizeof(int) * ((size_t)L.max_wg + 1), 256);
    L.wt_off = off; off = align_up(off + sizeof(unsigned short) * (size_t)E * (d > 0 ? d : 0), 256);
    L.total = off;
    return L;
}

static bool shape_ok(int T, int E, int k, int C)
{
    return T >= 1 && T <= (1 << kMaxTBits) && E >= 1 && E <= kMaxE && k >= 1 && k <= E && k <= kMaxK && C >= 1;
}

static maxscore_opts resolve(const maxscore_opts *o)
{
    maxscore_opts r = {1.0f, 20, 200000, 12, MAXSCORE_ASSIGN_EXACT, 0u, nullptr, 0};
    if (o) {
        r = *o;
        if (r.quant_shift == 0) r.quant_shift = 20;
        if (r.max_rounds <= 0) r.max_rounds = 200000;
        if (r.eps_div < 2) r.eps_div = 12;
        if (r.eps_start < 0) r.eps_start = 0;
    }
    return r;
}

static int32_t check_ws(const void *ws, size_t bytes, int T, int E, int k)
{
    if (!ws || ((uintptr_t)ws % 256) != 0) return MAXSCORE_ERR_WORKSPACE;
    if (bytes < workspace_layout(T, E, k).total) return MAXSCORE_ERR_WORKSPACE;
    return MAXSCORE_OK;
}

// The projection can compute the scores in its own epilogue (and skip the logits if the caller passes none).
static bool fused_scores_ok(int dtype, int d, int E, const void *x, const void *wt, const float *logits,
                            const float *scores, const int32_t *q)
{
    return gemm_softtopk_supported(dtype, d, E, x, wt) &&
           ((((uintptr_t)logits) | ((uintptr_t)scores) | ((uintptr_t)q)) % 16) == 0;
}

}  // namespace maxscore

using namespace maxscore;

extern "C" {

size_t maxscore_workspace_bytes(int32_t T, int32_t d, int32_t E, int32_t k, int32_t C)
{
    if (!shape_ok(T, E, k, C) || d < 0) return 0;
    size_t need = workspace_layout(T, E, k, d).total;
    const int Ce = C < T ? C : T;
    if ((long long)T * k > (long long)E * Ce) {       // the exact solver then works on a padded copy of the rewards
        const size_t os = oversub_workspace_bytes(T, E, k);
        need = os > need ? os : need;
    }
    return need;
}

int32_t maxscore_router_logits(const void *x, const void *W, const float *bias, int32_t in_dtype, int32_t T,
                               int32_t d, int32_t E, float *logits, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    if (!x || !W || !logits) return MAXSCORE_ERR_NULL;
    if (T < 1 || d < 1 || E < 1 || E > kMaxE || T > (1 << kMaxTBits)) return MAXSCORE_ERR_SHAPE;
    if (in_dtype != MAXSCORE_DTYPE_BF16 && in_dtype != MAXSCORE_DTYPE_FP32) return MAXSCORE_ERR_DTYPE;
    void *wt = nullptr;     // optional scratch for the transposed weight: d*E 16-bit values, 256-byte aligned
    if (workspace && ((uintptr_t)workspace % 256) == 0 && workspace_bytes >= (size_t)d * E * 2) wt = workspace;
    return gemm_run(x, W, bias, in_dtype, T, d, E, logits, wt, (hipStream_t)stream);
}

int32_t maxscore_softtopk(const float *logits, int32_t T, int32_t E, int32_t k, float t, int32_t quant_shift,
                          float *scores, int32_t *q, void *stream)
{
    if (!logits || (!scores && !q)) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1) || quant_shift < 1 || quant_shift > 24 || !(t >= 0.f) || t > 64.f)
        return MAXSCORE_ERR_SHAPE;
    return softtopk_run(logits, T, E, k, t, quant_shift, scores, q, (hipStream_t)stream);
}

int32_t maxscore_softtopk_reading(const float *logits, int32_t T, int32_t E, int32_t k, float t, int32_t quant_shift,
                                  int32_t reading, float *scores, int32_t *q, void *stream)
{
    if (!logits || (!scores && !q)) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1) || quant_shift < 1 || quant_shift > 24 || !(t >= 0.f) || t > 64.f)
        return MAXSCORE_ERR_SHAPE;
    if (reading < MAXSCORE_SOFTTOPK_A || reading > MAXSCORE_SOFTTOPK_C) return MAXSCORE_ERR_SHAPE;
    return softtopk_run(logits, T, E, k, t, quant_shift, scores, q, (hipStream_t)stream, reading);
}

int32_t maxscore_assign_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, int32_t C,
                            const maxscore_opts *opts, int32_t *assign, int64_t *prices, int64_t *price_scale,
                            maxscore_stats *stats, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q || !assign) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, C)) return MAXSCORE_ERR_SHAPE;
    const int Ce = C < T ? C : T;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, k);
    if (rc) return rc;
    maxscore_opts o = resolve(opts);
    if (stats) std::memset(stats, 0, sizeof(*stats));
    if ((long long)T * k > (long long)E * Ce)
        return oversub_run(q, T, E, k, Ce, o, assign, prices, price_scale, stats, (char *)workspace, workspace_bytes,
                           (hipStream_t)stream);
    return solver_run(q, T, E, k, Ce, o, assign, prices, price_scale, stats, (char *)workspace,
                      (hipStream_t)stream);
}

int32_t maxscore_scores_op(const float *logits, int32_t T, int32_t E, int32_t k, int32_t op, int32_t quant_shift,
                           float *scores, int32_t *q, void *stream)
{
    if (!logits || (!scores && !q)) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1) || quant_shift < 1 || quant_shift > 24) return MAXSCORE_ERR_SHAPE;
    if (op < MAXSCORE_OP_SIGMOID || op > MAXSCORE_OP_GRADTOPK) return MAXSCORE_ERR_SHAPE;
    return scores_op_run(logits, T, E, k, op, quant_shift, scores, q, (hipStream_t)stream);
}

int32_t maxscore_aux_loss(const float *scores, const int32_t *expert_offsets, int32_t T, int32_t E, float lambda,
                          float *loss, float *mean_scores, float *dscores_col, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    if (!scores || !expert_offsets || !loss) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, 1, 1)) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, 1);
    if (rc) return rc;
    return aux_loss_run(scores, expert_offsets, T, E, lambda, loss, mean_scores, dscores_col, (char *)workspace,
                        (hipStream_t)stream);
}

int32_t maxscore_gates_backward(const float *logits, const float *scores, const int32_t *assign,
                                const float *dgates, const float *dscores_col, int32_t T, int32_t E, int32_t k,
                                float *dlogits, void *stream)
{
    if (!logits || !scores || !assign || !dgates || !dlogits) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1)) return MAXSCORE_ERR_SHAPE;
    return gates_backward_run(logits, scores, assign, dgates, dscores_col, T, E, k, dlogits, (hipStream_t)stream);
}

int32_t maxscore_assign_iter_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, int32_t C, int32_t max_rounds,
                                 int32_t *assign, int64_t *total, int32_t *flow, int32_t *rounds, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (!q || !assign) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, C)) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, k);
    if (rc) return rc;
    if (max_rounds < 0) max_rounds = 1000;
    return iter_run(q, T, E, k, C, max_rounds, assign, total, flow, rounds, (char *)workspace, (hipStream_t)stream);
}

int32_t maxscore_assign_caps_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, const int32_t *capacity,
                                 const maxscore_opts *opts, int32_t *assign, int64_t *prices, int64_t *price_scale,
                                 maxscore_stats *stats, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q || !assign || !capacity) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1)) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, k);
    if (rc) return rc;
    maxscore_opts o = resolve(opts);
    if (stats) std::memset(stats, 0, sizeof(*stats));
    const int32_t *cap_dev = nullptr;
    long long room = 0;
    int cmax = 1;
    rc = caps_to_device(capacity, T, E, k, (char *)workspace, &cap_dev, &room, &cmax, (hipStream_t)stream);
    if (rc) return rc;
    return solver_run(q, T, E, k, cmax, o, assign, prices, price_scale, stats, (char *)workspace, (hipStream_t)stream,
                      cap_dev, room);
}

int32_t maxscore_assign_kvec_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, const int32_t *kvec, int32_t C,
                                 const int32_t *capacity, const maxscore_opts *opts, int32_t *assign,
                                 int64_t *prices, int64_t *price_scale, maxscore_stats *stats, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (!q || !assign || !kvec) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, capacity ? 1 : C)) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, k);
    if (rc) return rc;
    maxscore_opts o = resolve(opts);
    if (stats) std::memset(stats, 0, sizeof(*stats));
    long long demand = 0;
    rc = kvec_check(kvec, T, E, k, (char *)workspace, &demand, (hipStream_t)stream);
    if (rc) return rc;
    if (capacity) {
        const int32_t *cap_dev = nullptr;
        long long room = 0;
        int cmax = 1;
        rc = caps_to_device(capacity, T, E, k, (char *)workspace, &cap_dev, &room, &cmax, (hipStream_t)stream, demand);
        if (rc) return rc;
        return solver_run(q, T, E, k, cmax, o, assign, prices, price_scale, stats, (char *)workspace,
                          (hipStream_t)stream, cap_dev, room, kvec, demand);
    }
    const int Ce = C < T ? C : T;
    if (demand > (long long)E * Ce) return MAXSCORE_ERR_OVERSUBSCRIBED;
    return solver_run(q, T, E, k, Ce, o, assign, prices, price_scale, stats, (char *)workspace, (hipStream_t)stream,
                      nullptr, 0, kvec, demand);
}

int32_t maxscore_assign_top1_residual_i32(const int32_t *q, int32_t T, int32_t E, int32_t C,
                                          const maxscore_opts *opts, int32_t *q_residual, int32_t *assign,
                                          int32_t *residual_capacity, int64_t *total, int32_t *flow,
                                          maxscore_stats *stats, void *workspace, size_t workspace_bytes,
                                          void *stream)
{
    if (!q || !q_residual || !assign) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, 2, C)) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, 2);
    if (rc) return rc;
    maxscore_opts o = resolve(opts);
    if (stats) std::memset(stats, 0, sizeof(*stats));
    return alg1_run(q, T, E, C, o, q_residual, assign, residual_capacity, total, flow, stats, (char *)workspace,
                    (hipStream_t)stream);
}

int32_t maxscore_assign_top1_sinkhorn(const float *scores, int32_t T, int32_t E, int32_t C, float tau,
                                      int32_t n_iter, int32_t *assign, float *plan, int32_t *residual_capacity,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (!scores || !assign) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, 2, C) || !(tau > 0.f) || n_iter < 0 || n_iter > 100000) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, 2);
    if (rc) return rc;
    return sinkhorn_run(scores, T, E, C, tau, n_iter, assign, plan, residual_capacity, (char *)workspace,
                        (hipStream_t)stream);
}

int32_t maxscore_gates(const float *scores, const int32_t *assign, int32_t T, int32_t E, int32_t k, float *gates,
                       void *stream)
{
    if (!scores || !assign || !gates) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1)) return MAXSCORE_ERR_SHAPE;
    return gates_run(scores, assign, T, E, k, gates, (hipStream_t)stream);
}

int32_t maxscore_dispatch(const int32_t *assign, const float *gates, int32_t T, int32_t E, int32_t k,
                          int32_t *expert_offsets, int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!assign || !expert_offsets || !disp_token || !token_pos) return MAXSCORE_ERR_NULL;
    if ((disp_gate != nullptr) != (gates != nullptr)) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1)) return MAXSCORE_ERR_SHAPE;
    int32_t rc = check_ws(workspace, workspace_bytes, T, E, k);
    if (rc) return rc;
    return dispatch_run(assign, gates, T, E, k, expert_offsets, disp_token, disp_gate, token_pos,
                        (char *)workspace, (hipStream_t)stream);
}

int32_t maxscore_dispatch_tokens(const void *x, int32_t in_dtype, const int32_t *expert_offsets,
                                 const int32_t *disp_token, int32_t T, int32_t d, int32_t E, int32_t C,
                                 void *expert_in, void *stream)
{
    if (!x || !expert_offsets || !disp_token || !expert_in) return MAXSCORE_ERR_NULL;
    if (T < 1 || T > (1 << kMaxTBits) || d < 1 || E < 1 || E > kMaxE || C < 1) return MAXSCORE_ERR_SHAPE;
    if (in_dtype != MAXSCORE_DTYPE_BF16 && in_dtype != MAXSCORE_DTYPE_FP32) return MAXSCORE_ERR_DTYPE;
    return dispatch_tokens_run(x, in_dtype, expert_offsets, disp_token, T, d, E, C, expert_in, (hipStream_t)stream);
}

int32_t maxscore_combine(const void *expert_out, int32_t in_dtype, const int32_t *assign, const int32_t *token_pos,
                         const float *gates, int32_t T, int32_t d, int32_t E, int32_t k, int32_t C, float *y,
                         void *stream)
{
    if (!expert_out || !assign || !token_pos || !gates || !y) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, C) || d < 1) return MAXSCORE_ERR_SHAPE;
    if (in_dtype != MAXSCORE_DTYPE_BF16 && in_dtype != MAXSCORE_DTYPE_FP32) return MAXSCORE_ERR_DTYPE;
    return combine_run(expert_out, in_dtype, assign, token_pos, gates, T, d, E, k, C, y, (hipStream_t)stream);
}

// A pair of events per host thread for the a5 + a6 time of the routing calls (created once, kept).
static int32_t route_events(hipEvent_t *a, hipEvent_t *b)
{
    static thread_local hipEvent_t ev[2] = {nullptr, nullptr};
    static thread_local int ev_dev = -1;
    int dev = 0;
    MS_HIP(hipGetDevice(&dev));
    if (ev_dev != dev) {                 // first call of the thread (or the thread moved to another device)
        MS_HIP(hipEventCreate(&ev[0]));
        MS_HIP(hipEventCreate(&ev[1]));
        ev_dev = dev;
    }
    *a = ev[0];
    *b = ev[1];
    return MAXSCORE_OK;
}

// a4..a6 on scores and rewards that are already in place (the common tail of the maxscore_route_* calls).
static int32_t route_from_rewards(const float *scores, const int32_t *q, int T, int E, int k, int C,
                                  const maxscore_opts &o, int32_t *assign, float *gates, int32_t *expert_offsets,
                                  int32_t *disp_token, float *disp_gate, int32_t *token_pos, int64_t *prices,
                                  maxscore_stats *stats, char *ws, size_t ws_bytes, hipStream_t s)
{
    const int Ce = C < T ? C : T;
    int32_t src;
    hipEvent_t ev_a = nullptr, ev_b = nullptr;
    {
        int32_t rc = route_events(&ev_a, &ev_b);
        if (rc) return rc;
    }
    auto finish = [&](int32_t status) -> int32_t {       // end of a5 + a6: wait for the stream, report their time
        if (hipEventRecord(ev_b, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return MAXSCORE_ERR_HIP;
        float t = 0.f;
        if (stats && hipEventElapsedTime(&t, ev_a, ev_b) == hipSuccess) stats->gates_dispatch_ms = t;
        return status;
    };
    if (o.assignment == MAXSCORE_ASSIGN_ITER) {
        int64_t total = 0;
        int32_t flow = 0, rounds = 0;
        src = iter_run(q, T, E, k, C, o.max_rounds, assign, &total, &flow, &rounds, ws, s);
        if (stats) {
            stats->total_score_q = total;
            stats->flow_value = flow;
            stats->rounds = rounds;
            stats->status = src;
        }
    } else if ((long long)T * k > (long long)E * Ce) {
        // more demand than capacity: every expert ends full, rows come back with empty slots (-1) at their end
        src = oversub_run(q, T, E, k, Ce, o, assign, prices, nullptr, stats, ws, ws_bytes, s);
    } else {
        // After a converged solve the final bid pass has left every pair as a key, sorted by expert inside each block
        // of rows: gates and dispatch come from there.  They are enqueued behind the solve before the call waits for
        // it (the kernels stay inside their buffers on any state; if the solve did not converge the general kernels
        // below overwrite what they wrote).
        struct AfterCtx {
            const float *scores; const int32_t *assign; int T, E, k; float *gates; int32_t *offsets, *disp_token;
            float *disp_gate; int32_t *token_pos; char *ws; hipEvent_t ev_start, ev_b;
        } ctx = {scores, assign, T, E, k, gates, expert_offsets, disp_token, disp_gate, token_pos, ws, nullptr, ev_b};
        SolverAfter after = [](void *c, const SolverGeometry &g, hipStream_t st, hipEvent_t solve_end) -> int32_t {
            AfterCtx *a = (AfterCtx *)c;
            a->ev_start = solve_end;         // gates and dispatch are timed from the end of the solve (no event of their own)
            int32_t rc = dispatch_from_keys(g, a->scores, a->assign, a->T, a->E, a->k, a->gates, a->offsets,
                                            a->disp_token, a->disp_gate, a->token_pos, a->ws, st);
            if (rc) return rc;
            MS_HIP(hipEventRecord(a->ev_b, st));
            return MAXSCORE_OK;
        };
        SolverGeometry geom = {0, 0, 0};
        src = solver_run(q, T, E, k, Ce, o, assign, prices, nullptr, stats, ws, s, nullptr, 0, nullptr, 0, &geom, after,
                         &ctx);
        if (src == MAXSCORE_OK && geom.n_wg > 0) {
            float t = 0.f;           // the solve has waited for the stream: both events are complete
            if (stats && ctx.ev_start && hipEventElapsedTime(&t, ctx.ev_start, ev_b) == hipSuccess)
                stats->gates_dispatch_ms = t;
            return src;
        }
    }
    if (src != MAXSCORE_OK && src != MAXSCORE_ERR_NOT_CONVERGED) return src;
    MS_HIP(hipEventRecord(ev_a, s));
    int32_t rc = gates_run(scores, assign, T, E, k, gates, s);
    if (rc) return rc;
    rc = dispatch_run(assign, gates, T, E, k, expert_offsets, disp_token, disp_gate, token_pos, ws, s);
    if (rc) return rc;
    return finish(src);
}

// Argument checks shared by the maxscore_route_* calls (everything after the scores exist).
static int32_t route_check(int T, int E, int k, int C, const maxscore_opts &o, const void *workspace,
                           size_t workspace_bytes)
{
    if (!shape_ok(T, E, k, C)) return MAXSCORE_ERR_SHAPE;
    if (o.assignment != MAXSCORE_ASSIGN_EXACT && o.assignment != MAXSCORE_ASSIGN_ITER) return MAXSCORE_ERR_SHAPE;
    if (o.quant_shift < 1 || o.quant_shift > 24 || !(o.t >= 0.f) || o.t > 64.f) return MAXSCORE_ERR_SHAPE;
    const int Ce = C < T ? C : T;
    // with more demand than capacity both kinds of assignment leave empty slots; the exact solver then pads the
    // problem with k more experts
    if (o.assignment == MAXSCORE_ASSIGN_EXACT && (long long)T * k > (long long)E * Ce && E + k > kMaxE)
        return MAXSCORE_ERR_OVERSUBSCRIBED;
    return check_ws(workspace, workspace_bytes, T, E, k);
}

int32_t maxscore_route_scores(const float *scores, int32_t T, int32_t E, int32_t k, int32_t C,
                              const maxscore_opts *opts, int32_t *q_out, int32_t *assign, float *gates,
                              int32_t *expert_offsets, int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                              int64_t *prices, maxscore_stats *stats, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    if (!scores || !q_out || !assign || !gates || !expert_offsets || !disp_token || !disp_gate || !token_pos)
        return MAXSCORE_ERR_NULL;
    maxscore_opts o = resolve(opts);
    int32_t rc = route_check(T, E, k, C, o, workspace, workspace_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (stats) std::memset(stats, 0, sizeof(*stats));
    rc = quantise_run(scores, T, E, o.quant_shift, q_out, s);
    if (rc) return rc;
    return route_from_rewards(scores, q_out, T, E, k, C, o, assign, gates, expert_offsets, disp_token, disp_gate,
                              token_pos, prices, stats, (char *)workspace, workspace_bytes, s);
}

int32_t maxscore_route_logits(const float *logits, int32_t T, int32_t E, int32_t k, int32_t C,
                              const maxscore_opts *opts, float *scores_out, int32_t *q_out, int32_t *assign,
                              float *gates, int32_t *expert_offsets, int32_t *disp_token, float *disp_gate,
                              int32_t *token_pos, int64_t *prices, maxscore_stats *stats, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    if (!logits || !scores_out || !q_out || !assign || !gates || !expert_offsets || !disp_token || !disp_gate ||
        !token_pos)
        return MAXSCORE_ERR_NULL;
    maxscore_opts o = resolve(opts);
    int32_t rc = route_check(T, E, k, C, o, workspace, workspace_bytes);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (stats) std::memset(stats, 0, sizeof(*stats));
    rc = softtopk_run(logits, T, E, k, o.t, o.quant_shift, scores_out, q_out, s);
    if (rc) return rc;
    return route_from_rewards(scores_out, q_out, T, E, k, C, o, assign, gates, expert_offsets, disp_token,
                              disp_gate, token_pos, prices, stats, (char *)workspace, workspace_bytes, s);
}

int32_t maxscore_route_xw(const void *x, const void *W, const float *bias, int32_t in_dtype, int32_t T, int32_t d,
                          int32_t E, int32_t k, int32_t C, const maxscore_opts *opts, float *logits_out,
                          float *scores_out, int32_t *q_out, int32_t *assign, float *gates,
                          int32_t *expert_offsets, int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                          int64_t *prices, maxscore_stats *stats, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (!x || !W) return MAXSCORE_ERR_NULL;
    if (d < 1) return MAXSCORE_ERR_SHAPE;
    if (in_dtype != MAXSCORE_DTYPE_BF16 && in_dtype != MAXSCORE_DTYPE_FP32) return MAXSCORE_ERR_DTYPE;
    if (!shape_ok(T, E, k, C)) return MAXSCORE_ERR_SHAPE;
    if (!scores_out || !q_out || !assign || !gates || !expert_offsets || !disp_token || !disp_gate || !token_pos)
        return MAXSCORE_ERR_NULL;
    const maxscore_opts o = resolve(opts);
    int32_t rc = route_check(T, E, k, C, o, workspace, workspace_bytes);
    if (rc) return rc;
    void *wt = nullptr;
    {
        WorkspaceLayout L = workspace_layout(T, E, k, d);
        if (workspace_bytes >= L.total) wt = (char *)workspace + L.wt_off;
    }
    hipStream_t s = (hipStream_t)stream;
    if (fused_scores_ok(in_dtype, d, E, x, wt, logits_out, scores_out, q_out)) {
        // a1..a3 in one kernel: the scores come straight out of the projection's accumulators
        if (stats) std::memset(stats, 0, sizeof(*stats));
        rc = gemm_softtopk_run(x, W, bias, in_dtype, T, d, E, k, o.t, o.quant_shift, logits_out, scores_out, q_out, wt,
                               s);
        if (rc) return rc;
        return route_from_rewards(scores_out, q_out, T, E, k, C, o, assign, gates, expert_offsets, disp_token,
                                  disp_gate, token_pos, prices, stats, (char *)workspace, workspace_bytes, s);
    }
    if (!logits_out) return MAXSCORE_ERR_NULL;          // the two-kernel form keeps the logits in the caller's buffer
    rc = gemm_run(x, W, bias, in_dtype, T, d, E, logits_out, wt, s);
    if (rc) return rc;
    return maxscore_route_logits(logits_out, T, E, k, C, opts, scores_out, q_out, assign, gates, expert_offsets,
                                 disp_token, disp_gate, token_pos, prices, stats, workspace, workspace_bytes,
                                 stream);
}

int32_t maxscore_router_softtopk(const void *x, const void *W, const float *bias, int32_t in_dtype, int32_t T,
                                 int32_t d, int32_t E, int32_t k, float t, int32_t quant_shift, float *logits_out,
                                 float *scores, int32_t *q, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !W || (!scores && !q)) return MAXSCORE_ERR_NULL;
    if (!shape_ok(T, E, k, 1) || d < 1 || quant_shift < 1 || quant_shift > 24 || !(t >= 0.f) || t > 64.f)
        return MAXSCORE_ERR_SHAPE;
    if (in_dtype != MAXSCORE_DTYPE_BF16 && in_dtype != MAXSCORE_DTYPE_FP32) return MAXSCORE_ERR_DTYPE;
    void *wt = nullptr;     // optional scratch for the transposed weight: d*E 16-bit values, 256-byte aligned
    if (workspace && ((uintptr_t)workspace % 256) == 0 && workspace_bytes >= (size_t)d * E * 2) wt = workspace;
    hipStream_t s = (hipStream_t)stream;
    if (fused_scores_ok(in_dtype, d, E, x, wt, logits_out, scores, q))
        return gemm_softtopk_run(x, W, bias, in_dtype, T, d, E, k, t, quant_shift, logits_out, scores, q, wt, s);
    if (!logits_out) return MAXSCORE_ERR_NULL;
    int32_t rc = gemm_run(x, W, bias, in_dtype, T, d, E, logits_out, wt, s);
    if (rc) return rc;
    return softtopk_run(logits_out, T, E, k, t, quant_shift, scores, q, s);
}

void maxscore_set_kernel_timing(int32_t on) { g_kernel_timing = on ? 1 : 0; }

int32_t maxscore_copy_bytes(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return MAXSCORE_ERR_NULL;
    if (bytes % 16 != 0) return MAXSCORE_ERR_SHAPE;
    return copy_run(src, dst, bytes, (hipStream_t)stream);
}

const char *maxscore_status_string(int32_t status)
{
    switch (status) {
        case MAXSCORE_OK: return "ok";
        case MAXSCORE_ERR_NULL: return "a required pointer is NULL";
        case MAXSCORE_ERR_SHAPE: return "unsupported or inconsistent sizes";
        case MAXSCORE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case MAXSCORE_ERR_DTYPE: return "unknown input dtype";
        case MAXSCORE_ERR_HIP: return "HIP runtime error";
        case MAXSCORE_ERR_OVERSUBSCRIBED: return "T*k exceeds E*min(C,T)";
        case MAXSCORE_ERR_RANGE: return "reward range too wide";
        case MAXSCORE_ERR_NOT_CONVERGED: return "solver hit max_rounds";
        default: return "unknown status";
    }
}

}  // extern "C"
