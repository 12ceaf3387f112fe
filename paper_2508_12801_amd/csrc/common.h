// Shared host/device declarations of the MaxScore routing library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "maxscore.h"

namespace maxscore {

constexpr int kMaxE = 1024;
#ifndef MS_DISP_TILE
#define MS_DISP_TILE 1024
#endif
constexpr int kDispTile = MS_DISP_TILE;   // slots of the pair list owned by one wavefront in the dispatch kernels
constexpr int kMaxK = 64;
constexpr int kMaxTBits = 21;
constexpr int64_t kBidBig = (int64_t)1 << 40;   // bid of a token that has no alternative left
constexpr int kCand = 32;          // lowest keys per expert handed to the tail pass (16 beyond 256 experts, 8 beyond 512)
constexpr int kEps0Shift = 8;      // the auction's first phase runs at eps0 <= S * (reward range) / 2^8
constexpr int kTailMaxE = 1024;    // the tail pass keeps all candidate lists in LDS (= kMaxE: it always runs)

// Device-resident control block of one assignment solve.
struct SolverState {
    long long eps;         // current epsilon (in units of 1/S of a reward unit)
    long long eps_prev;    // epsilon of the previous phase (0 in the first phase)
    long long beta;        // price-lowering factor applied between phases when capacity is slack
    long long qmin, qmax;  // reward range
    long long total;       // sum of q over chosen pairs (finalize)
    int sbits;             // S = 1 << sbits > E
    int tbits;             // token id bits inside a bid key
    int eps_div;
    int max_rounds;
    int round;
    int phases;
    int done;              // 1 once the final phase is quiescent (or on error)
    int status;
    int moves;             // drops + fills of the current bid pass
    int blocks_done;       // completion counter of the select pass
    int flow;
    int slack;             // E*Ce - T*k > 0
    int wide;              // 1: prices near 2^30, the bid pass must use 64-bit values
    int tail_go;           // the select pass built candidate lists: the tail pass may run
    int after_tail;        // the tail pass changed the state: the next round cannot be declared quiescent
    int tail_block;        // the tail pass could not proceed: the next select pass must do a normal select
    int tail_gos;          // rounds so far in which the select pass handed over to the tail pass
    int tail_runs, tail_iters;   // diagnostics
    int warm;              // how many steps back up the eps ladder are still allowed (a start from given prices, or
                           // phases that were ended early, may have left the prices further off than their eps assumes)
    int early_off;         // set once the ladder has been climbed back up: from then on no phase ends early
    int phase_start;       // round at which the current phase began
    long long eps0;        // first-phase epsilon of a cold start (upper end of the eps ladder)
    long long stop_eps;    // the phase with eps <= stop_eps is the last one of the auction (1: it runs to the optimum
                           // itself; above 1 the cycle-cancelling finisher takes over from there)
    long long fin_bound;   // finisher: arcs whose reduced cost is at or above this are left out of the arc matrix
    int fin;               // finisher: 0 not in use, 1 pending (more passes needed), 2 optimum certified, 3 gave up
    int fin_passes;        // arc-matrix passes so far
    int fin_cycles;        // negative cycles cancelled so far
    int fin_dirty;         // cycles cancelled since the arc matrix was last rebuilt
    int phase_round[28];   // round index at which each phase ended (diagnostic)
};

struct WorkspaceLayout {
    size_t state_off, theta_off, gcount_off, klist_off, wcnt_off, wmoves_off, cand_off, tiles_off, cap_off, aux_off,
        wt_off, dbase_off, fin_off, finm_off, tri_off, total;
    int n_tiles, max_wg;
};

// How the last solve laid out its bid keys (what the dispatch needs to read them): the key blocks of the final bid
// pass hold one key per (token, expert) pair, sorted by expert inside each block of `rows` consecutive tokens.
struct SolverGeometry {
    int rows;        // token rows per bid workgroup = per key block
    int n_wg;        // number of key blocks
    int tbits;       // the token id sits in the low tbits bits of a key
};

WorkspaceLayout workspace_layout(int T, int E, int k, int d = 0);

inline bool hip_ok(hipError_t e) { return e == hipSuccess; }

#define MS_HIP(call)                                   \
    do {                                               \
        if ((call) != hipSuccess) return MAXSCORE_ERR_HIP; \
    } while (0)

// --- solver.hip
// cap: optional device array of E per-expert capacities (each <= T) with sum `room`; NULL = Ce for all.
// kvec: optional device array of T per-token k (each 0..k) with sum `demand`; NULL = k for all.
// after: optional work the caller wants behind the solve on the same stream (the routing calls' gates and dispatch).
// It is enqueued before the call waits for the stream, so the device goes from the solve straight into it; it
// runs whatever the solve's status turns out to be and must therefore be safe on any state the solver can leave
// (the caller redoes it another way when the status is not MAXSCORE_OK).
// solve_end: the event the solver has just recorded behind its last kernel (it stays valid until the calling thread
// solves again on this device); work timed from there needs no start event of its own.
typedef int32_t (*SolverAfter)(void *ctx, const SolverGeometry &g, hipStream_t s, hipEvent_t solve_end);
int32_t solver_run(const int32_t *q, int T, int E, int k, int Ce, const maxscore_opts &o, int32_t *assign,
                   int64_t *prices, int64_t *price_scale, maxscore_stats *stats, char *ws, hipStream_t s,
                   const int32_t *cap = nullptr, long long room = 0, const int32_t *kvec = nullptr,
                   long long demand = 0, SolverGeometry *geom = nullptr, SolverAfter after = nullptr,
                   void *after_ctx = nullptr);
// Checks a device array of T per-token k (each 0..k) and returns its sum in *demand (synchronises the stream).
int32_t kvec_check(const int32_t *kvec, int T, int E, int k, char *ws, long long *demand, hipStream_t s);
// --- finish.hip
// Exact finish from a quiescent auction state at a coarse eps (every token holds its experts): cancels the negative
// cycles of the expert graph until none is left and replaces the prices by exact ones.  One call enqueues the passes
// first_pass .. first_pass + passes - 1 of total_passes, each a pair of (arc matrix, Bellman-Ford + cancelling) that
// exits at once unless st->fin is 1, and a last kernel that reports to host_words[0..3]: {1 certified | 2 the auction
// goes on | 3 not finished, passes left; cycles cancelled so far; st->fin; round}.  retry: when the auction has to
// go on it stops again one rung further down (the finisher can be enqueued anew, from pass 0) instead of running to
// eps = 1.  Supports E <= kFinMaxE (beyond 256 experts without the arc matrix: a first pass whose arc list is not
// complete hands back to the auction).
constexpr int kFinMaxE = 1024;
constexpr int kFinMatrixMaxE = 256;       // its arc matrix (one token per expert pair) serves up to this many experts
constexpr int kFinMovedCap = 4096;        // tokens the finisher may move in one solve (more: the auction goes on)
int32_t finish_enqueue(const int32_t *q, int32_t *assign, SolverState *st, long long *theta2, const int *loads2,
                       const int *cap, int Ce, int T, int E, int k, char *ws, int rows, int n_wg, int first_pass,
                       int passes, int total_passes, long long bound_mult, int *host_words, int retry, hipStream_t s);
size_t finish_area_bytes(int T);          // bytes of WorkspaceLayout::fin_off's region
// One bit per token, set for the tokens the finisher has moved since its first pass of this attempt (the region's
// first (T + 31) / 32 + 1 words).
inline const unsigned *finish_moved_bits(const char *ws, const WorkspaceLayout &L) { return (const unsigned *)(ws + L.fin_off); }
// Arc lists of the finisher's first pass: key block w owns a segment of consecutive entries, an equal share of a
// region of fin_tri_entries() entries; the region is sized so that a share is never smaller than fin_seg_cap(rows, k)
// for any geometry the solver picks (rows * k <= 1024 per block).
inline int fin_seg_cap(int rows, int k)
{
    const int c = rows * k / 4;
    return c < 16 ? 16 : c;
}
inline size_t fin_tri_entries(int T, int k, int max_wg) { return ((size_t)T + 1024) * k / 4 + 16 * (size_t)max_wg + 16; }
// --- oversub.hip
// Exact assignment with more demand than capacity (T*k > E*Ce): every expert ends full, the placed pairs have the
// maximum score, rows come back with their experts first and -1 in the slots left empty.  Needs E + k <= kMaxE and
// oversub_workspace_bytes() of workspace (0: not supported for these sizes).  Synchronises the stream.
size_t oversub_workspace_bytes(int T, int E, int k);
int32_t oversub_run(const int32_t *q, int T, int E, int k, int Ce, const maxscore_opts &o, int32_t *assign,
                    int64_t *prices, int64_t *price_scale, maxscore_stats *stats, char *ws, size_t ws_bytes,
                    hipStream_t s);
// --- softtopk.hip
int32_t softtopk_run(const float *logits, int T, int E, int k, float t, int shift, float *scores, int32_t *q,
                     hipStream_t s, int reading = MAXSCORE_SOFTTOPK_A);
int32_t quantise_run(const float *scores, int T, int E, int shift, int32_t *q, hipStream_t s);
int32_t gates_run(const float *scores, const int32_t *assign, int T, int E, int k, float *gates, hipStream_t s);
// --- dispatch.hip
int32_t dispatch_run(const int32_t *assign, const float *gates, int T, int E, int k, int32_t *offsets,
                     int32_t *disp_token, float *disp_gate, int32_t *token_pos, char *ws, hipStream_t s);
// Stable position of every entry of `list` (n expert ids, -1 = none) among the entries of the same expert, and
// the exclusive prefix sums of the per-expert counts; disp_token / disp_gate may be null.  `tiles` needs
// n_tiles*E + kMaxE ints with n_tiles = ceil(n / kDispTile).
// a5 + a6 straight from the key blocks of a converged solve in the same workspace (every token holds k experts):
// gates, expert offsets, both dispatch lists and the positions, in two launches.
int32_t dispatch_from_keys(const SolverGeometry &g, const float *scores, const int32_t *assign, int T, int E, int k,
                           float *gates, int32_t *offsets, int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                           char *ws, hipStream_t s);
int32_t dispatch_core(const int32_t *list, const float *gates, size_t n, int E, int k, int32_t *offsets,
                      int32_t *disp_token, float *disp_gate, int32_t *token_pos, int *tiles, int n_tiles,
                      hipStream_t s);
// --- iter.hip
int32_t iter_run(const int32_t *q, int T, int E, int k, int C, int max_rounds, int32_t *assign, int64_t *total,
                 int32_t *flow, int32_t *rounds, char *ws, hipStream_t s);
// --- operators.hip
int32_t scores_op_run(const float *logits, int T, int E, int k, int op, int shift, float *scores, int32_t *q,
                      hipStream_t s);
int32_t top1_run(const int32_t *q, int T, int E, int32_t *top1, hipStream_t s);
int32_t assign_total_run(const int32_t *q, const int32_t *assign, int T, int E, int k, void *state16, int64_t *total,
                         int32_t *flow, hipStream_t s);
// --- alg1.hip
// Validates a host capacity vector (each >= 0, clamped to T, sum >= demand; demand < 0 stands for T*k) and
// copies it into the workspace.
int32_t caps_to_device(const int32_t *caps_host, int T, int E, int k, char *ws, const int32_t **cap_dev,
                       long long *room, int *cmax, hipStream_t s, long long demand = -1);
int32_t alg1_run(const int32_t *q, int T, int E, int C, const maxscore_opts &o, int32_t *q_residual,
                 int32_t *assign, int32_t *caps_out, int64_t *total, int32_t *flow, maxscore_stats *stats, char *ws,
                 hipStream_t s);
// --- sinkhorn.hip
int32_t sinkhorn_run(const float *scores, int T, int E, int C, float tau, int n_iter, int32_t *assign, float *plan,
                     int32_t *caps_host, char *ws, hipStream_t s);
// --- training.hip
int32_t aux_loss_run(const float *scores, const int32_t *offsets, int T, int E, float lam, float *loss,
                     float *mean_scores, float *dscores_col, char *ws, hipStream_t s);
int32_t gates_backward_run(const float *logits, const float *scores, const int32_t *assign, const float *dgates,
                           const float *dscores_col, int T, int E, int k, float *dlogits, hipStream_t s);
// --- movement.hip
int32_t dispatch_tokens_run(const void *x, int dtype, const int32_t *offsets, const int32_t *disp_token, int T, int d,
                            int E, int C, void *out, hipStream_t s);
int32_t combine_run(const void *buf, int dtype, const int32_t *assign, const int32_t *token_pos, const float *gates,
                    int T, int d, int E, int k, int C, float *y, hipStream_t s);
// --- gemm.hip
int32_t gemm_run(const void *x, const void *W, const float *bias, int dtype, int T, int d, int E, float *logits,
                 void *wt_scratch, hipStream_t s);
// a1 + a2 + a3 in one kernel (the scores come out of the projection's accumulators): bf16 inputs, E in {32, 64, 128},
// d a multiple of 64, the transposed-weight scratch given.  logits may be null (then they are never written).
bool gemm_softtopk_supported(int dtype, int d, int E, const void *x, const void *wt_scratch);
int32_t gemm_softtopk_run(const void *x, const void *W, const float *bias, int dtype, int T, int d, int E, int k,
                          float t, int shift, float *logits, float *scores, int32_t *q, void *wt_scratch,
                          hipStream_t s);
int32_t copy_run(const void *src, void *dst, size_t bytes, hipStream_t s);

extern int g_kernel_timing;

}  // namespace maxscore
