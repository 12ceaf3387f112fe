/*
 * maxscore.h - C ABI of the MaxScore routing hot path on one AMD MI355X (gfx950).
 *
 * Method: "Maximum Score Routing For Mixture-of-Experts" (arXiv 2508.12801), Section 3.2.
 * Notation follows the paper: T = n tokens, E = e experts, k experts per token, C = c capacity
 * per expert, d = model width, t = SoftTopk temperature.
 *
 * Path (each step is one or more HIP kernels; nothing runs on the host except launches,
 * argument checks and the convergence poll of the solver):
 *
 *   a1  logits  L = x . W_g (+ bias)                Eq. 2, Algorithm 1 step 2
 *   a2  scores  A = SoftTopk_t^(k)(L) per token row  Eq. 6 (Table 2 row 1 for the softmax inside)
 *   a3  rewards q = round_half_even(A * 2^shift)     integer form of the affinities A_ij
 *   a4  assignment P: binary, <= k distinct experts per token, <= C tokens per expert,
 *       maximum number of ones first, then maximum sum P_ij q_ij
 *                                                    Eq. 7-8, Table 1 (min-cost max-flow)
 *   a5  gates   g[i,s] = A[i, assign[i,s]]           Eq. 2 (affinity of the selected experts)
 *   a6  dispatch into per-expert buffers             Section 2.3 (capacity c = k*n/e buffers)
 *
 * Conventions common to every entry point
 *   - Every data pointer is DEVICE memory owned by the caller, row-major, densely packed, and
 *     must stay valid until the stream has executed the call.  Outputs are fully overwritten.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - `workspace` is device scratch of at least maxscore_workspace_bytes(...) bytes, 256-byte
 *     aligned.  Two calls may overlap only if they use different workspaces.
 *   - Return value: MAXSCORE_OK or a negative MAXSCORE_ERR_* code.  Argument errors are found on
 *     the host before anything is launched.  No entry point throws or allocates device memory.
 *   - Entry points that contain the assignment step (a4) pace their launches by the solver's progress and
 *     therefore SYNCHRONISE `stream` before returning; the others only enqueue work.  The progress words (rounds
 *     done, end of the solve, the finisher's report) and the final solver state live in two small blocks of pinned
 *     host memory (under 1 KiB together) that the first such call of a host thread allocates per device and keeps
 *     until the process ends; the calling thread polls them while the solve runs (one solve at a time per host
 *     thread; different threads may solve concurrently on different streams with different workspaces).
 *   - Supported sizes: 1 <= k <= E <= 1024, k <= 64, 1 <= T <= 2^21, C >= 1 (C > T acts as T).
 *   - More demand than capacity, T*k > E*min(C,T) (never with a capacity c' = c_f*k*n/e, c_f >= 1, of Section 2.3):
 *     Eq. 7's equalities cannot all hold then; with the capacities of Table 1 the problem is still a flow problem
 *     (Section 3.2), and the exact assignment is its solution: every expert ends full (E*min(C,T) pairs, the
 *     maximum flow) and the placed pairs have the maximum score.  Rows come back with their experts first and -1
 *     in the slots left empty; gates are 0 there and the dispatch lists hold the placed pairs only.  It is solved
 *     with k padding experts, so it needs E + k <= 1024 (MAXSCORE_ERR_OVERSUBSCRIBED otherwise) and the larger
 *     workspace that maxscore_workspace_bytes reports for such T, E, k, C.
 */
#ifndef MAXSCORE_H
#define MAXSCORE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MAXSCORE_OK = 0,
    MAXSCORE_ERR_NULL = -1,           /* a required pointer is NULL */
    MAXSCORE_ERR_SHAPE = -2,          /* T, E, k, C, d outside the supported sizes, or k > E */
    MAXSCORE_ERR_WORKSPACE = -3,      /* workspace NULL, misaligned or too small */
    MAXSCORE_ERR_DTYPE = -4,          /* unknown input dtype code */
    MAXSCORE_ERR_HIP = -5,            /* a HIP call or kernel launch failed */
    MAXSCORE_ERR_OVERSUBSCRIBED = -6, /* more demand than capacity in a form that is not solved: T*k > E*min(C,T) with
                                         E + k > 1024, or a capacity vector whose sum is below the demand */
    MAXSCORE_ERR_RANGE = -7,          /* reward range too wide for the solver's 64-bit bids */
    MAXSCORE_ERR_NOT_CONVERGED = -8   /* max_rounds reached: the assignment returned is feasible (<= C tokens per
                                         expert, distinct experts per token) but neither complete nor optimal:
                                         slots the solver still had to move are empty (-1) */
};

enum { MAXSCORE_DTYPE_BF16 = 0, MAXSCORE_DTYPE_FP32 = 1 };

/* Options.  Pass NULL for the defaults {t = 1, quant_shift = 20, max_rounds = 200000, eps_div = 12, exact
 * assignment, no flags, no starting prices}.  Zero in a field stands for its default. */
typedef struct {
    float t;              /* SoftTopk temperature of Eq. 6 */
    int32_t quant_shift;  /* rewards are round(A * 2^quant_shift); 1..24 */
    int32_t max_rounds;   /* cap on solver rounds (bid pass + select pass) */
    int32_t eps_div;      /* eps-scaling ratio between solver phases, >= 2 */
    int32_t assignment;   /* maxscore_route_* only: MAXSCORE_ASSIGN_EXACT (0, the exact solver) or
                             MAXSCORE_ASSIGN_ITER (1, iterative rerouting: prices are not written,
                             stats carry total, flow and the number of rerouting rounds) */
    uint32_t flags;       /* MAXSCORE_FLAG_* */
    const int64_t *prices_in; /* exact solver: NULL, or DEVICE array of E starting prices in the units of the
                             `prices` output (1/price_scale of a q unit; price_scale depends on E only), e.g. the
                             prices a previous call returned for a batch routed by the same W_g.  Any values >= 0 are
                             legal: the result is the same optimum, only the number of rounds changes.  (A forward
                             auction only raises prices, so a start that is too high on some experts makes all the
                             others climb: measured on successive batches of one router it saves nothing.) */
    int64_t eps_start;    /* with prices_in: eps of the first phase in the same units (it is rounded down to a power
                             of eps_div; 0 = one step below the cold-start value).  A phase that runs longer than 48 rounds
                             after a start from given prices goes back up one step of the eps ladder (at most as many
                             steps in all as the start skipped). */
} maxscore_opts;
#define MAXSCORE_ASSIGN_EXACT 0
#define MAXSCORE_ASSIGN_ITER 1
#define MAXSCORE_FLAG_NO_TAIL_PASS 1u   /* exact solver: dense rounds only (slower; same optimum) */
#define MAXSCORE_FLAG_NO_FINISHER 2u    /* exact solver: the auction runs down to eps = 1 itself instead of handing
                                           its last phases to the cycle-cancelling finisher (slower; same optimum) */

/* Filled on the HOST when the call returns (may be NULL). */
typedef struct {
    int64_t total_score_q; /* sum of q over the chosen pairs */
    int32_t flow_value;    /* number of chosen pairs */
    int32_t rounds;        /* solver rounds executed (auction rounds: bid pass + select pass) */
    int32_t phases;        /* eps-scaling phases executed (restarts included) */
    int32_t status;        /* MAXSCORE_OK, MAXSCORE_ERR_RANGE or MAXSCORE_ERR_NOT_CONVERGED */
    float solver_ms;       /* device time of a4 between two events on `stream` */
    float bid_ms;          /* summed device time of the bid-pass launches inside a4 (0 unless
                              timing was switched on with maxscore_set_kernel_timing) */
    int32_t bid_launches;  /* bid-pass launches that did work (0 unless timing is on) */
    float select_ms;       /* summed device time of the select-pass launches of the same rounds, the tail pass
                              that runs inside some of them included (0 unless timing is on) */
    float gates_dispatch_ms; /* maxscore_route_* only: device time of a5 + a6 between two events on `stream` */
    int32_t finish_passes; /* passes of the cycle-cancelling finisher (0: the auction ran to eps = 1 itself) */
    int32_t finish_cycles; /* negative cycles it cancelled */
} maxscore_stats;

/* Bytes of device scratch the calls below need for these sizes (0 on invalid sizes). */
size_t maxscore_workspace_bytes(int32_t T, int32_t d, int32_t E, int32_t k, int32_t C);

/* a1.  logits[T,E] (fp32) = x[T,d] . W[d,E] + bias[E].  x and W are bf16 (16-bit patterns,
 * fp32 accumulation on the matrix cores) or fp32 according to in_dtype; bias may be NULL.
 * `workspace` is optional here: with at least 2*d*E bytes (256-byte aligned) the bf16 path first
 * writes a transposed copy of W into it and runs its fast kernel; with NULL it uses a slower one. */
int32_t maxscore_router_logits(const void *x, const void *W, const float *bias, int32_t in_dtype,
                               int32_t T, int32_t d, int32_t E, float *logits, void *workspace,
                               size_t workspace_bytes, void *stream);

/* a2 + a3.  Per row: p = softmax(logits); rank r (1 = largest, ties to the lower index);
 * scores = p * (1 + t*(min(r,k) - 1)), the level-by-level reading of Eq. 6;
 * q = round_half_even(scores * 2^shift).  scores and/or q may be NULL. */
int32_t maxscore_softtopk(const float *logits, int32_t T, int32_t E, int32_t k, float t,
                          int32_t quant_shift, float *scores, int32_t *q, void *stream);

/* a2 + a3 under the other readings that the print of Eq. 6 admits (it has no base case, and its SE term does not
 * depend on the recursion level).  Everything as maxscore_softtopk; `reading`:
 *   MAXSCORE_SOFTTOPK_A   what maxscore_softtopk computes: level 1 is Softmax(a), level m = 2..k masks the m-1
 *                         largest entries: p_i * (1 + t * (min(rank_i, k) - 1));
 *   MAXSCORE_SOFTTOPK_A1  level 0 is Softmax(a), level m = 1..k masks the m largest: p_i * (1 + t * min(rank_i - 1, k));
 *   MAXSCORE_SOFTTOPK_B   the mask as printed, the k largest entries at every level 2..k: p_i inside the top k,
 *                         p_i * (1 + t * (k - 1)) outside;
 *   MAXSCORE_SOFTTOPK_C   as A with SE renormalised over the entries it is added to (every level adds a
 *                         distribution scaled by t, as the iterated operators of Table 2 do).
 * The routing entry points use reading A. */
enum { MAXSCORE_SOFTTOPK_A = 0, MAXSCORE_SOFTTOPK_A1 = 1, MAXSCORE_SOFTTOPK_B = 2, MAXSCORE_SOFTTOPK_C = 3 };
int32_t maxscore_softtopk_reading(const float *logits, int32_t T, int32_t E, int32_t k, float t,
                                  int32_t quant_shift, int32_t reading, float *scores, int32_t *q, void *stream);

/* a4.  Exact assignment on integer rewards q[T,E] (Eq. 7-8, Table 1: maximum flow, then maximum score).
 *   assign[T,k] : expert ids per token, distinct, ascending slot order is arbitrary.  With more demand than
 *                 capacity (see above) a row holds fewer than k experts, first in the row, then -1; the prices
 *                 then belong to the padded problem and certify nothing by themselves.
 *   prices[E]   : (may be NULL) int64 expert prices in units of 1/price_scale of a q unit;
 *                 every token holds k experts whose price_scale*q_ij - price_j is within 1 of
 *                 its best alternatives, and unfilled experts have price 0 (the dual side of
 *                 Eq. 7-8 that certifies the optimum).  price_scale[1] (may be NULL) receives
 *                 the scale, a power of two > E.
 * Synchronises `stream`. */
int32_t maxscore_assign_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, int32_t C,
                            const maxscore_opts *opts, int32_t *assign, int64_t *prices,
                            int64_t *price_scale, maxscore_stats *stats, void *workspace,
                            size_t workspace_bytes, void *stream);

/* a5.  gates[T,k] = scores[i, assign[i,s]] (0 where assign < 0). */
int32_t maxscore_gates(const float *scores, const int32_t *assign, int32_t T, int32_t E, int32_t k,
                       float *gates, void *stream);

/* a6.  Dispatch.  expert_offsets[E+1] = exclusive prefix sum of tokens per expert; inside expert j
 * tokens appear in ascending token id; disp_token[T*k], disp_gate[T*k] list the pairs in that
 * order; token_pos[T,k] is the position of pair (i, assign[i,s]) inside its expert's buffer, so
 * its address in a padded [E, C] capacity buffer is assign[i,s]*C + token_pos[i,s].
 * disp_gate / gates may both be NULL. */
int32_t maxscore_dispatch(const int32_t *assign, const float *gates, int32_t T, int32_t E, int32_t k,
                          int32_t *expert_offsets, int32_t *disp_token, float *disp_gate,
                          int32_t *token_pos, void *workspace, size_t workspace_bytes, void *stream);

/* a6 for callers that cannot allocate or hand over scratch memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as maxscore_dispatch, without the
 * workspace arguments: the per-tile expert counts live in a 1 MiB device array that is part of the library (every
 * GPU the library runs on holds its copy until the process ends).  Limit: ceil(T*k / 1024) * E + 1024 <= 262144
 * (T*k <= 2^21 pairs at E = 128); larger problems return MAXSCORE_ERR_WORKSPACE.  The call allocates nothing, on
 * the host or on the device, and only enqueues work.  The device of `stream` must be the current device.  All
 * calls on one GPU share that array: two calls that overlap in time on the same GPU (different streams) race;
 * calls on one stream, or on different GPUs, do not. */
int32_t maxscore_dispatch_static(const int32_t *assign, const float *gates, int32_t T, int32_t E, int32_t k,
                                 int32_t *expert_offsets, int32_t *disp_token, float *disp_gate,
                                 int32_t *token_pos, void *stream);

/* Other routing operators of Table 2 (Section 3.1) in place of SoftTopk: scores[T, E] and/or the integer
 * rewards q = round-half-even(score * 2^quant_shift) (either output may be NULL, not both).
 *   MAXSCORE_OP_SIGMOID   y = 1 / (1 + e^-x)
 *   MAXSCORE_OP_SOFTKMAX  y^(m) = y^(m-1) + Softmax((1 - y^(m-1)) * x), m = 1..k
 *   MAXSCORE_OP_ITERTOPK  y^(m) = y^(m-1) + w e^x / sum_j w_j e^x_j with w = 1 - y^(m-1), m = 1..k
 *   MAXSCORE_OP_GRADTOPK  g^(m) = x + log(e^{z^(m-1)} - e^{g^(m-1)}), z^(m) = logsumexp(g^(m)) - log m,
 *                         y^(m) = e^{g^(m) - z^(m)}, evaluated in the equal form y^(m) = m w e^x / sum_j w_j e^x_j;
 *                         a row in which some level-(m-1) value exceeds 1 turns NaN (the logarithm has no value)
 * The table gives no base case: y^(0) = 0 (GradTopk: g^(1) = x) is used, so level 1 is Softmax.  IterTopk is evaluated as printed
 * (its weights may turn negative from level 3 on; a row whose weighted sum reaches 0 gives non-finite
 * values).  The integer rewards are only meaningful when score * 2^quant_shift fits 32 bits.  Only enqueues. */
#define MAXSCORE_OP_SIGMOID 1
#define MAXSCORE_OP_SOFTKMAX 2
#define MAXSCORE_OP_ITERTOPK 3
#define MAXSCORE_OP_GRADTOPK 4
int32_t maxscore_scores_op(const float *logits, int32_t T, int32_t E, int32_t k, int32_t op, int32_t quant_shift,
                           float *scores, int32_t *q, void *stream);

/* Training-side by-products.
 *
 * maxscore_aux_loss: the load-balance loss of Eq. 9 (Section 4.1),
 *   loss = lambda * (1/E) * sum_j mean_i(scores[i, j]) * mean_i(P[i, j]),
 * with the column counts of P taken from expert_offsets[E+1] (output of maxscore_dispatch).  Device outputs:
 * loss[1]; mean_scores[E] (may be NULL); dscores_col[E] (may be NULL) = d loss / d scores[i, j], which is the
 * same for every token i: lambda / (E*T) * mean_i(P[i, j]) (P is a constant).  Column sums are accumulated in
 * a fixed order (fp32 inside a block of rows, fp64 across blocks): the result is deterministic.  Workspace as
 * for the other calls (any k); only enqueues.
 *
 * maxscore_gates_backward: d loss / d logits through the gates of Eq. 2 with the SoftTopk scores of Eq. 6.
 * The rank multipliers of Eq. 6 are piecewise constant in the logits, so with A = scores and p = Softmax(logits)
 *   dlogits[i, l] = gA[i, l]*A[i, l] - p[i, l] * sum_j gA[i, j]*A[i, j],
 *   gA[i, j] = sum over slots s with assign[i, s] == j of dgates[i, s]  (+ dscores_col[j] if given).
 * logits, scores [T, E]; assign, dgates [T, k]; dscores_col [E] or NULL; dlogits [T, E] out.  Only enqueues. */
int32_t maxscore_aux_loss(const float *scores, const int32_t *expert_offsets, int32_t T, int32_t E, float lambda,
                          float *loss, float *mean_scores, float *dscores_col, void *workspace,
                          size_t workspace_bytes, void *stream);
int32_t maxscore_gates_backward(const float *logits, const float *scores, const int32_t *assign,
                                const float *dgates, const float *dscores_col, int32_t T, int32_t E, int32_t k,
                                float *dlogits, void *stream);

/* a4 with one capacity per expert (the vector c of Eq. 7; in Table 1 the arc Expert_j -> Sink gets capacity
 * capacity[j]).  capacity is a HOST array of E values >= 0 (values above T act as T); their sum must be at least
 * T*k (MAXSCORE_ERR_OVERSUBSCRIBED otherwise).  Everything else as maxscore_assign_i32. */
int32_t maxscore_assign_caps_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, const int32_t *capacity,
                                 const maxscore_opts *opts, int32_t *assign, int64_t *prices, int64_t *price_scale,
                                 maxscore_stats *stats, void *workspace, size_t workspace_bytes, void *stream);

/* a4 with one k per token (the vector k of Eq. 7; in Table 1 the arc Source -> Token_i gets capacity kvec[i]).
 * kvec is a DEVICE array of T values in 0..k; k is the row width of assign (k <= E, k <= 64).  Token i ends with
 * exactly kvec[i] distinct experts in assign[i, 0..kvec[i]-1]; the remaining slots of its row hold -1, so
 * maxscore_gates, maxscore_dispatch and the movement calls take the result as it is.  Capacities: C for every
 * expert (capacity == NULL), or the HOST array capacity[E] as in maxscore_assign_caps_i32 (C is then ignored).
 * The capacities must sum to at least sum_i kvec[i] (MAXSCORE_ERR_OVERSUBSCRIBED otherwise; with one C for all
 * experts every token can then ship all its units, with unequal capacities that is the caller's business as in
 * maxscore_assign_caps_i32); an entry of kvec outside 0..k gives MAXSCORE_ERR_SHAPE.  The call reads kvec back
 * once to check it (it synchronises the stream before the solve as well as after).  Optimality is the same
 * statement as for maxscore_assign_i32: with the returned prices every token holds its kvec[i] best experts by
 * price_scale*q_ij - price_j up to 1 unit, which is below the resolution of the integer rewards.  Everything
 * else as maxscore_assign_i32. */
int32_t maxscore_assign_kvec_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, const int32_t *kvec, int32_t C,
                                 const int32_t *capacity, const maxscore_opts *opts, int32_t *assign,
                                 int64_t *prices, int64_t *price_scale, maxscore_stats *stats, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* Algorithm 1 (Section 3.2, top-2 routing) with its residual problem solved exactly: every token takes its
 * highest-reward expert whatever the load (ties to the lower id); that entry of the reward matrix is set to 0
 * (q_residual[T, E], device, out: the caller provides the storage); the capacities become max(0, C - load_j)
 * (residual_capacity[E], HOST out, may be NULL); each token then gets one more expert by the exact assignment
 * with k = 1 on the residual problem.  The paper solves that step approximately with Sinkhorn, whose iteration
 * count, regulariser and rounding it does not give; this entry point gives the exact answer the approximation
 * aims at.  assign[T, 2] device out = (top-1 expert, second expert or -1); total (sum of q over both choices)
 * and flow (number of pairs) are HOST pointers and may be NULL; stats describe the residual solve.  Because the
 * top-1 stage ignores the load, an expert can end above C, and because step 5 zeroes an entry instead of
 * forbidding it, a token's second expert can be its first one again.  MAXSCORE_ERR_OVERSUBSCRIBED if the
 * residual capacities sum to less than T.  Synchronises the stream. */
int32_t maxscore_assign_top1_residual_i32(const int32_t *q, int32_t T, int32_t E, int32_t C,
                                          const maxscore_opts *opts, int32_t *q_residual, int32_t *assign,
                                          int32_t *residual_capacity, int64_t *total, int32_t *flow,
                                          maxscore_stats *stats, void *workspace, size_t workspace_bytes,
                                          void *stream);

/* Algorithm 1 with its last step done by Sinkhorn, as in the paper.  The paper names the algorithm only; the
 * regulariser tau, the iteration count n_iter and the rounding are this library's reading:
 *   top-1 per token on scores[T, E] (ties to the lower expert id); residual capacities max(0, C - load_j);
 *   residual affinities a' = scores with the top-1 entry set to 0;
 *   K_ij = exp((a'_ij - max_j a'_ij) / tau) on experts with residual capacity, else 0;
 *   column targets m_j = cap_j * T / sum(cap);  v = 1;  n_iter times: u_i = 1 / sum_j K_ij v_j,
 *   v_j = m_j / sum_i K_ij u_i;  plan_ij = u_i K_ij v_j (u = 1 when n_iter = 0);
 *   second expert = arg-max_j plan_ij (ties to the lower id), -1 when the row is all zero.
 * assign[T, 2] device out; plan[T, E] device out or NULL; residual_capacity[E] HOST out or NULL (the call then
 * synchronises the stream, otherwise it only enqueues).  tau > 0, 0 <= n_iter <= 100000, E >= 2.  The rounded
 * second choices follow the capacities only approximately.  fp32 arithmetic; column sums are added in a fixed
 * order, so results are reproducible for a given shape. */
int32_t maxscore_assign_top1_sinkhorn(const float *scores, int32_t T, int32_t E, int32_t C, float tau,
                                      int32_t n_iter, int32_t *assign, float *plan, int32_t *residual_capacity,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* Iterative rerouting (Section 2.3, the second stage drawn in Figure 1(c); the assignment step of the
 * "-I" variants of Section 4): a fast greedy alternative to maxscore_assign_i32 on the same integer rewards.
 * Stage 1 keeps, per expert, the first C of the tokens' top-k choices taken in the order (choice rank, token
 * id); stage 2 runs synchronous rounds in which every token proposes, for its holes in slot order, its best
 * experts among those with room at the start of the round (not held, not proposed twice), and an expert
 * accepts proposals in the order (slot, token id) while it has room; rounds end when nobody can propose.
 * The paper states the two stages in a sentence; these orders are this library's reading.
 *
 * q[T, E] device; assign[T, k] device out (slot s holds the token's s-th choice or its replacement, -1 = hole
 * that nobody could take).  total (sum of q over the chosen pairs), flow (number of pairs) and rounds (stage-2
 * rounds that had proposals) are host pointers and may be NULL.  max_rounds < 0 means 1000; max_rounds = 0
 * stops after stage 1, which is plain top-k routing with token dropping (Section 2.3, Figure 1(b)).  Any C >= 1 is
 * accepted (no over-subscription error: holes simply stay).  The call synchronises the stream; workspace as for
 * maxscore_assign_i32.  Returns MAXSCORE_ERR_NOT_CONVERGED if proposals were still pending after max_rounds
 * (the assignment is feasible all the same). */
int32_t maxscore_assign_iter_i32(const int32_t *q, int32_t T, int32_t E, int32_t k, int32_t C, int32_t max_rounds,
                                 int32_t *assign, int64_t *total, int32_t *flow, int32_t *rounds, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* Activation movement around the experts (the step after the routing path; Eq. 1 and the capacity
 * buffers of Section 2.3).
 *
 * maxscore_dispatch_tokens: expert_in[E, C, d] (same element type as x) receives, in slot s of expert j,
 * row disp_token[expert_offsets[j] + s] of x[T, d]; the slots past the expert's count are set to zero.
 * Every expert must hold at most C tokens (true for the outputs of a6 when the same C was used in a4).
 *
 * maxscore_combine: y[T, d] (fp32) = sum over s of gates[i, s] * expert_out[assign[i, s], token_pos[i, s], :]
 * with fp32 accumulation; slots with assign < 0 contribute nothing.  expert_out is [E, C, d] bf16 or fp32.
 * Both only enqueue work; rows whose byte length is a multiple of 16 (and 16-byte aligned buffers) take
 * the fast path. */
int32_t maxscore_dispatch_tokens(const void *x, int32_t in_dtype, const int32_t *expert_offsets,
                                 const int32_t *disp_token, int32_t T, int32_t d, int32_t E, int32_t C,
                                 void *expert_in, void *stream);
int32_t maxscore_combine(const void *expert_out, int32_t in_dtype, const int32_t *assign, const int32_t *token_pos,
                         const float *gates, int32_t T, int32_t d, int32_t E, int32_t k, int32_t C, float *y,
                         void *stream);

/* a2..a6 from given logits.  scores_out[T,E] and q_out[T,E] are required (they are the working
 * storage of a2/a3).  Synchronises `stream`. */
int32_t maxscore_route_logits(const float *logits, int32_t T, int32_t E, int32_t k, int32_t C,
                              const maxscore_opts *opts, float *scores_out, int32_t *q_out,
                              int32_t *assign, float *gates, int32_t *expert_offsets,
                              int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                              int64_t *prices, maxscore_stats *stats, void *workspace,
                              size_t workspace_bytes, void *stream);

/* a3..a6 from given scores A[T,E] (fp32; e.g. affinities produced by another operator): rewards
 * q_out[T,E] = round_half_even(A * 2^quant_shift) (required: the working storage of a3), then the assignment on
 * them (Eq. 7-8), gates[i,s] = A[i, assign[i,s]] (Eq. 2) and the dispatch (Section 2.3).  Algorithm 1's
 * Require/Ensure: affinities in, P out.  Synchronises `stream`. */
int32_t maxscore_route_scores(const float *scores, int32_t T, int32_t E, int32_t k, int32_t C,
                              const maxscore_opts *opts, int32_t *q_out, int32_t *assign, float *gates,
                              int32_t *expert_offsets, int32_t *disp_token, float *disp_gate,
                              int32_t *token_pos, int64_t *prices, maxscore_stats *stats, void *workspace,
                              size_t workspace_bytes, void *stream);

/* a1 + a2 + a3: scores[T,E] and/or q[T,E] from x and W_g (Eq. 2, then Eq. 6 and the rounding), in one kernel where
 * maxscore_route_xw can do so (same conditions, `workspace` as for maxscore_router_logits; logits_out may then be
 * NULL), else by the two kernels of maxscore_router_logits and maxscore_softtopk through logits_out (required
 * then).  Only enqueues work. */
int32_t maxscore_router_softtopk(const void *x, const void *W, const float *bias, int32_t in_dtype, int32_t T,
                                 int32_t d, int32_t E, int32_t k, float t, int32_t quant_shift, float *logits_out,
                                 float *scores, int32_t *q, void *workspace, size_t workspace_bytes, void *stream);

/* a1..a6 from x and W_g.  With bf16 inputs, E in {32, 64, 128}, d a multiple of 64 and the workspace of
 * maxscore_workspace_bytes(T, d, ...) the projection computes the SoftTopk scores and the rewards in its own
 * epilogue (a1..a3 in one kernel, Eq. 2 -> Eq. 6; scores and rewards bit-equal to the separate kernels'); then
 * logits_out may be NULL and the logits are never written.  Otherwise logits_out[T,E] is required
 * (MAXSCORE_ERR_NULL).  Synchronises `stream`. */
int32_t maxscore_route_xw(const void *x, const void *W, const float *bias, int32_t in_dtype,
                          int32_t T, int32_t d, int32_t E, int32_t k, int32_t C,
                          const maxscore_opts *opts, float *logits_out, float *scores_out,
                          int32_t *q_out, int32_t *assign, float *gates, int32_t *expert_offsets,
                          int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                          int64_t *prices, maxscore_stats *stats, void *workspace,
                          size_t workspace_bytes, void *stream);

/* Switch per-launch HIP-event timing of the solver's bid and select passes on (1) or off (0, default).
 * Timing adds three event records per round; it is meant for benchmarks. */
void maxscore_set_kernel_timing(int32_t on);

/* Plain device-to-device copy kernel of `bytes` bytes (multiple of 16), used by the benchmark to
 * calibrate memory counters and to measure achievable bandwidth. */
int32_t maxscore_copy_bytes(const void *src, void *dst, size_t bytes, void *stream);

const char *maxscore_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* MAXSCORE_H */
