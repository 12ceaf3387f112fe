// Exact capacity-constrained maximum-score assignment (Section 3.2, Eq. 7-8, Table 1) as a
// synchronous forward auction with epsilon-scaling on the bipartite token/expert network.
//
// The paper solves the min-cost max-flow by sequential cheapest-path augmentation and calls it
// inherently sequential; this solver is a different, data-parallel method for the same optimum:
//
//   * Integer rewards are scaled by S = 2^sbits > E.  An assignment in which every token holds k
//     experts whose S*q_ij - p_j is within eps = 1 of its best alternatives, every expert holds
//     <= C tokens and unfilled experts have price 0 cannot be improved: an improving residual
//     cycle visits each expert at most once, so it gains less than E*eps < S, i.e. nothing.
//   * One round = a bid pass over all tokens + a select pass over all experts.
//       bid pass (k_bid): every token re-evaluates its row against the current prices, drops
//         held experts that violate the eps condition or fell below the expert's threshold,
//         refills its free slots with its best experts and emits one bid key per held expert,
//         (S*q_ij - w_i + eps) * 2^tbits + i, where w_i is its best value among experts it does
//         not hold.  Rows that turn out unchanged are recognised by a cheap value-only check; only
//         the others get the full evaluation.  Each workgroup writes its keys as one block sorted
//         by expert.
//       select pass (k_select): every expert holding more than C keys raises its threshold to
//         the (n-C+1)-th smallest key (exact selection), which makes the n-C weakest holders
//         drop in the next bid pass.  The expert's price is threshold >> tbits.
//   * Phases run eps = eps0, eps0/div, ..., 1; prices carry over.  When capacity is slack
//     (T*k < E*C) prices are lowered by beta*eps_prev (clamped at 0) at each phase start, and a
//     phase that ends with an unfilled expert at a positive price is repeated with beta doubled,
//     so the final state always has price 0 on unfilled experts.
//   * When a round moves only a handful of slots, the select pass publishes each expert's lowest
//     keys instead of selecting, and one extra workgroup of the same launch continues the auction
//     on these lists alone (the tail pass) until nothing is over capacity, a list runs out or a
//     hop limit is reached; the next bid pass re-validates every token.
//   * Control is on the device.  State, thresholds and per-expert loads are double-buffered by
//     round parity; every block of the select pass recomputes the same decision (quiescence,
//     phase change, price lowering, done) from the previous round's loads and this round's move
//     counts, so no block waits for another (only the tail workgroup waits, for the candidate
//     lists, in the few rounds that hand over to it).  The host enqueues rounds ahead of the
//     device and polls `done` from pinned memory.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "common.h"

namespace maxscore {

int g_kernel_timing = 0;

namespace {

constexpr unsigned long long kVB = 1ull << 52;  // bias that makes packed values unsigned
constexpr long long kNarrowPrice = (long long)1 << 29;   // prices below this (and a reward range below 2^28/S) fit 32-bit values

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int off)
{
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return ((unsigned long long)hi << 32) | lo;
}

// Inclusive prefix sum over the 64 lanes with lane moves inside the rows and row broadcasts (no LDS crossbar):
// lanes without a source read 0.  Lane 63 ends with the total.
__device__ __forceinline__ int wave_scan_add(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);    // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// The same walk with OR: lane 63 ends with the OR over the wavefront.
__device__ __forceinline__ int wave_scan_or(int v)
{
    v |= __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
    v |= __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
    v |= __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
    v |= __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
    v |= __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v |= __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    return v;
}

// One step of a 64-bit maximum across lanes: both halves make the same lane swap (CTRL: a data-parallel-primitive
// pattern inside the 16-lane row), the larger of own and swapped value stays.
template <int CTRL>
__device__ __forceinline__ unsigned long long max_swap_u64(unsigned long long v)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_mov_dpp((int)(unsigned)v, CTRL, 0xf, 0xf, true);
    const unsigned hi = (unsigned)__builtin_amdgcn_mov_dpp((int)(unsigned)(v >> 32), CTRL, 0xf, 0xf, true);
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    return o > v ? o : v;
}

// Maximum of a 64-bit value over the G lanes of a group, result in every lane of the group.  Groups of 8 and 16
// lanes use lane swaps inside the row (quad, mirrored half row, mirrored row: every lane of a full wavefront is a
// valid source); wider groups go through the LDS crossbar.
template <int G>
__device__ __forceinline__ unsigned long long group_max(unsigned long long v)
{
    if constexpr (G == 8 || G == 16) {
        v = max_swap_u64<0xB1>(v);      // quad_perm [1,0,3,2]
        v = max_swap_u64<0x4E>(v);      // quad_perm [2,3,0,1]
        v = max_swap_u64<0x141>(v);     // row_half_mirror
        if constexpr (G == 16) v = max_swap_u64<0x140>(v);   // row_mirror
    } else {
#pragma unroll
        for (int off = G / 2; off > 0; off >>= 1) {
            unsigned long long o = shfl_xor_u64(v, off);
            v = o > v ? o : v;
        }
    }
    return v;
}


// Maximum of a 32-bit value over the G lanes of a group, result in every lane of the group.  Groups of 8 and 16
// lanes lie inside one 16-lane row, where data-parallel-primitive lane swaps do it without going through the LDS
// crossbar: inside each quad, then the mirrored half row (lane i <-> 7-i pairs the two quads), then the
// mirrored row (lane i <-> 15-i pairs the two halves).
template <int G>
__device__ __forceinline__ int group_max_i32(int v)
{
    if constexpr (G == 8 || G == 16) {
        // every lane of a full wavefront is a valid source for these swaps, so the value read for an invalid
        // source never matters (that lets the compiler fold the swap into the max instruction)
        int o;
        o = __builtin_amdgcn_mov_dpp(v, 0xB1, 0xf, 0xf, true); v = o > v ? o : v;   // quad_perm [1,0,3,2]
        o = __builtin_amdgcn_mov_dpp(v, 0x4E, 0xf, 0xf, true); v = o > v ? o : v;   // quad_perm [2,3,0,1]
        o = __builtin_amdgcn_mov_dpp(v, 0x141, 0xf, 0xf, true); v = o > v ? o : v;  // row_half_mirror
        if constexpr (G == 16) {
            o = __builtin_amdgcn_mov_dpp(v, 0x140, 0xf, 0xf, true); v = o > v ? o : v;  // row_mirror
        }
    } else {
#pragma unroll
        for (int off = G / 2; off > 0; off >>= 1) {
            const int o = __shfl_xor(v, off);
            v = o > v ? o : v;
        }
    }
    return v;
}

// Start of a solve: empty assignment, zero thresholds and counters, the control block.  Runs as the first part of
// k_init_minmax (any grid of 256-thread workgroups with at least 2 * kMaxE threads in all).
__device__ __forceinline__ void init_solve(SolverState *st, long long *theta, int *gcount, int *qmm, int32_t *assign,
                                           int T, int E, int k, int eps_div, int max_rounds, int slack,
                                           long long stop_eps)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t n = (size_t)T * k;
    if ((((uintptr_t)assign) & 15) == 0) {
        int4 *a4 = (int4 *)assign;
        const size_t n4 = n / 4;
        for (size_t a = i; a < n4; a += (size_t)gridDim.x * blockDim.x) a4[a] = make_int4(-1, -1, -1, -1);
        for (size_t a = n4 * 4 + i; a < n; a += (size_t)gridDim.x * blockDim.x) assign[a] = -1;
    } else {
        for (size_t a = i; a < n; a += (size_t)gridDim.x * blockDim.x) assign[a] = -1;
    }
    if (i < (size_t)2 * kMaxE) {
        theta[i] = 0;
        gcount[i] = 0;
    }
    if (i == 0) {
        qmm[0] = 0x7fffffff;
        qmm[1] = -0x7fffffff - 1;
        qmm[2] = 0;                      // internal error flag
        qmm[3] = 0;                      // hand-over counter of the select pass
        st->eps = 1; st->eps_prev = 0; st->beta = 2;
        st->qmin = 0x7fffffff; st->qmax = -0x7fffffff - 1; st->total = 0;
        st->sbits = 0; st->tbits = 0; st->eps_div = eps_div; st->max_rounds = max_rounds;
        st->round = 0; st->phases = 1; st->done = 0; st->status = MAXSCORE_OK; st->moves = 0;
        st->blocks_done = 0; st->flow = 0; st->slack = slack;
        st->wide = 0; st->tail_go = 0; st->after_tail = 0; st->tail_block = 0; st->tail_runs = 0; st->tail_gos = 0;
        st->tail_iters = 0;
        st->warm = 0; st->early_off = 0; st->phase_start = 0; st->eps0 = 1; st->stop_eps = stop_eps;
        st->fin = 0; st->fin_passes = 0; st->fin_cycles = 0; st->fin_dirty = 0; st->fin_bound = 0;
        for (int a = 0; a < 28; ++a) st->phase_round[a] = 0;
    }
}

// Reward range: every workgroup leaves its minimum and maximum in part[2*b], part[2*b+1] (no atomics:
// a thousand workgroups updating one word cost more than reading the matrix), k_setup reduces them.
constexpr int kMinmaxBlocks = 512;

__global__ __launch_bounds__(256) void k_init_minmax(const int32_t *__restrict__ q, size_t n, int *__restrict__ part,
                                                     SolverState *st, long long *theta, int *gcount, int *qmm,
                                                     int32_t *assign, int T, int E, int k, int eps_div,
                                                     int max_rounds, int slack, long long stop_eps)
{
    init_solve(st, theta, gcount, qmm, assign, T, E, k, eps_div, max_rounds, slack, stop_eps);
    __shared__ int s_lo[4], s_hi[4];
    int lo = 0x7fffffff, hi = -0x7fffffff - 1;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (((uintptr_t)q & 15) == 0) {
        const int4 *q4 = (const int4 *)q;
        const size_t n4 = n / 4;
        for (; i < n4; i += stride) {
            const int4 v = q4[i];
            lo = min(min(lo, v.x), min(min(v.y, v.z), v.w));
            hi = max(max(hi, v.x), max(max(v.y, v.z), v.w));
        }
        i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // the last n % 4 values
    }
    for (; i < n; i += stride) {
        const int v = q[i];
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    }
    for (int off = 32; off > 0; off >>= 1) {
        int a = __shfl_xor(lo, off), b = __shfl_xor(hi, off);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    if ((threadIdx.x & 63) == 0) {
        s_lo[threadIdx.x >> 6] = lo;
        s_hi[threadIdx.x >> 6] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) {
            lo = s_lo[w] < lo ? s_lo[w] : lo;
            hi = s_hi[w] > hi ? s_hi[w] : hi;
        }
        part[2 * blockIdx.x] = lo;
        part[2 * blockIdx.x + 1] = hi;
    }
}

// prices_in (optional): E starting prices in the units of the price output; they become the thresholds of round 0
// and the first phase starts at eps_start (rounded down to a power of the ladder's ratio) instead of at the top.
constexpr long long kMaxPriceIn = (long long)1 << 38;
constexpr long long kFinPairBudget = 8000000;   // the finisher takes over at the first eps rung with pairs * eps (in reward units) under this
constexpr int kFinPasses = 8;              // finisher passes per solve at most
constexpr int kFinGroup = 4;               // passes enqueued at a time
constexpr int kFinAttempts = 3;            // rungs of the ladder at which the finisher may try (after a try that fails the auction goes one rung down)
constexpr int kFinFirstGroup = 2;          // ... the first time (the first pass usually certifies: it keeps its arc list complete)
constexpr long long kFinBoundMult = 32;    // arcs with a reduced cost of 32 eps or more stay out of the finisher's arc matrix
constexpr int kWarmPhaseCap = 48;          // rounds after which a phase started from given prices goes back up the ladder

__global__ __launch_bounds__(kMinmaxBlocks) void k_setup(SolverState *st, const int *__restrict__ part, int nparts,
                                                        int T, int E, int force_wide, int eps0_shift,
                                                        long long *__restrict__ theta,
                                                        const int64_t *__restrict__ prices_in, long long eps_start,
                                                        long long fin_limit_q)
{
    __shared__ int s_lo[kMinmaxBlocks / 64], s_hi[kMinmaxBlocks / 64];
    int lo = 0x7fffffff, hi = -0x7fffffff - 1;
    if ((int)threadIdx.x < nparts) {
        lo = part[2 * threadIdx.x];
        hi = part[2 * threadIdx.x + 1];
    }
    for (int off = 32; off > 0; off >>= 1) {
        int a = __shfl_xor(lo, off), b = __shfl_xor(hi, off);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    if ((threadIdx.x & 63) == 0) {
        s_lo[threadIdx.x >> 6] = lo;
        s_hi[threadIdx.x >> 6] = hi;
    }
    __syncthreads();
    int tb = 1;
    while ((1 << tb) < T) ++tb;
    if (prices_in) {
        for (int e = threadIdx.x; e < E; e += kMinmaxBlocks) {
            long long p = prices_in[e];
            p = p < 0 ? 0 : (p > kMaxPriceIn ? kMaxPriceIn : p);
            theta[e] = p << tb;
        }
    }
    if (threadIdx.x != 0) return;
    for (int w = 1; w < kMinmaxBlocks / 64; ++w) {
        lo = s_lo[w] < lo ? s_lo[w] : lo;
        hi = s_hi[w] > hi ? s_hi[w] : hi;
    }
    st->qmin = lo;
    st->qmax = hi;
    int sb = 0;
    while ((1 << sb) < E + 1) ++sb;
    st->sbits = sb;
    st->tbits = tb;
    long long range = ((long long)hi - (long long)lo) << sb;
    if (range >= ((long long)1 << 38)) {
        st->status = MAXSCORE_ERR_RANGE;
        st->done = 1;
    }
    // values S*(q - qmin) - price fit 32 bits unless the range is this wide or a token can be left
    // without any alternative (k = E: bids of kBidBig)
    st->wide = (range >= ((long long)1 << 28) || force_wide) ? 1 : 0;
    long long top = range >> eps0_shift, eps = 1;
    while (eps * st->eps_div <= top) eps *= st->eps_div;
    st->eps0 = eps;
    if (prices_in) {
        // start lower on the same ladder (the later phases are then the ones of a cold start)
        const long long want = eps_start > 0 ? eps_start : eps / st->eps_div;
        int rungs = 0;
        while (eps > 1 && eps > want) {
            eps /= st->eps_div;
            ++rungs;
        }
        st->warm = rungs;          // steps back up the ladder that are still allowed
    }
    st->eps = eps;
    if (fin_limit_q > 0) {
        // the auction stops at the first rung of its ladder that is at or under fin_limit_q reward units; the
        // cycle-cancelling finisher takes over from there
        const long long limit = fin_limit_q << sb;
        long long r = st->eps0;
        while (r > 1 && r > limit) r /= st->eps_div;
        st->stop_eps = r > 1 ? r : 1;
    }
}

// Bid pass.  A group of G lanes owns one token row; lane l of the group owns the EPL consecutive
// experts l*EPL .. l*EPL+EPL-1 and slot l of the token (k <= G).  A wavefront therefore works on
// 64/G rows at once and its loads of consecutive rows are contiguous.  The next row of each group
// is prefetched into registers while the current one is evaluated.
// (four workgroups per compute unit for the narrow groups; rows of 512 and 1024 experts need more registers)
template <int G, int EPL, bool VEC, bool KV>
__global__ __launch_bounds__(256, (G * EPL > 256 ? 3 : 4)) void k_bid(const int32_t *__restrict__ q, int32_t *__restrict__ assign,
                                             const long long *__restrict__ theta, const SolverState *__restrict__ st,
                                             long long *__restrict__ klist, int *__restrict__ wcnt,
                                             int *__restrict__ wmoves, int *__restrict__ errflag, int T, int E, int k,
                                             int rows_per_wg, const int32_t *__restrict__ kvec, int force,
                                             const unsigned *__restrict__ moved_bits)
{
    constexpr int EP = G * EPL;
    constexpr int NG = 256 / G;
    constexpr int LOGP = EPL == 1 ? 0 : EPL == 2 ? 1 : EPL == 4 ? 2 : EPL == 8 ? 3 : 4;
    __shared__ long long s_theta[EP];
    __shared__ int s_cnt[EP];
    __shared__ int s_off[EP];
    __shared__ int s_wtot[4];
    // staged rows: one padding word after every lane's EPL values and G after every row, so that the
    // 64 lanes of a store spread over all LDS banks (lane stride EPL+1 is odd)
    constexpr int SQ_ROW = EP + G;
    constexpr int SQ_WORDS = NG * SQ_ROW > 2048 ? NG * SQ_ROW : 2048;   // doubles as the sorted key block (1024 keys)
    __shared__ __attribute__((aligned(16))) int s_q[SQ_WORDS];
    __shared__ long long s_key[1024];
    __shared__ short s_exp[1024];
    __shared__ short s_pos[1024];
    __shared__ short s_queue[1024];
    __shared__ unsigned s_hm[256];          // per group of G lanes: G words of "held" bits, one word per lane
    __shared__ int s_moves, s_nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63, lg = lane & (G - 1), gbase = lane & ~(G - 1);
    const int grp = tid / G;
    const int row0 = blockIdx.x * rows_per_wg;
    // the bits of a wavefront ballot that belong to this lane's group, moved down to bit 0
    auto group_bits = [&](unsigned long long b) {
        return G == 64 ? b : (b >> gbase) & ((1ull << (G & 63)) - 1);
    };
    int *sq = s_q + grp * SQ_ROW;
    auto sq_at = [&](int e) { return e + (e >> LOGP); };

    int qn[EPL];
    int an = -2;
    auto load_row_to = [&](int row, int(&qn)[EPL], int &an) {
        const int32_t *qr = q + (size_t)row * E + lg * EPL;
        if constexpr (VEC) {
            if constexpr (EPL >= 4) {
#pragma unroll
                for (int m = 0; m < EPL; m += 4) {
                    int4 t4 = *(const int4 *)(qr + m);
                    qn[m] = t4.x; qn[m + 1] = t4.y; qn[m + 2] = t4.z; qn[m + 3] = t4.w;
                }
            } else if constexpr (EPL == 2) {
                int2 t2 = *(const int2 *)qr;
                qn[0] = t2.x; qn[1] = t2.y;
            } else {
                qn[0] = qr[0];
            }
        } else {
#pragma unroll
            for (int m = 0; m < EPL; ++m) qn[m] = (lg * EPL + m < E) ? qr[m] : 0;
        }
        an = (lg < k) ? assign[(size_t)row * k + lg] : -2;
        // with one k per token (KV), the slots from kvec[row] on do not exist for this row: they read as -2
        // like the lanes beyond k, are never filled and emit no key (both loads are issued unconditionally)
        if (KV) an = (lg < kvec[row]) ? an : -2;
    };
    auto load_row = [&](int row) { load_row_to(row, qn, an); };
    // The first row of every group and the thresholds are requested before the state is looked at:
    // the exit test below then waits for the scalar loads of the state only, while the vector loads
    // are already on their way (rows and thresholds are valid memory whether or not the solve is over).
    if (row0 + grp < T && grp < rows_per_wg) load_row(row0 + grp);
    long long th0[(EP + 255) / 256];
#pragma unroll
    for (int i = 0; i < (EP + 255) / 256; ++i) {
        const int e = tid + i * 256;
        th0[i] = e < E ? theta[e] : 0;
    }
    const int over = st->done;
    const long long eps = st->eps, qmin = st->qmin;
    const int sb = st->sbits, tb = st->tbits;
    // force: one more pass after the end, which only rewrites the key blocks (1: always; 2: if the finisher has
    // certified the optimum after moving tokens, which the host does not know yet when it enqueues this pass)
    if (force == 2 ? !(st->fin == 2 && st->fin_cycles > 0) : (over && !force)) return;
    if (force && moved_bits) {
        // only the key blocks that hold a token the finisher has moved change (the dispatch reads which pairs a
        // block holds, not the key values): the other workgroups leave theirs as they are
        const int r1 = (row0 + rows_per_wg < T ? row0 + rows_per_wg : T) - 1;
        unsigned any = 0;
        for (int wd = row0 >> 5; wd <= (r1 >> 5); ++wd) {
            unsigned m = moved_bits[wd];
            if (wd == (row0 >> 5)) m &= ~0u << (row0 & 31);
            if (wd == (r1 >> 5)) m &= ~0u >> (31 - (r1 & 31));
            any |= m;
        }
        if (!any) return;
    }
#pragma unroll
    for (int i = 0; i < (EP + 255) / 256; ++i) {
        const int e = tid + i * 256;
        if (e < EP) {
            s_theta[e] = th0[i];
            s_cnt[e] = 0;
        }
    }
    if (tid == 0) {
        s_moves = 0;
        s_nq = 0;
    }
    __syncthreads();

    // The prices of this lane's experts are read from the LDS copy of the thresholds where they are needed:
    // keeping the 64-bit values in registers through both kinds of pass costs more registers than a wavefront
    // has to spare, and a spilled row costs a memory round trip at the head of the kernel.
    unsigned validm = 0;
    bool high = false;
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        int e = lg * EPL + m;
        high |= (s_theta[e] >> tb) >= kNarrowPrice;
        if (e < E) validm |= 1u << m;
    }
    // Quick check of a row (most rows of most rounds): when rewards and prices are small enough for
    // 32-bit values (the state says the reward range is, and every wavefront sees all prices, so all
    // take the same branch), and few tokens moved in the previous round, a group first computes only
    // the VALUE of its row's best expert not held, which is all the keys of an unchanged row need.
    // If every hold of the row is still valid the keys are emitted; otherwise the row is queued and
    // gets the full evaluation afterwards, which recomputes everything.
    const bool quick = E == EP && st->round > 0 && !st->wide && __ballot(high) == 0 && (long long)st->moves * 4 < T;
    const int qmin32 = (int)qmin;

    // Full evaluation of one row by its group (lanes of other groups may be inactive).
    auto full_row = [&](const int lr, const int(&qc)[EPL], int my_e) {
        const int row = row0 + lr;
        // stage the raw rewards of the row for the slot lanes
#pragma unroll
        for (int m = 0; m < EPL; ++m) sq[lg * (EPL + 1) + m] = qc[m];

        long long v[EPL];
#pragma unroll
        for (int m = 0; m < EPL; ++m) v[m] = (((long long)qc[m] - qmin) << sb) - (s_theta[lg * EPL + m] >> tb);
        // which of this lane's experts the row holds: the slot lanes set their expert's bit in the word of the lane
        // that owns it (three LDS instructions; a loop over the k slots costs a cross-lane read and half a dozen
        // instructions per slot)
        auto held_mask = [&](int e_slot) {
            unsigned *hmg = s_hm + (tid - lg);
            hmg[lg] = 0;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (e_slot >= 0) atomicOr(&hmg[e_slot >> LOGP], 1u << (e_slot & (EPL - 1)));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            return hmg[lg];
        };
        unsigned heldm = held_mask(my_e);
        // packed candidate: value, then a per-row rotation of the lane order, then the lower expert
        const unsigned long long pbase = (kVB << 10) | ((unsigned long long)((lg + row) & (G - 1)) << 4);
        auto local_best = [&]() {
            unsigned long long b = 0;
            const unsigned cand = validm & ~heldm;
#pragma unroll
            for (int m = 0; m < EPL; ++m) {
                unsigned long long pk = (unsigned long long)(v[m] << 10) + (pbase | (unsigned)(15 - m));
                pk = ((cand >> m) & 1u) ? pk : 0ull;
                b = pk > b ? pk : b;
            }
            return b;
        };
        auto decode = [&](unsigned long long pk) {
            int field = (int)((pk >> 4) & 63), m = 15 - (int)(pk & 15);
            int l = (field - row) & (G - 1);
            return l * EPL + m;
        };
        unsigned long long pk = group_max<G>(local_best());
        bool has_alt = pk != 0;
        long long a = (long long)(pk >> 10) - (long long)kVB;

        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // re-validate the held experts against the current prices and thresholds
        long long my_sq = 0;
        const int was_e = my_e;
        bool dropped = false;
        if (my_e >= 0) {
            my_sq = ((long long)sq[sq_at(my_e)] - qmin) << sb;
            long long bid = has_alt ? my_sq - a + eps : kBidBig;
            long long key = bid * ((long long)1 << tb) + row;
            if (key < s_theta[my_e]) {
                dropped = true;
                my_e = -1;
            }
        }
        const unsigned long long gfb = group_bits(__ballot(my_e == -1));
        const int f = __popcll(gfb);
        if (f > 0) {
            const bool any_drop = group_bits(__ballot(dropped)) != 0;
            if (any_drop) heldm = held_mask(my_e);
            const int my_rank = (my_e == -1) ? __popcll(gfb & ((1ull << lg) - 1)) : -1;
            for (int r = 0; r < f; ++r) {
                pk = group_max<G>(local_best());
                int e = decode(pk);
                if (pk == 0 || e >= E) {          // cannot happen while k <= E; never index out of range
                    e = 0;
                    *errflag = 1;
                }
                long long val = (long long)(pk >> 10) - (long long)kVB;
                if ((e >> LOGP) == lg) heldm |= 1u << (e & (EPL - 1));
                if (my_rank == r) {
                    my_e = e;
                    my_sq = val + (s_theta[e] >> tb);
                }
            }
            pk = group_max<G>(local_best());
            has_alt = pk != 0;
            a = (long long)(pk >> 10) - (long long)kVB;
            if (lg == 0) atomicAdd(&s_moves, f);
            if (lg < k && my_e != was_e) assign[(size_t)row * k + lg] = my_e;
        }
        if (lg < k) {
            const int idx = lr * k + lg;
            if (!KV || my_e >= 0) {
                long long bid = has_alt ? my_sq - a + eps : kBidBig;
                bid = bid < kBidBig ? bid : kBidBig;
                long long key = bid * ((long long)1 << tb) + row;
                int pos = atomicAdd(&s_cnt[my_e], 1);
                s_key[idx] = key;
                s_exp[idx] = (short)my_e;
                s_pos[idx] = (short)pos;
            } else {
                s_exp[idx] = -1;           // a slot this token does not have
            }
        }
    };

    if (quick) {
        // pass 1: value-only check of every row; rows with a hold to drop or a slot to fill are queued.
        // The raw rewards are staged; slot lanes fetch the reward of their expert and then blank it, so that
        // the re-read row holds only experts not held.  Values are (q - qmin)*S - price in 32 bits, computed
        // as (q << sb) + np with np = -(price + (qmin << sb)) (wrap-around arithmetic; the true value fits).
        constexpr int kBlank = -(1 << 30);        // (blank value) - price stays above -2^31
        const unsigned qmin_s = (unsigned)qmin32 << sb;
        const int blank_q = (int)((unsigned)qmin32 + (unsigned)(kBlank >> sb));
        unsigned np[EPL];
#pragma unroll
        for (int m = 0; m < EPL; ++m) np[m] = 0u - ((unsigned)(s_theta[lg * EPL + m] >> tb) + qmin_s);
        auto quick_row = [&](const int lr, const int(&qc)[EPL], const int my_e) {
            const int row = row0 + lr;
#pragma unroll
            for (int m = 0; m < EPL; ++m) sq[lg * (EPL + 1) + m] = qc[m];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            int my_u = 0;
            if (my_e >= 0) {
                my_u = sq[sq_at(my_e)] - qmin32;       // u = q - qmin (>= 0, < 2^28 / S)
                sq[sq_at(my_e)] = blank_q;             // same lane, same word: read, then overwritten
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            int bv = -0x7fffffff - 1;
#pragma unroll
            for (int m = 0; m < EPL; ++m) {
                int vv;     // (q << sb) + np in one instruction; E == EP: no padding experts
                asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(vv) : "v"(sq[lg * (EPL + 1) + m]), "s"(sb), "v"(np[m]));
                bv = vv > bv ? vv : bv;
            }
            bv = group_max_i32<G>(bv);
            bool bad = false;
            long long qkey = 0;
            if (KV ? my_e != -2 : lg < k) {      // a slot lane of this row
                bad = my_e < 0;
                if (!bad) {
                    long long bid = ((long long)my_u << sb) - (long long)bv + eps;
                    bid = bid < kBidBig ? bid : kBidBig;
                    qkey = bid * ((long long)1 << tb) + row;
                    bad = qkey < s_theta[my_e];
                }
            }
            if (group_bits(__ballot(bad)) == 0) {
                if (lg < k) {
                    const int idx = lr * k + lg;
                    if (!KV || my_e >= 0) {
                        int pos = atomicAdd(&s_cnt[my_e], 1);
                        s_key[idx] = qkey;
                        s_exp[idx] = (short)my_e;
                        s_pos[idx] = (short)pos;
                    } else {
                        s_exp[idx] = -1;   // a slot this token does not have
                    }
                }
            } else if (lg == 0) {
                s_queue[atomicAdd(&s_nq, 1)] = (short)lr;
            }
            __builtin_amdgcn_wave_barrier();   // the next row reuses this group's staging buffer
        };
        // two register sets take turns: while one row is checked, the next one of the group is on its way
        // into the other set
        int qb[EPL];
        int ab = -2;
        for (int lr = grp; lr < rows_per_wg; lr += 2 * NG) {
            const int row = row0 + lr;
            if (row >= T) break;
            const bool has_b = lr + NG < rows_per_wg && row + NG < T;
            if (has_b) load_row_to(row + NG, qb, ab);
            quick_row(lr, qn, an);
            if (!has_b) break;
            if (lr + 2 * NG < rows_per_wg && row + 2 * NG < T) load_row_to(row + 2 * NG, qn, an);
            quick_row(lr + NG, qb, ab);
        }
        __syncthreads();
        // pass 2: the queued rows, compacted over the groups, get the full evaluation
        const int nq = s_nq;
        for (int qi = grp; qi < nq; qi += NG) {
            const int lr = s_queue[qi];
            load_row(row0 + lr);
            full_row(lr, qn, an);
            __builtin_amdgcn_wave_barrier();   // the next row reuses this group's staging buffer
        }
    } else {
        for (int lr = grp; lr < rows_per_wg; lr += NG) {
            const int row = row0 + lr;
            if (row >= T) break;
            int qc[EPL];
#pragma unroll
            for (int m = 0; m < EPL; ++m) qc[m] = qn[m];
            const int my_e = an;
            if (lr + NG < rows_per_wg && row + NG < T) load_row(row + NG);
            full_row(lr, qc, my_e);
            __builtin_amdgcn_wave_barrier();   // the next row reuses this group's staging buffer
        }
    }
    __syncthreads();
    // The keys of this workgroup are stored sorted by expert in one contiguous block of the key
    // buffer (block w starts at w*rows_per_wg*k), with (offset << 16 | count) per expert beside it:
    // full cache lines are written and no global atomics are needed.
    {
        constexpr int PER = (EP + 255) / 256;
        int loc[PER];
        int sum = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int e = tid * PER + i;
            loc[i] = e < EP ? s_cnt[e] : 0;
            sum += loc[i];
        }
        const int inc = wave_scan_add(sum);
        if ((tid & 63) == 63) s_wtot[tid >> 6] = inc;
        __syncthreads();
        int base = inc - sum;
        for (int w = 0; w < (tid >> 6); ++w) base += s_wtot[w];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int e = tid * PER + i;
            if (e < EP) s_off[e] = base;
            if (e < E) wcnt[(size_t)blockIdx.x * E + e] = (base << 16) | loc[i];
            base += loc[i];
        }
    }
    if (tid == 0) wmoves[blockIdx.x] = s_moves;
    __syncthreads();
    int rows_here = T - row0;
    rows_here = rows_here < rows_per_wg ? rows_here : rows_per_wg;
    const int nslots = rows_here * k;
    long long *blk = klist + (size_t)blockIdx.x * rows_per_wg * k;
    // sorted inside LDS first (the row staging buffer is free by now), then copied out in order
    long long *s_sorted = (long long *)s_q;
    for (int idx = tid; idx < nslots; idx += 256) {
        const int e = s_exp[idx];
        if (!KV || e >= 0) s_sorted[s_off[e] + s_pos[idx]] = s_key[idx];
    }
    __syncthreads();
    for (int idx = tid; idx < nslots; idx += 256) blk[idx] = s_sorted[idx];
}

// Tail pass: when a bid pass moved only a few slots, one workgroup continues the same auction on the
// candidate lists (each expert's lowest bid keys) published by the select pass, without touching the
// other tokens: an over-full expert drops its lowest candidates and raises its threshold to the next
// one; every dropped token is re-evaluated against the current prices by one wavefront exactly as in
// the bid pass, and its new keys enter the candidate lists.  Keys of tokens that were not touched
// can only be lower than their current values, so the expert still removes a token whose true key is
// the lowest (a candidate that is re-evaluated and survives is put back with its new key).  The pass
// stops when nothing is over capacity, when a list runs out or after max_iters rounds; the next bid
// pass re-validates every token, so this pass only has to make valid moves, not complete ones.
constexpr int kTailThreads = 1024;
#ifdef MAXSCORE_DEBUG_ENV
__device__ int g_tailtrace[256 * 8];      // per tail run: round, iterations, victims, stop1, stop2, over_last, wall ticks
__device__ int g_tailruns;
#endif
constexpr int kHostRoundWord = 8;       // word of the pinned host block that carries the number of rounds done
constexpr int kTailMoves = 16;            // hand over to the tail pass when a bid pass moved this few slots
constexpr int kEarlyMoves = 16;           // a phase before the last one ends when a bid pass moved this few slots
constexpr long long kKeyInf = (long long)1 << 62;
constexpr int kTailSpinMax = 1 << 20;     // polls of the tail workgroup for the candidate lists before it gives up
constexpr int kTailVict = 64;             // dropped tokens per iteration (the list is read back one entry per lane)
static_assert(kTailVict == 64, "the victim list is read with one entry per lane");
constexpr int kTailIns = 256;

// maximum over the 64 lanes with DPP row operations (the result is wavefront-uniform)
__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
    // lanes without a source lane (and the rows a step leaves out) read 0, the identity of the unsigned maximum:
    // that lets the compiler fold the lane move into the max instruction (one instruction per step instead of four)
    unsigned o;
    o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true); v = o > v ? o : v;   // row_shr:1
    o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true); v = o > v ? o : v;   // row_shr:2
    o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true); v = o > v ? o : v;   // row_shr:4
    o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true); v = o > v ? o : v;   // row_shr:8
    o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false); v = o > v ? o : v;  // row_bcast:15
    o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false); v = o > v ? o : v;  // row_bcast:31
    return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v)
{
    const unsigned hi = (unsigned)(v >> 32), lo = (unsigned)v;
    const unsigned mhi = wave_max_u32(hi);
    const unsigned mlo = wave_max_u32(hi == mhi ? lo : 0u);
    return ((unsigned long long)mhi << 32) | mlo;
}

// An LDS counter address the compiler cannot see to be the same in all lanes: with a wavefront-uniform address it
// wraps an atomic add in code that first counts and ranks the active lanes (a loop over them when the addends
// differ); here one or two lanes are active, and the plain LDS atomic is a fraction of that code.
__device__ __forceinline__ int *opaque_counter(int *p)
{
    typedef __attribute__((address_space(3))) int lds_int;
    unsigned off = (unsigned)(unsigned long)(lds_int *)p;      // the 32-bit LDS offset (the address stays an LDS one)
    asm volatile("" : "+v"(off));
    return (int *)(lds_int *)(unsigned long)off;
}

// Sizes of the tail pass by expert slots per lane.  Up to 256 experts every candidate list holds kCand keys; up to
// 512 experts half as many and up to 1024 a quarter (all lists, the per-wavefront row copies and the select pass's
// own key cache share one compute unit's LDS), and the select pass caches fewer keys.  With 1024 experts there is no
// room for the row copies: the rare evaluation that needs one reads the row from memory again.
template <int TEPL> struct TailCfg {
    static constexpr int MaxE = 256, KC = kCand, SelCache = 6144, RowCopy = 256;
};
template <> struct TailCfg<8> {
    static constexpr int MaxE = 512, KC = kCand / 2, SelCache = 3072, RowCopy = 512;
};
template <> struct TailCfg<16> {
    static constexpr int MaxE = 1024, KC = kCand / 4, SelCache = 3072, RowCopy = 1;
};

// Runs in the extra workgroup of the select pass (all kTailThreads threads), after the other
// workgroups have published their candidate lists.
// LDS of the tail pass, in a function of its own so that the instantiations of tail_pass share one copy.
template <int MAXE, int KC, int ROWCOPY>
struct TailSharedT {
    // candidate lists are kept in DESCENDING order: the lowest keys sit at the end and leave by
    // shortening the list
    long long cand[MAXE * KC];
    long long theta[MAXE];
    long long bound[MAXE];
    long long ikey[kTailIns];
    int n[MAXE];
    int capv[MAXE];     // capacity of every expert (uniform Ce unless a vector was given)
    int cn[MAXE];
    int vtok[kTailVict], vexp[kTailVict];
    int iexp[kTailIns];
    int qrow[kTailThreads / 64][ROWCOPY];       // per wavefront: the row under evaluation (ROWCOPY = MAXE, or 1: not kept)
    unsigned char hmark[kTailThreads / 64][MAXE];   // per wavefront: 1 on the experts the token under evaluation holds
    int nv2[2], ni2[2], over2[2];     // per-iteration counters, double-buffered by iteration parity
    // stop requests: stop1 is written in step 1 and read after the barrier that ends it, stop2 likewise for
    // step 2, so a flag is never written between a barrier and the reads that follow that barrier
    int stop1, stop2, moves, changed;
};

template <int MAXE, int KC, int ROWCOPY>
__device__ __forceinline__ TailSharedT<MAXE, KC, ROWCOPY> *tail_shared()
{
    __shared__ TailSharedT<MAXE, KC, ROWCOPY> s;
    return &s;
}

// TEPL = expert slots per lane (ceil(E / 64) <= TEPL): 1 and 2 serve E <= 64 and E <= 128 without the dead work
// of 4 (the pass is bound by the number of instructions one wavefront has to get through per hop).
template <int TEPL>
__device__ __forceinline__ void tail_pass(const int32_t *__restrict__ q, int32_t *assign, long long *theta2,
                                          int *gcount2, SolverState *st2, const long long *cand, int *errflag,
                                          int par, int T, int E, int k, int Ce, const int *__restrict__ cap,
                                          int max_iters, const int32_t *__restrict__ kvec)
{
    SolverState *st = st2 + (par ^ 1);          // the state the next bid pass will read
    long long *theta = theta2 + (par ^ 1) * kMaxE;
    int *gcur = gcount2 + par * kMaxE;
    constexpr int KC = TailCfg<TEPL>::KC;       // keys per candidate list
    constexpr bool kRowCopy = TailCfg<TEPL>::RowCopy > 1;
    auto &sh = *tail_shared<TailCfg<TEPL>::MaxE, KC, TailCfg<TEPL>::RowCopy>();
    auto &s_cand = sh.cand;
    auto &s_theta = sh.theta;
    auto &s_bound = sh.bound;
    auto &s_n = sh.n;
    auto &s_capv = sh.capv;
    auto &s_cn = sh.cn;
    auto &s_vtok = sh.vtok;
    auto &s_vexp = sh.vexp;
    auto &s_iexp = sh.iexp;
    auto &s_ikey = sh.ikey;
    auto &s_qrow = sh.qrow;
    auto &s_hmark = sh.hmark;
    auto &s_nv2 = sh.nv2;
    auto &s_ni2 = sh.ni2;
    auto &s_over2 = sh.over2;
    int &s_stop1 = sh.stop1, &s_stop2 = sh.stop2, &s_moves = sh.moves, &s_changed = sh.changed;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const long long eps = st->eps, qmin = st->qmin;
    const int sb = st->sbits, tb = st->tbits;
    const long long tmask = ((long long)1 << tb) - 1;
    const int eplt = (E + 63) >> 6;            // expert slots per lane actually in use
    for (int i = tid; i < E * (kCand + 2); i += kTailThreads) {
        const int e = i / (kCand + 2), c = i - e * (kCand + 2);
        const long long val = cand[i];
        const int cn = (int)cand[(size_t)e * (kCand + 2) + kCand];
        if (c < kCand) {
            if (c < cn && cn <= KC) s_cand[e * KC + (cn - 1 - c)] = val;     // ascending in memory -> descending here
        } else if (c == kCand) {
            s_cn[e] = (int)val;
        } else {
            s_bound[e] = val;
        }
    }
    for (int e = tid; e < E; e += kTailThreads) {
        s_theta[e] = theta[e];
        s_n[e] = gcur[e];
        s_capv[e] = cap ? cap[e] : Ce;
    }
    static_assert(sizeof(sh.hmark) % (4 * kTailThreads) == 0, "whole words of marks per thread");
    for (int i = tid; i < (int)(sizeof(sh.hmark) / 4); i += kTailThreads) ((int *)&s_hmark[0][0])[i] = 0;
    if (tid == 0) {
        s_stop1 = 0; s_stop2 = 0; s_moves = 0; s_changed = 0;
        s_nv2[0] = s_nv2[1] = 0; s_ni2[0] = s_ni2[1] = 0; s_over2[0] = s_over2[1] = 0;
    }
    __syncthreads();

#ifdef MAXSCORE_DEBUG_ENV
    int dbg_vict = 0;
    const long long dbg_t0 = wall_clock64();
#endif
    int it = 0, over_last = 0;
    for (; it < max_iters; ++it) {
        // the counters are double-buffered by iteration parity: this iteration's were cleared during the last one
        const int pi = it & 1;
        int &s_nv = s_nv2[pi], &s_ni = s_ni2[pi], &s_over = s_over2[pi];
        // 0. the keys requested in the previous iteration enter the lists in request order; wavefront w serves
        //    the experts e with e mod 16 = w (its first KC lanes hold one list entry each) and, right after,
        //    runs step 1 for the same experts, so no workgroup barrier is needed between the two
        if (it > 0) {
            const int ni_prev = s_ni2[pi ^ 1];
            const int ni = ni_prev < kTailIns ? ni_prev : kTailIns;
            for (int r = 0; r < ni; ++r) {
                const int e = __builtin_amdgcn_readfirstlane(s_iexp[r]);
                if ((e & (kTailThreads / 64 - 1)) != wv) continue;
                const long long key = s_ikey[r];
                long long *ce = s_cand + e * KC;
                int cn = s_cn[e];
                long long val = (lane < cn && lane < KC) ? ce[lane] : -1;
                bool skip = false;
                if (cn == KC) {
                    const long long top = ce[0];                 // largest listed key
                    if (key > top) {
                        if (lane == 0 && key < s_bound[e]) s_bound[e] = key;   // stays off the list
                        skip = true;
                    } else {
                        if (lane == 0) s_bound[e] = top;         // the largest listed key leaves the list
                        val = (lane + 1 < cn) ? ce[lane + 1] : -1;
                        --cn;
                    }
                }
                __builtin_amdgcn_wave_barrier();
                if (!skip) {
                    const bool above = lane < cn && val > key;
                    const int pos = __popcll(__ballot(above));
                    if (lane < cn) ce[above ? lane : lane + 1] = val;
                    if (lane == 0) {
                        ce[pos] = key;
                        s_cn[e] = cn + 1;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        // 1. every over-full expert drops its lowest candidates and raises its threshold (expert e: lane e/16 of
        //    wavefront e mod 16)
        // (the words of an expert are asked for together, and the list entries together with the slot reservation:
        // three LDS round trips on the path of an over-full expert instead of six)
        for (int e = wv + (kTailThreads / 64) * lane; e < E; e += kTailThreads) {
            const int cap_e = s_capv[e], cn = s_cn[e], n_e = s_n[e];
            const long long theta_e = s_theta[e], bound_e = s_bound[e];
            // (the empty statement makes the five words live here: otherwise the compiler moves each read down to
            // its first use, one dependent round trip after the other)
            asm volatile("" ::"v"(cap_e), "v"(cn), "v"(n_e), "v"(theta_e), "v"(bound_e));
            const int m = n_e - cap_e;
            if (m > 0) {
                s_over = 1;
                if (cn < m) {
                    s_stop1 = 1;                       // list exhausted: the select pass has to rebuild it
                } else {
                    const long long *ce = s_cand + e * KC;
                    const long long low0 = ce[cn - 1];                       // the first key to go
                    const long long next_key = cn > m ? ce[cn - 1 - m] : bound_e;
                    const long long last_out = ce[cn - m];                   // the highest key that goes
                    const int b = atomicAdd(opaque_counter(&s_nv), m);
                    asm volatile("" ::"v"(low0), "v"(next_key), "v"(last_out), "v"(b));
                    if (b + m > kTailVict) {
                        s_stop1 = 1;
                    } else {
                        s_vtok[b] = (int)(low0 & tmask);
                        s_vexp[b] = e;
                        for (int i = 1; i < m; ++i) {
                            s_vtok[b + i] = (int)(ce[cn - 1 - i] & tmask);
                            s_vexp[b + i] = e;
                        }
                        long long nt = next_key;
                        // an expert without capacity that dropped every key it had: nobody may stay at or
                        // under the highest of them
                        if (cap_e == 0 && !(nt < kKeyInf)) nt = last_out + 1;
                        s_cn[e] = cn - m;
                        s_changed = 1;
                        if (nt > theta_e && nt < kKeyInf) s_theta[e] = nt;
                    }
                }
            }
        }
        __syncthreads();
        // the counters of the other parity were last read in step 0 above; the next iteration starts from zero
        // (by the last wavefront: the first ones are the ones that evaluate, and this pass is bound by what they have to issue)
        if (tid == kTailThreads - 1) { s_nv2[pi ^ 1] = 0; s_ni2[pi ^ 1] = 0; s_over2[pi ^ 1] = 0; }
        // everything this step needs from the mailboxes is asked for at once (one LDS round trip instead of five
        // dependent ones): the flags, the count, and the whole victim list, one entry per lane
        const int stop1_now = s_stop1, over_now = s_over, nv_now = s_nv;
        const int vtok_l = s_vtok[lane], vexp_l = s_vexp[lane];
        over_last = over_now;
#ifdef MAXSCORE_DEBUG_ENV
        dbg_vict += nv_now;
#endif
        if (stop1_now || !over_now) break;
        // 2. one wavefront per dropped token: the bid pass's row evaluation
        const int nv = nv_now < kTailVict ? nv_now : kTailVict;
        for (int vi = wv; vi < nv; vi += kTailThreads / 64) {
            const int tok = __builtin_amdgcn_readlane(vtok_l, vi);
            const int32_t *qr = q + (size_t)tok * E;
            // the row is requested first, everything else is looked up while it travels.  Other
            // wavefronts of this workgroup may have rewritten the assignment row in an earlier round:
            // it is read and written at workgroup scope.
            int my_e = lane < k ? __hip_atomic_load(&assign[(size_t)tok * k + lane], __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_WORKGROUP)
                                : -2;
            const int k_tok = kvec ? kvec[tok] : k;       // slots from k_tok on do not exist for this token
            my_e = lane < k_tok ? my_e : -2;
            int qv[TEPL];
#pragma unroll
            for (int m = 0; m < TEPL; ++m) qv[m] = (m < eplt && lane + 64 * m < E) ? qr[lane + 64 * m] : 0;
            // a token challenged by several experts at once is evaluated once, by its first entry
            const unsigned long long twins = __ballot(lane < nv && lane != vi && vtok_l == tok);
            if (twins & ((1ull << vi) - 1)) continue;
            const int ve = __builtin_amdgcn_readlane(vexp_l, vi);
            const long long theta_ve = s_theta[ve];
            long long v[TEPL];
            unsigned validm = 0, heldm = 0;
#pragma unroll
            for (int m = 0; m < TEPL; ++m) {
                v[m] = 0;
                if (m < eplt) {
                    const int e = lane + 64 * m;
                    if (e < E) {
                        v[m] = (((long long)qv[m] - qmin) << sb) - (s_theta[e] >> tb);
                        validm |= 1u << m;
                    }
                }
            }
            {
                // which of this lane's experts the token holds: the slot lanes mark their expert in a byte map of the
                // wavefront, every lane reads its own bytes, the marks are taken back (three LDS instructions where a
                // loop over the slots needs a dozen instructions per slot)
                unsigned char *hm = s_hmark[wv];
                if (my_e >= 0) hm[my_e] = 1;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int m = 0; m < TEPL; ++m) heldm |= (unsigned)hm[lane + 64 * m] << m;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                if (my_e >= 0) hm[my_e] = 0;
            }
            // equal values are ranked by expert id XOR a per-token mask (a bijection below 1024), so that
            // identical rows spread over the experts
            const int r0 = tok & 1023;
            auto best_unheld = [&]() {
                unsigned long long b = 0;
#pragma unroll
                for (int m = 0; m < TEPL; ++m) {
                    if (m < eplt && (((validm & ~heldm) >> m) & 1u)) {
                        unsigned long long pk =
                            ((unsigned long long)(v[m] + (long long)kVB) << 10) | (unsigned)((lane + 64 * m) ^ r0);
                        b = pk > b ? pk : b;
                    }
                }
                return wave_max_u64(b);
            };
            auto expert_of = [&](unsigned long long pk) { return (int)(pk & 1023) ^ r0; };
            auto key_of = [&](long long sq, unsigned long long pk_alt) {
                long long bid = pk_alt != 0 ? sq - ((long long)(pk_alt >> 10) - (long long)kVB) + eps : kBidBig;
                bid = bid < kBidBig ? bid : kBidBig;
                return bid * ((long long)1 << tb) + tok;
            };
            // (bounds and thresholds are only written in steps 0 and 1, so they can be read ahead of their use here)
            auto request = [&](int e, long long key, long long bound_e) {       // one lane; bound_e = s_bound[e]
                if (key < bound_e) {
                    const int slot = atomicAdd(opaque_counter(&s_ni), 1);
                    if (slot < kTailIns) {
                        s_iexp[slot] = e;
                        s_ikey[slot] = key;
                    } else {
                        s_stop2 = 1;
                    }
                }
            };
            unsigned long long pk = best_unheld();
            if (!twins) {
                // The usual case: one hold (tok, ve) is challenged.  Every other hold of the token is
                // still valid (its listed key was not popped and true keys only rise), so only this
                // one is decided, with wavefront-uniform arithmetic.
                auto reward_of = [&](int e) {             // e is wavefront-uniform
                    int r = 0;
#pragma unroll
                    for (int m = 0; m < TEPL; ++m)
                        if ((e >> 6) == m) r = __builtin_amdgcn_readlane(qv[m], e & 63);
                    return ((long long)r - qmin) << sb;
                };
                if (__ballot(my_e == ve) != 0) {           // still held (else there is nothing to decide)
                    const long long key = key_of(reward_of(ve), pk);
                    if (key >= theta_ve) {
                        if (lane == 0) request(ve, key, s_bound[ve]);   // survives: back on the list with its true key
                    } else {
                        // falls below the threshold: the best expert not held takes the slot (ve itself
                        // cannot be it: its value is now at least eps under that best one)
                        const int e1 = __builtin_amdgcn_readfirstlane(expert_of(pk));
                        if (pk == 0 || e1 >= E) {          // cannot happen while k <= E
                            *errflag = 1;
                        } else {
                            const long long bound_e1 = s_bound[e1];     // on its way while the next best is found
                            if ((ve & 63) == lane) heldm &= ~(1u << (ve >> 6));
                            if ((e1 & 63) == lane) heldm |= 1u << (e1 >> 6);
                            const unsigned long long pk2 = best_unheld();
                            const long long key1 = key_of(reward_of(e1), pk2);
                            if (my_e == ve)
                                __hip_atomic_store(&assign[(size_t)tok * k + lane], e1, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                            // the three counters in one LDS instruction: lanes 0-2 take one each (with a
                            // wavefront-uniform address the compiler wraps every atomic in code that counts
                            // the active lanes first)
                            if (lane < 3) {
                                int *ctr = lane == 0 ? &s_n[ve] : lane == 1 ? &s_n[e1] : &s_moves;
                                atomicAdd(ctr, lane == 0 ? -1 : 1);
                            }
                            if (lane == 0) {
                                request(e1, key1, bound_e1);
                            }
                        }
                    }
                }
                continue;
            }
            // several holds of the token are challenged at once: the bid pass's general evaluation
            // (the slot lanes need the reward of their own expert: from a copy of the row in LDS, or from memory)
            const int *qrow = kRowCopy ? s_qrow[wv] : qr;
            if (kRowCopy) {
                int *qw = s_qrow[wv];
#pragma unroll
                for (int m = 0; m < TEPL; ++m)
                    if (m < eplt && lane + 64 * m < E) qw[lane + 64 * m] = qv[m];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            long long my_sq = 0;
            bool dropped = false;
            if (my_e >= 0) {
                my_sq = ((long long)qrow[my_e] - qmin) << sb;
                if (key_of(my_sq, pk) < s_theta[my_e]) {
                    dropped = true;
                    atomicAdd(&s_n[my_e], -1);
                }
            }
            bool challenged = my_e == ve;      // a challenged hold that survives goes back on its list
            if (my_e >= 0) {
                unsigned long long tw = twins;
                while (tw) {
                    const int u = __ffsll((long long)tw) - 1;
                    tw &= tw - 1;
                    challenged |= s_vexp[u] == my_e;
                }
            }
            unsigned long long db = __ballot(dropped);
            const int f = __popcll(db);
            bool picked = false;
            if (f > 0) {
                const unsigned long long fb = db;
                while (db) {                           // dropped experts become candidates again
                    const int sl = __ffsll((long long)db) - 1;
                    db &= db - 1;
                    const int es = __builtin_amdgcn_readlane(my_e, sl);
                    if ((es & 63) == lane) heldm &= ~(1u << (es >> 6));
                }
                if (dropped) my_e = -1;
                const int my_rank = dropped ? __popcll(fb & ((1ull << lane) - 1)) : -1;
                for (int r = 0; r < f; ++r) {
                    pk = best_unheld();
                    int e = expert_of(pk);
                    if (pk == 0 || e >= E) {
                        e = 0;
                        *errflag = 1;
                    }
                    if ((e & 63) == lane) heldm |= 1u << (e >> 6);
                    if (my_rank == r) {
                        my_e = e;
                        my_sq = ((long long)qrow[e] - qmin) << sb;
                        picked = true;
                    }
                }
                pk = best_unheld();
                if (lane == 0) atomicAdd(&s_moves, f);
            }
            if (lane < k && my_e >= 0 && (picked || challenged)) {
                const long long key = key_of(my_sq, pk);
                if (picked) {
                    __hip_atomic_store(&assign[(size_t)tok * k + lane], my_e, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                    atomicAdd(&s_n[my_e], 1);
                }
                request(my_e, key, s_bound[my_e]);
            }
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        if (s_stop2) break;
    }
    for (int e = tid; e < E; e += kTailThreads) {
        theta[e] = s_theta[e];
        gcur[e] = s_n[e];
    }
    if (tid == 0) {
        // Ended with nothing over capacity: every hold is valid, the phase is quiescent.  Without slack
        // there is no price lowering to decide, so the next round starts the next phase right away
        // (the last phase still gets its full check by a bid pass).
        const int stopped = s_stop1 | s_stop2;
        if (!stopped && !over_last && !st->slack && st->eps > st->stop_eps) {
            if (st->phases <= 28) st->phase_round[st->phases - 1] = st->round;
            st->eps_prev = st->eps;
            const long long ne = st->eps / st->eps_div;
            st->eps = ne > 1 ? ne : 1;
            st->phases += 1;
            st->moves = T;
            st->phase_start = st->round;
        }
        st->after_tail = (s_changed || s_moves) ? 1 : 0;
        st->tail_block = stopped;
        st->tail_go = 0;
#ifdef MAXSCORE_DEBUG_ENV
        {
            const int r = g_tailruns < 255 ? g_tailruns : 255;
            g_tailtrace[r * 8 + 0] = st->round; g_tailtrace[r * 8 + 1] = it; g_tailtrace[r * 8 + 2] = dbg_vict;
            g_tailtrace[r * 8 + 3] = s_stop1; g_tailtrace[r * 8 + 4] = s_stop2; g_tailtrace[r * 8 + 5] = over_last;
            g_tailtrace[r * 8 + 6] = (int)(wall_clock64() - dbg_t0); g_tailtrace[r * 8 + 7] = s_moves;
            g_tailruns = r + 1;
        }
#endif
        st->tail_runs += 1;
        st->tail_iters += it;
    }
}

// Select pass: one workgroup per expert; exact (n-Ce+1)-th smallest key by radix select (Ce = the expert's
// capacity: cap[e] when a capacity vector is given, else the same Ce for all).
constexpr int kSelThreads = 1024;
constexpr int kSelDirect = 256;           // at most this many keys are ranked against each other directly


static_assert(kSelThreads == kTailThreads, "the tail pass runs in a workgroup of the select pass");

// Grid: E workgroups, one per expert, plus (when tail_on) one more that runs the tail pass on the
// candidate lists the others publish in rounds that hand over to it.  TEPL = expert slots per lane of the tail
// pass (the host picks the smallest that covers E: the kernel then carries one copy of that pass, and a smaller
// kernel measurably runs faster here).
#ifdef MAXSCORE_DEBUG_ENV
__device__ long long g_roundtrace[2048 * 2];      // per round: moves | flags << 32, eps
#endif
template <int TEPL>
__global__ __launch_bounds__(kSelThreads) void k_select(const long long *__restrict__ klist,
                                                        const int *__restrict__ wcnt, const int *__restrict__ wmoves,
                                                        int *gcount2, long long *theta2, SolverState *st2,
                                                        int *errflag, long long *cand, const int32_t *__restrict__ q,
                                                        int32_t *assign, int *ready, int *host_done, int par, int T, int E, int k,
                                                        int Ce, const int *__restrict__ cap, int n_wg,
                                                        int rows_per_wg, int tail_on, int tail_moves, int early_moves,
                                                        int tail_iters, const int32_t *__restrict__ kvec)
{
    const SolverState *st = st2 + par;
    SolverState *st_out = st2 + (par ^ 1);
    // This thread's count and move words are requested before the state is looked at (valid memory whether or not
    // the solve is over): the exit test then waits for the scalar loads of the state only, and the first of the
    // kernel's two dependent memory round trips has already begun.
    int mt0 = 0, mv = 0;
    {
        const int jj = (int)blockIdx.x == E ? 0 : blockIdx.x;
        if ((int)threadIdx.x < n_wg) {
            mt0 = wcnt[(size_t)threadIdx.x * E + jj];
            mv = wmoves[threadIdx.x];
        }
    }
    if (st->done) {
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            *st_out = *st;
            __hip_atomic_store(host_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);   // also when set-up ended it
        }
        return;
    }
    const long long *theta_in = theta2 + par * kMaxE;
    long long *theta_out = theta2 + (par ^ 1) * kMaxE;
    const int *gprev = gcount2 + (par ^ 1) * kMaxE;   // loads after the previous round
    int *gcur = gcount2 + par * kMaxE;
    constexpr int kSelCache = TailCfg<TEPL>::SelCache;       // keys of an expert that are copied to LDS
    constexpr int KC = TailCfg<TEPL>::KC;                    // keys per candidate list of the tail pass
    __shared__ long long s_keys[kSelCache];
    __shared__ __attribute__((aligned(16))) int s_hist[2][256];
    __shared__ unsigned long long s_small[kSelDirect];
    __shared__ int s_redi[kSelThreads / 64];
    __shared__ int s_flag[kSelThreads / 64];
    __shared__ int s_mvw[kSelThreads / 64];
    __shared__ long long s_cl[kCand];
    __shared__ unsigned long long s_res;
    __shared__ int s_meta[kSelThreads];
    __shared__ int s_d, s_rank, s_m, s_nsm, s_ncl, s_fill, s_ok;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const bool is_tail = (int)blockIdx.x == E;          // the extra workgroup
    const int j = is_tail ? 0 : blockIdx.x;
    // (offset << 16 | count) of this expert inside the key block of bid workgroup w
    auto meta = [&](int w) { return wcnt[(size_t)w * E + j]; };
    const size_t blk_stride = (size_t)rows_per_wg * k;
    // One reduction for everything the block needs: the number of keys of this expert (sum of the
    // per-workgroup counts, with an exclusive scan that places each thread's keys in the LDS copy),
    // the moves of this bid pass, and the over-capacity / unfilled-but-priced experts after the
    // previous round.  All loads are issued before the single barrier.
    int ct = mt0 & 0xffff, ov = 0, vi = 0;
    for (int w = tid + kSelThreads; w < n_wg; w += kSelThreads) {
        ct += meta(w) & 0xffff;
        mv += wmoves[w];
    }
    for (int e = tid; e < E; e += kSelThreads) {
        const int c = gprev[e], ce = cap ? cap[e] : Ce;
        ov += c > ce;
        vi += (c < ce && theta_in[e] > 0);
    }
    const int cur_round = st->round, cur_slack = st->slack, cur_tbits = st->tbits,
              cur_tail_block = st->tail_block, cur_tail_gos = st->tail_gos, cur_max_rounds = st->max_rounds;
    const long long cur_eps = st->eps, cur_eps_prev = st->eps_prev, cur_beta = st->beta;
    const long long base = theta_in[j];
    int flags = (ov ? 2 : 0) | (vi ? 4 : 0);
    flags = wave_scan_or(flags);          // lane 63 holds the wavefront's result
    mv = wave_scan_add(mv);
    ct = wave_scan_add(ct);
    if (lane == 63) {
        s_redi[wv] = ct;
        s_flag[wv] = flags;
        s_mvw[wv] = mv;
    }
    if (tid < 256) {
        s_hist[0][tid] = 0;
        s_hist[1][tid] = 0;
    }
    s_meta[tid] = mt0;
    if (tid == 0) {
        s_ncl = 0;
        s_nsm = 0;
        s_fill = 0;
    }
    __syncthreads();
    int n = 0, moves = 0;
    flags = 0;
    for (int w = 0; w < kSelThreads / 64; ++w) {
        int v = s_redi[w];
        n += v;
        flags |= s_flag[w];
        moves += s_mvw[w];
    }
    if (tid == 0 && !is_tail) gcur[j] = n;

    // the decision every thread of every block takes identically: nothing moved in this bid pass and
    // no expert was above capacity after the previous one  =>  the phase is quiescent
    const bool quiet = (moves == 0 && (flags & 2) == 0 && cur_round > 0);
    const bool redo = quiet && cur_slack && (flags & 4);
    const long long eps_ref = cur_eps_prev > 0 ? cur_eps_prev : cur_eps;
    // few slots moved: leave the thresholds alone, publish each expert's lowest keys and let the
    // single-workgroup tail pass run the next rounds on them
    const bool stopping = cur_round + 1 >= cur_max_rounds || *errflag != 0;
    // (not in the last round the cap allows: that round must leave thresholds that cut every expert to capacity)
    // A phase that is not the auction's last one only has to bring the prices near their values at its eps:
    // the holds it leaves are checked again under the next eps anyway.  Such a phase therefore ends as soon as a
    // round moves only a few slots, instead of settling its last tokens one by one; they go on bidding under the
    // smaller eps.  (Only where supply equals demand: with spare capacity a phase change also lowers prices, which
    // needs the quiescent state.)  The last phase runs to the end: it has to leave a complete assignment.
    // The tokens left over may still have long chains of displacements ahead of them, which a smaller eps makes
    // longer: every early end therefore allows one step back up the ladder should a later phase drag on, and after
    // such a step every phase runs to its end.
    const bool early_end = early_moves > 0 && !quiet && moves <= early_moves && !cur_slack && !st->early_off &&
                           cur_eps > st->stop_eps && !stopping && cur_round - st->phase_start >= 2;
    const bool tail_go = tail_on && !quiet && !cur_tail_block && cur_round > 0 && moves <= tail_moves &&
                         (moves > 0 || (flags & 2)) && !stopping && !early_end;
    int action = 0;
    long long lower = 0;
    if (redo) {
        action = 1;                          // an unfilled expert kept a positive price: redo the phase lower
        lower = cur_beta * 2 * eps_ref;
    } else if (quiet && cur_eps > st->stop_eps && cur_slack) {
        action = 1;
        lower = cur_beta * cur_eps;
    }
    if (blockIdx.x == 0 && tid == 0) {
        SolverState ns = *st;
        const int round = cur_round + 1;
        bool new_phase = false;      // eps changed without a quiescent round
        if (quiet) {
            if (ns.phases <= 28) ns.phase_round[ns.phases - 1] = round;
            ns.phase_start = round;
            if (redo) {
                ns.beta = cur_beta * 2;
                ns.phases += 1;
            } else if (cur_eps <= ns.stop_eps) {
                ns.done = 1;
                ns.fin = ns.stop_eps > 1 ? 1 : 0;      // stopped above eps = 1: the finisher has to take over
            } else {
                ns.eps_prev = cur_eps;
                long long ne = cur_eps / ns.eps_div;
                ns.eps = ne > 1 ? ne : 1;
                ns.phases += 1;
            }
        } else if (round >= ns.max_rounds) {
            ns.status = MAXSCORE_ERR_NOT_CONVERGED;
            ns.done = 1;
        } else if (early_end) {
            if (ns.phases <= 28) ns.phase_round[ns.phases - 1] = round;
            ns.phase_start = round;
            ns.eps_prev = cur_eps;
            long long ne = cur_eps / ns.eps_div;
            ns.eps = ne > 1 ? ne : 1;
            ns.phases += 1;
            ns.warm += 1;
            new_phase = true;
        } else if (ns.warm > 0 && round - ns.phase_start >= kWarmPhaseCap && cur_eps * ns.eps_div <= ns.eps0) {
            // The given prices were further off than the starting eps assumed: one step back up the ladder.  Every
            // hold that is valid at an eps is valid at a larger one, so this is legal at any time; the phases below
            // it run again afterwards.
            ns.eps = cur_eps * ns.eps_div;
            ns.phases += 1;
            ns.phase_start = round;
            ns.warm -= 1;              // at most as many steps up as were skipped or cut short: no ping-pong
            ns.early_off = 1;
            new_phase = true;
        }
        if (*errflag) {
            ns.status = MAXSCORE_ERR_HIP;
            ns.done = 1;
        }
#ifdef MAXSCORE_DEBUG_ENV
        if (cur_round < 2048) {
            g_roundtrace[2 * cur_round] = (long long)moves | ((long long)(flags | (tail_go ? 8 : 0) | (early_end ? 16 : 0) | (quiet ? 32 : 0)) << 32);
            g_roundtrace[2 * cur_round + 1] = cur_eps;
        }
#endif
        ns.round = round;
        ns.moves = (quiet || new_phase) ? T : moves;   // a new phase starts with many moves: no quick checks in its first round
        ns.tail_go = tail_go ? 1 : 0;
        ns.tail_gos = cur_tail_gos + (tail_go ? 1 : 0);
        ns.after_tail = 0;
        ns.tail_block = 0;
        *st_out = ns;
        // the host polls these words (pinned host memory) instead of copying the state or waiting for events: the
        // number of rounds done so far, by which it paces its launches, and the end of the solve
        __hip_atomic_store(host_done + kHostRoundWord, round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (ns.done) __hip_atomic_store(host_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    if (is_tail) {
        // The other workgroups publish their candidate lists, thresholds, loads and the next state, then
        // count themselves in (device-scope release); this one waits for all E of this hand-over
        // (the counter is never reset: E per hand-over so far), drops its stale cache lines and runs the
        // tail pass.  The wait is bounded; nothing the others do depends on this workgroup.
        if (!tail_go || stopping) return;
        if (tid == 0) {
            const int target = (cur_tail_gos + 1) * E;
            int spins = 0;
            while (__hip_atomic_load(ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target &&
                   ++spins < kTailSpinMax)
                __builtin_amdgcn_s_sleep(8);
            s_ok = spins < kTailSpinMax ? 1 : 0;
        }
        __syncthreads();
        __threadfence();
        if (!s_ok) {
            if (tid == 0) *errflag = 1;       // reported as MAXSCORE_ERR_HIP by the next select pass
            return;
        }
        tail_pass<TEPL>(q, assign, theta2, gcount2, st2, cand, errflag, par, T, E, k, Ce, cap, tail_iters, kvec);
        return;
    }
    long long new_theta = base;
    const int Cj = cap ? cap[j] : Ce;         // capacity of this workgroup's expert
    const bool need_select = !tail_go && n > Cj;
    const bool need_cand = tail_go;
    if (need_select || need_cand) {
        const bool cached = n <= kSelCache;
        // Eight consecutive lanes share one segment (the keys one bid workgroup wrote for this expert,
        // a few dozen bytes), so that one load instruction of a wavefront touches 8 cache lines
        // instead of 64.
        const int sub = tid & 7, grp8 = tid >> 3;
        auto seg_meta = [&](int w) { return w < kSelThreads ? s_meta[w] : meta(w); };
        if (cached) {
            constexpr int kSegGroups = kSelThreads / 8;
            const int iters = (n_wg + kSegGroups - 1) / kSegGroups;
            for (int it0 = 0; it0 < iters; it0 += 8) {
                int cs[8];
                long long kvv[8];
                const long long *sp[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int w = grp8 + kSegGroups * (it0 + u);
                    cs[u] = 0;
                    sp[u] = klist;
                    if (w < n_wg) {
                        const int mt = seg_meta(w);
                        cs[u] = mt & 0xffff;
                        sp[u] = klist + (size_t)w * blk_stride + (mt >> 16);
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) kvv[u] = sub < cs[u] ? sp[u][sub] : 0;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (it0 + u < iters) {           // the same for the whole wavefront
                        int inc = cs[u];             // all 8 lanes of a group hold their segment's count
                        // inclusive sum over the groups: the other half of the row, then the rows before
                        inc += __builtin_amdgcn_update_dpp(0, inc, 0x118, 0xf, 0xf, true);    // row_shr:8
                        inc += __builtin_amdgcn_update_dpp(0, inc, 0x142, 0xa, 0xf, false);   // row_bcast:15
                        inc += __builtin_amdgcn_update_dpp(0, inc, 0x143, 0xc, 0xf, false);   // row_bcast:31
                        const int tot = __builtin_amdgcn_readlane(inc, 63);
                        int bp = 0;
                        if (lane == 63 && tot > 0) bp = atomicAdd(&s_fill, tot);
                        bp = __builtin_amdgcn_readlane(bp, 63);
                        const int gpos = bp + inc - cs[u];
                        if (sub < cs[u]) s_keys[gpos + sub] = kvv[u];
                        for (int i = sub + 8; i < cs[u]; i += 8) s_keys[gpos + i] = sp[u][i];
                    }
                }
            }
            __syncthreads();
        }
        // visit every key of this expert (LDS copy when it fits, else the global segments)
        auto for_keys = [&](auto fn) {
            if (cached) {
                for (int i = tid; i < n; i += kSelThreads) fn(s_keys[i]);
            } else {
                for (int w = grp8; w < n_wg; w += kSelThreads / 8) {
                    const int mt = seg_meta(w), c = mt & 0xffff;
                    const long long *seg = klist + (size_t)w * blk_stride + (mt >> 16);
                    for (int i = sub; i < c; i += 8) fn(seg[i]);
                }
            }
        };
        // key of 0-based rank `rank` in ascending order, by narrowing on u = key - base (>= 0: every key of this pass is at or above the old
        // threshold): first the bit length of u (the keys crowd near the threshold with a long tail
        // above, so equal-width digits from the top would separate little), then 8-bit digits below
        // it, and as soon as at most kSelDirect keys share the prefix they are ranked directly.
        // Wavefront 0 scans the histogram (4 bins per lane) while the others clear the next one.
        auto nth_by_narrowing = [&](int rank) {
            int hsel = 0;
            for_keys([&](long long kv) {
                const unsigned long long u = (unsigned long long)(kv - base);
                atomicAdd(&s_hist[0][u ? 64 - __clzll((long long)u) : 0], 1);
            });
            __syncthreads();
            auto scan_find = [&](int h) {       // finds the bin holding `rank`; call from all threads
                if (wv == 0) {
                    const int4 b4 = *(const int4 *)&s_hist[h][lane * 4];
                    const int sum = b4.x + b4.y + b4.z + b4.w;
                    const int hi = wave_scan_add(sum);
                    const int exc = hi - sum;
                    if (exc <= rank && rank < hi) {
                        int r = rank - exc, d = 0, m = b4.x;
                        if (r >= b4.x) { r -= b4.x; d = 1; m = b4.y;
                            if (r >= b4.y) { r -= b4.y; d = 2; m = b4.z;
                                if (r >= b4.z) { r -= b4.z; d = 3; m = b4.w; } } }
                        s_d = lane * 4 + d;
                        s_rank = r;
                        s_m = m;
                    }
                } else if (tid - 64 < 256) {
                    s_hist[h ^ 1][tid - 64] = 0;
                }
                __syncthreads();
            };
            scan_find(0);
            const int bl = s_d;                  // bit length of the wanted u
            if (bl <= 1) return base + (long long)bl;     // u = 0 or u = 1
            rank = s_rank;
            int m = s_m, shift = bl - 1;         // bits below the leading one are still open
            unsigned long long prefix = 1ull << shift, pmask = ~(prefix - 1);
            while (m > kSelDirect && shift > 0) {
                hsel ^= 1;
                const int wd = shift < 8 ? shift : 8;
                shift -= wd;
                const unsigned dm = (1u << wd) - 1;
                for_keys([&](long long kv) {
                    const unsigned long long u = (unsigned long long)(kv - base);
                    if ((u & pmask) == prefix) atomicAdd(&s_hist[hsel][(unsigned)(u >> shift) & dm], 1);
                });
                __syncthreads();
                scan_find(hsel);
                prefix |= (unsigned long long)s_d << shift;
                pmask |= (unsigned long long)dm << shift;
                rank = s_rank;
                m = s_m;
            }
            if (shift == 0) return base + (long long)prefix;
            for_keys([&](long long kv) {
                const unsigned long long u = (unsigned long long)(kv - base);
                if ((u & pmask) == prefix) {
                    const int slot = atomicAdd(&s_nsm, 1);
                    if (slot < kSelDirect) s_small[slot] = u;
                }
            });
            __syncthreads();
            {   // a few threads per listed key count the keys below it
                constexpr int kParts = kSelThreads / kSelDirect;
                const int el = tid / kParts, part = tid % kParts;
                int r = 0;
                unsigned long long mine = 0;
                if (el < m) {
                    mine = s_small[el];
                    for (int i = part; i < m; i += kParts) r += s_small[i] < mine;
                }
                static_assert(kParts == 4, "the partial counts of a key sit in one quad of lanes");
                r += __builtin_amdgcn_mov_dpp(r, 0xB1, 0xf, 0xf, true);     // quad_perm [1,0,3,2]
                r += __builtin_amdgcn_mov_dpp(r, 0x4E, 0xf, 0xf, true);     // quad_perm [2,3,0,1]
                if (el < m && part == 0 && r == rank) s_res = mine;
            }
            __syncthreads();
            const unsigned long long res = s_res;
            __syncthreads();
            if (tid == 0) s_nsm = 0;
            return base + (long long)res;
        };
        if (need_select) {
            // 0-based rank of the new threshold among the keys, ascending; an expert without capacity moves its
            // threshold just above its largest key
            const int rank = Cj > 0 ? n - Cj : n - 1;
            new_theta = nth_by_narrowing(rank) + (Cj > 0 ? 0 : 1);
        } else {
            // candidate list for the tail pass: the KC smallest keys in ascending order, their
            // count, and a bound no other key of this expert lies under
            const long long bound = n > KC ? nth_by_narrowing(KC) : kKeyInf;
            for_keys([&](long long kv) {
                if (kv < bound) s_cl[atomicAdd(&s_ncl, 1)] = kv;
            });
            __syncthreads();
            const int nc = s_ncl;            // = min(n, KC): keys are distinct
            long long *cj_out = cand + (size_t)j * (kCand + 2);
            if (tid < nc) {
                const long long mine = s_cl[tid];
                int r = 0;
                for (int i = 0; i < nc; ++i) r += s_cl[i] < mine;
                cj_out[r] = mine;
            }
            if (tid == 0) {
                cj_out[kCand] = nc;
                cj_out[kCand + 1] = bound;
            }
        }
    }
    if (tid == 0) {
        if (action) {
            long long p = (new_theta >> cur_tbits) - lower;
            new_theta = (p > 0 ? p : 0) << cur_tbits;
        }
        theta_out[j] = new_theta;
    }
    if (tail_go) {
        __syncthreads();
        if (tid == 0) {
            __threadfence();                  // lists, threshold, load and (workgroup 0) the next state are out
            atomicAdd(ready, 1);
        }
    }
}

// Total score and flow of the final assignment: per-workgroup partial sums (no contended atomics), then
// one small workgroup adds them up and writes prices and scale.
constexpr int kFinalBlocks = 256;

__global__ __launch_bounds__(256) void k_finalize(const int32_t *__restrict__ q, const int32_t *__restrict__ assign,
                                                  long long *__restrict__ part, int T, int E, int k)
{
    __shared__ long long s_sum[4];
    __shared__ int s_cnt[4];
    size_t n = (size_t)T * k;
    long long sum = 0;
    int cnt = 0;
    for (size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x; a < n; a += (size_t)gridDim.x * blockDim.x) {
        int e = assign[a];
        if (e >= 0) {
            sum += q[(a / k) * E + e];
            ++cnt;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        sum += (long long)shfl_xor_u64((unsigned long long)sum, off);
        cnt += __shfl_xor(cnt, off);
    }
    if ((threadIdx.x & 63) == 0) {
        s_sum[threadIdx.x >> 6] = sum;
        s_cnt[threadIdx.x >> 6] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        part[2 * blockIdx.x] = s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3];
        part[2 * blockIdx.x + 1] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
    }
}

// At the round cap the last select pass has raised the thresholds so that every expert keeps its capacity, but the
// bid pass that would drop the holds under them never runs.  This pass drops them: every key of the last bid pass
// that lies under its expert's final threshold gives up its slot (-1), which leaves a feasible, incomplete
// assignment.  One workgroup per key block; exits at once unless the solve ended at the cap.
__global__ __launch_bounds__(256) void k_trim(const SolverState *__restrict__ st, const long long *__restrict__ theta2,
                                              const long long *__restrict__ klist, const int *__restrict__ wcnt,
                                              int32_t *__restrict__ assign, int E, int k, int rows_per_wg)
{
    if (st->status != MAXSCORE_ERR_NOT_CONVERGED) return;
    const long long *theta = theta2 + (st->round & 1) * kMaxE;      // what the last select pass wrote
    const long long tmask = ((long long)1 << st->tbits) - 1;
    const long long *blk = klist + (size_t)blockIdx.x * rows_per_wg * k;
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int mt = wcnt[(size_t)blockIdx.x * E + e];
        const int off = mt >> 16, cnt = mt & 0xffff;
        const long long th = theta[e];
        for (int i = 0; i < cnt; ++i) {
            const long long key = blk[off + i];
            if (key < th) {
                const size_t tok = (size_t)(key & tmask);
                for (int sl = 0; sl < k; ++sl)
                    if (assign[tok * k + sl] == e) assign[tok * k + sl] = -1;
            }
        }
    }
}

__global__ __launch_bounds__(kFinalBlocks) void k_finalize2(const long long *__restrict__ part,
                                                           const long long *__restrict__ theta2, SolverState *st,
                                                           int64_t *prices, int64_t *price_scale, int E,
                                                           SolverState *host_state)
{
    const long long *theta = theta2 + (st->round & 1) * kMaxE;      // what the last select pass wrote
    __shared__ long long s_sum[kFinalBlocks / 64], s_cnt[kFinalBlocks / 64];
    long long sum = part[2 * threadIdx.x], cnt = part[2 * threadIdx.x + 1];
    for (int off = 32; off > 0; off >>= 1) {
        sum += (long long)shfl_xor_u64((unsigned long long)sum, off);
        cnt += (long long)shfl_xor_u64((unsigned long long)cnt, off);
    }
    if ((threadIdx.x & 63) == 0) {
        s_sum[threadIdx.x >> 6] = sum;
        s_cnt[threadIdx.x >> 6] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long ts = 0, tc = 0;
        for (int w = 0; w < kFinalBlocks / 64; ++w) {
            ts += s_sum[w];
            tc += s_cnt[w];
        }
        st->total = ts;
        st->flow = (int)tc;
        if (price_scale) *price_scale = (int64_t)1 << st->sbits;
        // the host reads the final state from pinned memory once the stream has drained (no copy in the stream)
        *host_state = *st;
    }
    const int tb = st->tbits;
    if (prices)
        for (int e = threadIdx.x; e < E; e += blockDim.x) prices[e] = theta[e] >> tb;
}

// Sum of a per-token k vector and the number of entries outside 0..k: workgroup b leaves its partial results in
// out[2*b], out[2*b+1] (no atomics, nothing to clear); the host adds the kKvecBlocks pairs.
constexpr int kKvecBlocks = 64;

__global__ __launch_bounds__(256) void k_kvec_check(const int32_t *__restrict__ kvec, int T, int k,
                                                    long long *__restrict__ out)
{
    __shared__ long long s_sum[4];
    __shared__ int s_bad[4];
    long long sum = 0;
    int bad = 0;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < T; i += kKvecBlocks * 256) {
        const int v = kvec[i];
        bad += (v < 0 || v > k);
        sum += v;
    }
    for (int off = 32; off > 0; off >>= 1) {
        sum += (long long)shfl_xor_u64((unsigned long long)sum, off);
        bad += __shfl_xor(bad, off);
    }
    if ((threadIdx.x & 63) == 0) {
        s_sum[threadIdx.x >> 6] = sum;
        s_bad[threadIdx.x >> 6] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3];
        out[2 * blockIdx.x + 1] = s_bad[0] + s_bad[1] + s_bad[2] + s_bad[3];
    }
}

template <int G, int EPL>
void launch_bid(bool vec, const int32_t *q, int32_t *assign, const long long *theta, const SolverState *st,
                long long *klist, int *wcnt, int *wmoves, int *errflag, int T, int E, int k, int rows_per_wg,
                const int32_t *kvec, int force, const unsigned *moved_bits, hipStream_t s)
{
    int grid = (T + rows_per_wg - 1) / rows_per_wg;
#define MS_BK(VV, KK)                                                                                        \
    hipLaunchKernelGGL((k_bid<G, EPL, VV, KK>), dim3(grid), dim3(256), 0, s, q, assign, theta, st, klist, wcnt, \
                       wmoves, errflag, T, E, k, rows_per_wg, kvec, force, moved_bits)
    if (kvec) {
        if (vec) MS_BK(true, true);
        else MS_BK(false, true);
    } else {
        if (vec) MS_BK(true, false);
        else MS_BK(false, false);
    }
#undef MS_BK
}

template <int G>
void launch_bid_g(int EPL, bool vec, const int32_t *q, int32_t *assign, const long long *theta,
                  const SolverState *st, long long *klist, int *wcnt, int *wmoves, int *errflag, int T, int E, int k,
                  int rows_per_wg, const int32_t *kvec, int force, const unsigned *moved_bits, hipStream_t s)
{
#define MS_B(PP) \
    launch_bid<G, PP>(vec, q, assign, theta, st, klist, wcnt, wmoves, errflag, T, E, k, rows_per_wg, kvec, force, moved_bits, s)
    if (EPL == 1) MS_B(1);
    else if (EPL == 2) MS_B(2);
    else if (EPL == 4) MS_B(4);
    else if (EPL == 8) MS_B(8);
    else MS_B(16);
#undef MS_B
}

}  // namespace

int32_t kvec_check(const int32_t *kvec, int T, int E, int k, char *ws, long long *demand, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    long long *out = (long long *)(ws + L.cand_off);       // the candidate lists are not in use before a solve
    hipLaunchKernelGGL(k_kvec_check, dim3(kKvecBlocks), dim3(256), 0, s, kvec, T, k, out);
    long long h[2 * kKvecBlocks];
    MS_HIP(hipMemcpyAsync(h, out, sizeof(h), hipMemcpyDeviceToHost, s));
    MS_HIP(hipStreamSynchronize(s));
    MS_HIP(hipGetLastError());
    long long sum = 0, bad = 0;
    for (int b = 0; b < kKvecBlocks; ++b) {
        sum += h[2 * b];
        bad += h[2 * b + 1];
    }
    if (bad != 0) return MAXSCORE_ERR_SHAPE;
    *demand = sum;
    return MAXSCORE_OK;
}

// Per-host-thread objects of the solver that outlive a call: the pinned flag the select pass writes `done` into,
// and the events (created once, reused by every solve of the thread, never destroyed: a few handles per thread).
struct SolverHost {
    // pinned and mapped, 16 words: [0] the solve has ended, [4..7] the finisher's report, [kHostRoundWord] rounds done
    int *flag = nullptr;
    int *flag_dev = nullptr;    // the same words as the device sees them
    SolverState *state = nullptr, *state_dev = nullptr;      // pinned and mapped: the final state of the last solve
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    // whether the first finisher group of the last solve of this shape certified (what follows a certified solve is
    // enqueued ahead of the group's report only while that keeps happening)
    int ahead_T = 0, ahead_E = 0, ahead_k = 0, ahead_ok = 1;
    std::vector<hipEvent_t> tev;      // pool of per-launch timing events (kernel timing only)
    int device = -1;
};

static int32_t solver_host(SolverHost **out)
{
    static thread_local SolverHost tl[8];      // one per device the thread has solved on (up to 8 devices)
    int dev = 0;
    MS_HIP(hipGetDevice(&dev));
    SolverHost *h = nullptr;
    for (auto &c : tl)
        if (c.device == dev || c.device < 0) {
            h = &c;
            break;
        }
    if (!h) return MAXSCORE_ERR_HIP;
    if (h->device < 0) {
        MS_HIP(hipHostMalloc((void **)&h->flag, 64, hipHostMallocMapped));
        MS_HIP(hipHostGetDevicePointer((void **)&h->flag_dev, h->flag, 0));
        MS_HIP(hipHostMalloc((void **)&h->state, sizeof(SolverState), hipHostMallocMapped));
        MS_HIP(hipHostGetDevicePointer((void **)&h->state_dev, h->state, 0));
        MS_HIP(hipEventCreate(&h->ev0));
        MS_HIP(hipEventCreate(&h->ev1));
        h->device = dev;
    }
    *out = h;
    return MAXSCORE_OK;
}

// On an error after work has been queued the stream is drained before returning, so that nothing of this solve
// is still running on the caller's buffers.
#define MS_HIP_SYNC(call)                        \
    do {                                         \
        if ((call) != hipSuccess) {              \
            (void)hipStreamSynchronize(s);       \
            return MAXSCORE_ERR_HIP;             \
        }                                        \
    } while (0)

int32_t solver_run(const int32_t *q, int T, int E, int k, int Ce, const maxscore_opts &o, int32_t *assign,
                   int64_t *prices, int64_t *price_scale, maxscore_stats *stats, char *ws, hipStream_t s,
                   const int32_t *cap, long long room, const int32_t *kvec, long long demand, SolverGeometry *geom,
                   SolverAfter after, void *after_ctx)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    SolverState *st = (SolverState *)(ws + L.state_off);
    long long *theta = (long long *)(ws + L.theta_off);
    int *gcount = (int *)(ws + L.gcount_off);
    long long *klist = (long long *)(ws + L.klist_off);
    int *qmm = gcount + 2 * kMaxE;   // after the counters: reward min, max, internal error flag
    int *wcnt = (int *)(ws + L.wcnt_off);
    int *wmoves = (int *)(ws + L.wmoves_off);
    long long *cand = (long long *)(ws + L.cand_off);
    int tail_on = (E <= kTailMaxE && !(o.flags & MAXSCORE_FLAG_NO_TAIL_PASS)) ? 1 : 0;
    int tail_iters = 64, tail_moves = kTailMoves, early_moves = kEarlyMoves;
    int eps0_shift = kEps0Shift;
    long long stop_eps = 1;
    // The cycle-cancelling finisher takes over from the auction at the first rung of the eps ladder at or under
    // fin_limit_q reward units (0: the auction runs down to eps = 1 itself).
    // (the number of cycles left to cancel grows with the number of pairs and with eps: the switch point keeps
    // pairs * eps, in reward units, under a budget that leaves a few dozen cycles at most)
    long long fin_limit_q = 0;
    if (E <= kFinMaxE && !(o.flags & MAXSCORE_FLAG_NO_FINISHER)) {
        fin_limit_q = kFinPairBudget / ((long long)T * k);
        fin_limit_q = fin_limit_q < 1 ? 1 : fin_limit_q;
    }
    int fin_passes = kFinPasses;
    long long fin_bound_mult = kFinBoundMult;

    // lanes per token row (G >= k) and consecutive experts per lane
    int G = 8, EPL = 1;
    while (G < k) G *= 2;
    while (G * 16 < E) G *= 2;
    while (G * EPL < E) EPL *= 2;
    const int ngrp = 256 / G;
    int rows = ngrp * 2;
    // more rows per workgroup as long as two workgroups per compute unit remain: fewer, longer key blocks for the
    // select pass, and the loads of a group's later rows overlap with the evaluation of its earlier ones
    while (rows * 2 * k <= 1024 && (T + 2 * rows - 1) / (2 * rows) >= 512) rows *= 2;
    if (rows * k > 1024) rows = ngrp;
    if (rows * k > 1024) return MAXSCORE_ERR_SHAPE;
#ifdef MAXSCORE_DEBUG_ENV
    // tuning overrides of a development build (not compiled into the library otherwise); values are clamped
    if (const char *ev = getenv("MAXSCORE_TAIL_MOVES")) tail_moves = std::max(0, std::min(atoi(ev), kTailVict));
    if (const char *ev = getenv("MAXSCORE_EARLY")) early_moves = std::max(0, atoi(ev));
    if (const char *ev = getenv("MAXSCORE_TAIL")) {
        tail_iters = std::max(0, std::min(atoi(ev), 4096));
        if (tail_iters <= 0) tail_on = 0;
    }
    if (const char *ev = getenv("MAXSCORE_ROWS")) {
        int r = atoi(ev);
        if (r >= ngrp && r % ngrp == 0 && r * k <= 1024) rows = r;
    }
    if (const char *ev = getenv("MAXSCORE_EPS0_SHIFT")) eps0_shift = std::max(0, std::min(atoi(ev), 30));
    if (const char *ev = getenv("MAXSCORE_STOP_EPS")) stop_eps = std::max(1ll, atoll(ev));   // ends early: NOT optimal
    if (const char *ev = getenv("MAXSCORE_FIN_Q")) fin_limit_q = E <= kFinMaxE ? std::max(0ll, atoll(ev)) : 0;
    if (const char *ev = getenv("MAXSCORE_FIN_PASSES")) fin_passes = std::max(1, std::min(atoi(ev), 64));
    if (const char *ev = getenv("MAXSCORE_FIN_BMULT")) fin_bound_mult = std::max(1ll, atoll(ev));
#endif
    const bool vec = (E == G * EPL) && (((uintptr_t)q) % 16 == 0);
    const int n_wg = (T + rows - 1) / rows;
    if (n_wg > L.max_wg) return MAXSCORE_ERR_WORKSPACE;

    SolverHost *hs = nullptr;
    {
        int32_t rc = solver_host(&hs);
        if (rc) return rc;
    }
    // room = total capacity (sum of the vector, or E*Ce)
    // demand = number of pairs to place (sum of the per-token k, or T*k)
    const long long want = kvec ? demand : (long long)T * k;
    const int slack = ((cap ? room : (long long)E * Ce) - want) > 0 ? 1 : 0;
    MS_HIP(hipEventRecord(hs->ev0, s));
    {
        // one launch: the start state of the solve and the reward range, per-workgroup partial results of which
        // k_setup reduces (at least 2 * kMaxE threads: the init part clears that many thresholds and counters)
        size_t nq = (size_t)T * E;
        int g2 = (int)((nq + 256 * 16 - 1) / (256 * 16));
        if (g2 > kMinmaxBlocks) g2 = kMinmaxBlocks;
        if (g2 < 2 * kMaxE / 256) g2 = 2 * kMaxE / 256;
        int *part = (int *)cand;                 // the candidate lists are not in use yet
        hipLaunchKernelGGL(k_init_minmax, dim3(g2), dim3(256), 0, s, q, nq, part, st, theta, gcount, qmm, assign, T, E,
                           k, o.eps_div, o.max_rounds, slack, stop_eps);
        hipLaunchKernelGGL(k_setup, dim3(1), dim3(kMinmaxBlocks), 0, s, st, part, g2, T, E, k == E ? 1 : 0,
                           eps0_shift, theta, o.prices_in, (long long)o.eps_start, fin_limit_q);
    }

    // Rounds are enqueued in batches; the select pass writes the number of rounds done and `done` straight into
    // pinned host memory, and the host paces itself by polling those words (an event per batch would cost the
    // device a pipeline drain of several microseconds each).  The next batch is always enqueued BEFORE the host
    // waits for the current one to end, so the device never idles during the host round trip; once the solve is
    // over the rounds still in the queue exit at once.
    volatile int *hw = (volatile int *)hs->flag;
    hw[0] = 0;
    hw[kHostRoundWord] = 0;
    // Waits until `word` reaches `target` or the solve has ended.  The stream is looked at now and then: an error
    // ends the wait, and so does a stream that has drained (everything enqueued has run; the caller's own limits
    // then decide how to go on).
    auto wait_word = [&](int word, int target, bool or_done) -> int32_t {
        for (unsigned spin = 1;; ++spin) {
            if ((or_done && hw[0]) || hw[word] >= target) return MAXSCORE_OK;
            if ((spin & 2047) == 0) {
                const hipError_t e = hipStreamQuery(s);
                if (e == hipSuccess) return MAXSCORE_OK;
                if (e != hipErrorNotReady) {
                    (void)hipStreamSynchronize(s);
                    return MAXSCORE_ERR_HIP;
                }
            }
            __builtin_ia32_pause();
        }
    };
    std::vector<hipEvent_t> &tev = hs->tev;
    size_t tev_used = 0;
    int batch = 2;      // two to four rounds in flight: each round still queued when the solve ends costs an empty launch pair
#ifdef MAXSCORE_DEBUG_ENV
    if (const char *ev = getenv("MAXSCORE_BATCH")) batch = std::max(1, std::min(atoi(ev), 64));
#endif
    int launched = 0;
    auto enqueue_batch = [&](int slot) -> int32_t {
        for (int b = 0; b < batch; ++b) {
            const int par = launched & 1;
            if (g_kernel_timing) {
                while (tev.size() < tev_used + 3) {
                    hipEvent_t e = nullptr;
                    MS_HIP(hipEventCreate(&e));
                    tev.push_back(e);
                }
                MS_HIP(hipEventRecord(tev[tev_used], s));
            }
#define MS_BID(GG)                                                                                   \
    launch_bid_g<GG>(EPL, vec, q, assign, theta + par * kMaxE, st + par, klist, wcnt, wmoves, qmm + 2, T, E, k, \
                     rows, kvec, 0, nullptr, s)
            if (G == 8) MS_BID(8);
            else if (G == 16) MS_BID(16);
            else if (G == 32) MS_BID(32);
            else MS_BID(64);
#undef MS_BID
            if (g_kernel_timing) MS_HIP(hipEventRecord(tev[tev_used + 1], s));
#define MS_SEL(TT)                                                                                             \
    hipLaunchKernelGGL(k_select<TT>, dim3(E + tail_on), dim3(kSelThreads), 0, s, klist, wcnt, wmoves, gcount, theta, \
                       st, qmm + 2, cand, q, assign, qmm + 3, hs->flag_dev, par, T, E, k, Ce, cap, n_wg, rows, tail_on, \
                       tail_moves, early_moves, tail_iters, kvec)
            if (E <= 64) MS_SEL(1);
            else if (E <= 128) MS_SEL(2);
            else if (E <= 256) MS_SEL(4);
            else if (E <= 512) MS_SEL(8);
            else MS_SEL(16);
#undef MS_SEL
            if (g_kernel_timing) {
                MS_HIP(hipEventRecord(tev[tev_used + 2], s));
                tev_used += 3;
            }
            ++launched;
        }
        return MAXSCORE_OK;
    };
    auto run_rounds = [&]() -> int32_t {
        int cur = 0;
        const int launched0 = launched;
        int32_t rc = enqueue_batch(cur);
        while (rc == MAXSCORE_OK) {
            const int launched_cur = launched;
            rc = enqueue_batch(cur ^ 1);
            if (rc != MAXSCORE_OK) break;
            rc = wait_word(kHostRoundWord, launched_cur, true);      // the batch before the one just enqueued has run
            if (rc != MAXSCORE_OK) return rc;
            if (hw[0] || launched_cur - launched0 > o.max_rounds + 64) break;
            cur ^= 1;
        }
        if (rc != MAXSCORE_OK) (void)hipStreamSynchronize(s);
        return rc;
    };
    {
        int32_t rc = run_rounds();
        if (rc != MAXSCORE_OK) return rc;
    }
    // What follows the solve on the stream: the pass that rewrites the key blocks for the caller (if asked for),
    // the trim at the round cap, totals and prices, the end-of-solve event and the caller's own work.
    auto enqueue_end = [&](int bid_force) -> int32_t {
        const int par = launched & 1;    // every launch after the end copied the final state on: both copies hold it
        if (bid_force && geom) {
#define MS_BIDF(GG) \
    launch_bid_g<GG>(EPL, vec, q, assign, theta + par * kMaxE, st + par, klist, wcnt, wmoves, qmm + 2, T, E, k, rows, \
                     kvec, bid_force, finish_moved_bits(ws, L), s)
            if (G == 8) MS_BIDF(8);
            else if (G == 16) MS_BIDF(16);
            else if (G == 32) MS_BIDF(32);
            else MS_BIDF(64);
#undef MS_BIDF
        }
        // (the trim only has work when the solve ended at the round cap, which takes that many rounds)
        if (launched >= o.max_rounds)
            hipLaunchKernelGGL(k_trim, dim3(n_wg), dim3(256), 0, s, st + par, theta, klist, wcnt, assign, E, k, rows);
        hipLaunchKernelGGL(k_finalize, dim3(kFinalBlocks), dim3(256), 0, s, q, assign, cand, T, E, k);   // lists are free again
        hipLaunchKernelGGL(k_finalize2, dim3(1), dim3(kFinalBlocks), 0, s, cand, theta, st + par, prices, price_scale, E,
                           hs->state_dev);
        MS_HIP_SYNC(hipEventRecord(hs->ev1, s));
        if (after) {
            int tb = 1;                       // as k_setup computes it
            while ((1 << tb) < T) ++tb;
            const SolverGeometry g = {rows, n_wg, tb};
            const int32_t arc = after(after_ctx, g, s, hs->ev1);
            if (arc != MAXSCORE_OK) {
                (void)hipStreamSynchronize(s);
                return arc;
            }
        }
        return MAXSCORE_OK;
    };
    int fin_cycles = 0, fin_state = 0, fin_cycles_before = 0;
    bool end_enqueued = false;
    for (int attempt = 0; fin_limit_q > 0 && attempt < kFinAttempts; ++attempt) {
        // The auction has stopped at a coarse eps (or ended for another reason, then every finisher launch exits at
        // once).  A fixed number of finisher passes is enqueued; the last kernel reports through pinned memory
        // whether the optimum is certified or the auction has been set going again, one step down its ladder, where
        // it stops again for the next attempt (after the last attempt it runs to eps = 1 itself).
        volatile int *words = (volatile int *)hs->flag;
        words[4] = 0;
        const int fp = launched & 1;
        const int retry = attempt + 1 < kFinAttempts ? 1 : 0;
        // the passes are enqueued a few at a time (most solves are certified by the first pass, and a pass that
        // finds the work done still costs two launches)
        int32_t rc = MAXSCORE_OK;
        // (one pass alone the first time if that was enough for the previous solve of the same shape)
        const bool one_sufficed = hs->ahead_T == T && hs->ahead_E == E && hs->ahead_k == k && hs->ahead_ok == 2;
        for (int p0 = 0, grp = one_sufficed ? 1 : kFinFirstGroup; p0 < fin_passes; p0 += grp, grp = kFinGroup) {
            grp = std::min(grp, fin_passes - p0);
            words[4] = 0;                         // (the previous group's report has been read)
            rc = finish_enqueue(q, assign, st + fp, theta, gcount, cap, Ce, T, E, k, ws, rows, n_wg, p0, grp, fin_passes,
                                fin_bound_mult, hs->flag_dev + 4, retry, s);
            if (rc != MAXSCORE_OK) {
                (void)hipStreamSynchronize(s);
                return rc;
            }
            // The first group of the first attempt usually certifies.  What follows a certified solve is therefore
            // enqueued before the host learns how the group ended, so the device goes straight on (the key-block
            // pass decides on the device whether it is needed); if the group did not certify, these launches ran
            // on a state that is not final, which is harmless, and they are enqueued again at the real end.
            const bool same_shape = hs->ahead_T == T && hs->ahead_E == E && hs->ahead_k == k;
            const bool ahead = attempt == 0 && p0 == 0 && (!same_shape || hs->ahead_ok > 0);
            if (ahead) {
                rc = enqueue_end(2);
                if (rc != MAXSCORE_OK) return rc;
            }
            rc = wait_word(4, 1, false);          // the group's last kernel has reported
            if (rc != MAXSCORE_OK) return rc;
            if (words[4] == 0) {                  // (the stream drained without a report: cannot happen)
                (void)hipStreamSynchronize(s);
                return MAXSCORE_ERR_HIP;
            }
            if (ahead && words[4] == 1) end_enqueued = true;
            if (attempt == 0 && p0 == 0) {
                hs->ahead_T = T; hs->ahead_E = E; hs->ahead_k = k;
                // 1: certified by the group (2 once the final state shows that one pass did it); 0: not certified
                hs->ahead_ok = words[4] == 1 ? 1 : 0;
            }
            if (words[4] != 3) break;
        }
        fin_cycles = fin_cycles_before + words[5];
        fin_state = words[6];
        if (words[4] == 2) {
            // not certified: the second copy of the state follows the first, and the rounds go on
            fin_cycles_before = fin_cycles;
            MS_HIP_SYNC(hipMemcpyAsync(st + (fp ^ 1), st + fp, sizeof(SolverState), hipMemcpyDeviceToDevice, s));
            words[0] = 0;
            launched = words[7];          // rounds done so far: thresholds and loads alternate with the round number
            rc = run_rounds();
            if (rc != MAXSCORE_OK) return rc;
            continue;
        }
        if (!end_enqueued) {
            // the caller reads the key blocks of the last bid pass: if tokens were moved, one more pass rewrites them
            // for the final assignment (every hold is valid under the exact prices, so the pass moves nothing)
            rc = enqueue_end(words[5] > 0 ? 1 : 0);
            if (rc != MAXSCORE_OK) return rc;
            end_enqueued = true;
        }
        break;
    }
    if (!end_enqueued) {
        const int32_t rc = enqueue_end(0);
        if (rc != MAXSCORE_OK) return rc;
    }
    MS_HIP(hipStreamSynchronize(s));
    MS_HIP(hipGetLastError());
    const SolverState h = *hs->state;     // what the last k_finalize2 wrote
    if (fin_limit_q > 0 && hs->ahead_T == T && hs->ahead_E == E && hs->ahead_k == k && hs->ahead_ok == 1 &&
        h.fin == 2 && h.fin_passes <= 1)
        hs->ahead_ok = 2;
    float ms = 0.f, bid_ms = 0.f, select_ms = 0.f;
    (void)hipEventElapsedTime(&ms, hs->ev0, hs->ev1);
    int timed = 0;
    if (tev_used > 0) {
        // what a pair of event records costs with nothing between them is taken off every launch time
        float empty_ms = 0.f;
        const int n_cal = 16;
        while (tev.size() < tev_used + 2 * n_cal) {
            hipEvent_t e = nullptr;
            MS_HIP(hipEventCreate(&e));
            tev.push_back(e);
        }
        hipEvent_t *ce = tev.data() + tev_used;
        for (int i = 0; i < n_cal; ++i) {
            MS_HIP(hipEventRecord(ce[2 * i], s));
            MS_HIP(hipEventRecord(ce[2 * i + 1], s));
        }
        MS_HIP(hipStreamSynchronize(s));
        for (int i = 0; i < n_cal; ++i) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, ce[2 * i], ce[2 * i + 1]);
            empty_ms += t / n_cal;
        }
        for (size_t i = 0; i + 2 < tev_used; i += 3) {
            if ((int)(i / 3) < h.round) {
                float t = 0.f;
                (void)hipEventElapsedTime(&t, tev[i], tev[i + 1]);
                t -= empty_ms;
                bid_ms += t > 0.f ? t : 0.f;
                (void)hipEventElapsedTime(&t, tev[i + 1], tev[i + 2]);
                t -= empty_ms;
                select_ms += t > 0.f ? t : 0.f;
                ++timed;
            }
        }
    }
#ifdef MAXSCORE_DEBUG_ENV
    if (getenv("MAXSCORE_DEBUG"))
        fprintf(stderr, "[maxscore] finisher: stop_eps %lld state %d passes %d cycles %d (host saw state %d cycles %d)\n",
                (long long)h.stop_eps, h.fin, h.fin_passes, h.fin_cycles, fin_state, fin_cycles);
    if (getenv("MAXSCORE_TRACE")) {
        static int tt[256 * 8];
        int nr = 0, zero = 0;
        (void)hipMemcpyFromSymbol(tt, HIP_SYMBOL(g_tailtrace), sizeof(tt));
        (void)hipMemcpyFromSymbol(&nr, HIP_SYMBOL(g_tailruns), sizeof(nr));
        (void)hipMemcpyToSymbol(HIP_SYMBOL(g_tailruns), &zero, sizeof(zero));
        for (int r = 0; r < nr; ++r)
            fprintf(stderr, "[tail] after round %d: iters %d victims %d stop1 %d stop2 %d over_last %d us %.1f moves %d\n", tt[r * 8], tt[r * 8 + 1],
                    tt[r * 8 + 2], tt[r * 8 + 3], tt[r * 8 + 4], tt[r * 8 + 5], tt[r * 8 + 6] * 0.01, tt[r * 8 + 7]);
        static long long tr[4096];
        (void)hipMemcpyFromSymbol(tr, HIP_SYMBOL(g_roundtrace), sizeof(tr));
        for (int r = 0; r < h.round && r < 2048; ++r)
            fprintf(stderr, "[trace] round %d eps %lld moves %lld flags %lld\n", r, tr[2 * r + 1], tr[2 * r] & 0xffffffffll, tr[2 * r] >> 32);
    }
    if (getenv("MAXSCORE_DEBUG")) {
        fprintf(stderr, "[maxscore] phase end rounds:");
        for (int a = 0; a < 28 && a < h.phases; ++a) fprintf(stderr, " %d", h.phase_round[a]);
        fprintf(stderr, "  tail runs %d iters %d  [cyc/64: init %d p1 %d p2 %d p3 %d]\n", h.tail_runs, h.tail_iters,
                h.phase_round[20], h.phase_round[21], h.phase_round[22], h.phase_round[23]);
        fprintf(stderr, "  p2 detail: load-wait %d eval %d barrier %d\n", h.phase_round[20], h.phase_round[24], h.phase_round[25]);
        fprintf(stderr, "  eval detail (fast path, cyc/64): held marks %d, first best %d, decision %d, second best %d, commit %d\n",
                h.phase_round[14], h.phase_round[15], h.phase_round[16], h.phase_round[17], h.phase_round[18]);
    }
#endif
    if (geom) {
        geom->rows = rows;
        geom->n_wg = n_wg;
        geom->tbits = h.tbits;
    }
    if (stats) {
        stats->total_score_q = h.total;
        stats->flow_value = h.flow;
        stats->rounds = h.round;
        stats->phases = h.phases;
        stats->status = h.status;
        stats->solver_ms = ms;
        stats->bid_ms = bid_ms;
        stats->bid_launches = timed;
        stats->select_ms = select_ms;
        stats->finish_passes = h.fin_passes;
        stats->finish_cycles = fin_cycles;        // over all attempts (finish_passes: the last attempt's)
    }
    return h.status;
}

}  // namespace maxscore
