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
//         not hold.  Keys are appended to a per-expert list.
//       select pass (k_select): every expert holding more than C keys raises its threshold to
//         the (n-C+1)-th smallest key (exact radix select), which makes the n-C weakest holders
//         drop in the next bid pass.  The expert's price is threshold >> tbits.
//   * Phases run eps = eps0, eps0/div, ..., 1; prices carry over.  When capacity is slack
//     (T*k < E*C) prices are lowered by beta*eps_prev (clamped at 0) at each phase start, and a
//     phase that ends with an unfilled expert at a positive price is repeated with beta doubled,
//     so the final state always has price 0 on unfilled experts.
//   * The last block of the select pass is the controller: it detects quiescence, advances the
//     phase and raises `done`.  The host only enqueues rounds and polls `done`.
#include <vector>

#include "common.h"

namespace maxscore {

int g_kernel_timing = 0;

namespace {

constexpr unsigned long long kVB = 1ull << 52;  // bias that makes packed values unsigned

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int off)
{
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return ((unsigned long long)hi << 32) | lo;
}

template <int G>
__device__ __forceinline__ unsigned long long group_max(unsigned long long v)
{
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) {
        unsigned long long o = shfl_xor_u64(v, off);
        v = o > v ? o : v;
    }
    return v;
}

__global__ void k_init(SolverState *st, long long *theta, int *gcount, int *qmm, int32_t *assign, int T, int E,
                       int k, int eps_div, int max_rounds, int slack)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t n = (size_t)T * k;
    for (size_t a = i; a < n; a += (size_t)gridDim.x * blockDim.x) assign[a] = -1;
    if (i < (size_t)kMaxE) {
        theta[i] = 0;
        gcount[i] = 0;
    }
    if (i == 0) {
        qmm[0] = 0x7fffffff;
        qmm[1] = -0x7fffffff - 1;
        st->eps = 1; st->eps_prev = 0; st->beta = 2;
        st->qmin = 0x7fffffff; st->qmax = -0x7fffffff - 1; st->total = 0;
        st->sbits = 0; st->tbits = 0; st->eps_div = eps_div; st->max_rounds = max_rounds;
        st->round = 0; st->phases = 1; st->done = 0; st->status = MAXSCORE_OK; st->moves = 0;
        st->blocks_done = 0; st->flow = 0; st->slack = slack;
    }
}

__global__ __launch_bounds__(256) void k_minmax(const int32_t *__restrict__ q, size_t n, int *qmin, int *qmax)
{
    int lo = 0x7fffffff, hi = -0x7fffffff - 1;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        int v = q[i];
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    }
    for (int off = 32; off > 0; off >>= 1) {
        int a = __shfl_xor(lo, off), b = __shfl_xor(hi, off);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    if ((threadIdx.x & 63) == 0) {
        atomicMin(qmin, lo);
        atomicMax(qmax, hi);
    }
}

__global__ void k_setup(SolverState *st, const int *qmin, const int *qmax, int T, int E)
{
    st->qmin = *qmin;
    st->qmax = *qmax;
    int sb = 0;
    while ((1 << sb) < E + 1) ++sb;
    int tb = 1;
    while ((1 << tb) < T) ++tb;
    st->sbits = sb;
    st->tbits = tb;
    long long range = ((long long)*qmax - (long long)*qmin) << sb;
    if (range >= ((long long)1 << 38)) {
        st->status = MAXSCORE_ERR_RANGE;
        st->done = 1;
    }
    long long top = range >> 4, eps = 1;
    while (eps * st->eps_div <= top) eps *= st->eps_div;
    st->eps = eps;
}

// Bid pass.  A group of G lanes owns one token row; lane l of the group owns experts l, l+G, ...
// (EPL per lane) and slot l of the token (k <= G).
template <int G, int EPL>
__global__ __launch_bounds__(256) void k_bid(const int32_t *__restrict__ q, int32_t *__restrict__ assign,
                                             const long long *__restrict__ theta, SolverState *__restrict__ st,
                                             long long *__restrict__ klist, int *__restrict__ gcount, int T,
                                             int E, int k, int rows_per_wg)
{
    if (st->done) return;
    constexpr int EP = G * EPL;
    __shared__ long long s_theta[EP];
    __shared__ int s_cnt[EP];
    __shared__ int s_base[EP];
    __shared__ long long s_key[1024];
    __shared__ short s_exp[1024];
    __shared__ short s_pos[1024];
    __shared__ int s_moves;

    const int tid = threadIdx.x;
    const long long eps = st->eps, qmin = st->qmin;
    const int sb = st->sbits, tb = st->tbits;
    for (int e = tid; e < EP; e += 256) {
        s_theta[e] = e < E ? theta[e] : 0;
        s_cnt[e] = 0;
    }
    if (tid == 0) s_moves = 0;
    __syncthreads();

    const int lane = tid & 63, lg = lane & (G - 1), gbase = lane & ~(G - 1);
    const int grp = tid / G, ngrp = 256 / G;
    const int row0 = blockIdx.x * rows_per_wg;
    const unsigned long long gmask = (G == 64) ? ~0ull : (((1ull << G) - 1) << gbase);

    for (int lr = grp; lr < rows_per_wg; lr += ngrp) {
        const int row = row0 + lr;
        if (row >= T) break;
        const int32_t *qr = q + (size_t)row * E;
        const int r0 = row % E;

        long long v[EPL];
        unsigned validm = 0, heldm = 0;
#pragma unroll
        for (int m = 0; m < EPL; ++m) {
            int e = lg + m * G;
            if (e < E) {
                v[m] = (((long long)qr[e] - qmin) << sb) - (s_theta[e] >> tb);
                validm |= 1u << m;
            } else {
                v[m] = 0;
            }
        }
        int my_e = (lg < k) ? assign[(size_t)row * k + lg] : -2;
        for (int s = 0; s < k; ++s) {
            int es = __shfl(my_e, s, G);
            if (es >= 0 && (es & (G - 1)) == lg) heldm |= 1u << (es / G);
        }
        auto local_best = [&]() {
            unsigned long long b = 0;
#pragma unroll
            for (int m = 0; m < EPL; ++m) {
                if (((validm & ~heldm) >> m) & 1u) {
                    int tieb = lg + m * G - r0;
                    if (tieb < 0) tieb += E;
                    unsigned long long pk = ((unsigned long long)(v[m] + (long long)kVB) << 10) | (unsigned)(1023 - tieb);
                    b = pk > b ? pk : b;
                }
            }
            return b;
        };
        unsigned long long pk = group_max<G>(local_best());
        bool has_alt = pk != 0;
        long long a = (long long)(pk >> 10) - (long long)kVB;

        // re-validate the held experts against the current prices and thresholds
        long long my_sq = 0;
        const int was_e = my_e;
        bool dropped = false;
        if (my_e >= 0) {
            my_sq = ((long long)qr[my_e] - qmin) << sb;
            long long bid = has_alt ? my_sq - a + eps : kBidBig;
            long long key = bid * ((long long)1 << tb) + row;
            if (key < s_theta[my_e]) {
                dropped = true;
                my_e = -1;
            }
        }
        const unsigned long long gfb = (__ballot(my_e == -1) & gmask) >> gbase;
        const int f = __popcll(gfb);
        if (f > 0) {
            const bool any_drop = ((__ballot(dropped) & gmask) != 0);
            if (any_drop) {
                heldm = 0;
                for (int s = 0; s < k; ++s) {
                    int es = __shfl(my_e, s, G);
                    if (es >= 0 && (es & (G - 1)) == lg) heldm |= 1u << (es / G);
                }
            }
            const int my_rank = (my_e == -1) ? __popcll(gfb & ((1ull << lg) - 1)) : -1;
            for (int r = 0; r < f; ++r) {
                pk = group_max<G>(local_best());
                int e = 1023 - (int)(pk & 1023) + r0;
                if (e >= E) e -= E;
                if (pk == 0 || e >= E) {          // cannot happen while k <= E; never index out of range
                    e = 0;
                    st->status = MAXSCORE_ERR_HIP;
                }
                long long val = (long long)(pk >> 10) - (long long)kVB;
                if ((e & (G - 1)) == lg) heldm |= 1u << (e / G);
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
            long long bid = has_alt ? my_sq - a + eps : kBidBig;
            bid = bid < kBidBig ? bid : kBidBig;
            long long key = bid * ((long long)1 << tb) + row;
            int pos = atomicAdd(&s_cnt[my_e], 1);
            int idx = lr * k + lg;
            s_key[idx] = key;
            s_exp[idx] = (short)my_e;
            s_pos[idx] = (short)pos;
        }
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256) {
        int c = s_cnt[e];
        s_base[e] = c ? atomicAdd(&gcount[e], c) : 0;
    }
    if (tid == 0 && s_moves) atomicAdd(&st->moves, s_moves);
    __syncthreads();
    int rows_here = T - row0;
    rows_here = rows_here < rows_per_wg ? rows_here : rows_per_wg;
    const int nslots = rows_here * k;
    for (int idx = tid; idx < nslots; idx += 256) {
        int e = s_exp[idx];
        klist[(size_t)e * T + s_base[e] + s_pos[idx]] = s_key[idx];
    }
}

// Select pass: one workgroup per expert; exact (n-Ce+1)-th smallest key by radix select.
constexpr int kSelThreads = 1024;
constexpr int kSelCache = 6144;

__global__ __launch_bounds__(kSelThreads) void k_select(const long long *__restrict__ klist, int *gcount,
                                                        long long *theta, SolverState *st, int T, int E, int Ce)
{
    if (st->done) return;
    __shared__ long long s_keys[kSelCache];
    __shared__ int s_hist[256];
    __shared__ unsigned long long s_red[kSelThreads / 64];
    __shared__ int s_d, s_rank, s_last, s_over, s_viol, s_action;
    __shared__ long long s_lower;
    const int tid = threadIdx.x, j = blockIdx.x;
    const int n = gcount[j];
    if (n > Ce) {
        const long long base = theta[j];
        const long long *keys = klist + (size_t)j * T;
        const bool cached = n <= kSelCache;
        unsigned long long umax = 0;
        for (int i = tid; i < n; i += kSelThreads) {
            long long kv = keys[i];
            if (cached) s_keys[i] = kv;
            unsigned long long u = (unsigned long long)(kv - base);
            umax = u > umax ? u : umax;
        }
        for (int off = 32; off > 0; off >>= 1) {
            unsigned long long o = shfl_xor_u64(umax, off);
            umax = o > umax ? o : umax;
        }
        if ((tid & 63) == 0) s_red[tid >> 6] = umax;
        __syncthreads();
        umax = 0;
        for (int w = 0; w < kSelThreads / 64; ++w) umax = s_red[w] > umax ? s_red[w] : umax;
        int nd = 1;
        while (nd < 8 && (umax >> (8 * nd)) != 0) ++nd;
        unsigned long long prefix = 0, pmask = 0;
        int rank = n - Ce;   // 0-based rank of the new threshold among the keys, ascending
        for (int pass = nd - 1; pass >= 0; --pass) {
            const int shift = pass * 8;
            if (tid < 256) s_hist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < n; i += kSelThreads) {
                unsigned long long u = (unsigned long long)((cached ? s_keys[i] : keys[i]) - base);
                if ((u & pmask) == prefix) atomicAdd(&s_hist[(int)((u >> shift) & 255)], 1);
            }
            __syncthreads();
            if (tid == 0) {
                int cum = 0, dsel = 0;
                for (; dsel < 256; ++dsel) {
                    if (cum + s_hist[dsel] > rank) break;
                    cum += s_hist[dsel];
                }
                s_d = dsel;
                s_rank = rank - cum;
            }
            __syncthreads();
            prefix |= (unsigned long long)s_d << shift;
            pmask |= 255ull << shift;
            rank = s_rank;
        }
        if (tid == 0) theta[j] = base + (long long)prefix;
    }

    // controller: the last block to finish decides what the next round does
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(&st->blocks_done, 1) == (int)gridDim.x - 1);
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (tid == 0) { s_over = 0; s_viol = 0; s_action = 0; s_lower = 0; }
    __syncthreads();
    const int tb = st->tbits;
    for (int e = tid; e < E; e += kSelThreads) {
        int c = __atomic_load_n(&gcount[e], __ATOMIC_RELAXED);
        long long th = __atomic_load_n(&theta[e], __ATOMIC_RELAXED);
        if (c > Ce) atomicAdd(&s_over, 1);
        if (c < Ce && th > 0) atomicAdd(&s_viol, 1);
    }
    __syncthreads();
    if (tid == 0) {
        const int round = st->round + 1;
        const bool quiet = (st->moves == 0 && s_over == 0);
        if (quiet) {
            if (st->slack && s_viol > 0 && st->eps_prev > 0) {
                st->beta *= 2;          // an unfilled expert kept a positive price: redo the phase lower
                s_action = 1;
                s_lower = st->beta * st->eps_prev;
                st->phases++;
            } else if (st->eps == 1) {
                st->done = 1;
            } else {
                st->eps_prev = st->eps;
                long long ne = st->eps / st->eps_div;
                st->eps = ne > 1 ? ne : 1;
                st->phases++;
                if (st->slack) {
                    s_action = 1;
                    s_lower = st->beta * st->eps_prev;
                }
            }
        } else if (round >= st->max_rounds) {
            st->status = MAXSCORE_ERR_NOT_CONVERGED;
            st->done = 1;
        }
        st->round = round;
        st->moves = 0;
        st->blocks_done = 0;
    }
    __syncthreads();
    for (int e = tid; e < E; e += kSelThreads) {
        gcount[e] = 0;
        if (s_action) {
            long long p = (theta[e] >> tb) - s_lower;
            theta[e] = (p > 0 ? p : 0) << tb;
        }
    }
}

__global__ __launch_bounds__(256) void k_finalize(const int32_t *__restrict__ q, const int32_t *__restrict__ assign,
                                                  const long long *__restrict__ theta, SolverState *st,
                                                  int64_t *prices, int64_t *price_scale, int T, int E, int k)
{
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
    if ((threadIdx.x & 63) == 0 && cnt) {
        atomicAdd((unsigned long long *)&st->total, (unsigned long long)sum);
        atomicAdd(&st->flow, cnt);
    }
    if (blockIdx.x == 0) {
        const int tb = st->tbits;
        if (prices)
            for (int e = threadIdx.x; e < E; e += blockDim.x) prices[e] = theta[e] >> tb;
        if (price_scale && threadIdx.x == 0) *price_scale = (int64_t)1 << st->sbits;
    }
}

template <int G, int EPL>
void launch_bid(const int32_t *q, int32_t *assign, const long long *theta, SolverState *st, long long *klist,
                int *gcount, int T, int E, int k, int rows_per_wg, hipStream_t s)
{
    int grid = (T + rows_per_wg - 1) / rows_per_wg;
    hipLaunchKernelGGL((k_bid<G, EPL>), dim3(grid), dim3(256), 0, s, q, assign, theta, st, klist, gcount, T, E, k,
                       rows_per_wg);
}

}  // namespace

int32_t solver_run(const int32_t *q, int T, int E, int k, int Ce, const maxscore_opts &o, int32_t *assign,
                   int64_t *prices, int64_t *price_scale, maxscore_stats *stats, char *ws, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    SolverState *st = (SolverState *)(ws + L.state_off);
    long long *theta = (long long *)(ws + L.theta_off);
    int *gcount = (int *)(ws + L.gcount_off);
    long long *klist = (long long *)(ws + L.klist_off);
    int *qmm = gcount + kMaxE;   // two ints after the counters: reward min / max

    // group size / elements per lane
    int G = 8, EPL = 1;
    while (G < 64 && G < E) G *= 2;
    while (G * EPL < E) EPL *= 2;
    const int ngrp = 256 / G;
    int rows = (T + 1023) / 1024;
    if (rows > 1024 / k) rows = 1024 / k;
    rows = ((rows + ngrp - 1) / ngrp) * ngrp;
    if (rows * k > 1024) rows = (1024 / k / ngrp) * ngrp;
    if (rows < 1) return MAXSCORE_ERR_SHAPE;

    const int slack = ((long long)E * Ce - (long long)T * k) > 0 ? 1 : 0;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    MS_HIP(hipEventCreate(&ev0));
    MS_HIP(hipEventCreate(&ev1));
    MS_HIP(hipEventRecord(ev0, s));
    {
        size_t n = (size_t)T * k;
        int grid = (int)((n + 255) / 256);
        if (grid < 4) grid = 4;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(k_init, dim3(grid), dim3(256), 0, s, st, theta, gcount, qmm, assign, T, E, k,
                           o.eps_div, o.max_rounds, slack);
        size_t nq = (size_t)T * E;
        int g2 = (int)((nq + 256 * 16 - 1) / (256 * 16));
        if (g2 > 2048) g2 = 2048;
        if (g2 < 1) g2 = 1;
        hipLaunchKernelGGL(k_minmax, dim3(g2), dim3(256), 0, s, q, nq, qmm, qmm + 1);
        hipLaunchKernelGGL(k_setup, dim3(1), dim3(1), 0, s, st, qmm, qmm + 1, T, E);
    }

    std::vector<hipEvent_t> tev;
    int batch = 8, launched = 0;
    int h_done = 0;
    while (!h_done) {
        for (int b = 0; b < batch; ++b) {
            if (g_kernel_timing) {
                hipEvent_t e0, e1;
                MS_HIP(hipEventCreate(&e0));
                MS_HIP(hipEventCreate(&e1));
                tev.push_back(e0);
                tev.push_back(e1);
                MS_HIP(hipEventRecord(e0, s));
            }
#define MS_BID(GG, PP) launch_bid<GG, PP>(q, assign, theta, st, klist, gcount, T, E, k, rows, s)
            if (G == 8) MS_BID(8, 1);
            else if (G == 16) MS_BID(16, 1);
            else if (G == 32) MS_BID(32, 1);
            else if (EPL == 1) MS_BID(64, 1);
            else if (EPL == 2) MS_BID(64, 2);
            else if (EPL == 4) MS_BID(64, 4);
            else if (EPL == 8) MS_BID(64, 8);
            else MS_BID(64, 16);
#undef MS_BID
            if (g_kernel_timing) MS_HIP(hipEventRecord(tev.back(), s));
            hipLaunchKernelGGL(k_select, dim3(E), dim3(kSelThreads), 0, s, klist, gcount, theta, st, T, E, Ce);
            ++launched;
        }
        MS_HIP(hipMemcpyAsync(&h_done, &st->done, sizeof(int), hipMemcpyDeviceToHost, s));
        MS_HIP(hipStreamSynchronize(s));
        if (launched > o.max_rounds + 64) break;
        if (batch < 64) batch *= 2;
    }
    hipLaunchKernelGGL(k_finalize, dim3(256), dim3(256), 0, s, q, assign, theta, st, prices, price_scale, T, E, k);
    MS_HIP(hipEventRecord(ev1, s));
    SolverState h;
    MS_HIP(hipMemcpyAsync(&h, st, sizeof(h), hipMemcpyDeviceToHost, s));
    MS_HIP(hipStreamSynchronize(s));
    MS_HIP(hipGetLastError());
    float ms = 0.f, bid_ms = 0.f;
    (void)hipEventElapsedTime(&ms, ev0, ev1);
    int timed = 0;
    for (size_t i = 0; i + 1 < tev.size(); i += 2) {
        if ((int)(i / 2) < h.round) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, tev[i], tev[i + 1]);
            bid_ms += t;
            ++timed;
        }
        (void)hipEventDestroy(tev[i]);
        (void)hipEventDestroy(tev[i + 1]);
    }
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    if (stats) {
        stats->total_score_q = h.total;
        stats->flow_value = h.flow;
        stats->rounds = h.round;
        stats->phases = h.phases;
        stats->status = h.status;
        stats->solver_ms = ms;
        stats->bid_ms = bid_ms;
        stats->bid_launches = timed;
        stats->reserved = 0;
    }
    return h.status;
}

}  // namespace maxscore
