// Iterative rerouting (Section 2.3; the assignment step of the "-I" variants of Section 4): top-k with
// capacity, then the dropped pairs are re-proposed, round by round, to the best expert that still has room.
// A fast heuristic beside the exact solver; it works on the same integer rewards, so every decision is an
// integer comparison.
//
// Orders (the paper leaves them open; these are fixed here so that the result is one well-defined assignment):
//   stage 1  pairs are taken by (choice rank, token id); an expert keeps the first C pairs naming it;
//   stage 2  at the start of a round the experts with room are fixed; a token fills its holes in slot order with
//            its best experts among those (not held, not yet proposed this round); proposals are taken by
//            (slot, token id) and an expert accepts while it has room; rounds repeat until nobody proposes.
// Both orders are "stable position inside the expert" of a slot-major pair list, which the dispatch kernels
// already compute; every round is propose -> positions -> accept.
#include <climits>

#include "common.h"

namespace maxscore {
namespace {

struct IterState {
    unsigned long long total;
    int flow;
    int nprop;     // proposals of the last round
    int rounds;    // rounds that had proposals
    int pad;
};

// Best live expert of a row spread over a wavefront (lane l holds experts l, l+64, ...; bit c of `live` says
// whether the lane's c-th expert may still be chosen): largest reward, ties to the lower expert id; -1 if no
// expert is live.
template <int EPL>
__device__ inline int wave_best(const int (&val)[EPL], unsigned live)
{
    int m = INT_MIN;
#pragma unroll
    for (int c = 0; c < EPL; ++c)
        if (((live >> c) & 1) && val[c] > m) m = val[c];
    for (int off = 32; off >= 1; off >>= 1) {
        const int o = __shfl_xor(m, off);
        m = o > m ? o : m;
    }
    int e = -1;
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
        const unsigned long long b = __ballot(((live >> c) & 1) && val[c] == m);
        if (e < 0 && b) e = 64 * c + __ffsll((long long)b) - 1;
    }
    return e;
}

__device__ inline unsigned drop_expert(unsigned live, int e, int lane)
{
    return (e >= 0 && lane == (e & 63)) ? live & ~(1u << (e >> 6)) : live;
}

// choice[s*T + i] <- the token's s-th best expert, s < k (slot-major list).  One wavefront per token row;
// lane l holds experts l, l+64, ...
template <int EPL>
__global__ __launch_bounds__(256) void k_iter_topk(const int32_t *__restrict__ q, int T, int E, int k,
                                                   int32_t *__restrict__ choice)
{
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = wave; row < T; row += n_waves) {
        int val[EPL];
        unsigned live = 0;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            val[c] = e < E ? q[(size_t)row * E + e] : 0;
            live |= (e < E ? 1u : 0u) << c;
        }
        int mine = -1;
        for (int s = 0; s < k; ++s) {
            const int e = wave_best<EPL>(val, live);
            live = drop_expert(live, e, lane);
            if (lane == s) mine = e;
        }
        if (lane < k) choice[(size_t)lane * T + row] = mine;
    }
}

// assign[i, s] <- choice if the pair is among the first C of its expert, else -1; load <- min(C, count).
__global__ __launch_bounds__(256) void k_iter_keep(const int32_t *__restrict__ choice, const int32_t *__restrict__ pos,
                                                   const int32_t *__restrict__ offsets, int T, int E, int k, int C,
                                                   int32_t *__restrict__ assign, int *__restrict__ load,
                                                   IterState *__restrict__ st)
{
    const size_t n = (size_t)T * k;
    const size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (a < n) {
        const size_t i = a / k, s = a % k, idx = s * T + i;
        assign[a] = pos[idx] < C ? choice[idx] : -1;
    }
    if (blockIdx.x == 0) {
        for (int j = threadIdx.x; j < E; j += blockDim.x) {
            const int cnt = offsets[j + 1] - offsets[j];
            load[j] = cnt < C ? cnt : C;
        }
        if (threadIdx.x == 0) {
            st->total = 0;
            st->flow = 0;
            st->nprop = 0;
            st->rounds = 0;
        }
    }
}

// prop[s*T + i] <- expert proposed for hole s of token i, or -1.
template <int EPL>
__global__ __launch_bounds__(256) void k_iter_propose(const int32_t *__restrict__ q,
                                                      const int32_t *__restrict__ assign,
                                                      const int *__restrict__ load, int T, int E, int k, int C,
                                                      int32_t *__restrict__ prop)
{
    __shared__ unsigned char s_room[kMaxE];
    for (int j = threadIdx.x; j < E; j += blockDim.x) s_room[j] = load[j] < C;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = wave; row < T; row += n_waves) {
        const int slot = lane < k ? assign[(size_t)row * k + lane] : 0;
        unsigned long long holes = __ballot(slot < 0);
        int mine = -1;
        if (holes) {
            int val[EPL];
            unsigned live = 0;
#pragma unroll
            for (int c = 0; c < EPL; ++c) {
                const int e = lane + 64 * c;
                const bool ok = e < E && s_room[e];
                val[c] = ok ? q[(size_t)row * E + e] : 0;
                live |= (ok ? 1u : 0u) << c;
            }
            for (int s = 0; s < k; ++s) live = drop_expert(live, __shfl(slot, s), lane);
            while (holes) {
                const int s = __ffsll((long long)holes) - 1;
                holes &= holes - 1;
                const int e = wave_best<EPL>(val, live);
                if (e < 0) break;
                live = drop_expert(live, e, lane);
                if (lane == s) mine = e;
            }
        }
        if (lane < k) prop[(size_t)lane * T + row] = mine;
    }
}

// A proposal is accepted when its position among the proposals of its expert is below the room left.
__global__ __launch_bounds__(256) void k_iter_accept(const int32_t *__restrict__ prop, const int32_t *__restrict__ pos,
                                                     const int32_t *__restrict__ offsets,
                                                     const int *__restrict__ load, int *__restrict__ load_next, int T,
                                                     int E, int k, int C, int32_t *__restrict__ assign,
                                                     IterState *__restrict__ st)
{
    const size_t n = (size_t)T * k;
    const size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (a < n) {
        const size_t i = a / k, s = a % k, idx = s * T + i;
        const int e = prop[idx];
        if (e >= 0 && pos[idx] < C - load[e]) assign[a] = e;
    }
    if (blockIdx.x == 0) {
        for (int j = threadIdx.x; j < E; j += blockDim.x) {
            const int cnt = offsets[j + 1] - offsets[j], room = C - load[j];
            load_next[j] = load[j] + (cnt < room ? cnt : room);
        }
        if (threadIdx.x == 0) {
            const int np = offsets[E];
            st->nprop = np;
            if (np > 0) st->rounds += 1;
        }
    }
}

__global__ __launch_bounds__(256) void k_iter_total(const int32_t *__restrict__ q, const int32_t *__restrict__ assign,
                                                    int T, int E, int k, IterState *__restrict__ st)
{
    __shared__ long long s_sum[4];
    __shared__ int s_cnt[4];
    const size_t n = (size_t)T * k;
    long long sum = 0;
    int cnt = 0;
    for (size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x; a < n; a += (size_t)gridDim.x * blockDim.x) {
        const int e = assign[a];
        if (e >= 0) {
            sum += q[(a / k) * E + e];
            ++cnt;
        }
    }
    for (int off = 32; off >= 1; off >>= 1) {
        sum += __shfl_xor(sum, off);
        cnt += __shfl_xor(cnt, off);
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) {
        s_sum[wv] = sum;
        s_cnt[wv] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        atomicAdd(&st->total, (unsigned long long)(s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3]));
        atomicAdd(&st->flow, s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3]);
    }
}

template <int EPL>
void launch_topk(const int32_t *q, int T, int E, int k, int32_t *choice, hipStream_t s)
{
    const int grid = T < 4 * 2048 ? (T + 3) / 4 : 2048;
    hipLaunchKernelGGL(k_iter_topk<EPL>, dim3(grid), dim3(256), 0, s, q, T, E, k, choice);
}

template <int EPL>
void launch_propose(const int32_t *q, const int32_t *assign, const int *load, int T, int E, int k, int C,
                    int32_t *prop, hipStream_t s)
{
    const int grid = T < 4 * 2048 ? (T + 3) / 4 : 2048;
    hipLaunchKernelGGL(k_iter_propose<EPL>, dim3(grid), dim3(256), 0, s, q, assign, load, T, E, k, C, prop);
}

}  // namespace

int32_t top1_run(const int32_t *q, int T, int E, int32_t *top1, hipStream_t s)
{
    const int epl = (E + 63) / 64;
    if (epl <= 1) launch_topk<1>(q, T, E, 1, top1, s);
    else if (epl <= 2) launch_topk<2>(q, T, E, 1, top1, s);
    else if (epl <= 4) launch_topk<4>(q, T, E, 1, top1, s);
    else if (epl <= 8) launch_topk<8>(q, T, E, 1, top1, s);
    else launch_topk<16>(q, T, E, 1, top1, s);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t assign_total_run(const int32_t *q, const int32_t *assign, int T, int E, int k, void *state16,
                         int64_t *total, int32_t *flow, hipStream_t s)
{
    IterState *st = (IterState *)state16;
    IterState h = {};
    MS_HIP(hipMemcpyAsync(st, &h, sizeof(h), hipMemcpyHostToDevice, s));
    const size_t n = (size_t)T * k;
    int grid = (int)((n + 255) / 256);
    if (grid > 256) grid = 256;
    hipLaunchKernelGGL(k_iter_total, dim3(grid), dim3(256), 0, s, q, assign, T, E, k, st);
    MS_HIP(hipGetLastError());
    MS_HIP(hipMemcpyAsync(&h, st, sizeof(h), hipMemcpyDeviceToHost, s));
    MS_HIP(hipStreamSynchronize(s));
    if (total) *total = (int64_t)h.total;
    if (flow) *flow = h.flow;
    return MAXSCORE_OK;
}

int32_t iter_run(const int32_t *q, int T, int E, int k, int C, int max_rounds, int32_t *assign, int64_t *total,
                 int32_t *flow, int32_t *rounds, char *ws, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    const size_t n = (size_t)T * k;
    int32_t *list = (int32_t *)(ws + L.klist_off);     // slot-major choices, later proposals
    int32_t *pos = list + n;
    int32_t *offsets = (int32_t *)(ws + L.theta_off);
    int *load = (int *)(ws + L.gcount_off);            // two buffers of kMaxE, alternating by round
    IterState *st = (IterState *)(ws + L.state_off);
    int *tiles = (int *)(ws + L.tiles_off);
    const int epl = (E + 63) / 64;
    const int pair_grid = (int)((n + 255) / 256);

    if (epl <= 1) launch_topk<1>(q, T, E, k, list, s);
    else if (epl <= 2) launch_topk<2>(q, T, E, k, list, s);
    else if (epl <= 4) launch_topk<4>(q, T, E, k, list, s);
    else if (epl <= 8) launch_topk<8>(q, T, E, k, list, s);
    else launch_topk<16>(q, T, E, k, list, s);
    int32_t rc = dispatch_core(list, nullptr, n, E, 1, offsets, nullptr, nullptr, pos, tiles, L.n_tiles, s);
    if (rc) return rc;
    hipLaunchKernelGGL(k_iter_keep, dim3(pair_grid), dim3(256), 0, s, list, pos, offsets, T, E, k, C, assign, load, st);

    IterState h = {};
    int r = 0;
    bool open = false;          // the last round still had proposals
    while (r < max_rounds) {
        const int batch = max_rounds - r < 2 ? max_rounds - r : 2;   // two rounds per host check
        for (int b = 0; b < batch; ++b, ++r) {
            const int *cur = load + (r & 1) * kMaxE;
            int *next = load + ((r + 1) & 1) * kMaxE;
            if (epl <= 1) launch_propose<1>(q, assign, cur, T, E, k, C, list, s);
            else if (epl <= 2) launch_propose<2>(q, assign, cur, T, E, k, C, list, s);
            else if (epl <= 4) launch_propose<4>(q, assign, cur, T, E, k, C, list, s);
            else if (epl <= 8) launch_propose<8>(q, assign, cur, T, E, k, C, list, s);
            else launch_propose<16>(q, assign, cur, T, E, k, C, list, s);
            rc = dispatch_core(list, nullptr, n, E, 1, offsets, nullptr, nullptr, pos, tiles, L.n_tiles, s);
            if (rc) return rc;
            hipLaunchKernelGGL(k_iter_accept, dim3(pair_grid), dim3(256), 0, s, list, pos, offsets, cur, next, T, E,
                               k, C, assign, st);
        }
        MS_HIP(hipMemcpyAsync(&h, st, sizeof(h), hipMemcpyDeviceToHost, s));
        MS_HIP(hipStreamSynchronize(s));
        open = h.nprop > 0;
        if (!open) break;
    }
    const int tot_grid = pair_grid < 256 ? pair_grid : 256;
    hipLaunchKernelGGL(k_iter_total, dim3(tot_grid), dim3(256), 0, s, q, assign, T, E, k, st);
    MS_HIP(hipGetLastError());
    MS_HIP(hipMemcpyAsync(&h, st, sizeof(h), hipMemcpyDeviceToHost, s));
    MS_HIP(hipStreamSynchronize(s));
    if (total) *total = (int64_t)h.total;
    if (flow) *flow = h.flow;
    if (rounds) *rounds = h.rounds;
    return open ? MAXSCORE_ERR_NOT_CONVERGED : MAXSCORE_OK;
}

}  // namespace maxscore
