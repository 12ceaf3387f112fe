// Exact assignment when demand exceeds capacity (T*k > E*min(C,T)): maximum flow first, then maximum score.
//
// Eq. 7 prints equalities that cannot all hold in this case; Table 1 gives every arc a capacity, so the problem
// read as a flow problem still has a solution: every expert ends up full, E*C pairs are placed, and among all such
// placements the score is maximal (Section 3.2, Eq. 7-8, Table 1).  A token then ships fewer than k units.
//
// The solver handles it as a problem it already solves.  k padding experts are appended, each with room for every
// token and the same reward PAD for all tokens, PAD so far below every real reward that one more real pair always
// outweighs whatever a rearrangement of the others can lose: an exchange cycle of the expert graph visits each of
// the E + k experts at most once, so it changes the score of real pairs by at most (E + k) * range, and PAD lies
// (E + k + 1) * (range + 1) below the smallest reward.  With the padding every token holds k experts again
// (capacity suffices), the optimum of the padded problem uses as few padding pairs as possible (that is the
// maximum flow), and what it pays for the real pairs is the maximum score at that flow.  A hold on a padding expert
// is an empty slot: the rows come back with the real experts first and -1 after them.
//
// Where the auction starts.  Every real expert ends full and its last token is indifferent between it and a padding
// expert, so its price ends at S * (q - PAD) >= S * (lo - PAD) for some reward q of its own (S the solver's scale
// factor, lo the smallest real reward).  From zero prices the auction would climb that height, E + k + 1 times
// the reward range, in steps of eps, through thousands of rounds; it is started instead with S * (lo - PAD) on
// every real expert and 0 on the padding experts (never full: their price stays 0), at the eps a problem with the
// real reward range starts from.  Net of these prices a real expert is worth S * (q - lo) >= 0 to a token and a
// padding expert 0, and the auction only has to resolve differences inside the real range.  (Starting prices do not
// change the optimum the solver returns, only its rounds.)
#include <vector>

#include "common.h"

namespace maxscore {
namespace {

constexpr int kOsBlocks = 256;

__global__ __launch_bounds__(256) void k_os_minmax(const int32_t *__restrict__ q, size_t n, int *__restrict__ part)
{
    int lo = 0x7fffffff, hi = -0x7fffffff - 1;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const int v = q[i];
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    }
    for (int off = 32; off > 0; off >>= 1) {
        const int a = __shfl_xor(lo, off), b = __shfl_xor(hi, off);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    __shared__ int s_lo[4], s_hi[4];
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

// q2[T, E + k]: the rewards, then k columns of PAD; start[E + k]: the starting prices
__global__ __launch_bounds__(256) void k_os_pad(const int32_t *__restrict__ q, int32_t *__restrict__ q2, int T, int E,
                                                int E2, int pad, int *holes, int64_t *__restrict__ start,
                                                long long start_real)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) holes[0] = 0;
    if (blockIdx.x == 0)
        for (int e = threadIdx.x; e < E2; e += 256) start[e] = e < E ? start_real : 0;
    const size_t n = (size_t)T * E2;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const size_t row = i / E2;
        const int e = (int)(i - row * E2);
        q2[i] = e < E ? q[row * E + e] : pad;
    }
}

// Padding experts become empty slots; the real experts of a row keep their order and come first.  holes[0] counts
// the empty slots of the whole batch.
__global__ __launch_bounds__(256) void k_os_unpad(int32_t *assign, int T, int E, int k, int *holes)
{
    const int row = blockIdx.x * 256 + threadIdx.x;
    int h = 0;
    if (row < T) {
        int32_t *a = assign + (size_t)row * k;
        int w = 0;
        for (int s = 0; s < k; ++s) {
            const int e = a[s];
            if (e >= 0 && e < E) a[w++] = e;
        }
        h = k - w;
        for (; w < k; ++w) a[w] = -1;
    }
    for (int off = 32; off > 0; off >>= 1) h += __shfl_xor(h, off);
    if ((threadIdx.x & 63) == 0 && h) atomicAdd(holes, h);
}

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

size_t oversub_workspace_bytes(int T, int E, int k)
{
    const int E2 = E + k;
    if (E2 > kMaxE) return 0;
    return up256(workspace_layout(T, E2, k).total) + up256(sizeof(int32_t) * (size_t)T * E2) +
           2 * up256(sizeof(int64_t) * E2) + 256;
}

int32_t oversub_run(const int32_t *q, int T, int E, int k, int Ce, const maxscore_opts &o, int32_t *assign,
                    int64_t *prices, int64_t *price_scale, maxscore_stats *stats, char *ws, size_t ws_bytes,
                    hipStream_t s)
{
    const int E2 = E + k;
    if (E2 > kMaxE) return MAXSCORE_ERR_OVERSUBSCRIBED;          // no room for the padding experts
    if (ws_bytes < oversub_workspace_bytes(T, E, k)) return MAXSCORE_ERR_WORKSPACE;
    const size_t solver_bytes = up256(workspace_layout(T, E2, k).total);
    int32_t *q2 = (int32_t *)(ws + solver_bytes);
    int64_t *prices2 = (int64_t *)(ws + solver_bytes + up256(sizeof(int32_t) * (size_t)T * E2));
    int64_t *start = (int64_t *)((char *)prices2 + up256(sizeof(int64_t) * E2));
    int *holes_dev = (int *)((char *)start + up256(sizeof(int64_t) * E2));

    // reward range (the partial results use the head of the region the padded rewards will fill)
    const size_t n = (size_t)T * E;
    int nb = (int)((n + 256 * 16 - 1) / (256 * 16));
    nb = nb < 1 ? 1 : (nb > kOsBlocks ? kOsBlocks : nb);
    int *part = (int *)q2;
    hipLaunchKernelGGL(k_os_minmax, dim3(nb), dim3(256), 0, s, q, n, part);
    int hp[2 * kOsBlocks];
    MS_HIP(hipMemcpyAsync(hp, part, sizeof(int) * 2 * nb, hipMemcpyDeviceToHost, s));
    MS_HIP(hipStreamSynchronize(s));
    long long lo = hp[0], hi = hp[1];
    for (int b = 1; b < nb; ++b) {
        lo = hp[2 * b] < lo ? hp[2 * b] : lo;
        hi = hp[2 * b + 1] > hi ? hp[2 * b + 1] : hi;
    }
    const long long pad = lo - (long long)(E2 + 1) * (hi - lo + 1);
    if (pad < -((long long)1 << 30)) return MAXSCORE_ERR_RANGE;  // the padded rewards must stay 32-bit values
    long long start_real = 0, eps_start = 1;

    {
        const size_t n2 = (size_t)T * E2;
        int grid = (int)((n2 + 256 * 8 - 1) / (256 * 8));
        grid = grid < 1 ? 1 : (grid > 8192 ? 8192 : grid);
        int sb = 0;                      // the solver's scale factor for E2 experts: S = 2^sb > E2
        while ((1 << sb) < E2 + 1) ++sb;
        start_real = (lo - pad) << sb;
        eps_start = ((hi - lo) << sb) >> kEps0Shift;
        hipLaunchKernelGGL(k_os_pad, dim3(grid), dim3(256), 0, s, q, q2, T, E, E2, (int)pad, holes_dev, start,
                           start_real);
    }
    maxscore_opts o2 = o;                // (prices the caller may have given refer to another problem: not used)
    o2.prices_in = start;
    o2.eps_start = eps_start > 1 ? eps_start : 1;
    std::vector<int32_t> caps(E2);
    for (int e = 0; e < E2; ++e) caps[e] = e < E ? Ce : T;
    const int32_t *cap_dev = nullptr;
    long long room = 0;
    int cmax = 1;
    int32_t rc = caps_to_device(caps.data(), T, E2, k, ws, &cap_dev, &room, &cmax, s);
    if (rc) return rc;
    maxscore_stats st2;
    st2 = maxscore_stats();
    rc = solver_run(q2, T, E2, k, cmax, o2, assign, prices2, price_scale, &st2, ws, s, cap_dev, room);
    if (rc != MAXSCORE_OK && rc != MAXSCORE_ERR_NOT_CONVERGED) return rc;
    hipLaunchKernelGGL(k_os_unpad, dim3((T + 255) / 256), dim3(256), 0, s, assign, T, E, k, holes_dev);
    int holes = 0;
    MS_HIP(hipMemcpyAsync(&holes, holes_dev, sizeof(int), hipMemcpyDeviceToHost, s));
    if (prices) MS_HIP(hipMemcpyAsync(prices, prices2, sizeof(int64_t) * E, hipMemcpyDeviceToDevice, s));
    MS_HIP(hipStreamSynchronize(s));
    MS_HIP(hipGetLastError());
    if (stats) {
        *stats = st2;
        // the solver counted the padding pairs (its own holes, after a round cap, count for nothing there)
        const long long placed2 = st2.flow_value;
        const long long pads = placed2 - ((long long)T * k - holes);
        stats->total_score_q = st2.total_score_q - pads * pad;
        stats->flow_value = (int32_t)((long long)T * k - holes);
    }
    return rc;
}

}  // namespace maxscore
