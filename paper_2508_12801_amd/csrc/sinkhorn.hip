// Algorithm 1 (Section 3.2) with its last step done the paper's way: Sinkhorn on the residual problem.
// The paper names the algorithm only; regulariser, iteration count and rounding are this library's reading:
//   top-1 per token (ties to the lower expert id), residual capacities caps_j = max(0, C - load_j), residual
//   affinities a' = scores with the top-1 entry set to 0;
//   K_ij = exp((a'_ij - max_j a'_ij) / tau) on experts with caps_j > 0, else 0 (the row shift is absorbed by u);
//   column targets m_j = caps_j * T / sum(caps);  v = 1;  n_iter times: u_i = 1 / sum_j K_ij v_j,
//   v_j = m_j / sum_i K_ij u_i;  plan_ij = u_i K_ij v_j;  second expert = arg-max_j plan_ij (ties to the lower
//   id; -1 when the row is all zero).
// One wavefront per token row, lane l holds experts l, l+64, ...; K is recomputed from the scores in every pass
// (it is cheaper than storing it), column sums go through per-workgroup partial results added in a fixed order.
#include "common.h"

namespace maxscore {
namespace {

constexpr int kSkBlocksMax = 1024;

__device__ inline float sk_wave_max(float v)
{
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

__device__ inline float sk_wave_sum(float v)
{
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// first lane-major position holding the row maximum: expert with the largest value, ties to the lower id
template <int EPL>
__device__ inline int sk_argmax(const float (&x)[EPL], const bool (&in)[EPL], float mx)
{
    int e = -1;
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
        const unsigned long long b = __ballot(in[c] && x[c] == mx);
        if (e < 0 && b) e = 64 * c + __ffsll((long long)b) - 1;
    }
    return e;
}

template <int EPL>
__global__ __launch_bounds__(256) void k_sk_top1(const float *__restrict__ scores, int T, int E,
                                                 int32_t *__restrict__ top1)
{
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = wave; row < T; row += n_waves) {
        float x[EPL];
        bool in[EPL];
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            in[c] = e < E;
            x[c] = in[c] ? scores[(size_t)row * E + e] : -INFINITY;
            mx = fmaxf(mx, x[c]);
        }
        mx = sk_wave_max(mx);
        const int e = sk_argmax<EPL>(x, in, mx);
        if (lane == 0) top1[row] = e;
    }
}

// caps, column targets and the starting v from the top-1 counts (one workgroup)
__global__ __launch_bounds__(1024) void k_sk_init(const int32_t *__restrict__ offsets, int T, int E, int C,
                                                  int32_t *__restrict__ caps, float *__restrict__ targets,
                                                  float *__restrict__ v)
{
    __shared__ long long s_w[16];
    const int j = threadIdx.x;
    int cap = 0;
    if (j < E) {
        const int left = C - (offsets[j + 1] - offsets[j]);
        cap = left > 0 ? left : 0;
    }
    long long sum = cap;
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if ((j & 63) == 0) s_w[j >> 6] = sum;
    __syncthreads();
    long long tot = 0;
    for (int w = 0; w < 16; ++w) tot += s_w[w];
    if (j < E) {
        caps[j] = cap;
        targets[j] = tot > 0 ? (float)((double)cap * (double)T / (double)tot) : 0.f;
        v[j] = 1.f;
    }
}

// u_i = 1 / sum_j K_ij v_j for the rows of this workgroup, and the workgroup's partial sums of K_ij u_i per
// column.  LAST: also the plan's arg-max (and the plan itself) with the v of the last column update.
template <int EPL>
__global__ __launch_bounds__(256) void k_sk_row(const float *__restrict__ scores, const int32_t *__restrict__ top1,
                                                const float *__restrict__ targets, const float *__restrict__ v,
                                                int T, int E, float inv_tau, float *__restrict__ u,
                                                float *__restrict__ part)
{
    extern __shared__ float s_sk[];        // [4][E] column partials of the four wavefronts
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    float vv[EPL], acc[EPL];
    bool in[EPL];
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
        const int e = lane + 64 * c;
        in[c] = e < E;
        vv[c] = (in[c] && targets[e] > 0.f) ? v[e] : 0.f;      // closed experts: K = 0
        acc[c] = 0.f;
    }
    for (int row = wave; row < T; row += n_waves) {
        const int t1 = top1[row];
        float x[EPL];
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            x[c] = in[c] ? (e == t1 ? 0.f : scores[(size_t)row * E + e]) : -INFINITY;
            mx = fmaxf(mx, x[c]);
        }
        mx = sk_wave_max(mx);
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            x[c] = (in[c] && targets[lane + 64 * c] > 0.f) ? expf((x[c] - mx) * inv_tau) : 0.f;   // K_ij
            s += x[c] * vv[c];
        }
        s = sk_wave_sum(s);
        const float ui = 1.f / s;
        if (lane == 0) u[row] = ui;
#pragma unroll
        for (int c = 0; c < EPL; ++c) acc[c] += x[c] * ui;
    }
#pragma unroll
    for (int c = 0; c < EPL; ++c)
        if (in[c]) s_sk[wv * E + lane + 64 * c] = acc[c];
    __syncthreads();
    for (int j = threadIdx.x; j < E; j += 256)
        part[(size_t)blockIdx.x * E + j] = (s_sk[j] + s_sk[E + j]) + (s_sk[2 * E + j] + s_sk[3 * E + j]);
}

// v_j = targets_j / sum over workgroups of part[b][j] (one workgroup; partials added in a fixed order)
__global__ __launch_bounds__(1024) void k_sk_col(const float *__restrict__ part, int n_blocks,
                                                 const float *__restrict__ targets, int E, int epad,
                                                 float *__restrict__ v)
{
    __shared__ double s_red[1024];
    const int tid = threadIdx.x, groups = 1024 / epad;
    {
        const int j = tid % epad, g = tid / epad;
        double sum = 0.0;
        if (j < E) {
#pragma unroll 8
            for (int b = g; b < n_blocks; b += groups) sum += (double)part[(size_t)b * E + j];
        }
        s_red[g * epad + j] = sum;
    }
    __syncthreads();
    if (tid < E) {
        double sum = 0.0;
        for (int g = 0; g < groups; ++g) sum += s_red[g * epad + tid];
        const float m = targets[tid];
        v[tid] = m > 0.f ? (float)((double)m / (sum > 1e-300 ? sum : 1e-300)) : 0.f;
    }
}

template <int EPL>
__global__ __launch_bounds__(256) void k_sk_round(const float *__restrict__ scores, const int32_t *__restrict__ top1,
                                                  const float *__restrict__ targets, const float *__restrict__ v,
                                                  const float *__restrict__ u, int use_u, int T, int E,
                                                  float inv_tau, int32_t *__restrict__ assign,
                                                  float *__restrict__ plan)
{
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    float vv[EPL];
    bool in[EPL];
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
        const int e = lane + 64 * c;
        in[c] = e < E;
        vv[c] = (in[c] && targets[e] > 0.f) ? v[e] : 0.f;
    }
    for (int row = wave; row < T; row += n_waves) {
        const int t1 = top1[row];
        const float ui = use_u ? u[row] : 1.f;
        float x[EPL];
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            x[c] = in[c] ? (e == t1 ? 0.f : scores[(size_t)row * E + e]) : -INFINITY;
            mx = fmaxf(mx, x[c]);
        }
        mx = sk_wave_max(mx);
        float pm = -INFINITY;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const float kij = (in[c] && targets[lane + 64 * c] > 0.f) ? expf((x[c] - mx) * inv_tau) : 0.f;
            x[c] = in[c] ? ui * kij * vv[c] : -INFINITY;
            if (plan && in[c]) plan[(size_t)row * E + lane + 64 * c] = x[c];
            pm = fmaxf(pm, x[c]);          // fmaxf ignores a NaN operand
        }
        pm = sk_wave_max(pm);
        int second = -1;
        if (pm > 0.f) second = sk_argmax<EPL>(x, in, pm);
        if (lane == 0) {
            assign[2 * (size_t)row] = t1;
            assign[2 * (size_t)row + 1] = second;
        }
    }
}

template <int EPL>
int32_t run_epl(const float *scores, int T, int E, int C, float tau, int n_iter, int32_t *assign, float *plan,
                int32_t *caps_host, char *ws, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, 1);
    int32_t *top1 = (int32_t *)(ws + L.aux_off), *pos = top1 + T;
    int32_t *offsets = (int32_t *)(ws + L.theta_off);
    float *targets = (float *)(ws + L.gcount_off), *v = targets + kMaxE;
    int32_t *caps = (int32_t *)(ws + L.cap_off);
    float *u = (float *)(ws + L.klist_off);
    float *part = (float *)(ws + L.wcnt_off);
    int grid = T < 4 * kSkBlocksMax ? (T + 3) / 4 : kSkBlocksMax;
    if (grid > L.max_wg) grid = L.max_wg;
    const float inv_tau = 1.f / tau;
    int epad = 1;
    while (epad < E) epad <<= 1;

    hipLaunchKernelGGL(k_sk_top1<EPL>, dim3(grid), dim3(256), 0, s, scores, T, E, top1);
    int32_t rc = dispatch_core(top1, nullptr, (size_t)T, E, 1, offsets, nullptr, nullptr, pos,
                               (int *)(ws + L.tiles_off), L.n_tiles, s);
    if (rc) return rc;
    hipLaunchKernelGGL(k_sk_init, dim3(1), dim3(1024), 0, s, offsets, T, E, C, caps, targets, v);
    for (int it = 0; it < n_iter; ++it) {
        hipLaunchKernelGGL(k_sk_row<EPL>, dim3(grid), dim3(256), (size_t)4 * E * sizeof(float), s, scores, top1,
                           targets, v, T, E, inv_tau, u, part);
        hipLaunchKernelGGL(k_sk_col, dim3(1), dim3(1024), 0, s, part, grid, targets, E, epad, v);
    }
    hipLaunchKernelGGL(k_sk_round<EPL>, dim3(grid), dim3(256), 0, s, scores, top1, targets, v, u, n_iter > 0 ? 1 : 0,
                       T, E, inv_tau, assign, plan);
    MS_HIP(hipGetLastError());
    if (caps_host) {
        MS_HIP(hipMemcpyAsync(caps_host, caps, sizeof(int32_t) * E, hipMemcpyDeviceToHost, s));
        MS_HIP(hipStreamSynchronize(s));
    }
    return MAXSCORE_OK;
}

}  // namespace

int32_t sinkhorn_run(const float *scores, int T, int E, int C, float tau, int n_iter, int32_t *assign, float *plan,
                     int32_t *caps_host, char *ws, hipStream_t s)
{
    const int epl = (E + 63) / 64;
    if (epl <= 1) return run_epl<1>(scores, T, E, C, tau, n_iter, assign, plan, caps_host, ws, s);
    if (epl <= 2) return run_epl<2>(scores, T, E, C, tau, n_iter, assign, plan, caps_host, ws, s);
    if (epl <= 4) return run_epl<4>(scores, T, E, C, tau, n_iter, assign, plan, caps_host, ws, s);
    if (epl <= 8) return run_epl<8>(scores, T, E, C, tau, n_iter, assign, plan, caps_host, ws, s);
    return run_epl<16>(scores, T, E, C, tau, n_iter, assign, plan, caps_host, ws, s);
}

}  // namespace maxscore
