// Other routing operators of Table 2 (Section 3.1) as alternatives to SoftTopk for the affinity scores:
// Sigmoid, SoftKmax, IterTopk and GradTopk.  The table gives the recursions without a base case; y^(0) = 0 is
// used (for GradTopk: g^(1) = x), so that level 1 of every recursion is Softmax(x).  One wavefront per token row; lane l holds experts l, l+64, ...
#include "common.h"

namespace maxscore {
namespace {

__device__ inline float wave_max_f(float v)
{
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

__device__ inline float wave_sum_f(float v)
{
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

template <int EPL>
__global__ __launch_bounds__(256) void k_scores_op(const float *__restrict__ logits, int T, int E, int k, int op,
                                                   float scale, float *__restrict__ scores,
                                                   int32_t *__restrict__ q)
{
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = wave; row < T; row += n_waves) {
        float x[EPL], y[EPL];
        bool in[EPL];
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            in[c] = e < E;
            x[c] = in[c] ? logits[(size_t)row * E + e] : 0.f;
            y[c] = 0.f;
        }
        if (op == MAXSCORE_OP_SIGMOID) {
#pragma unroll
            for (int c = 0; c < EPL; ++c) y[c] = 1.f / (1.f + expf(-x[c]));
        } else if (op == MAXSCORE_OP_SOFTKMAX) {
            for (int m = 0; m < k; ++m) {
                float g[EPL];
                float mx = -INFINITY;
#pragma unroll
                for (int c = 0; c < EPL; ++c) {
                    g[c] = in[c] ? (1.f - y[c]) * x[c] : -INFINITY;
                    mx = fmaxf(mx, g[c]);
                }
                mx = wave_max_f(mx);
                float z = 0.f;
#pragma unroll
                for (int c = 0; c < EPL; ++c) {
                    g[c] = expf(g[c] - mx);
                    z += g[c];
                }
                const float inv = 1.f / wave_sum_f(z);
#pragma unroll
                for (int c = 0; c < EPL; ++c) y[c] += g[c] * inv;
            }
        } else if (op == MAXSCORE_OP_GRADTOPK) {
            // g^(m) = x + log(e^{z^(m-1)} - e^{g^(m-1)}) and y = e^{g - z} with z = logsumexp(g) - log m give
            // y^(m) = m * w e^x / sum_j w_j e^{x_j}, w = 1 - y^(m-1) (w = 1 at level 1); the logarithm has no
            // value for w < 0: the row turns NaN as in the printed form
            float mx = -INFINITY;
#pragma unroll
            for (int c = 0; c < EPL; ++c) mx = fmaxf(mx, in[c] ? x[c] : -INFINITY);
            mx = wave_max_f(mx);
            float ex[EPL];
#pragma unroll
            for (int c = 0; c < EPL; ++c) ex[c] = in[c] ? expf(x[c] - mx) : 0.f;
            for (int m = 1; m <= k; ++m) {
                float term[EPL];
                float z = 0.f;
#pragma unroll
                for (int c = 0; c < EPL; ++c) {
                    const float w = m == 1 ? 1.f : 1.f - y[c];
                    term[c] = !in[c] ? 0.f : (w > 0.f ? w * ex[c] : (w == 0.f ? 0.f : NAN));
                    z += term[c];
                }
                const float scale_m = (float)m / wave_sum_f(z);
#pragma unroll
                for (int c = 0; c < EPL; ++c) y[c] = term[c] * scale_m;
            }
        } else {   // MAXSCORE_OP_ITERTOPK
            float mx = -INFINITY;
#pragma unroll
            for (int c = 0; c < EPL; ++c) mx = fmaxf(mx, in[c] ? x[c] : -INFINITY);
            mx = wave_max_f(mx);
            float ex[EPL];
#pragma unroll
            for (int c = 0; c < EPL; ++c) ex[c] = in[c] ? expf(x[c] - mx) : 0.f;
            for (int m = 0; m < k; ++m) {
                float we[EPL];
                float z = 0.f;
#pragma unroll
                for (int c = 0; c < EPL; ++c) {
                    we[c] = (1.f - y[c]) * ex[c];
                    z += we[c];
                }
                const float inv = 1.f / wave_sum_f(z);
#pragma unroll
                for (int c = 0; c < EPL; ++c) y[c] += we[c] * inv;
            }
        }
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            if (in[c]) {
                if (scores) scores[(size_t)row * E + e] = y[c];
                if (q) q[(size_t)row * E + e] = (int32_t)rintf(y[c] * scale);
            }
        }
    }
}

template <int EPL>
void launch_op(const float *logits, int T, int E, int k, int op, float scale, float *scores, int32_t *q,
               hipStream_t s)
{
    const int grid = T < 4 * 4096 ? (T + 3) / 4 : 4096;
    hipLaunchKernelGGL(k_scores_op<EPL>, dim3(grid), dim3(256), 0, s, logits, T, E, k, op, scale, scores, q);
}

}  // namespace

int32_t scores_op_run(const float *logits, int T, int E, int k, int op, int shift, float *scores, int32_t *q,
                      hipStream_t s)
{
    const float scale = (float)(1 << shift);
    const int epl = (E + 63) / 64;
    if (epl <= 1) launch_op<1>(logits, T, E, k, op, scale, scores, q, s);
    else if (epl <= 2) launch_op<2>(logits, T, E, k, op, scale, scores, q, s);
    else if (epl <= 4) launch_op<4>(logits, T, E, k, op, scale, scores, q, s);
    else if (epl <= 8) launch_op<8>(logits, T, E, k, op, scale, scores, q, s);
    else launch_op<16>(logits, T, E, k, op, scale, scores, q, s);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

}  // namespace maxscore
