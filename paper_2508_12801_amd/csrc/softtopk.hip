// a2 + a3: SoftTopk scores and integer rewards per token row (Eq. 6; softmax of Table 2 row 1),
// and a5: gates gathered at the assigned pairs (Eq. 2).
//
// Eq. 6 is taken level by level: level 1 is Softmax(a); level m = 2..k adds t*Softmax(a)_i to the
// entries that are not among the m-1 largest of a.  An entry of descending rank r (1-based, equal
// logits ranked by lower index) therefore ends as p_i * (1 + t*(min(r,k) - 1)).
#include "common.h"

namespace maxscore {
namespace {

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int off)
{
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return ((unsigned long long)hi << 32) | lo;
}

// order-preserving map float -> uint32 (finite inputs)
__device__ __forceinline__ unsigned ord_f32(float x)
{
    unsigned u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// A group of G lanes owns one row; lane l owns columns l, l+G, ... (EPL per lane).
template <int G, int EPL>
__global__ __launch_bounds__(256) void k_softtopk(const float *__restrict__ logits, int T, int E, int k, float t,
                                                  float qscale, float *__restrict__ scores,
                                                  int32_t *__restrict__ q)
{
    const int tid = threadIdx.x, lane = tid & 63, lg = lane & (G - 1);
    const int grp = tid / G, ngrp = 256 / G;
    for (int row = blockIdx.x * ngrp + grp; row < T; row += gridDim.x * ngrp) {
        const float *lr = logits + (size_t)row * E;
        float x[EPL];
        float mx = -3.4e38f;
#pragma unroll
        for (int m = 0; m < EPL; ++m) {
            int e = lg + m * G;
            x[m] = e < E ? lr[e] : -3.4e38f;
            mx = fmaxf(mx, x[m]);
        }
#pragma unroll
        for (int off = G / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        float ex[EPL];
        float sum = 0.f;
#pragma unroll
        for (int m = 0; m < EPL; ++m) {
            int e = lg + m * G;
            ex[m] = e < E ? expf(x[m] - mx) : 0.f;
            sum += ex[m];
        }
#pragma unroll
        for (int off = G / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
        const float inv = 1.0f / sum;

        // ranks 1..k-1 by repeated arg-max; everything else has min(rank, k) = k
        int rk[EPL];
#pragma unroll
        for (int m = 0; m < EPL; ++m) rk[m] = k;
        unsigned taken = 0;
        if (t != 0.f) {
            for (int r = 1; r < k; ++r) {
                unsigned long long best = 0;
#pragma unroll
                for (int m = 0; m < EPL; ++m) {
                    int e = lg + m * G;
                    if (e < E && !((taken >> m) & 1u)) {
                        unsigned long long pk = ((unsigned long long)ord_f32(x[m]) << 10) | (unsigned)(1023 - e);
                        best = pk > best ? pk : best;
                    }
                }
#pragma unroll
                for (int off = G / 2; off > 0; off >>= 1) {
                    unsigned long long o = shfl_xor_u64(best, off);
                    best = o > best ? o : best;
                }
                int e = 1023 - (int)(best & 1023);
                if ((e & (G - 1)) == lg) {
                    int m = e / G;
#pragma unroll
                    for (int mm = 0; mm < EPL; ++mm)
                        if (mm == m) rk[mm] = r;
                    taken |= 1u << m;
                }
            }
        }
#pragma unroll
        for (int m = 0; m < EPL; ++m) {
            int e = lg + m * G;
            if (e < E) {
                float p = ex[m] * inv;
                float sc = p * (1.0f + t * (float)(rk[m] - 1));
                if (scores) scores[(size_t)row * E + e] = sc;
                if (q) q[(size_t)row * E + e] = __float2int_rn(sc * qscale);
            }
        }
    }
}

__global__ __launch_bounds__(256) void k_gates(const float *__restrict__ scores, const int32_t *__restrict__ assign,
                                               size_t n, int E, int k, float *__restrict__ gates)
{
    for (size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x; a < n; a += (size_t)gridDim.x * blockDim.x) {
        int e = assign[a];
        gates[a] = e >= 0 ? scores[(a / k) * E + e] : 0.f;
    }
}

}  // namespace

int32_t softtopk_run(const float *logits, int T, int E, int k, float t, int shift, float *scores, int32_t *q,
                     hipStream_t s)
{
    int G = 8, EPL = 1;
    while (G < 64 && G < E) G *= 2;
    while (G * EPL < E) EPL *= 2;
    const int ngrp = 256 / G;
    int grid = (T + ngrp - 1) / ngrp;
    if (grid > 8192) grid = 8192;
    const float qscale = (float)(1 << shift);
#define MS_ST(GG, PP) \
    hipLaunchKernelGGL((k_softtopk<GG, PP>), dim3(grid), dim3(256), 0, s, logits, T, E, k, t, qscale, scores, q)
    if (G == 8) MS_ST(8, 1);
    else if (G == 16) MS_ST(16, 1);
    else if (G == 32) MS_ST(32, 1);
    else if (EPL == 1) MS_ST(64, 1);
    else if (EPL == 2) MS_ST(64, 2);
    else if (EPL == 4) MS_ST(64, 4);
    else if (EPL == 8) MS_ST(64, 8);
    else MS_ST(64, 16);
#undef MS_ST
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t gates_run(const float *scores, const int32_t *assign, int T, int E, int k, float *gates, hipStream_t s)
{
    size_t n = (size_t)T * k;
    int grid = (int)((n + 255) / 256);
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(k_gates, dim3(grid), dim3(256), 0, s, scores, assign, n, E, k, gates);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

}  // namespace maxscore
