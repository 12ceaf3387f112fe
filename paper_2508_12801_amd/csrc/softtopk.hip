// a2 + a3: SoftTopk scores and integer rewards per token row (Eq. 6; softmax of Table 2 row 1),
// and a5: gates gathered at the assigned pairs (Eq. 2).
//
// Eq. 6 is taken level by level: level 1 is Softmax(a); level m = 2..k adds t*Softmax(a)_i to the
// entries that are not among the m-1 largest of a.  An entry of descending rank r (1-based, equal
// logits ranked by lower index) therefore ends as p_i * (1 + t*(min(r,k) - 1)).
//
// Eq. 6 prints no base case and an SE term that does not depend on the level, so other readings exist; they are
// kept behind an argument (MAXSCORE_SOFTTOPK_*).  All of them end as p_i * (1 + t * w) with a weight w that
// depends on the rank r of the entry alone:
//   A   (above)                                   w = min(r, k) - 1
//   A1  level 0 is Softmax, level m = 1..k masks the m largest:      w = min(r - 1, k)
//   B   the printed mask (the k largest) at every level 2..k:        w = 0 for r <= k, k - 1 otherwise
//   C   A with SE renormalised over the entries it is added to:      w = sum over m = 2..min(r, k) of
//                                                                        1 / (mass of p outside the m-1 largest)
#include "common.h"
#include "softtopk_row.h"

namespace maxscore {
namespace {

// A group of G lanes owns one row.  Vector path (E == G*EPL): lane l owns the 4-column pieces l, l+G, l+2G, ...
// of the row, so each 16-byte load instruction of a wavefront covers whole 128-byte lines of 64/G consecutive
// rows.  Scalar path: lane l owns the EPL consecutive columns l*EPL .. l*EPL+EPL-1.
template <int G, int EPL, bool VEC>
__global__ __launch_bounds__(256) void k_softtopk(const float *__restrict__ logits, int T, int E, int k, float t,
                                                  float qscale, float *__restrict__ scores,
                                                  int32_t *__restrict__ q, int reading)
{
    const int tid = threadIdx.x, lane = tid & 63, lg = lane & (G - 1);
    const int grp = tid / G, ngrp = 256 / G;
    constexpr bool kVec = VEC && EPL >= 4;
    auto colof = [&](int m) { return kVec ? ((m >> 2) * (4 * G) + lg * 4 + (m & 3)) : (lg * EPL + m); };
    for (int row = blockIdx.x * ngrp + grp; row < T; row += gridDim.x * ngrp) {
        const float *lr = logits + (size_t)row * E + lg * EPL;
        float x[EPL];
        if (kVec) {
#pragma unroll
            for (int m = 0; m < EPL; m += 4) {
                float4 v4 = *(const float4 *)(logits + (size_t)row * E + colof(m));
                x[m] = v4.x; x[m + 1] = v4.y; x[m + 2] = v4.z; x[m + 3] = v4.w;
            }
        } else {
#pragma unroll
            for (int m = 0; m < EPL; ++m) x[m] = (lg * EPL + m < E) ? lr[m] : -3.4e38f;
        }
        float sc[EPL];
        int qq[EPL];
        softtopk_row<G, EPL, kVec>(x, lg, E, k, t, qscale, reading, sc, qq);
        const size_t o0 = (size_t)row * E + lg * EPL;
        if (kVec) {
#pragma unroll
            for (int m = 0; m < EPL; m += 4) {
                const size_t o = (size_t)row * E + colof(m);
                if (scores) *(float4 *)(scores + o) = make_float4(sc[m], sc[m + 1], sc[m + 2], sc[m + 3]);
                if (q) *(int4 *)(q + o) = make_int4(qq[m], qq[m + 1], qq[m + 2], qq[m + 3]);
            }
        } else {
#pragma unroll
            for (int m = 0; m < EPL; ++m) {
                if (lg * EPL + m < E) {
                    if (scores) scores[o0 + m] = sc[m];
                    if (q) q[o0 + m] = qq[m];
                }
            }
        }
    }
}

// a3 alone: q = round-half-even(score * 2^shift) for scores that were computed elsewhere
__global__ __launch_bounds__(256) void k_quantise(const float *__restrict__ scores, size_t n, float qscale,
                                                  int32_t *__restrict__ q)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (((((uintptr_t)scores) | ((uintptr_t)q)) & 15) == 0) {
        const size_t n4 = n / 4;
        for (; i < n4; i += stride) {
            const float4 v = ((const float4 *)scores)[i];
            ((int4 *)q)[i] = make_int4(__float2int_rn(v.x * qscale), __float2int_rn(v.y * qscale),
                                       __float2int_rn(v.z * qscale), __float2int_rn(v.w * qscale));
        }
        i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // the last n % 4 values
    }
    for (; i < n; i += stride) q[i] = __float2int_rn(scores[i] * qscale);
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
                     hipStream_t s, int reading)
{
    int G = 8, EPL = 1;
    while (G * 16 < E) G *= 2;
    while (G * EPL < E) EPL *= 2;
    const int ngrp = 256 / G;
    int grid = (T + ngrp - 1) / ngrp;
    if (grid > 4096) grid = 4096;
    const float qscale = (float)(1 << shift);
    const bool vec = (E == G * EPL) && EPL >= 4 &&
                     ((((uintptr_t)logits) | ((uintptr_t)scores) | ((uintptr_t)q)) % 16 == 0);
#define MS_ST2(GG, PP)                                                                                              \
    do {                                                                                                            \
        if (vec)                                                                                                    \
            hipLaunchKernelGGL((k_softtopk<GG, PP, true>), dim3(grid), dim3(256), 0, s, logits, T, E, k, t, qscale, \
                               scores, q, reading);                                                                 \
        else                                                                                                        \
            hipLaunchKernelGGL((k_softtopk<GG, PP, false>), dim3(grid), dim3(256), 0, s, logits, T, E, k, t,        \
                               qscale, scores, q, reading);                                                         \
    } while (0)
#define MS_ST(GG)                    \
    do {                             \
        if (EPL == 1) MS_ST2(GG, 1); \
        else if (EPL == 2) MS_ST2(GG, 2); \
        else if (EPL == 4) MS_ST2(GG, 4); \
        else if (EPL == 8) MS_ST2(GG, 8); \
        else MS_ST2(GG, 16);         \
    } while (0)
    if (G == 8) MS_ST(8);
    else if (G == 16) MS_ST(16);
    else if (G == 32) MS_ST(32);
    else MS_ST(64);
#undef MS_ST
#undef MS_ST2
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t quantise_run(const float *scores, int T, int E, int shift, int32_t *q, hipStream_t s)
{
    const size_t n = (size_t)T * E;
    int grid = (int)((n / 4 + 255) / 256);
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(k_quantise, dim3(grid), dim3(256), 0, s, scores, n, (float)(1 << shift), q);
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
