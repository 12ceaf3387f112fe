// One token row of a2 + a3 (Eq. 6; softmax of Table 2 row 1), shared by the score kernel and by the projection
// kernel that computes the scores in its epilogue.  A group of G lanes owns the row; in the vector layout lane l
// owns the 4-column pieces l, l+G, l+2G, ... (columns (m >> 2) * 4G + 4l + (m & 3) for its m-th value), in the
// scalar layout the EPL consecutive columns l*EPL .. l*EPL+EPL-1.  Both kernels run the same instructions on the
// same values in the same lanes, so their scores and rewards are bit-equal.
#pragma once

#include "common.h"

namespace maxscore {

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

// x: this lane's logits of the row (columns at or beyond E must hold -3.4e38f); sc, qq: its scores and rewards.
template <int G, int EPL, bool kVec>
__device__ __forceinline__ void softtopk_row(const float (&x)[EPL], int lg, int E, int k, float t, float qscale,
                                             int reading, float (&sc)[EPL], int (&qq)[EPL])
{
    auto colof = [&](int m) { return kVec ? ((m >> 2) * (4 * G) + lg * 4 + (m & 3)) : (lg * EPL + m); };
    float mx = -3.4e38f;
#pragma unroll
    for (int m = 0; m < EPL; ++m) mx = fmaxf(mx, x[m]);
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float ex[EPL];
    float sum = 0.f;
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        // fast exponential (exp2 of the scaled argument): the argument is in [-87, 0], its scaling costs at most
        // |x| * 2^-24 of relative error, 1.5e-6 at x = -16, below which a probability is under 1e-7
        ex[m] = (colof(m) < E) ? __expf(x[m] - mx) : 0.f;
        sum += ex[m];
    }
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    const float inv = 1.0f / sum;

    // the largest entries one by one (equal logits: lower column first), each with the weight of its rank; the
    // entries that are never picked share the weight of the ranks beyond
    const int n_pick = (reading == MAXSCORE_SOFTTOPK_A1 || reading == MAXSCORE_SOFTTOPK_B) ? k : k - 1;
    float wv[EPL];
    float w_run = 0.f;                 // reading C: the weight of the rank being picked
    unsigned taken = 0;
    if (t != 0.f) {
        for (int r = 1; r <= n_pick; ++r) {
            unsigned bo = 0;
            int bm = -1;
#pragma unroll
            for (int m = 0; m < EPL; ++m) {
                const unsigned o = ord_f32(x[m]);
                const bool take = (colof(m) < E) && !((taken >> m) & 1u) && (bm < 0 || o > bo);
                bo = take ? o : bo;
                bm = take ? m : bm;
            }
            unsigned long long best =
                bm >= 0 ? (((unsigned long long)bo << 10) | (unsigned)(1023 - colof(bm))) : 0ull;
#pragma unroll
            for (int off = G / 2; off > 0; off >>= 1) {
                unsigned long long o = shfl_xor_u64(best, off);
                best = o > best ? o : best;
            }
            const int e = 1023 - (int)(best & 1023);
            const bool mine = kVec ? (((e >> 2) & (G - 1)) == lg) : (e / EPL == lg);
            if (mine) {
                const int m = kVec ? ((e / (4 * G)) * 4 + (e & 3)) : (e % EPL);
                const float w = reading == MAXSCORE_SOFTTOPK_B ? 0.f
                              : reading == MAXSCORE_SOFTTOPK_C ? w_run : (float)(r - 1);
#pragma unroll
                for (int mm = 0; mm < EPL; ++mm)
                    if (mm == m) wv[mm] = w;
                taken |= 1u << m;
            }
            if (reading == MAXSCORE_SOFTTOPK_C) {
                // mass outside the r largest, summed over what is left (no cancellation on peaked rows)
                float rest = 0.f;
#pragma unroll
                for (int m = 0; m < EPL; ++m) rest += ((taken >> m) & 1u) ? 0.f : ex[m];
#pragma unroll
                for (int off = G / 2; off > 0; off >>= 1) rest += __shfl_xor(rest, off);
                w_run += rest > 0.f ? 1.0f / (rest * inv) : 0.f;      // (nothing left: the entries beyond are 0 anyway)
            }
        }
    }
    const float w_rest = reading == MAXSCORE_SOFTTOPK_A1 ? (float)k
                       : reading == MAXSCORE_SOFTTOPK_C  ? w_run : (float)(k - 1);
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        const float p = ex[m] * inv;
        const float w = ((taken >> m) & 1u) ? wv[m] : w_rest;
        sc[m] = p * (1.0f + t * w);
        qq[m] = __float2int_rn(sc[m] * qscale);
    }
}

}  // namespace maxscore
