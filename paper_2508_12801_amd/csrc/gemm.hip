// a1: router projection  logits = x . W_g (+ bias)   (Eq. 2, Algorithm 1 step 2).
//
// bf16 inputs run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  The output
// is only E <= 128 columns wide per workgroup, so the kernel is bound by streaming x from HBM:
// each workgroup owns 128 token rows, walks d in steps of 64, stages the x tile and the transposed
// W tile in LDS and prefetches the next tiles into registers while the matrix cores work.  The fast
// kernel (k_gemm_bf16_wtc) reads x with whole-line loads and restores the operand layout through LDS.
// fp32 inputs (the tiny configuration) use a plain FMA kernel.
#include "common.h"
#include "softtopk_row.h"

namespace maxscore {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int BM = 128, BK = 64, LDP = BK + 8;   // LDS row pitch in bf16 elements (pad 16 B)

// 16-byte load of 8 bf16 starting at element (r, c) of a row-major [R, Ccols] matrix, zero outside.
template <bool ALIGNED>
__device__ __forceinline__ u32x4 load8(const unsigned short *__restrict__ p, int r, int c, int R, int Ccols)
{
    u32x4 out = {0u, 0u, 0u, 0u};
    if (r >= R || c >= Ccols) return out;
    const unsigned short *src = p + (size_t)r * Ccols + c;
    if (ALIGNED && c + 8 <= Ccols) {
        out = *(const u32x4 *)src;
    } else {
        unsigned short tmp[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) tmp[i] = (c + i < Ccols) ? src[i] : (unsigned short)0;
        out.x = tmp[0] | ((unsigned)tmp[1] << 16);
        out.y = tmp[2] | ((unsigned)tmp[3] << 16);
        out.z = tmp[4] | ((unsigned)tmp[5] << 16);
        out.w = tmp[6] | ((unsigned)tmp[7] << 16);
    }
    return out;
}

// NT = number of 32-column output tiles per workgroup (BN = 32*NT <= 128).
template <int NT, bool ALIGNED>
__global__ __launch_bounds__(256) void k_gemm_bf16(const unsigned short *__restrict__ x,
                                                   const unsigned short *__restrict__ W,
                                                   const float *__restrict__ bias, int T, int d, int E,
                                                   float *__restrict__ out)
{
    constexpr int BN = 32 * NT;
    __shared__ __attribute__((aligned(16))) unsigned short sA[BM * LDP];
    __shared__ __attribute__((aligned(16))) unsigned short sB[BN * LDP];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int row0 = blockIdx.x * BM, col0 = blockIdx.y * 128;

    // global -> register staging: A tile 128 x 64 (4 x 16 B per thread), B tile 64 x BN
    const int a_r = tid >> 3, a_c = (tid & 7) * 8;              // + 32 rows per pass
    constexpr int B_VEC_PER_ROW = BN / 8;                        // 16-byte vectors per k-row
    constexpr int B_VECS = BK * B_VEC_PER_ROW;                   // per tile
    constexpr int B_PER_THREAD = (B_VECS + 255) / 256;
    u32x4 ra[4], rb[B_PER_THREAD];

    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) ra[p] = load8<ALIGNED>(x, row0 + a_r + 32 * p, k0 + a_c, T, d);
#pragma unroll
        for (int p = 0; p < B_PER_THREAD; ++p) {
            int v = tid + 256 * p;
            int kr = v / B_VEC_PER_ROW, nc = (v % B_VEC_PER_ROW) * 8;
            rb[p] = (v < B_VECS) ? load8<ALIGNED>(W, k0 + kr, col0 + nc, d, E) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < 4; ++p) *(u32x4 *)&sA[(a_r + 32 * p) * LDP + a_c] = ra[p];
#pragma unroll
        for (int p = 0; p < B_PER_THREAD; ++p) {
            int v = tid + 256 * p;
            if (v < B_VECS) {
                int kr = v / B_VEC_PER_ROW, nc = (v % B_VEC_PER_ROW) * 8;
                unsigned w4[4] = {rb[p].x, rb[p].y, rb[p].z, rb[p].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {      // transpose: sB[n][k]
                    sB[(nc + 2 * i) * LDP + kr] = (unsigned short)(w4[i] & 0xffffu);
                    sB[(nc + 2 * i + 1) * LDP + kr] = (unsigned short)(w4[i] >> 16);
                }
            }
        }
    };

    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;

    fetch(0);
    for (int k0 = 0; k0 < d; k0 += BK) {
        __syncthreads();            // previous tile fully consumed
        stash();
        __syncthreads();
        if (k0 + BK < d) fetch(k0 + BK);
        const int ar = wave * 32 + (lane & 31), kq = 8 * (lane >> 5);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 a = *(const bf16x8 *)&sA[ar * LDP + kk + kq];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                bf16x8 b = *(const bf16x8 *)&sB[(nt * 32 + (lane & 31)) * LDP + kk + kq];
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[nt], 0, 0, 0);
            }
        }
    }
    // epilogue: acc[nt][4*j + i] is row 8*j + 4*(lane/32) + i, column lane%32 of the 32 x 32 tile
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int col = col0 + nt * 32 + (lane & 31);
        if (col >= E) continue;
        const float bv = bias ? bias[col] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int row = row0 + wave * 32 + 8 * j + 4 * (lane >> 5) + i;
                if (row < T) out[(size_t)row * E + col] = acc[nt][4 * j + i] + bv;
            }
    }
}

// Transposed copy of the router weight: wt[E, d] <- W[d, E] (bf16 patterns), so that both MFMA
// operands are contiguous along the reduction index.
__global__ __launch_bounds__(256) void k_transpose_w(const unsigned short *__restrict__ W,
                                                     unsigned short *__restrict__ wt, int d, int E)
{
    __shared__ unsigned short tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const int k0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    for (int r = ty; r < 32; r += 8) {
        const int kk = k0 + r, n = n0 + tx;
        tile[r][tx] = (kk < d && n < E) ? W[(size_t)kk * E + n] : (unsigned short)0;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r, kk = k0 + tx;
        if (n < E && kk < d) wt[(size_t)n * d + kk] = tile[tx][r];
    }
}

// Main bf16 kernel (d % 8 == 0, 16-byte aligned x and wt).  Workgroup = 4 wavefronts = 128 token rows
// x (32*NT) experts; wavefront w owns rows 32w..32w+31.  Per 64-wide slab of d: the A fragments come
// straight from global memory into registers (each lane reads 16 bytes per MFMA step: row l%32,
// columns 8*(l/32).. of the step), the transposed-W slab goes through a double-buffered LDS tile shared
// by the four wavefronts.  The next slab of both is requested before the MFMAs of the current one.
template <int NT>
__global__ __launch_bounds__(256) void k_gemm_bf16_wt(const unsigned short *__restrict__ x,
                                                      const unsigned short *__restrict__ wt,
                                                      const float *__restrict__ bias, int T, int d, int E,
                                                      float *__restrict__ out)
{
    constexpr int BN = 32 * NT;
    __shared__ __attribute__((aligned(16))) unsigned short sB[2][BN * LDP];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int row0 = blockIdx.x * BM, col0 = blockIdx.y * 128;
    const int arow = row0 + wave * 32 + (lane & 31), kq = 8 * (lane >> 5);
    const bool arow_ok = arow < T;
    const unsigned short *xrow = x + (size_t)(arow_ok ? arow : 0) * d;

    // B staging: BN rows x 64 columns = BN*8 16-byte vectors, B_PER per thread
    constexpr int B_VECS = BN * 8;
    constexpr int B_PER = (B_VECS + 255) / 256;
    // Two slabs of A are in flight per wavefront (x is the stream that has to come from HBM: with one
    // slab ahead the bytes in flight bound the kernel well below the memory rate); the transposed-W slab
    // comes from L2 and stays one ahead.
    u32x4 ra[2][4], rb[B_PER];
    auto fetch_a = [&](int k0, u32x4(&dst)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int kk = k0 + 16 * j + kq;
            dst[j] = (arow_ok && kk < d) ? *(const u32x4 *)(xrow + kk) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto fetch_b = [&](int k0) {
#pragma unroll
        for (int p = 0; p < B_PER; ++p) {
            const int v = tid + 256 * p;
            const int n = v >> 3, kk = k0 + (v & 7) * 8;
            rb[p] = (v < B_VECS && col0 + n < E && kk < d) ? *(const u32x4 *)(wt + (size_t)(col0 + n) * d + kk)
                                                           : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto stash_b = [&](int buf) {
#pragma unroll
        for (int p = 0; p < B_PER; ++p) {
            const int v = tid + 256 * p;
            if (v < B_VECS) *(u32x4 *)&sB[buf][(v >> 3) * LDP + (v & 7) * 8] = rb[p];
        }
    };
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;

    fetch_a(0, ra[0]);
    fetch_b(0);
    fetch_a(BK, ra[1]);
    stash_b(0);
    int buf = 0;
    auto step = [&](int k0, u32x4(&cur)[4]) {
        u32x4 a_cur[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) a_cur[j] = cur[j];
        __syncthreads();                         // sB[buf] is complete; sB[buf^1] is free again
        const bool more = k0 + BK < d;
        if (more) fetch_b(k0 + BK);
        if (k0 + 2 * BK < d) fetch_a(k0 + 2 * BK, cur);      // this register set is free again
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bf16x8 a = __builtin_bit_cast(bf16x8, a_cur[j]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                bf16x8 b = *(const bf16x8 *)&sB[buf][(nt * 32 + (lane & 31)) * LDP + 16 * j + kq];
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[nt], 0, 0, 0);
            }
        }
        if (more) stash_b(buf ^ 1);
        buf ^= 1;
    };
    for (int k0 = 0; k0 < d; k0 += 2 * BK) {
        step(k0, ra[0]);
        if (k0 + BK < d) step(k0 + BK, ra[1]);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int col = col0 + nt * 32 + (lane & 31);
        if (col >= E) continue;
        const float bv = bias ? bias[col] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int row = row0 + wave * 32 + 8 * j + 4 * (lane >> 5) + i;
                if (row < T) out[(size_t)row * E + col] = acc[nt][4 * j + i] + bv;
            }
    }
}

// Same tiling, but x reaches the matrix cores through a wavefront-private LDS tile: every global load
// instruction then reads whole 128-byte lines (8 rows x 128 B, 8 lanes per row) instead of 32 rows x 32 B in the
// MFMA operand layout, which is what the memory pipeline prefers; the operand layout is restored by the LDS
// read.  Needs d to be a multiple of 64.
//
// FUSE: the workgroup holds whole rows (E = 32 * NT columns, one workgroup column), so the SoftTopk scores and the
// integer rewards of Eq. 6 are computed here, from the accumulators, instead of writing the logits and reading
// them back in a second kernel: every wavefront passes its 32 rows through LDS, 16 at a time, into the layout of
// the score kernel (8 lanes per row, 16-byte pieces) and runs that kernel's row routine on them.  The logits are
// written only if the caller wants them.
template <int NT, int RB, int NS, bool FUSE>
__global__ __launch_bounds__(256) void k_gemm_bf16_wtc(const unsigned short *__restrict__ x,
                                                       const unsigned short *__restrict__ wt,
                                                       const float *__restrict__ bias, int T, int d, int E,
                                                       float *__restrict__ out, float *__restrict__ scores,
                                                       int32_t *__restrict__ q, int k, float t, float qscale)
{
    constexpr int BN = 32 * NT;
    constexpr int RW = 32 * RB;                  // rows per wavefront
    constexpr int NL = 4 * RB;                   // global loads per lane and slab
    __shared__ __attribute__((aligned(16))) unsigned short sB[2][BN * LDP];
    __shared__ __attribute__((aligned(16))) unsigned short sA[4][RW * LDP];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int row0 = blockIdx.x * (4 * RW), col0 = blockIdx.y * 128;
    const int kq = 8 * (lane >> 5);
    const int lr = lane >> 3, lc = (lane & 7) * 8;          // loader: row inside a group of 8, column of the slab
    const unsigned short *xp[NL];
    bool ok[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int r = row0 + wave * RW + 8 * i + lr;
        ok[i] = r < T;
        xp[i] = x + (size_t)(ok[i] ? r : 0) * d + lc;
    }
    constexpr int B_VECS = BN * 8;
    constexpr int B_PER = (B_VECS + 255) / 256;
    u32x4 ra[NS][NL], rb[B_PER];          // NS slabs of x in flight per wavefront
    auto fetch_a = [&](int k0, u32x4(&dst)[NL]) {
#pragma unroll
        for (int i = 0; i < NL; ++i) dst[i] = ok[i] ? *(const u32x4 *)(xp[i] + k0) : u32x4{0u, 0u, 0u, 0u};
    };
    auto fetch_b = [&](int k0) {
#pragma unroll
        for (int p = 0; p < B_PER; ++p) {
            const int v = tid + 256 * p;
            const int n = v >> 3, kk = k0 + (v & 7) * 8;
            rb[p] = (v < B_VECS && col0 + n < E) ? *(const u32x4 *)(wt + (size_t)(col0 + n) * d + kk)
                                                 : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto stash_b = [&](int buf) {
#pragma unroll
        for (int p = 0; p < B_PER; ++p) {
            const int v = tid + 256 * p;
            if (v < B_VECS) *(u32x4 *)&sB[buf][(v >> 3) * LDP + (v & 7) * 8] = rb[p];
        }
    };
    f32x16 acc[RB][NT];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][nt][i] = 0.f;

    // Workgroups walk d in rotated orders: at any moment they read different column slabs of x, which spreads
    // the 2*d-byte row stride over the memory channels.
    const int nslab = d / BK;
    const int rot = (int)((blockIdx.x * 7u + (blockIdx.x >> 5)) % (unsigned)nslab);
    auto kof = [&](int i) {
        int sidx = i + rot;
        if (sidx >= nslab) sidx -= nslab;
        return sidx * BK;
    };
    fetch_a(kof(0), ra[0]);
    fetch_b(kof(0));
#pragma unroll
    for (int i = 1; i < NS; ++i)
        if (i < nslab) fetch_a(kof(i), ra[i]);
    stash_b(0);
    int buf = 0;
    unsigned short *myA = sA[wave];
    auto step = [&](int it, u32x4(&cur)[NL]) {
#pragma unroll
        for (int i = 0; i < NL; ++i) *(u32x4 *)&myA[(8 * i + lr) * LDP + lc] = cur[i];
        __syncthreads();                         // sB[buf] and this wavefront's x tile are complete
        const bool more = it + 1 < nslab;
        if (more) fetch_b(kof(it + 1));
        if (it + NS < nslab) fetch_a(kof(it + NS), cur);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bf16x8 a[RB];
#pragma unroll
            for (int b = 0; b < RB; ++b) a[b] = *(const bf16x8 *)&myA[(32 * b + (lane & 31)) * LDP + 16 * j + kq];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                bf16x8 bv = *(const bf16x8 *)&sB[buf][(nt * 32 + (lane & 31)) * LDP + 16 * j + kq];
#pragma unroll
                for (int b = 0; b < RB; ++b)
                    acc[b][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[b], bv, acc[b][nt], 0, 0, 0);
            }
        }
        if (more) stash_b(buf ^ 1);
        buf ^= 1;
    };
    for (int it = 0; it < nslab; it += NS) {
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (it + i < nslab) step(it + i, ra[i]);
    }
    if constexpr (FUSE) {
        static_assert(RB == 1, "the fused epilogue handles 32 rows per wavefront");
        constexpr int EPLS = BN / 8;                 // values per lane with 8 lanes per row
        constexpr int SP = BN + 4;                   // pitch of a staged row in floats
        static_assert(4 * 16 * SP * sizeof(float) <= sizeof(sB), "the staged rows reuse the W tiles");
        __syncthreads();                             // every wavefront is done with the W tiles
        float *stage = (float *)&sB[0][0] + wave * (16 * SP);
        float bvs[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bvs[nt] = bias ? bias[nt * 32 + (lane & 31)] : 0.f;
        const int lg = lane & 7, rl = lane >> 3;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        stage[(8 * jj + 4 * (lane >> 5) + i) * SP + nt * 32 + (lane & 31)] =
                            acc[0][nt][4 * (2 * half + jj) + i] + bvs[nt];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int r_local = 8 * pass + rl;
                const int row = row0 + wave * RW + 16 * half + r_local;
                float xv[EPLS];
#pragma unroll
                for (int m = 0; m < EPLS; m += 4) {
                    const float4 v4 = *(const float4 *)&stage[r_local * SP + (m >> 2) * 32 + lg * 4];
                    xv[m] = v4.x; xv[m + 1] = v4.y; xv[m + 2] = v4.z; xv[m + 3] = v4.w;
                }
                float sc[EPLS];
                int qq[EPLS];
                softtopk_row<8, EPLS, true>(xv, lg, E, k, t, qscale, MAXSCORE_SOFTTOPK_A, sc, qq);
                if (row < T) {
#pragma unroll
                    for (int m = 0; m < EPLS; m += 4) {
                        const size_t o = (size_t)row * E + (m >> 2) * 32 + lg * 4;
                        if (out) *(float4 *)(out + o) = make_float4(xv[m], xv[m + 1], xv[m + 2], xv[m + 3]);
                        if (scores) *(float4 *)(scores + o) = make_float4(sc[m], sc[m + 1], sc[m + 2], sc[m + 3]);
                        if (q) *(int4 *)(q + o) = make_int4(qq[m], qq[m + 1], qq[m + 2], qq[m + 3]);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();         // the next half overwrites the staged rows
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        return;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int col = col0 + nt * 32 + (lane & 31);
        if (col >= E) continue;
        const float bvs = bias ? bias[col] : 0.f;
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int row = row0 + wave * RW + 32 * b + 8 * j + 4 * (lane >> 5) + i;
                    if (row < T) out[(size_t)row * E + col] = acc[b][nt][4 * j + i] + bvs;
                }
    }
}

__global__ __launch_bounds__(256) void k_gemm_f32(const float *__restrict__ x, const float *__restrict__ W,
                                                  const float *__restrict__ bias, int T, int d, int E,
                                                  float *__restrict__ out)
{
    size_t n = (size_t)T * E;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        int row = (int)(o / E), col = (int)(o % E);
        float acc = 0.f;
        for (int m = 0; m < d; ++m) acc = fmaf(x[(size_t)row * d + m], W[(size_t)m * E + col], acc);
        out[o] = acc + (bias ? bias[col] : 0.f);
    }
}

__global__ __launch_bounds__(256) void k_copy16(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

}  // namespace

int32_t gemm_run(const void *x, const void *W, const float *bias, int dtype, int T, int d, int E, float *logits,
                 void *wt_scratch, hipStream_t s)
{
    if (dtype == MAXSCORE_DTYPE_FP32) {
        size_t n = (size_t)T * E;
        int grid = (int)((n + 255) / 256);
        if (grid > 8192) grid = 8192;
        hipLaunchKernelGGL(k_gemm_f32, dim3(grid), dim3(256), 0, s, (const float *)x, (const float *)W, bias, T, d,
                           E, logits);
        MS_HIP(hipGetLastError());
        return MAXSCORE_OK;
    }
    const unsigned short *xb = (const unsigned short *)x, *wb = (const unsigned short *)W;
    dim3 grid((T + BM - 1) / BM, (E + 127) / 128);
    int et = E >= 128 ? 128 : E;
    int nt = (et + 31) / 32;
    if (wt_scratch && d % 8 == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)wt_scratch % 16) == 0) {
        unsigned short *wt = (unsigned short *)wt_scratch;
        hipLaunchKernelGGL(k_transpose_w, dim3((d + 31) / 32, (E + 31) / 32), dim3(256), 0, s, wb, wt, d, E);
#define MS_GEMM3(NT_)                                                                                          \
    hipLaunchKernelGGL((k_gemm_bf16_wtc<NT_, 1, 2, false>), grid, dim3(256), 0, s, xb, wt, bias, T, d, E, logits, \
                       (float *)nullptr, (int32_t *)nullptr, 0, 0.f, 0.f)
        if (d % BK == 0) {
            if (nt == 1) MS_GEMM3(1);
            else if (nt == 2) MS_GEMM3(2);
            else if (nt == 3) MS_GEMM3(3);
            else MS_GEMM3(4);
            MS_HIP(hipGetLastError());
            return MAXSCORE_OK;
        }
#undef MS_GEMM3
#define MS_GEMM2(NT_) hipLaunchKernelGGL((k_gemm_bf16_wt<NT_>), grid, dim3(256), 0, s, xb, wt, bias, T, d, E, logits)
        if (nt == 1) MS_GEMM2(1);
        else if (nt == 2) MS_GEMM2(2);
        else if (nt == 3) MS_GEMM2(3);
        else MS_GEMM2(4);
#undef MS_GEMM2
        MS_HIP(hipGetLastError());
        return MAXSCORE_OK;
    }
    const bool aligned = (d % 8 == 0) && (E % 8 == 0) && (((uintptr_t)x | (uintptr_t)W) % 16 == 0);
#define MS_GEMM(NT_, AL_) \
    hipLaunchKernelGGL((k_gemm_bf16<NT_, AL_>), grid, dim3(256), 0, s, xb, wb, bias, T, d, E, logits)
    if (aligned) {
        if (nt == 1) MS_GEMM(1, true);
        else if (nt == 2) MS_GEMM(2, true);
        else if (nt == 3) MS_GEMM(3, true);
        else MS_GEMM(4, true);
    } else {
        if (nt == 1) MS_GEMM(1, false);
        else if (nt == 2) MS_GEMM(2, false);
        else if (nt == 3) MS_GEMM(3, false);
        else MS_GEMM(4, false);
    }
#undef MS_GEMM
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

bool gemm_softtopk_supported(int dtype, int d, int E, const void *x, const void *wt_scratch)
{
    return dtype == MAXSCORE_DTYPE_BF16 && (E == 32 || E == 64 || E == 128) && d >= BK && d % BK == 0 && wt_scratch &&
           ((uintptr_t)x % 16) == 0 && ((uintptr_t)wt_scratch % 16) == 0;
}

int32_t gemm_softtopk_run(const void *x, const void *W, const float *bias, int dtype, int T, int d, int E, int k,
                          float t, int shift, float *logits, float *scores, int32_t *q, void *wt_scratch,
                          hipStream_t s)
{
    if (!gemm_softtopk_supported(dtype, d, E, x, wt_scratch)) return MAXSCORE_ERR_SHAPE;
    if (((((uintptr_t)logits) | ((uintptr_t)scores) | ((uintptr_t)q)) % 16) != 0) return MAXSCORE_ERR_SHAPE;
    const unsigned short *xb = (const unsigned short *)x, *wb = (const unsigned short *)W;
    unsigned short *wt = (unsigned short *)wt_scratch;
    hipLaunchKernelGGL(k_transpose_w, dim3((d + 31) / 32, (E + 31) / 32), dim3(256), 0, s, wb, wt, d, E);
    dim3 grid((T + BM - 1) / BM, 1);
    const float qscale = (float)(1 << shift);
#define MS_GEMMF(NT_)                                                                                         \
    hipLaunchKernelGGL((k_gemm_bf16_wtc<NT_, 1, 2, true>), grid, dim3(256), 0, s, xb, wt, bias, T, d, E, logits, \
                       scores, q, k, t, qscale)
    if (E == 32) MS_GEMMF(1);
    else if (E == 64) MS_GEMMF(2);
    else MS_GEMMF(4);
#undef MS_GEMMF
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t copy_run(const void *src, void *dst, size_t bytes, hipStream_t s)
{
    size_t n = bytes / 16;
    int grid = (int)((n + 255) / 256);
    if (grid > 16384) grid = 16384;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(k_copy16, dim3(grid), dim3(256), 0, s, (const u32x4 *)src, (u32x4 *)dst, n);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

}  // namespace maxscore
