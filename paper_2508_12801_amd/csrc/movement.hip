// Activation movement around the experts (Eq. 1; the capacity buffers of Section 2.3):
//   dispatch_tokens: expert input buffers [E, C, d] <- rows of x in dispatch order, zero padding
//   combine:         y[i, :] = sum_s gate[i, s] * expert_out[assign[i, s], token_pos[i, s], :]
// Both are permutations of rows of d values: HBM-bound, nothing to compute but the gate-weighted sum.
// A row is moved as 16-byte vectors by consecutive lanes, so every load and store of a wavefront is one
// contiguous kilobyte; the per-row indices are wavefront-uniform and read through the scalar path.
#include "common.h"

namespace maxscore {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One wavefront per destination row (slot r = j*C + s of the [E, C, d] buffer), grid-stride over rows.
// vec_per_row = d * elem_bytes / 16.
__global__ __launch_bounds__(256) void k_dispatch_tokens(const u32x4 *__restrict__ x,
                                                         const int32_t *__restrict__ offsets,
                                                         const int32_t *__restrict__ disp_token, int T, int E, int C,
                                                         int vec_per_row, u32x4 *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const long long n_rows = (long long)E * C;
    const long long wave0 = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long long n_waves = (long long)gridDim.x * (blockDim.x >> 6);
    for (long long r = wave0; r < n_rows; r += n_waves) {
        const int j = (int)(r / C), s = (int)(r - (long long)j * C);
        const int o0 = offsets[j], cnt = offsets[j + 1] - o0;
        u32x4 *dst = out + r * vec_per_row;
        if (s < cnt) {
            const int tok = disp_token[o0 + s];
            const u32x4 *src = x + (size_t)(tok >= 0 && tok < T ? tok : 0) * vec_per_row;
            for (int c = lane; c < vec_per_row; c += 64) dst[c] = src[c];
        } else {
            for (int c = lane; c < vec_per_row; c += 64) dst[c] = u32x4{0u, 0u, 0u, 0u};
        }
    }
}

// Rows that are not a whole number of 16-byte vectors (or misaligned buffers): element by element.
template <typename TElem>
__global__ __launch_bounds__(256) void k_dispatch_tokens_elem(const TElem *__restrict__ x,
                                                              const int32_t *__restrict__ offsets,
                                                              const int32_t *__restrict__ disp_token, int T, int d,
                                                              int E, int C, TElem *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const long long n_rows = (long long)E * C;
    const long long wave0 = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long long n_waves = (long long)gridDim.x * (blockDim.x >> 6);
    for (long long r = wave0; r < n_rows; r += n_waves) {
        const int j = (int)(r / C), s = (int)(r - (long long)j * C);
        const int o0 = offsets[j], cnt = offsets[j + 1] - o0;
        TElem *dst = out + r * d;
        if (s < cnt) {
            const int tok = disp_token[o0 + s];
            const TElem *src = x + (size_t)(tok >= 0 && tok < T ? tok : 0) * d;
            for (int c = lane; c < d; c += 64) dst[c] = src[c];
        } else {
            for (int c = lane; c < d; c += 64) dst[c] = (TElem)0;
        }
    }
}

__device__ __forceinline__ float bf16_to_f32(unsigned short b) { return __uint_as_float((unsigned)b << 16); }

// One wavefront per token: every lane owns the 16-byte chunks lane, lane+64, ... of the row (at most
// kMaxChunks of them), accumulates the k gate-weighted expert rows in fp32 and writes fp32.
constexpr int kMaxChunks = 8;     // rows of up to 8 * 64 * 16 bytes (d <= 4096 bf16 / 2048 fp32) in one go

template <bool BF16>
__global__ __launch_bounds__(256) void k_combine(const u32x4 *__restrict__ buf, const int32_t *__restrict__ assign,
                                                 const int32_t *__restrict__ token_pos,
                                                 const float *__restrict__ gates, int T, int d, int E, int k, int C,
                                                 int vec_per_row, float *__restrict__ y)
{
    constexpr int EPV = BF16 ? 8 : 4;         // elements per 16-byte vector
    const int lane = threadIdx.x & 63;
    const long long wave0 = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long long n_waves = (long long)gridDim.x * (blockDim.x >> 6);
    for (long long i = wave0; i < T; i += n_waves) {
        for (int c0 = 0; c0 < vec_per_row; c0 += 64 * kMaxChunks) {
            float acc[kMaxChunks][EPV];
#pragma unroll
            for (int u = 0; u < kMaxChunks; ++u)
#pragma unroll
                for (int v = 0; v < EPV; ++v) acc[u][v] = 0.f;
            for (int s = 0; s < k; ++s) {
                const int e = assign[(size_t)i * k + s];
                if (e < 0) continue;                           // empty slot (wavefront-uniform)
                const int pos = token_pos[(size_t)i * k + s];
                // a place outside the expert's buffer (an assignment made with another capacity) is never read
                if (e >= E || pos < 0 || pos >= C) continue;
                const float g = gates[(size_t)i * k + s];
                const u32x4 *src = buf + ((size_t)e * C + pos) * vec_per_row;
                u32x4 vals[kMaxChunks];
#pragma unroll
                for (int u = 0; u < kMaxChunks; ++u) {
                    const int c = c0 + lane + 64 * u;
                    vals[u] = c < vec_per_row ? src[c] : u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < kMaxChunks; ++u) {
                    if (BF16) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const unsigned word = vals[u][w];
                            acc[u][2 * w] = fmaf(g, bf16_to_f32((unsigned short)(word & 0xffffu)), acc[u][2 * w]);
                            acc[u][2 * w + 1] = fmaf(g, bf16_to_f32((unsigned short)(word >> 16)), acc[u][2 * w + 1]);
                        }
                    } else {
#pragma unroll
                        for (int w = 0; w < 4; ++w) acc[u][w] = fmaf(g, __uint_as_float(vals[u][w]), acc[u][w]);
                    }
                }
            }
            float *yr = y + (size_t)i * d;
#pragma unroll
            for (int u = 0; u < kMaxChunks; ++u) {
                const int c = c0 + lane + 64 * u;
                if (c < vec_per_row) {
                    float4 *dst = (float4 *)(yr + (size_t)c * EPV);
                    dst[0] = float4{acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
                    if (BF16) dst[1] = float4{acc[u][4], acc[u][5], acc[u][6], acc[u][7]};
                }
            }
        }
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void k_combine_elem(const void *__restrict__ buf_, const int32_t *__restrict__ assign,
                                                      const int32_t *__restrict__ token_pos,
                                                      const float *__restrict__ gates, int T, int d, int E, int k,
                                                      int C, float *__restrict__ y)
{
    const size_t n = (size_t)T * d;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        const size_t i = o / d, c = o - i * d;
        float acc = 0.f;
        for (int s = 0; s < k; ++s) {
            const int e = assign[i * k + s];
            if (e < 0) continue;
            const int pos = token_pos[i * k + s];
            if (e >= E || pos < 0 || pos >= C) continue;      // outside the expert's buffer: never read
            const size_t at = ((size_t)e * C + pos) * d + c;
            const float v = BF16 ? bf16_to_f32(((const unsigned short *)buf_)[at]) : ((const float *)buf_)[at];
            acc = fmaf(gates[i * k + s], v, acc);
        }
        y[o] = acc;
    }
}

}  // namespace

int32_t dispatch_tokens_run(const void *x, int dtype, const int32_t *offsets, const int32_t *disp_token, int T, int d,
                            int E, int C, void *out, hipStream_t s)
{
    const int eb = dtype == MAXSCORE_DTYPE_BF16 ? 2 : 4;
    const long long n_rows = (long long)E * C;
    long long grid = (n_rows + 3) / 4;
    if (grid > 256 * 16) grid = 256 * 16;        // 16 workgroups of 4 wavefronts per compute unit, grid-stride
    if (grid < 1) grid = 1;
    const bool vec = ((size_t)d * eb) % 16 == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)out % 16) == 0;
    if (vec) {
        hipLaunchKernelGGL(k_dispatch_tokens, dim3((unsigned)grid), dim3(256), 0, s, (const u32x4 *)x, offsets,
                           disp_token, T, E, C, (int)((size_t)d * eb / 16), (u32x4 *)out);
    } else if (eb == 2) {
        hipLaunchKernelGGL((k_dispatch_tokens_elem<unsigned short>), dim3((unsigned)grid), dim3(256), 0, s,
                           (const unsigned short *)x, offsets, disp_token, T, d, E, C, (unsigned short *)out);
    } else {
        hipLaunchKernelGGL((k_dispatch_tokens_elem<unsigned int>), dim3((unsigned)grid), dim3(256), 0, s,
                           (const unsigned int *)x, offsets, disp_token, T, d, E, C, (unsigned int *)out);
    }
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t combine_run(const void *buf, int dtype, const int32_t *assign, const int32_t *token_pos, const float *gates,
                    int T, int d, int E, int k, int C, float *y, hipStream_t s)
{
    const int eb = dtype == MAXSCORE_DTYPE_BF16 ? 2 : 4;
    const bool vec = ((size_t)d * eb) % 16 == 0 && ((uintptr_t)buf % 16) == 0 && ((uintptr_t)y % 16) == 0;
    if (vec) {
        long long grid = ((long long)T + 3) / 4;
        if (grid > 256 * 16) grid = 256 * 16;
        if (grid < 1) grid = 1;
        const int vpr = (int)((size_t)d * eb / 16);
        if (eb == 2)
            hipLaunchKernelGGL((k_combine<true>), dim3((unsigned)grid), dim3(256), 0, s, (const u32x4 *)buf, assign,
                               token_pos, gates, T, d, E, k, C, vpr, y);
        else
            hipLaunchKernelGGL((k_combine<false>), dim3((unsigned)grid), dim3(256), 0, s, (const u32x4 *)buf, assign,
                               token_pos, gates, T, d, E, k, C, vpr, y);
    } else {
        size_t n = (size_t)T * d;
        long long grid = (long long)((n + 255) / 256);
        if (grid > 256 * 32) grid = 256 * 32;
        if (grid < 1) grid = 1;
        if (eb == 2)
            hipLaunchKernelGGL((k_combine_elem<true>), dim3((unsigned)grid), dim3(256), 0, s, buf, assign, token_pos,
                               gates, T, d, E, k, C, y);
        else
            hipLaunchKernelGGL((k_combine_elem<false>), dim3((unsigned)grid), dim3(256), 0, s, buf, assign,
                               token_pos, gates, T, d, E, k, C, y);
    }
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

}  // namespace maxscore
