// Training-side by-products of the routing path: the load-balance loss of Eq. 9 (Section 4.1) and the
// derivative of the gates (Eq. 2 with the SoftTopk scores of Eq. 6) with respect to the router logits.
//
// The rank multipliers of Eq. 6 are piecewise constant in the logits, so A_ij = m_ij * Softmax(L_i)_j gives
// dA_ij/dL_il = A_ij * (delta_jl - p_il): the backward pass needs the logits (for p) and the scores, not t or k.
#include "common.h"

namespace maxscore {
namespace {

constexpr int kColBlocksMax = 512;

// part[b][j] <- sum of scores[row][j] over the rows of block b.  blockDim = 256 = cols x rowlanes; a thread owns
// VEC adjacent columns (VEC = 4 when E is a multiple of 4) and keeps several row loads in flight.
template <int VEC>
__global__ __launch_bounds__(256) void k_colsum(const float *__restrict__ scores, int T, int E, int cols,
                                                int rows_per_block, float *__restrict__ part)
{
    extern __shared__ float s_acc[];     // [rowlanes][E]
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    const int rowlanes = 256 / cols, nvec = E / VEC;
    const int c = threadIdx.x % cols, rl = threadIdx.x / cols;
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = r0 + rows_per_block < T ? r0 + rows_per_block : T;
    const vec_t *src = reinterpret_cast<const vec_t *>(scores);
    for (int jv = c; jv < nvec; jv += cols) {
        vec_t acc = 0.f;
#pragma unroll 8
        for (int r = r0 + rl; r < r1; r += rowlanes) acc += src[(size_t)r * nvec + jv];
        *reinterpret_cast<vec_t *>(&s_acc[rl * E + jv * VEC]) = acc;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < E; j += 256) {
        float acc = 0.f;
        for (int l = 0; l < rowlanes; ++l) acc += s_acc[l * E + j];
        part[(size_t)blockIdx.x * E + j] = acc;
    }
}

// One workgroup: column means, the loss and its derivative with respect to the scores of a column.  Thread
// (j, g) adds the partial sums g, g+groups, ... of column j; the groups are then added in order.
__global__ __launch_bounds__(1024) void k_aux_final(const float *__restrict__ part, int n_blocks,
                                                    const int32_t *__restrict__ offsets, int T, int E, int epad,
                                                    float lam, float *__restrict__ loss,
                                                    float *__restrict__ mean_scores, float *__restrict__ dscores_col)
{
    __shared__ double s_red[1024];
    __shared__ double s_w[16];
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
    const int j = tid;
    double term = 0.0;
    if (j < E) {
        double sum = 0.0;
        for (int g = 0; g < groups; ++g) sum += s_red[g * epad + j];
        const double mean_a = sum / T;
        const double mean_p = (double)(offsets[j + 1] - offsets[j]) / T;
        term = mean_a * mean_p;
        if (mean_scores) mean_scores[j] = (float)mean_a;
        if (dscores_col) dscores_col[j] = (float)((double)lam / ((double)E * T) * mean_p);
    }
    for (int off = 32; off >= 1; off >>= 1) term += __shfl_xor(term, off);
    if ((j & 63) == 0) s_w[j >> 6] = term;
    __syncthreads();
    if (j == 0) {
        double tot = 0.0;
        for (int w = 0; w < 16; ++w) tot += s_w[w];
        *loss = (float)((double)lam * tot / E);
    }
}

// One wavefront per token row; lane l holds experts l, l+64, ...
template <int EPL>
__global__ __launch_bounds__(256) void k_gates_backward(const float *__restrict__ logits,
                                                        const float *__restrict__ scores,
                                                        const int32_t *__restrict__ assign,
                                                        const float *__restrict__ dgates,
                                                        const float *__restrict__ dscores_col, int T, int E, int k,
                                                        float *__restrict__ dlogits)
{
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int row = wave; row < T; row += n_waves) {
        float l[EPL], a[EPL], g[EPL];
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            const bool in = e < E;
            l[c] = in ? logits[(size_t)row * E + e] : -INFINITY;
            a[c] = in ? scores[(size_t)row * E + e] : 0.f;
            g[c] = (in && dscores_col) ? dscores_col[e] : 0.f;
            mx = fmaxf(mx, l[c]);
        }
        const int slot = lane < k ? assign[(size_t)row * k + lane] : -1;
        const float dg = lane < k ? dgates[(size_t)row * k + lane] : 0.f;
        for (int s = 0; s < k; ++s) {
            const int e = __shfl(slot, s);
            const float d = __shfl(dg, s);
#pragma unroll
            for (int c = 0; c < EPL; ++c)
                if (e == lane + 64 * c) g[c] += d;
        }
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        float z = 0.f, w = 0.f;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            l[c] = __expf(l[c] - mx);        // padded lanes: exp(-inf) = 0
            z += l[c];
            g[c] *= a[c];                    // w_j = gA_j * A_j
            w += g[c];
        }
        for (int off = 32; off >= 1; off >>= 1) {
            z += __shfl_xor(z, off);
            w += __shfl_xor(w, off);
        }
        const float scale = w / z;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            const int e = lane + 64 * c;
            if (e < E) dlogits[(size_t)row * E + e] = g[c] - l[c] * scale;
        }
    }
}

template <int EPL>
void launch_bwd(const float *logits, const float *scores, const int32_t *assign, const float *dgates,
                const float *dcol, int T, int E, int k, float *dlogits, hipStream_t s)
{
    const int grid = T < 4 * 4096 ? (T + 3) / 4 : 4096;
    hipLaunchKernelGGL(k_gates_backward<EPL>, dim3(grid), dim3(256), 0, s, logits, scores, assign, dgates, dcol, T, E,
                       k, dlogits);
}

}  // namespace

int32_t aux_loss_run(const float *scores, const int32_t *offsets, int T, int E, float lam, float *loss,
                     float *mean_scores, float *dscores_col, char *ws, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, 1);
    float *part = (float *)(ws + L.wcnt_off);          // n_blocks*E floats <= E*(T/4) ints
    const int vec = (E % 4 == 0 && ((uintptr_t)scores % 16) == 0) ? 4 : 1;
    int cols = 1;
    while (cols < E / vec && cols < 256) cols <<= 1;
    const int rowlanes = 256 / cols;
    int n_blocks = (T + 63) / 64;
    if (n_blocks > kColBlocksMax) n_blocks = kColBlocksMax;
    if (n_blocks > L.max_wg) n_blocks = L.max_wg;
    const int rows_per_block = (T + n_blocks - 1) / n_blocks;
    n_blocks = (T + rows_per_block - 1) / rows_per_block;
    const size_t shm = (size_t)rowlanes * E * sizeof(float);
    if (vec == 4)
        hipLaunchKernelGGL(k_colsum<4>, dim3(n_blocks), dim3(256), shm, s, scores, T, E, cols, rows_per_block, part);
    else
        hipLaunchKernelGGL(k_colsum<1>, dim3(n_blocks), dim3(256), shm, s, scores, T, E, cols, rows_per_block, part);
    int epad = 1;
    while (epad < E) epad <<= 1;
    hipLaunchKernelGGL(k_aux_final, dim3(1), dim3(1024), 0, s, part, n_blocks, offsets, T, E, epad, lam, loss,
                       mean_scores, dscores_col);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t gates_backward_run(const float *logits, const float *scores, const int32_t *assign, const float *dgates,
                           const float *dscores_col, int T, int E, int k, float *dlogits, hipStream_t s)
{
    const int epl = (E + 63) / 64;
    if (epl <= 1) launch_bwd<1>(logits, scores, assign, dgates, dscores_col, T, E, k, dlogits, s);
    else if (epl <= 2) launch_bwd<2>(logits, scores, assign, dgates, dscores_col, T, E, k, dlogits, s);
    else if (epl <= 4) launch_bwd<4>(logits, scores, assign, dgates, dscores_col, T, E, k, dlogits, s);
    else if (epl <= 8) launch_bwd<8>(logits, scores, assign, dgates, dscores_col, T, E, k, dlogits, s);
    else launch_bwd<16>(logits, scores, assign, dgates, dscores_col, T, E, k, dlogits, s);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

}  // namespace maxscore
