// a6: dispatch permutation into per-expert buffers (Section 2.3: every expert owns a buffer of
// c = k*n/e token places).  Pairs (token, expert) are ordered by expert and, inside an expert, by
// ascending token id, which is what a stable sort of the token-major pair list by expert gives.
//
// Four launches: per-tile expert histograms, a scan over tiles, a scan over experts, and a scatter that
// recomputes each pair's stable rank inside its tile.  A tile is kTile consecutive slots of the
// token-major [T, k] assignment and is owned by one wavefront.
#include "common.h"

namespace maxscore {
namespace {

constexpr int kTile = kDispTile;  // slots per wavefront tile
constexpr int kWavesPerWg = 4;

__global__ __launch_bounds__(256) void k_tile_hist(const int32_t *__restrict__ assign, size_t n, int E,
                                                   int *__restrict__ tiles, int n_tiles)
{
    extern __shared__ int s_cnt[];   // [kWavesPerWg][E]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = blockIdx.x * kWavesPerWg + wave;
    int *cnt = s_cnt + wave * E;
    for (int e = lane; e < E; e += 64) cnt[e] = 0;
    __syncthreads();
    if (tile < n_tiles) {
        size_t a0 = (size_t)tile * kTile;
        for (int c = lane; c < kTile; c += 64) {
            size_t a = a0 + c;
            if (a < n) {
                int e = assign[a];
                if (e >= 0) atomicAdd(&cnt[e], 1);
            }
        }
    }
    __syncthreads();
    if (tile < n_tiles)
        for (int e = lane; e < E; e += 64) tiles[(size_t)tile * E + e] = cnt[e];
}

// tiles[tile][e] <- number of pairs of expert e in earlier tiles; totals[e] <- pairs of expert e.
// One wavefront per expert: every lane scans a contiguous run of tiles, the lane totals are scanned
// with shuffles.
__global__ __launch_bounds__(64) void k_scan_tiles(int *__restrict__ tiles, int n_tiles, int E,
                                                   int *__restrict__ totals)
{
    const int e = blockIdx.x, lane = threadIdx.x;
    const int per = (n_tiles + 63) / 64;
    const int t0 = lane * per;
    int sum = 0;
    for (int i = 0; i < per; ++i) {
        const int tl = t0 + i;
        if (tl < n_tiles) sum += tiles[(size_t)tl * E + e];
    }
    int inc = sum;
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    int run = inc - sum;
    for (int i = 0; i < per; ++i) {
        const int tl = t0 + i;
        if (tl < n_tiles) {
            const int c = tiles[(size_t)tl * E + e];
            tiles[(size_t)tl * E + e] = run;
            run += c;
        }
    }
    if (lane == 63) totals[e] = inc;
}

__global__ __launch_bounds__(1024) void k_offsets(const int *__restrict__ totals, int E, int32_t *__restrict__ offsets)
{
    __shared__ int s_w[16];
    const int e = threadIdx.x, lane = e & 63, wv = e >> 6;
    const int c = e < E ? totals[e] : 0;
    int inc = c;
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) s_w[wv] = inc;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wv; ++w) base += s_w[w];
    if (e < E) offsets[e] = base + inc - c;
    if (e == E - 1) offsets[E] = base + inc;
}

__global__ __launch_bounds__(256) void k_scatter(const int32_t *__restrict__ assign, const float *__restrict__ gates,
                                                 size_t n, int E, int k, int ebits, const int *__restrict__ tiles,
                                                 int n_tiles, const int32_t *__restrict__ offsets,
                                                 int32_t *__restrict__ disp_token, float *__restrict__ disp_gate,
                                                 int32_t *__restrict__ token_pos)
{
    extern __shared__ int s_run[];   // [kWavesPerWg][E] running position per expert
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = blockIdx.x * kWavesPerWg + wave;
    if (tile >= n_tiles) return;     // whole wavefront leaves; no block barrier below
    int *run = s_run + wave * E;
    for (int e = lane; e < E; e += 64) run[e] = tiles[(size_t)tile * E + e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const size_t a0 = (size_t)tile * kTile;
    for (int c = 0; c < kTile; c += 64) {
        const size_t a = a0 + c + lane;
        const int e = a < n ? assign[a] : -1;
        // lanes holding the same expert: intersect the ballots of every bit of the expert id
        unsigned long long same = __ballot(e >= 0);
        for (int b = 0; b < ebits; ++b) {
            const unsigned long long bal = __ballot((e >> b) & 1);
            same &= ((e >> b) & 1) ? bal : ~bal;
        }
        int pos = -1;
        if (e >= 0) pos = run[e] + __popcll(same & ((1ull << lane) - 1));   // lane order = token order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (e >= 0 && lane == __ffsll((long long)same) - 1) run[e] += __popcll(same);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (a < n) {
            token_pos[a] = pos;
            if (e >= 0) {
                const int dst = offsets[e] + pos;
                if (disp_token) disp_token[dst] = (int32_t)(a / k);
                if (disp_gate) disp_gate[dst] = gates[a];
            }
        }
    }
}

// ---- a5 + a6 from the key blocks of a converged solve --------------------------------------------------------
// The final bid pass of the solver leaves, per block of `rows` consecutive tokens, one key per (token, expert)
// pair, sorted by expert, with (offset << 16 | count) per expert beside it; the token id sits in the low bits of a
// key.  That is the per-tile expert histogram and the expert-sorted pair list the dispatch needs: one scan over
// the blocks per expert, then one pass per block that ranks the few keys of a (block, expert) segment by token
// id, gathers the gate from the scores and writes both dispatch lists, the positions and the gates.

__global__ __launch_bounds__(256) void k_keys_scan(const int *__restrict__ wcnt, int n_wg, int E,
                                                   int *__restrict__ dbase, int *__restrict__ totals)
{
    __shared__ int s_w[4];
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int per = (n_wg + 255) / 256;
    const int w0 = tid * per;
    int sum = 0;
    for (int i = 0; i < per; ++i) {
        const int w = w0 + i;
        if (w < n_wg) sum += wcnt[(size_t)w * E + e] & 0xffff;
    }
    int inc = sum;
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) s_w[wv] = inc;
    __syncthreads();
    int run = inc - sum;
    for (int w = 0; w < wv; ++w) run += s_w[w];
    for (int i = 0; i < per; ++i) {
        const int w = w0 + i;
        if (w < n_wg) {
            dbase[(size_t)w * E + e] = run;
            run += wcnt[(size_t)w * E + e] & 0xffff;
        }
    }
    if (tid == 255) totals[e] = run;
}

constexpr int kKeysPerBlock = 1024;       // rows * k of a bid workgroup never exceeds this

__global__ __launch_bounds__(256) void k_keys_scatter(const long long *__restrict__ klist,
                                                      const int *__restrict__ wcnt, const int *__restrict__ dbase,
                                                      const int *__restrict__ totals,
                                                      const float *__restrict__ scores,
                                                      const int32_t *__restrict__ assign, int T, int E, int k,
                                                      int rows, int tbits, float *__restrict__ gates,
                                                      int32_t *__restrict__ offsets, int32_t *__restrict__ disp_token,
                                                      float *__restrict__ disp_gate, int32_t *__restrict__ token_pos)
{
    __shared__ long long s_key[kKeysPerBlock];
    __shared__ short s_e[kKeysPerBlock];
    __shared__ int s_assign[kKeysPerBlock];
    __shared__ int s_pos[kKeysPerBlock];
    __shared__ float s_gate[kKeysPerBlock];
    __shared__ int s_meta[kMaxE], s_base[kMaxE], s_off[kMaxE];
    __shared__ int s_w[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, w = blockIdx.x;
    const int row0 = w * rows;
    int rows_here = T - row0;
    rows_here = rows_here < rows ? rows_here : rows;
    const int nslots = rows_here * k;
    const long long tmask = ((long long)1 << tbits) - 1;
    const size_t n_pairs = (size_t)T * k;

    // expert offsets: exclusive scan of the totals (every block needs them; block 0 writes them out)
    {
        const int per = (E + 255) / 256;         // <= 4
        int loc[4] = {0, 0, 0, 0}, sum = 0;
        for (int i = 0; i < per; ++i) {
            const int e = tid * per + i;
            loc[i] = e < E ? totals[e] : 0;
            sum += loc[i];
        }
        int inc = sum;
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (lane == 63) s_w[wv] = inc;
        __syncthreads();
        int run = inc - sum;
        for (int v = 0; v < wv; ++v) run += s_w[v];
        for (int i = 0; i < per; ++i) {
            const int e = tid * per + i;
            if (e < E) {
                s_off[e] = run;
                if (w == 0) offsets[e] = run;
                run += loc[i];
                if (w == 0 && e == E - 1) offsets[E] = run;
            }
        }
    }
    for (int e = tid; e < E; e += 256) {
        s_meta[e] = wcnt[(size_t)w * E + e];
        s_base[e] = dbase[(size_t)w * E + e];
    }
    const long long *blk = klist + (size_t)w * rows * k;
    for (int i = tid; i < nslots; i += 256) {
        s_key[i] = blk[i];
        s_assign[i] = assign[(size_t)row0 * k + i];
        s_e[i] = -1;
        s_pos[i] = -1;
        s_gate[i] = 0.f;
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256) {
        const int off = s_meta[e] >> 16, cnt = s_meta[e] & 0xffff;
        for (int i = 0; i < cnt; ++i)
            if (off + i < nslots) s_e[off + i] = (short)e;
    }
    __syncthreads();
    for (int idx = tid; idx < nslots; idx += 256) {
        const int e = s_e[idx];
        if (e < 0) continue;
        const int off = s_meta[e] >> 16, cnt = s_meta[e] & 0xffff;
        if (off + cnt > nslots) continue;                  // never with the counts of this block's own bid pass
        const int tok = (int)(s_key[idx] & tmask);
        const int lr = tok - row0;
        if (lr < 0 || lr >= rows_here) continue;           // never with keys of this block
        int r = 0;
        for (int i = 0; i < cnt; ++i) r += (int)(s_key[off + i] & tmask) < tok;
        const int pos = s_base[e] + r;
        const size_t dst = (size_t)s_off[e] + pos;
        const float g = scores[(size_t)tok * E + e];
        if (dst < n_pairs) {
            disp_token[dst] = tok;
            disp_gate[dst] = g;
        }
        for (int sl = 0; sl < k; ++sl)
            if (s_assign[lr * k + sl] == e) {
                s_pos[lr * k + sl] = pos;
                s_gate[lr * k + sl] = g;
            }
    }
    __syncthreads();
    for (int i = tid; i < nslots; i += 256) {
        token_pos[(size_t)row0 * k + i] = s_pos[i];
        gates[(size_t)row0 * k + i] = s_gate[i];
    }
}

}  // namespace

int32_t dispatch_from_keys(const SolverGeometry &g, const float *scores, const int32_t *assign, int T, int E, int k,
                           float *gates, int32_t *offsets, int32_t *disp_token, float *disp_gate, int32_t *token_pos,
                           char *ws, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    if (g.rows * k > kKeysPerBlock || g.n_wg > L.max_wg || g.n_wg < 1) return MAXSCORE_ERR_SHAPE;
    const long long *klist = (const long long *)(ws + L.klist_off);
    const int *wcnt = (const int *)(ws + L.wcnt_off);
    int *dbase = (int *)(ws + L.dbase_off);
    int *totals = dbase + (size_t)E * L.max_wg;
    hipLaunchKernelGGL(k_keys_scan, dim3(E), dim3(256), 0, s, wcnt, g.n_wg, E, dbase, totals);
    hipLaunchKernelGGL(k_keys_scatter, dim3(g.n_wg), dim3(256), 0, s, klist, wcnt, dbase, totals, scores, assign, T, E,
                       k, g.rows, g.tbits, gates, offsets, disp_token, disp_gate, token_pos);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t dispatch_core(const int32_t *list, const float *gates, size_t n, int E, int k, int32_t *offsets,
                      int32_t *disp_token, float *disp_gate, int32_t *token_pos, int *tiles, int n_tiles,
                      hipStream_t s)
{
    const int grid = (n_tiles + kWavesPerWg - 1) / kWavesPerWg;
    const size_t shm = (size_t)kWavesPerWg * E * sizeof(int);
    hipLaunchKernelGGL(k_tile_hist, dim3(grid), dim3(256), shm, s, list, n, E, tiles, n_tiles);
    int *totals = tiles + (size_t)n_tiles * E;
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    hipLaunchKernelGGL(k_scan_tiles, dim3(E), dim3(64), 0, s, tiles, n_tiles, E, totals);
    hipLaunchKernelGGL(k_offsets, dim3(1), dim3(1024), 0, s, totals, E, offsets);
    hipLaunchKernelGGL(k_scatter, dim3(grid), dim3(256), shm, s, list, gates, n, E, k, ebits, tiles, n_tiles,
                       offsets, disp_token, disp_gate, token_pos);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

int32_t dispatch_run(const int32_t *assign, const float *gates, int T, int E, int k, int32_t *offsets,
                     int32_t *disp_token, float *disp_gate, int32_t *token_pos, char *ws, hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    return dispatch_core(assign, gates, (size_t)T * k, E, k, offsets, disp_token, disp_gate, token_pos,
                         (int *)(ws + L.tiles_off), L.n_tiles, s);
}

}  // namespace maxscore
