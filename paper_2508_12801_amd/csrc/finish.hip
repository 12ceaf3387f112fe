// Exact finish of the assignment (Eq. 7-8, Table 1) by cancelling negative cycles.
//
// The auction with eps-scaling spends its last phases on very little: the assignment it holds when the phase at a
// coarse eps (a few reward units) is quiescent already has the maximum flow and misses the optimum by a handful
// of exchanges.  Those are found directly.  With the token layer of Table 1's network contracted, the residual
// graph has the experts as nodes; the arc a -> b costs the smallest loss S*(q_ua - q_ub) over the tokens u that
// hold a and not b (moving u from a to b); a node Z stands for spare capacity (b -> Z is free when b has room,
// Z -> a is free when a holds a token).  The assignment is optimal iff this graph has no negative cycle, and then
// shortest-path distances give exact prices (the dual side of Eq. 7-8).  One pass:
//
//   k_fin_arcs    streams the rewards once and builds the arc matrix (smallest loss and its token per expert pair)
//                 in reduced form, loss - price_a + price_b, keeping only arcs under a bound (the others cannot lie
//                 on a negative cycle; this is verified at the end from the distances found);
//   k_fin_cycles  one workgroup: Bellman-Ford over the <= kFinMaxE + 1 nodes, cycles of the predecessor graph are negative
//                 cycles and are cancelled at once (the tokens on their arcs move, arcs of moved tokens leave the
//                 matrix), until the distances converge.  If anything was cancelled the matrix is incomplete and
//                 another pass follows; if nothing was, the optimum is certified and the prices are replaced.
//
// Everything is integer and deterministic (ties between tokens go to the lower token id).  When the finisher cannot
// certify (bound check fails, pass limit) the auction simply continues down its eps ladder from the state left here.
#include <algorithm>

#include "common.h"

namespace maxscore {
namespace {

constexpr unsigned long long kArcNone = ~0ull;
constexpr long long kRcBias = (long long)1 << 41;     // makes packed reduced costs unsigned
constexpr int kTokBits = kMaxTBits;                   // token id bits in a packed arc
constexpr int kCostInf = 1 << 30;                     // "no arc" in the 32-bit cost table (bounds stay below it)
constexpr long long kDistInf = (long long)1 << 60;
constexpr int kFinThreads = 1024;
constexpr int kFinMaxCyclesPerPass = 256;


__device__ __forceinline__ long long shfl_xor_i64(long long v, int off)
{
    unsigned lo = (unsigned)v, hi = (unsigned)((unsigned long long)v >> 32);
    lo = __shfl_xor(lo, off);
    hi = __shfl_xor(hi, off);
    return (long long)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ long long readlane_i64(long long v, int l)       // l is wavefront-uniform
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, l);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)((unsigned long long)v >> 32), l);
    return (long long)(((unsigned long long)hi << 32) | lo);
}

// Scratch of the finisher inside the workspace (WorkspaceLayout::fin_off): a bit per token that a cancelled cycle
// has moved, the list of those tokens, the expert loads and the node potentials carried from pass to pass.
struct FinArea {
    unsigned *bits;          // (T + 31) / 32 words
    int *n_moved;            // 1 counter (4 words reserved)
    int *list;               // kFinMovedCap token ids
    int *loads;              // kFinMaxE
    long long *pot;          // kFinMaxE + 2
};

__host__ __device__ inline FinArea fin_area(char *base, int T)
{
    FinArea f;
    size_t off = 0;
    f.bits = (unsigned *)(base + off); off += sizeof(unsigned) * (((size_t)T + 31) / 32 + 1);
    off = (off + 15) / 16 * 16;
    f.n_moved = (int *)(base + off); off += sizeof(int) * 4;
    f.list = (int *)(base + off); off += sizeof(int) * kFinMovedCap;
    f.loads = (int *)(base + off); off += sizeof(int) * kFinMaxE;
    off = (off + 15) / 16 * 16;
    f.pot = (long long *)(base + off);
    return f;
}

// Runs once when the auction has stopped at a coarse eps: clears the arc matrix and the moved-token marks and
// fixes the bound.
__global__ __launch_bounds__(kFinThreads) void k_fin_begin(SolverState *st, unsigned long long *M, char *fin_base,
                                                           int T, int E, long long bound_mult)
{
    if (st->fin != 1) return;
    FinArea fa = fin_area(fin_base, T);
    if (E <= kFinMatrixMaxE)
        for (int i = threadIdx.x; i < E * E; i += kFinThreads) M[i] = kArcNone;
    for (int i = threadIdx.x; i < (T + 31) / 32 + 1; i += kFinThreads) fa.bits[i] = 0u;
    if (threadIdx.x == 0) {
        long long b = bound_mult * st->eps;
        const long long cap = (long long)kCostInf - 1;
        st->fin_bound = b < cap ? b : cap;
        st->fin_passes = 0;
        st->fin_cycles = 0;
        st->fin_dirty = 0;
        fa.n_moved[0] = 0;
    }
}

// The arcs that token u offers: for the expert `only` it holds (or every expert it holds when only < 0) and every
// expert e it does not hold, the loss of moving it there in reduced form; arcs under the bound count.  With MIN they
// go into the matrix (smallest loss wins, then the lower token id); with an output list they are also written there
// in a fixed order (slot of the hold, then expert), the j-th of them at out_base + j while that is below out_end.
// Returns their number (the same in every lane).  One wavefront; lane l owns experts l, l + 64, ... (TEPL of them).  The assignment
// row is read at device scope: the Bellman-Ford workgroup calls this for tokens it has just moved.
__device__ __forceinline__ unsigned long long arc_pack(int cost, int a, int b)
{
    return ((unsigned long long)(unsigned)cost << 32) | (unsigned)((a << 16) | b);
}
__device__ __forceinline__ int arc_cost(unsigned long long w) { return (int)(unsigned)(w >> 32); }
__device__ __forceinline__ int arc_from(unsigned long long w) { return (int)((w >> 16) & 0xffff); }
__device__ __forceinline__ int arc_to(unsigned long long w) { return (int)(w & 0xffff); }

template <int TEPL, bool MIN>
__device__ __forceinline__ int token_arcs(const int32_t *__restrict__ q, const int32_t *assign,
                                          const long long (&p)[TEPL], int sb, int u, int only, long long B,
                                          unsigned long long *M, int E, int k, int lane, unsigned long long *out_arc,
                                          int *out_tok, int out_base, int out_end)
{
    const int a = lane < k ? __hip_atomic_load(&assign[(size_t)u * k + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                           : -1;
    long long v[TEPL];
#pragma unroll
    for (int m = 0; m < TEPL; ++m) {
        const int e = lane + 64 * m;
        const int qv = e < E ? q[(size_t)u * E + e] : 0;
        v[m] = (((long long)qv) << sb) - p[m];
    }
    unsigned heldm = 0;
    for (int s = 0; s < k; ++s) {
        const int h = __builtin_amdgcn_readlane(a, s);
        if (h >= 0 && (h & 63) == lane) heldm |= 1u << (h >> 6);
    }
    int cnt = 0;
    for (int s = 0; s < k; ++s) {
        const int h = __builtin_amdgcn_readlane(a, s);
        if (h < 0 || (only >= 0 && h != only)) continue;
        long long x = v[0];
#pragma unroll
        for (int m = 1; m < TEPL; ++m) x = (h >> 6) == m ? v[m] : x;
        const long long vh = readlane_i64(x, h & 63);
#pragma unroll
        for (int m = 0; m < TEPL; ++m) {
            const int e = lane + 64 * m;
            const long long rc = vh - v[m];
            const bool ok = e < E && !((heldm >> m) & 1u) && rc < B && rc > -kRcBias;
            const unsigned long long bal = __ballot(ok);
            if (ok) {
                if (MIN) {
                    const unsigned long long pk =
                        ((unsigned long long)(rc + kRcBias) << kTokBits) | (unsigned long long)u;
                    atomicMin(&M[(size_t)h * E + e], pk);
                }
                if (out_arc) {
                    const int pos = out_base + cnt + __popcll(bal & ((1ull << lane) - 1));
                    if (pos < out_end) {
                        out_arc[pos] = arc_pack((int)rc, h, e);
                        out_tok[pos] = u;
                    }
                }
            }
            cnt += __popcll(bal);
        }
    }
    return cnt;
}

// Arcs of one pass.  The bid keys of the auction's last round already hold, for every (token, expert) hold, how
// far the hold is above the token's best alternative: key >> tbits = S*q - best alternative + eps.  Only holds
// whose margin is under the bound can offer an arc under the bound, and they are few; so the key blocks are
// scanned (8 bytes per hold) and only the rows of those holds are read.  Tokens that a cancelled cycle has moved
// are taken from the list instead (their keys are out of date): all their holds are evaluated.
// Every arc goes into the matrix (smallest loss per expert pair).  The first pass also writes ALL arcs under the
// bound as a list, block w into its own segment of seg_cap entries in a fixed order (holds by their place in the
// key block, then by expert), with their number in tri_cnt[w] (-1: the segment is too small).  With the complete
// list the Bellman-Ford workgroup can keep the arcs up to date itself while it moves tokens, so one pass is enough.
// Grid: one workgroup per key block (n_wg), 256 threads.
template <int TEPL, bool MIN>
__global__ __launch_bounds__(256) void k_fin_arcs(const int32_t *__restrict__ q, const int32_t *assign,
                                                  const long long *__restrict__ theta2,
                                                  const SolverState *__restrict__ st,
                                                  const long long *__restrict__ klist, const int *__restrict__ wcnt,
                                                  unsigned long long *M, char *fin_base, int T, int E, int k,
                                                  int rows, unsigned long long *tri_arc, int *tri_tok, int *tri_cnt,
                                                  int seg_cap)
{
    if (st->fin != 1) return;
    __shared__ short s_e[1024];
    __shared__ short s_list[1024];
    __shared__ int s_cnt[1024];
    __shared__ long long s_p[kFinMaxE];
    __shared__ int s_wn[4], s_total;
    const FinArea fa = fin_area(fin_base, T);
    const long long B = st->fin_bound, eps = st->eps;
    const int sb = st->sbits, tb = st->tbits;
    const bool want_list = st->fin_passes == 0;
    const long long tmask = ((long long)1 << tb) - 1;
    const long long *theta = theta2 + (st->round & 1) * kMaxE;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, w = blockIdx.x;
    const int row0 = w * rows;
    int rows_here = T - row0;
    rows_here = rows_here < rows ? rows_here : rows;
    const int nslots = rows_here * k;
    for (int e = tid; e < E; e += 256) s_p[e] = theta[e] >> tb;
    for (int i = tid; i < nslots; i += 256) s_e[i] = -1;
    __syncthreads();
    for (int e = tid; e < E; e += 256) {
        const int mt = wcnt[(size_t)w * E + e];
        const int off = mt >> 16, cnt = mt & 0xffff;
        for (int i = 0; i < cnt; ++i)
            if (off + i < nslots) s_e[off + i] = (short)e;
    }
    __syncthreads();
    const long long *blk = klist + (size_t)w * rows * k;
    // the holds under the bound, in the order of their places in the key block
    int n = 0;
    for (int i0 = 0; i0 < nslots; i0 += 256) {
        const int idx = i0 + tid;
        bool take = false;
        if (idx < nslots) {
            const int e = s_e[idx];
            if (e >= 0) {
                const long long key = blk[idx];
                const long long margin = (key >> tb) - eps - s_p[e];   // the hold's value minus the best alternative's
                const int u = (int)(key & tmask);
                take = margin < B && u >= row0 && u < row0 + rows_here &&     // (never outside with keys of this block)
                       !(fa.bits[u >> 5] & (1u << (u & 31)));                // moved since: taken from the list
            }
        }
        const unsigned long long bal = __ballot(take);
        if (lane == 0) s_wn[wv] = __popcll(bal);
        __syncthreads();
        int before = n;
        for (int x = 0; x < wv; ++x) before += s_wn[x];
        if (take) s_list[before + __popcll(bal & ((1ull << lane) - 1))] = (short)idx;
        n += s_wn[0] + s_wn[1] + s_wn[2] + s_wn[3];
        __syncthreads();
    }
    long long p[TEPL];
#pragma unroll
    for (int m = 0; m < TEPL; ++m) p[m] = lane + 64 * m < E ? s_p[lane + 64 * m] : 0;
    for (int i = wv; i < n; i += 4) {
        const int idx = s_list[i];
        const int u = (int)(blk[idx] & tmask);
        const int c = token_arcs<TEPL, MIN>(q, assign, p, sb, u, s_e[idx], B, M, E, k, lane, nullptr, nullptr, 0, 0);
        if (lane == 0) s_cnt[i] = c;
    }
    if (want_list) {
        __syncthreads();
        if (wv == 0) {
            // exclusive prefix sums of the per-hold counts (one wavefront, chunks of 64 holds)
            int run = 0;
            for (int i0 = 0; i0 < n; i0 += 64) {
                const int c = i0 + lane < n ? s_cnt[i0 + lane] : 0;
                int inc = c;
                for (int off = 1; off < 64; off <<= 1) {
                    const int o = __shfl_up(inc, off);
                    if (lane >= off) inc += o;
                }
                if (i0 + lane < n) s_cnt[i0 + lane] = run + inc - c;
                run += __shfl(inc, 63);
            }
            if (lane == 0) {
                s_total = run;
                tri_cnt[w] = run <= seg_cap ? run : -1;
            }
        }
        __syncthreads();
        const int total = s_total;
        if (total > 0 && total <= seg_cap) {
            const int base = w * seg_cap;
            for (int i = wv; i < n; i += 4) {
                const int idx = s_list[i];
                const int u = (int)(blk[idx] & tmask);
                (void)token_arcs<TEPL, false>(q, assign, p, sb, u, s_e[idx], B, M, E, k, lane, tri_arc, tri_tok,
                                              base + s_cnt[i], base + seg_cap);
            }
        }
    }
    // the moved tokens, spread over all wavefronts of the grid (their arcs only matter to the matrix)
    if (MIN) {
        const int nm = fa.n_moved[0] < kFinMovedCap ? fa.n_moved[0] : kFinMovedCap;
        for (int i = w * 4 + wv; i < nm; i += gridDim.x * 4)
            (void)token_arcs<TEPL, true>(q, assign, p, sb, fa.list[i], -1, B, M, E, k, lane, nullptr, nullptr, 0, 0);
    }
}

// Sizes of the Bellman-Ford workgroup by expert slots per lane: nodes it has tables for and arcs its list can hold
// (more arcs: the auction goes on).  Beyond kFinMatrixMaxE experts only the complete arc list is used.
template <int TEPL> struct FinCfg {
    static constexpr int MaxE = 256, Arcs = 11264;
};
template <> struct FinCfg<8> {
    static constexpr int MaxE = 512, Arcs = 9984;
};
template <> struct FinCfg<16> {
    static constexpr int MaxE = 1024, Arcs = 7168;
};
constexpr int kFinChunkGroup = 16;            // chunks of the arc matrix whose loads are in flight together
constexpr long long kKeyBias = (long long)1 << 48;   // potentials stay far inside (-2^48, 2^48)
constexpr int kIdxBits = 14;
constexpr unsigned kIdxRoot = (1u << kIdxBits) - 1;  // "no predecessor arc"
constexpr long long kZCostMax = (long long)1 << 30;  // prices must stay under this for the spare-capacity arcs


template <int kFinMaxE, int kFinArcs>
struct FinSharedT {
    // arc i: reduced cost (signed, kCostInf = slot empty or arc withdrawn) in the high word, from << 16 | to in the
    // low one (16 bits each; nodes 0..E-1 experts, E = Z)
    unsigned long long arc[kFinArcs];
    int atok[kFinArcs];                       // token that realises arc i (-1 for the arcs of Z)
    // node labels: (potential + bias) << 14 | index of the arc that last lowered it; two copies (a sweep reads
    // one and lowers the other, so its result does not depend on the order in which threads run)
    unsigned long long key[2][kFinMaxE + 2];
    long long p[kFinMaxE];                    // prices the reduced costs refer to
    int jump[2][kFinMaxE + 2];
    int load[kFinMaxE], capv[kFinMaxE];
    int cyc[kFinMaxE + 2];                    // nodes of the cycle being cancelled
    int pred[kFinMaxE + 2];                   // predecessor of every node at the last check
    int cycflag[kFinMaxE + 2], cyclist[kFinMaxE + 2];     // smallest node of every cycle found by the check
    int moved[kFinMaxE + 2];
    int scan[kFinMatrixMaxE * kFinMatrixMaxE / kFinThreads][kFinThreads / 64];     // arcs per (chunk of the matrix, wavefront) while the list is built
    int moved_all[kFinMovedCap / 8];          // tokens moved in this pass, for the list in memory
    int changed[3];       // one flag per sweep, three in rotation (a flag is cleared two sweeps after its last read)
    int newcnt[kFinMaxE + 2];                 // arcs that every token moved by the current cycle offers anew
    int wsum[kFinThreads / 64];
    int n_arcs, n_found, n_cyc, n_moved, n_moved_all, give_up, dirty, cycles, bad;
    int complete;         // the arc list holds EVERY arc under the bound (kept so while tokens move): one pass can certify
    long long cyc_sum;
};
static_assert(sizeof(FinSharedT<FinCfg<4>::MaxE, FinCfg<4>::Arcs>) <= 160 * 1024 &&
                  sizeof(FinSharedT<FinCfg<8>::MaxE, FinCfg<8>::Arcs>) <= 160 * 1024 &&
                  sizeof(FinSharedT<FinCfg<16>::MaxE, FinCfg<16>::Arcs>) <= 160 * 1024,
              "the Bellman-Ford workgroup keeps everything in one compute unit's LDS");
static_assert(kFinMatrixMaxE * kFinMatrixMaxE / kFinThreads * (kFinThreads / 64) <= kFinThreads, "one count per thread in the prefix");
static_assert(FinCfg<16>::MaxE == kFinMaxE, "tables for every expert count the finisher accepts");

// Bellman-Ford with cancelling.  One workgroup of kFinThreads threads, E <= 64 * TEPL <= FinCfg<TEPL>::MaxE.
//
// The arcs under the bound are few (a few thousand of the E*E pairs), so they are kept as a list.  Node potentials
// (0 at the start) are lowered sweep by sweep, every thread relaxing its arcs, until no arc a -> b has
// pot[b] > pot[a] + cost: then no negative cycle exists among the arcs.  While arcs keep relaxing, every fourth
// sweep looks for a cycle in the predecessor graph; such a cycle is checked (its cost must be negative, every token
// on it must hold the expert it leaves and not the one it goes to) and cancelled.  The potentials are kept across
// a cancellation: any potentials that stop relaxing certify the arcs that are left, and a negative cycle keeps
// them relaxing.
template <int TEPL>
__global__ __launch_bounds__(kFinThreads) void k_fin_cycles(SolverState *st, unsigned long long *M, int32_t *assign,
                                                            long long *theta2, const int *__restrict__ loads2,
                                                            char *fin_base, const int *__restrict__ cap, int Ce,
                                                            int T, int E, int k, int last_pass,
                                                            const int32_t *__restrict__ q,
                                                            const unsigned long long *__restrict__ tri_arc,
                                                            const int *__restrict__ tri_tok,
                                                            const int *__restrict__ tri_cnt, int seg_cap, int n_wg)
{
    if (st->fin != 1) return;
    constexpr int kNodes = FinCfg<TEPL>::MaxE, kFinArcs = FinCfg<TEPL>::Arcs;
    __shared__ FinSharedT<kNodes, kFinArcs> sh;
    const FinArea fa = fin_area(fin_base, T);
    int *fin_loads = fa.loads;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int tb = st->tbits;
    const long long B = st->fin_bound;
    const int Z = E, R = E + 1;                 // Z = spare capacity, R = root of the search (no predecessor)
    const long long *theta = theta2 + (st->round & 1) * kMaxE;
    const int *loads = loads2 + ((st->round + 1) & 1) * kMaxE;      // what the last select pass counted
    const int first_pass = st->fin_passes == 0;

    if (tid == 0) {
        sh.give_up = 0;
        sh.dirty = 0;
        sh.cycles = 0;
        sh.changed[0] = sh.changed[1] = sh.changed[2] = 0;
        sh.n_moved_all = 0;
    }
    for (int e = tid; e < E; e += kFinThreads) {
        sh.p[e] = theta[e] >> tb;
        sh.load[e] = first_pass ? loads[e] : fin_loads[e];      // later passes carry their own count
        sh.capv[e] = cap ? cap[e] : Ce;
    }
    for (int v = tid; v < kNodes + 2; v += kFinThreads) {
        // potentials: 0 in the first pass, then what the previous pass ended with (any start is valid: potentials
        // only have to stop relaxing; a good start saves sweeps)
        const long long d0 = (first_pass || v > E) ? 0 : fa.pot[v];
        const unsigned long long k0 = ((unsigned long long)(d0 + kKeyBias) << kIdxBits) | kIdxRoot;
        sh.key[0][v] = k0;
        sh.key[1][v] = k0;
    }
    __syncthreads();
    // slots 0..E-1: e -> Z (e takes one more token), E..2E-1: Z -> e (e gives one away); then the token arcs, in
    // matrix order (every thread compacts a run of consecutive entries, so the list order is fixed)
    auto set_z_arcs = [&]() {
        for (int e = tid; e < E; e += kFinThreads) {
            const long long pe = sh.p[e];
            if (pe >= kZCostMax) sh.give_up = 1;
            sh.arc[e] = arc_pack((sh.load[e] < sh.capv[e] && pe < kZCostMax) ? (int)-pe : kCostInf, e, Z);   // 0 - p_e + p_Z
            sh.atok[e] = -1;
            sh.arc[E + e] = arc_pack((sh.load[e] > 0 && pe < kZCostMax) ? (int)pe : kCostInf, Z, e);         // 0 - p_Z + p_e
            sh.atok[E + e] = -1;
        }
    };
    set_z_arcs();
    {
        // First pass: the arc kernel has left every arc under the bound in per-block segments.  If no segment ran
        // over and all of them fit the list, they are taken in block order (a fixed order) and the list is complete.
        int mine = 0, bad_seg = 0;
        const int per = (n_wg + kFinThreads - 1) / kFinThreads, w0 = tid * per;
        if (first_pass) {
            for (int w = w0; w < w0 + per && w < n_wg; ++w) {
                const int c = tri_cnt[w];
                bad_seg |= c < 0;
                mine += c > 0 ? c : 0;
            }
        }
        int inc = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (lane == 63) sh.wsum[wv] = inc;
        const int any_bad = __syncthreads_or(bad_seg);
        int before = inc - mine, total = 0;
        for (int x = 0; x < kFinThreads / 64; ++x) {
            const int t = sh.wsum[x];
            before += x < wv ? t : 0;
            total += t;
        }
        const bool complete = first_pass && !any_bad && 2 * E + total <= kFinArcs;
        if (complete) {
            int pos = 2 * E + before;
            for (int w = w0; w < w0 + per && w < n_wg; ++w) {
                const int c = tri_cnt[w];
                for (int j = 0; j < c; ++j) {
                    sh.arc[pos] = tri_arc[(size_t)w * seg_cap + j];
                    sh.atok[pos] = tri_tok[(size_t)w * seg_cap + j];
                    ++pos;
                }
            }
        }
        if (tid == 0) {
            sh.complete = complete ? 1 : 0;
            if (complete) sh.n_arcs = 2 * E + total;
        }
        __syncthreads();
    }
    if (!sh.complete && E > kFinMatrixMaxE) {
        // no arc matrix for this many experts: the auction goes on
        if (tid == 0) {
            sh.n_arcs = 2 * E;
            sh.give_up = 1;
        }
    } else if (!sh.complete) {
        // The matrix is read in chunks of kFinThreads consecutive entries, kFinChunkGroup chunks' loads in flight at
        // a time; an arc's place in the list follows from the number of arcs before it in matrix order.  Two
        // readings: the first counts, the second places.
        const int n = E * E;
        const int n_chunks = (n + kFinThreads - 1) / kFinThreads;
        const int n_flat = n_chunks * (kFinThreads / 64);                 // counts in (chunk, wavefront) order
        const int n_sw = (n_flat + 63) / 64;                              // wavefronts that scan them
        for (int g0 = 0; g0 < n_chunks; g0 += kFinChunkGroup) {
            unsigned long long pk[kFinChunkGroup];
#pragma unroll
            for (int c = 0; c < kFinChunkGroup; ++c) {
                const int i = (g0 + c) * kFinThreads + tid;
                pk[c] = (g0 + c < n_chunks && i < n) ? M[i] : kArcNone;
            }
#pragma unroll
            for (int c = 0; c < kFinChunkGroup; ++c) {
                const unsigned long long bal = __ballot(pk[c] != kArcNone);
                if (lane == 0 && g0 + c < n_chunks) sh.scan[g0 + c][wv] = __popcll(bal);
            }
        }
        __syncthreads();
        int *flat = &sh.scan[0][0];
        if (wv < n_sw) {
            // exclusive prefix inside every wavefront of counts, the wavefront totals beside it
            const int v = tid < n_flat ? flat[tid] : 0;
            int inc = v;
            for (int off = 1; off < 64; off <<= 1) {
                const int o = __shfl_up(inc, off);
                if (lane >= off) inc += o;
            }
            if (tid < n_flat) flat[tid] = inc - v;
            if (lane == 63) sh.cyc[wv] = inc;
        }
        __syncthreads();
        int total = 0;
        for (int w4 = 0; w4 < n_sw; ++w4) total += sh.cyc[w4];
        for (int g0 = 0; g0 < n_chunks; g0 += kFinChunkGroup) {
            unsigned long long pk[kFinChunkGroup];
#pragma unroll
            for (int c = 0; c < kFinChunkGroup; ++c) {
                const int i = (g0 + c) * kFinThreads + tid;
                pk[c] = (g0 + c < n_chunks && i < n) ? M[i] : kArcNone;
            }
#pragma unroll
            for (int c = 0; c < kFinChunkGroup; ++c) {
                const unsigned long long bal = __ballot(pk[c] != kArcNone);
                if (pk[c] == kArcNone) continue;
                const int flat_i = (g0 + c) * (kFinThreads / 64) + wv;
                int base = 2 * E + flat[flat_i] + __popcll(bal & ((1ull << lane) - 1));
                for (int w4 = 0; w4 < flat_i / 64; ++w4) base += sh.cyc[w4];
                if (base < kFinArcs) {
                    const int i = (g0 + c) * kFinThreads + tid;
                    const int a = i / E, b = i - a * E;
                    sh.arc[base] = arc_pack((int)((long long)(pk[c] >> kTokBits) - kRcBias), a, b);
                    sh.atok[base] = (int)(pk[c] & ((1u << kTokBits) - 1));
                }
            }
        }
        if (tid == 0) {
            const int na = 2 * E + total;
            sh.n_arcs = na < kFinArcs ? na : kFinArcs;
            if (na > kFinArcs) sh.give_up = 1;          // more arcs than the list holds
        }
    }
    __syncthreads();
    int n_arcs = sh.n_arcs;

    // The first kRegArcs arcs of every thread (arc tid + j * kFinThreads) are kept in registers between sweeps, so
    // that a sweep issues all its label reads at once; they are read again whenever arcs have been withdrawn.
    constexpr int kRegArcs = 4;
    unsigned long long wreg[kRegArcs];
    auto load_arcs = [&]() {
#pragma unroll
        for (int j = 0; j < kRegArcs; ++j) {
            const int i = tid + j * kFinThreads;
            wreg[j] = i < n_arcs ? sh.arc[i] : arc_pack(kCostInf, 0, 0);
        }
    };
    load_arcs();
    bool converged = false, fresh = first_pass;     // fresh: the potentials started from zero and nothing was cancelled since
    int cur = 0;
    const int max_sweeps = 8 * (E + 2) + 16 * kFinMaxCyclesPerPass;
    for (int it = 0; it < max_sweeps && !sh.give_up; ++it) {
        // one sweep: labels are read from copy `cur` and lowered in the other copy (which starts equal to it)
        {
            const unsigned long long *kc = sh.key[cur];
            unsigned long long *kn = sh.key[cur ^ 1];
            // the copy to be lowered is two sweeps old (labels never rise): it first catches up with the current one
            for (int v = tid; v <= Z; v += kFinThreads) atomicMin(&kn[v], kc[v]);
            bool any = false;
            {
                long long da[kRegArcs], db[kRegArcs];
#pragma unroll
                for (int j = 0; j < kRegArcs; ++j) {
                    da[j] = (long long)(kc[arc_from(wreg[j])] >> kIdxBits);
                    db[j] = (long long)(kc[arc_to(wreg[j])] >> kIdxBits);
                }
#pragma unroll
                for (int j = 0; j < kRegArcs; ++j) {
                    const int c = arc_cost(wreg[j]);
                    const long long cand = da[j] + c;
                    if (c < kCostInf && cand < db[j]) {
                        atomicMin(&kn[arc_to(wreg[j])],
                                  ((unsigned long long)cand << kIdxBits) | (unsigned)(tid + j * kFinThreads));
                        any = true;
                    }
                }
            }
            for (int i = tid + kRegArcs * kFinThreads; i < n_arcs; i += kFinThreads) {
                const unsigned long long w = sh.arc[i];
                const int c = arc_cost(w);
                if (c >= kCostInf) continue;
                const int a = arc_from(w), b = arc_to(w);
                const long long da = (long long)(kc[a] >> kIdxBits), db = (long long)(kc[b] >> kIdxBits);
                const long long cand = da + c;
                if (cand < db) {
                    atomicMin(&kn[b], ((unsigned long long)cand << kIdxBits) | (unsigned)i);
                    any = true;
                }
            }
            if (any) sh.changed[it % 3] = 1;
        }
        if (tid == 0) sh.changed[(it + 1) % 3] = 0;      // last read before the previous barrier
        __syncthreads();
        cur ^= 1;
        if (!sh.changed[it % 3]) {
            // Stopped relaxing.  If nothing was cancelled this pass can certify, provided the potentials spread
            // less than the bound; potentials carried over from earlier passes can spread more than needed, so
            // in that case the sweeps run once more from zero (no cycle is left: they converge).
            if ((sh.dirty == 0 || sh.complete) && !fresh) {
                long long lo = kDistInf, hi = -kDistInf;
                for (int v = 0; v <= Z; ++v) {
                    const long long dv = (long long)(sh.key[cur][v] >> kIdxBits);
                    lo = dv < lo ? dv : lo;
                    hi = dv > hi ? dv : hi;
                }
                if (hi - lo >= B) {            // the same for every thread
                    __syncthreads();
                    for (int v = tid; v < kNodes + 2; v += kFinThreads) {
                        const unsigned long long k0 = ((unsigned long long)kKeyBias << kIdxBits) | kIdxRoot;
                        sh.key[0][v] = k0;
                        sh.key[1][v] = k0;
                    }
                    fresh = true;
                    __syncthreads();
                    continue;
                }
            }
            converged = true;
            break;
        }
        if ((it & 7) != 7) continue;
        // cycles of the predecessor graph: follow the predecessors 256 steps by pointer doubling; a node that does
        // not end at the root has landed on a cycle.  Every node has one predecessor, so the cycles are disjoint;
        // each is named by its smallest node (wavefront 0, a few nodes per lane; the others wait)
        if (wv == 0) {
            for (int v = lane; v <= R; v += 64) {
                int pv = R;
                if (v != R) {
                    const unsigned idx = (unsigned)(sh.key[cur][v] & kIdxRoot);
                    if (idx != kIdxRoot) pv = arc_from(sh.arc[idx]);
                }
                sh.jump[0][v] = pv;
                sh.pred[v] = pv;
                sh.cycflag[v] = 0;
            }
            int jb = 0;
            for (int rep = 0; rep < 8; ++rep) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                for (int v = lane; v <= R; v += 64) sh.jump[jb ^ 1][v] = sh.jump[jb][sh.jump[jb][v]];
                jb ^= 1;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            for (int v = lane; v <= Z; v += 64) {
                const int l = sh.jump[jb][v];
                if (l == R) continue;
                int m = l, x = sh.pred[l];
                for (int step = 0; step <= E + 1 && x != l && x != R; ++step) {
                    m = x < m ? x : m;
                    x = sh.pred[x];
                }
                if (x == l) sh.cycflag[m] = 1;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            // the flagged nodes in ascending order (the order in which the cycles are cancelled is fixed)
            int n_found = 0;
            for (int v0 = 0; v0 <= Z; v0 += 64) {
                const int v = v0 + lane;
                const bool f = v <= Z && sh.cycflag[v] != 0;
                const unsigned long long bal = __ballot(f);
                if (f) sh.cyclist[n_found + __popcll(bal & ((1ull << lane) - 1))] = v;
                n_found += __popcll(bal);
            }
            if (lane == 0) sh.n_found = n_found;
        }
        __syncthreads();
        const int n_found = sh.n_found;
        if (n_found == 0) continue;
        bool stop = false;
        int done_here = 0;
        for (int ci = 0; ci < n_found; ++ci) {
            if (sh.cycles >= kFinMaxCyclesPerPass) {
                stop = true;
                break;
            }
            // ---- cancel the cycle through sh.cyclist[ci] ----
            if (tid == 0) {
                // walking the predecessors lists the nodes x of the cycle; the arc into x is the one in its label.
                // An earlier cancellation of this round may have withdrawn one of its arcs: then it is left alone.
                const int c0 = sh.cyclist[ci];
                int n = 0, x = c0;
                long long sum = 0;
                bool ok = true;
                do {
                    sh.cyc[n++] = x;
                    const unsigned idx = (unsigned)(sh.key[cur][x] & kIdxRoot);
                    if (idx == kIdxRoot || arc_cost(sh.arc[idx]) >= kCostInf) {
                        ok = false;
                        break;
                    }
                    sum += arc_cost(sh.arc[idx]);
                    x = arc_from(sh.arc[idx]);
                } while (x != c0 && n <= E + 1);
                sh.n_cyc = (ok && x == c0 && sum < 0) ? n : 0;
                sh.cyc_sum = sum;
                sh.bad = 0;
                sh.n_moved = sh.n_cyc;            // moved[i] = the token on arc i of the cycle (-1: an arc of Z)
            }
            __syncthreads();
            const int n = sh.n_cyc;
            if (n == 0) {                                             // the same for every thread
                __syncthreads();                                      // (the next walk writes sh.n_cyc again)
                continue;
            }
            // every token move is checked before anything is changed: wavefront w takes the arcs w, w + 16, ...
            for (int i = wv; i < n; i += kFinThreads / 64) {
                const unsigned idx = (unsigned)(sh.key[cur][sh.cyc[i]] & kIdxRoot);
                const int u = sh.atok[idx];
                if (u < 0) continue;                                  // an arc of Z: no token moves
                const int a = arc_from(sh.arc[idx]), x = arc_to(sh.arc[idx]);
                const int sl = (lane < k && u < T) ? __hip_atomic_load(&assign[(size_t)u * k + lane], __ATOMIC_RELAXED,
                                                                       __HIP_MEMORY_SCOPE_AGENT)
                                                   : -1;
                const int n_a = __popcll(__ballot(lane < k && sl == a));
                const int n_x = __popcll(__ballot(lane < k && sl == x));
                if (lane == 0 && (u >= T || n_a != 1 || n_x != 0)) sh.bad = 1;
            }
            __syncthreads();
            if (sh.bad) {
                // a recorded arc that the assignment does not bear out: the finisher hands back to the auction
                if (tid == 0) sh.give_up = 1;
                stop = true;
                break;
            }
            for (int i = wv; i < n; i += kFinThreads / 64) {
                const unsigned idx = (unsigned)(sh.key[cur][sh.cyc[i]] & kIdxRoot);
                const int u = sh.atok[idx];
                const int a = arc_from(sh.arc[idx]), x = arc_to(sh.arc[idx]);
                if (u >= 0) {
                    if (lane < k && __hip_atomic_load(&assign[(size_t)u * k + lane], __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT) == a)
                        __hip_atomic_store(&assign[(size_t)u * k + lane], x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (lane == 0) {
                        sh.moved[i] = u;
                        // marked for the arc passes to come (its bid keys no longer describe it) and listed; a token
                        // listed twice is only evaluated twice
                        atomicOr(&fa.bits[u >> 5], 1u << (u & 31));
                        const int pos = atomicAdd(&sh.n_moved_all, 1);
                        if (pos < kFinMovedCap / 8) sh.moved_all[pos] = u;
                        else sh.give_up = 1;
                    }
                } else if (lane == 0) {
                    sh.moved[i] = -1;
                    if (x == Z) atomicAdd(&sh.load[a], 1);            // a keeps the token it received
                    else atomicAdd(&sh.load[x], -1);                  // x gives one away without getting one back
                }
            }
            if (tid == 0) {
                sh.dirty += 1;
                sh.cycles += 1;
            }
            ++done_here;
            __syncthreads();
            // arcs realised by a token that has moved are no longer known: they are withdrawn until the next pass
            {
                const int nm = sh.n_moved;
                for (int i = 2 * E + tid; i < n_arcs; i += kFinThreads) {
                    const int u = sh.atok[i];
                    bool hit = false;
                    for (int m = 0; m < nm; ++m) hit |= (sh.moved[m] == u);
                    if (hit) sh.arc[i] = arc_pack(kCostInf, 0, 0);
                }
                set_z_arcs();
            }
            __syncthreads();
            if (sh.complete) {
                // ... and, with a complete list, the arcs the moved tokens offer from where they are now join it
                // (counted first, then written behind the list in the order of the cycle), so the list stays complete
                const int nm = sh.n_moved;
                long long pp[TEPL];
#pragma unroll
                for (int m = 0; m < TEPL; ++m) pp[m] = lane + 64 * m < E ? sh.p[lane + 64 * m] : 0;
                const int sbq = st->sbits;
                for (int i = wv; i < nm; i += kFinThreads / 64) {
                    const int u = sh.moved[i];
                    bool skip = u < 0;
                    for (int j = 0; j < i; ++j) skip |= sh.moved[j] == u;      // a token on two arcs is taken once
                    const int c = skip ? 0
                                       : token_arcs<TEPL, false>(q, assign, pp, sbq, u, -1, B, M, E, k, lane, nullptr,
                                                              nullptr, 0, 0);
                    if (lane == 0) sh.newcnt[i] = skip ? -1 : c;
                }
                __syncthreads();
                if (tid == 0) {
                    int run = n_arcs;
                    for (int i = 0; i < nm; ++i) {
                        const int c = sh.newcnt[i];
                        sh.newcnt[i] = c < 0 ? -1 : run;
                        run += c < 0 ? 0 : c;
                    }
                    if (run > kFinArcs) sh.complete = 0;        // no room: from here on as without the list
                    else sh.n_arcs = run;
                }
                __syncthreads();
                if (sh.complete) {
                    for (int i = wv; i < nm; i += kFinThreads / 64)
                        if (sh.newcnt[i] >= 0)
                            (void)token_arcs<TEPL, false>(q, assign, pp, sbq, sh.moved[i], -1, B, M, E, k, lane, sh.arc,
                                                       sh.atok, sh.newcnt[i], kFinArcs);
                    n_arcs = sh.n_arcs;
                }
                __syncthreads();
            }
        }
        if (stop) {
            __syncthreads();
            break;
        }
        // The potentials stay; the predecessor arcs start again (an arc that is gone must not be followed, and what
        // is left of the other cycles shows again as soon as their nodes are lowered).
        for (int v = tid; v <= R; v += kFinThreads) {
            sh.key[0][v] |= kIdxRoot;
            sh.key[1][v] |= kIdxRoot;
        }
        __syncthreads();
        if (done_here > 0) {
            load_arcs();
            fresh = false;
        }
    }

    // ---- end of the pass ----
    __syncthreads();
    if (tid == 0) {
        st->fin_passes += 1;
        st->fin_cycles += sh.cycles;
        st->fin_dirty = sh.dirty;
    }
    if (sh.give_up || !converged) {
        if (tid == 0) st->fin = (sh.give_up || last_pass) ? 3 : 1;
    } else if (sh.dirty > 0 && !sh.complete) {
        if (tid == 0 && last_pass) st->fin = 3;               // still pending and no pass left
    } else {
        // nothing was cancelled and the potentials stopped relaxing: no negative cycle among the recorded arcs.
        // The arcs left out have reduced cost >= B; they stay non-negative under the new prices if the potentials
        // spread less than B.
        const unsigned long long *kc = sh.key[cur];
        long long lo = kDistInf, hi = -kDistInf;
        for (int v = lane; v <= Z; v += 64) {
            const long long dv = (long long)(kc[v] >> kIdxBits) - kKeyBias;
            lo = dv < lo ? dv : lo;
            hi = dv > hi ? dv : hi;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const long long a = shfl_xor_i64(lo, off), b = shfl_xor_i64(hi, off);
            lo = a < lo ? a : lo;
            hi = b > hi ? b : hi;
        }
        const bool ok = hi - lo < B;
        if (ok) {
            // exact prices: p_e - d_e + d_Z (>= 0 on every expert that holds a token, 0 where there is room)
            const long long dz = (long long)(kc[Z] >> kIdxBits) - kKeyBias;
            for (int e = tid; e < E; e += kFinThreads) {
                long long pn = sh.p[e] - ((long long)(kc[e] >> kIdxBits) - kKeyBias) + dz;
                pn = pn < 0 ? 0 : pn;
                theta2[e] = pn << tb;
                theta2[kMaxE + e] = pn << tb;
            }
        }
        if (tid == 0) st->fin = ok ? 2 : 3;
    }
    // the next pass starts from an empty matrix; the loads go with it
    if (!sh.give_up && sh.dirty > 0 && E <= kFinMatrixMaxE) {
        for (int i = tid; i < E * E; i += kFinThreads) M[i] = kArcNone;
    }
    for (int e = tid; e < E; e += kFinThreads) fin_loads[e] = sh.load[e];
    {
        // this pass's moved tokens join the list in memory (this workgroup is its only writer)
        const int have = fa.n_moved[0], add = sh.n_moved_all < kFinMovedCap / 8 ? sh.n_moved_all : kFinMovedCap / 8;
        const int room = kFinMovedCap - have;
        const int n_add = add < room ? add : room;
        for (int i = tid; i < n_add; i += kFinThreads) fa.list[have + i] = sh.moved_all[i];
        __syncthreads();
        if (tid == 0) {
            fa.n_moved[0] = have + n_add;
            if (n_add < add && st->fin == 1) st->fin = 3;          // the list is full: the auction goes on
        }
    }
    for (int v = tid; v <= E; v += kFinThreads) fa.pot[v] = (long long)(sh.key[cur][v] >> kIdxBits) - kKeyBias;
}

// After a group of passes: the host learns where the finisher stands (word 0: 1 = certified, 2 = the auction goes
// on, 3 = passes are left and the work is not finished).  After the last pass, or when the finisher gave up, an
// optimum that is not certified sends the auction one step further down its ladder from the state the finisher
// left (its exchanges only improved the assignment).  If attempts are left (retry), the auction stops again at
// that next rung and the finisher takes over once more; otherwise it runs to eps = 1 itself.  Either way its phases
// now run to quiescence: a phase that ends early leaves its longest chains to the next one, which is only sound
// while the finisher is sure to take the last of them.
__global__ void k_fin_end(SolverState *st, int T, int *host_words, int final, int retry)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int resumed = 0;
    if (st->fin == 1 && !final) {
        __hip_atomic_store(&host_words[1], st->fin_cycles, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(&host_words[2], st->fin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(&host_words[0], 3, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        return;
    }
    if (st->fin == 1 || st->fin == 3) {
        st->done = 0;
        st->eps_prev = st->eps;
        const long long ne = st->eps / st->eps_div;
        st->eps = ne > 1 ? ne : 1;
        st->stop_eps = retry ? st->eps : 1;
        st->early_off = 1;
        st->moves = T;
        st->phases += 1;
        st->phase_start = st->round;
        resumed = 1;
    }
    __hip_atomic_store(&host_words[3], st->round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&host_words[1], st->fin_cycles, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&host_words[2], st->fin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&host_words[0], resumed ? 2 : 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

}  // namespace

size_t finish_area_bytes(int T)
{
    FinArea f = fin_area((char *)0, T);
    return (size_t)((char *)(f.pot + kFinMaxE + 2) - (char *)0);
}

int32_t finish_enqueue(const int32_t *q, int32_t *assign, SolverState *st, long long *theta2, const int *loads2,
                       const int *cap, int Ce, int T, int E, int k, char *ws, int rows, int n_wg, int first_pass,
                       int passes, int total_passes, long long bound_mult, int *host_words, int retry, hipStream_t s)
{
    if (E > kFinMaxE || passes < 1 || first_pass < 0 || first_pass + passes > total_passes || bound_mult < 1 ||
        rows * k > 1024 || n_wg < 1)
        return MAXSCORE_ERR_SHAPE;
    WorkspaceLayout L = workspace_layout(T, E, k);
    unsigned long long *M = (unsigned long long *)(ws + L.finm_off);      // E*E entries of the kFinMatrixMaxE^2 there (not used beyond that)
    char *fin_base = ws + L.fin_off;
    if (finish_area_bytes(T) > L.wt_off - L.fin_off) return MAXSCORE_ERR_WORKSPACE;      // layout and area must agree
    const long long *klist = (const long long *)(ws + L.klist_off);
    const int *wcnt = (const int *)(ws + L.wcnt_off);
    const size_t tri_n = fin_tri_entries(T, k, L.max_wg);
    if ((size_t)n_wg * fin_seg_cap(rows, k) > tri_n || n_wg > L.max_wg) return MAXSCORE_ERR_WORKSPACE;
    // every key block gets an equal share of the region (at least fin_seg_cap(rows, k) entries: with few blocks
    // much more, so that the short key blocks of a small batch do not run over)
    const int seg_cap = (int)std::min<size_t>(tri_n / (size_t)n_wg, 4096);
    unsigned long long *tri_arc = (unsigned long long *)(ws + L.tri_off);
    int *tri_tok = (int *)(ws + L.tri_off + 8 * tri_n);
    int *tri_cnt = tri_tok + tri_n;
    if (first_pass == 0)
        hipLaunchKernelGGL(k_fin_begin, dim3(1), dim3(kFinThreads), 0, s, st, M, fin_base, T, E, bound_mult);
    for (int pass = first_pass; pass < first_pass + passes; ++pass) {
        if (E <= 64)
            hipLaunchKernelGGL((k_fin_arcs<1, true>), dim3(n_wg), dim3(256), 0, s, q, assign, theta2, st, klist, wcnt, M,
                               fin_base, T, E, k, rows, tri_arc, tri_tok, tri_cnt, seg_cap);
        else if (E <= 128)
            hipLaunchKernelGGL((k_fin_arcs<2, true>), dim3(n_wg), dim3(256), 0, s, q, assign, theta2, st, klist, wcnt, M,
                               fin_base, T, E, k, rows, tri_arc, tri_tok, tri_cnt, seg_cap);
        else if (E <= 256)
            hipLaunchKernelGGL((k_fin_arcs<4, true>), dim3(n_wg), dim3(256), 0, s, q, assign, theta2, st, klist, wcnt, M,
                               fin_base, T, E, k, rows, tri_arc, tri_tok, tri_cnt, seg_cap);
        else if (E <= 512)
            hipLaunchKernelGGL((k_fin_arcs<8, false>), dim3(n_wg), dim3(256), 0, s, q, assign, theta2, st, klist, wcnt, M,
                               fin_base, T, E, k, rows, tri_arc, tri_tok, tri_cnt, seg_cap);
        else
            hipLaunchKernelGGL((k_fin_arcs<16, false>), dim3(n_wg), dim3(256), 0, s, q, assign, theta2, st, klist, wcnt, M,
                               fin_base, T, E, k, rows, tri_arc, tri_tok, tri_cnt, seg_cap);
        const int last = pass == total_passes - 1 ? 1 : 0;
        if (E <= 128)
            hipLaunchKernelGGL(k_fin_cycles<2>, dim3(1), dim3(kFinThreads), 0, s, st, M, assign, theta2, loads2, fin_base,
                               cap, Ce, T, E, k, last, q, tri_arc, tri_tok, tri_cnt, seg_cap, n_wg);
        else if (E <= 256)
            hipLaunchKernelGGL(k_fin_cycles<4>, dim3(1), dim3(kFinThreads), 0, s, st, M, assign, theta2, loads2, fin_base,
                               cap, Ce, T, E, k, last, q, tri_arc, tri_tok, tri_cnt, seg_cap, n_wg);
        else if (E <= 512)
            hipLaunchKernelGGL(k_fin_cycles<8>, dim3(1), dim3(kFinThreads), 0, s, st, M, assign, theta2, loads2, fin_base,
                               cap, Ce, T, E, k, last, q, tri_arc, tri_tok, tri_cnt, seg_cap, n_wg);
        else
            hipLaunchKernelGGL(k_fin_cycles<16>, dim3(1), dim3(kFinThreads), 0, s, st, M, assign, theta2, loads2, fin_base,
                               cap, Ce, T, E, k, last, q, tri_arc, tri_tok, tri_cnt, seg_cap, n_wg);
    }
    hipLaunchKernelGGL(k_fin_end, dim3(1), dim3(64), 0, s, st, T, host_words,
                       first_pass + passes == total_passes ? 1 : 0, retry);
    MS_HIP(hipGetLastError());
    return MAXSCORE_OK;
}

}  // namespace maxscore
