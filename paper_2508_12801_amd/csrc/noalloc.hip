// maxscore_dispatch_static: the dispatch step (a6) for callers that cannot allocate or pass scratch memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The per-tile expert
// counts that maxscore_dispatch keeps in the caller's workspace live here in one file-scope device array.  Every
// GPU holds its own copy of that array at its own address, for as long as the process lives; the address is
// looked up once per device and only that address is ever handed to a kernel.
#include <mutex>

#include "common.h"

namespace maxscore {
namespace {

constexpr size_t kStaticWords = (size_t)1 << 18;          // 1 MiB of 32-bit counters per GPU
constexpr int kMaxDevices = 64;

static __device__ __align__(256) int scratch[kStaticWords];

std::mutex g_mu;
int *g_scratch_ptr[kMaxDevices];                          // device address of `scratch` on each GPU (null = not looked up)

// Device address of the scratch array on the current device; looked up on the first call per device.
int32_t scratch_address(int **out)
{
    int dev = -1;
    MS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MAXSCORE_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        int *p = nullptr;
        MS_HIP(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return MAXSCORE_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MAXSCORE_OK;
}

}  // namespace
}  // namespace maxscore

using namespace maxscore;

extern "C" int32_t maxscore_dispatch_static(const int32_t *assign, const float *gates, int32_t T, int32_t E,
                                            int32_t k, int32_t *expert_offsets, int32_t *disp_token,
                                            float *disp_gate, int32_t *token_pos, void *stream)
{
    if (!assign || !expert_offsets || !disp_token || !token_pos) return MAXSCORE_ERR_NULL;
    if ((disp_gate != nullptr) != (gates != nullptr)) return MAXSCORE_ERR_NULL;
    if (T < 1 || T > (1 << kMaxTBits) || E < 1 || E > kMaxE || k < 1 || k > E || k > kMaxK) return MAXSCORE_ERR_SHAPE;
    const size_t n = (size_t)T * k;
    const size_t n_tiles = (n + kDispTile - 1) / kDispTile;
    if (n_tiles * (size_t)E + kMaxE > kStaticWords) return MAXSCORE_ERR_WORKSPACE;   // beyond the built-in scratch
    int *tiles = nullptr;
    int32_t rc = scratch_address(&tiles);
    if (rc) return rc;
    return dispatch_core(assign, gates, n, E, k, expert_offsets, disp_token, disp_gate, token_pos, tiles,
                         (int)n_tiles, (hipStream_t)stream);
}
