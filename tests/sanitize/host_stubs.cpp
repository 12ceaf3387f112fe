// Host-only stand-ins for the kernel launchers behind the C ABI: every one reports success without touching a GPU.
// Linked with api.cpp under -fsanitize=address,undefined so that the argument validation and workspace carving of
// the boundary run on the CPU under the sanitizers.
#include "common.h"

namespace maxscore {

int g_kernel_timing = 0;

int32_t solver_run(const int32_t *, int, int, int, int, const maxscore_opts &, int32_t *, int64_t *, int64_t *,
                   maxscore_stats *, char *, hipStream_t, const int32_t *, long long, const int32_t *, long long,
                   SolverGeometry *, SolverAfter, void *)
{
    return MAXSCORE_OK;
}
size_t oversub_workspace_bytes(int T, int E, int k)
{
    if (E + k > kMaxE) return 0;
    return workspace_layout(T, E + k, k).total + sizeof(int32_t) * (size_t)T * (E + k) + sizeof(int64_t) * (E + k) + 1024;
}
int32_t oversub_run(const int32_t *, int T, int E, int k, int, const maxscore_opts &, int32_t *, int64_t *, int64_t *,
                    maxscore_stats *, char *, size_t ws_bytes, hipStream_t)
{
    if (E + k > kMaxE) return MAXSCORE_ERR_OVERSUBSCRIBED;
    if (ws_bytes < oversub_workspace_bytes(T, E, k)) return MAXSCORE_ERR_WORKSPACE;
    return MAXSCORE_OK;
}
int32_t dispatch_from_keys(const SolverGeometry &, const float *, const int32_t *, int, int, int, float *, int32_t *,
                           int32_t *, float *, int32_t *, char *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t kvec_check(const int32_t *, int, int, int, char *, long long *demand, hipStream_t)
{
    *demand = 0;
    return MAXSCORE_OK;
}
int32_t softtopk_run(const float *, int, int, int, float, int, float *, int32_t *, hipStream_t, int) { return MAXSCORE_OK; }
int32_t quantise_run(const float *, int, int, int, int32_t *, hipStream_t) { return MAXSCORE_OK; }
int32_t gates_run(const float *, const int32_t *, int, int, int, float *, hipStream_t) { return MAXSCORE_OK; }
int32_t dispatch_run(const int32_t *, const float *, int, int, int, int32_t *, int32_t *, float *, int32_t *, char *,
                     hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t dispatch_core(const int32_t *, const float *, size_t, int, int, int32_t *, int32_t *, float *, int32_t *,
                      int *, int, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t iter_run(const int32_t *, int, int, int, int, int, int32_t *, int64_t *, int32_t *, int32_t *, char *,
                 hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t scores_op_run(const float *, int, int, int, int, int, float *, int32_t *, hipStream_t) { return MAXSCORE_OK; }
int32_t top1_run(const int32_t *, int, int, int32_t *, hipStream_t) { return MAXSCORE_OK; }
int32_t assign_total_run(const int32_t *, const int32_t *, int, int, int, void *, int64_t *, int32_t *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t caps_to_device(const int32_t *caps_host, int T, int E, int k, char *, const int32_t **cap_dev, long long *room,
                       int *cmax, hipStream_t, long long demand)
{
    long long sum = 0;
    int mx = 0;
    for (int j = 0; j < E; ++j) {          // reads the caller's host array, as the real one does
        if (caps_host[j] < 0) return MAXSCORE_ERR_SHAPE;
        const int c = caps_host[j] < T ? caps_host[j] : T;
        sum += c;
        mx = c > mx ? c : mx;
    }
    if ((demand < 0 ? (long long)T * k : demand) > sum) return MAXSCORE_ERR_OVERSUBSCRIBED;
    *cap_dev = nullptr;
    *room = sum;
    *cmax = mx > 0 ? mx : 1;
    return MAXSCORE_OK;
}
int32_t alg1_run(const int32_t *, int, int, int, const maxscore_opts &, int32_t *, int32_t *, int32_t *, int64_t *,
                 int32_t *, maxscore_stats *, char *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t sinkhorn_run(const float *, int, int, int, float, int, int32_t *, float *, int32_t *, char *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t aux_loss_run(const float *, const int32_t *, int, int, float, float *, float *, float *, char *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t gates_backward_run(const float *, const float *, const int32_t *, const float *, const float *, int, int, int,
                           float *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t dispatch_tokens_run(const void *, int, const int32_t *, const int32_t *, int, int, int, int, void *,
                            hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t combine_run(const void *, int, const int32_t *, const int32_t *, const float *, int, int, int, int, int,
                    float *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t gemm_run(const void *, const void *, const float *, int, int, int, int, float *, void *, hipStream_t)
{
    return MAXSCORE_OK;
}
bool gemm_softtopk_supported(int dtype, int d, int E, const void *, const void *wt)
{
    return dtype == MAXSCORE_DTYPE_BF16 && (E == 32 || E == 64 || E == 128) && d % 64 == 0 && wt;
}
int32_t gemm_softtopk_run(const void *, const void *, const float *, int, int, int, int, int, float, int, float *,
                          float *, int32_t *, void *, hipStream_t)
{
    return MAXSCORE_OK;
}
int32_t copy_run(const void *, void *, size_t, hipStream_t) { return MAXSCORE_OK; }

}  // namespace maxscore

// the HIP calls api.cpp makes itself (around its launchers): nothing is queued in this build
extern "C" hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
extern "C" hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
extern "C" hipError_t hipEventCreate(hipEvent_t *e) { *e = nullptr; return hipSuccess; }
extern "C" hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
extern "C" hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
