// Algorithm 1 (Section 3.2, "Algorithm complexity optimization"): the top-2 split.  Every token first takes its
// highest-reward expert whatever the load (steps 4-5: that entry of the reward matrix is then set to 0), the
// capacities become max(0, C - load) (step 6), and each token gets one more expert from the residual problem
// (steps 7-9).  The paper solves the residual problem approximately with Sinkhorn and does not give its iteration
// count, regulariser or rounding; here it is solved exactly by the same solver, run with k = 1 and one capacity
// per expert.
#include <vector>

#include "common.h"

namespace maxscore {
namespace {

// q2 <- q with the top-1 entry of every row set to 0
__global__ __launch_bounds__(256) void k_residual(const int32_t *__restrict__ q, const int32_t *__restrict__ top1,
                                                  size_t n, int E, int32_t *__restrict__ q2)
{
    for (size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x; a < n; a += (size_t)gridDim.x * blockDim.x) {
        const size_t row = a / E;
        const int col = (int)(a - row * E);
        q2[a] = col == top1[row] ? 0 : q[a];
    }
}

__global__ __launch_bounds__(256) void k_pair(const int32_t *__restrict__ top1, const int32_t *__restrict__ second,
                                              int T, int32_t *__restrict__ assign)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < T) {
        assign[2 * (size_t)i] = top1[i];
        assign[2 * (size_t)i + 1] = second[i];
    }
}

}  // namespace

int32_t caps_to_device(const int32_t *caps_host, int T, int E, int k, char *ws, const int32_t **cap_dev,
                       long long *room, int *cmax, hipStream_t s, long long demand)
{
    WorkspaceLayout L = workspace_layout(T, E, k);
    std::vector<int32_t> eff(E);
    long long sum = 0;
    int mx = 0;
    for (int j = 0; j < E; ++j) {
        if (caps_host[j] < 0) return MAXSCORE_ERR_SHAPE;
        eff[j] = caps_host[j] < T ? caps_host[j] : T;
        sum += eff[j];
        mx = eff[j] > mx ? eff[j] : mx;
    }
    if ((demand < 0 ? (long long)T * k : demand) > sum) return MAXSCORE_ERR_OVERSUBSCRIBED;
    int32_t *dst = (int32_t *)(ws + L.cap_off);
    MS_HIP(hipMemcpyAsync(dst, eff.data(), sizeof(int32_t) * E, hipMemcpyHostToDevice, s));
    MS_HIP(hipStreamSynchronize(s));          // the host vector goes out of scope
    *cap_dev = dst;
    *room = sum;
    *cmax = mx > 0 ? mx : 1;
    return MAXSCORE_OK;
}

int32_t alg1_run(const int32_t *q, int T, int E, int C, const maxscore_opts &o, int32_t *q_residual,
                 int32_t *assign, int32_t *caps_out, int64_t *total, int32_t *flow, maxscore_stats *stats, char *ws,
                 hipStream_t s)
{
    WorkspaceLayout L = workspace_layout(T, E, 1);    // the layout the k = 1 solve below uses
    int32_t *top1 = (int32_t *)(ws + L.aux_off), *second = top1 + T;
    int32_t *offsets = (int32_t *)(ws + L.theta_off);
    int32_t rc = top1_run(q, T, E, top1, s);
    if (rc) return rc;
    // per-expert load of the top-1 choice (the position kernels also give the counts)
    rc = dispatch_core(top1, nullptr, (size_t)T, E, 1, offsets, nullptr, nullptr, second, (int *)(ws + L.tiles_off),
                       L.n_tiles, s);
    if (rc) return rc;
    std::vector<int32_t> off(E + 1), caps(E);
    MS_HIP(hipMemcpyAsync(off.data(), offsets, sizeof(int32_t) * (E + 1), hipMemcpyDeviceToHost, s));
    MS_HIP(hipStreamSynchronize(s));
    for (int j = 0; j < E; ++j) {
        const int left = C - (off[j + 1] - off[j]);
        caps[j] = left > 0 ? left : 0;
        if (caps_out) caps_out[j] = caps[j];
    }
    const size_t n = (size_t)T * E;
    int grid = (int)((n + 255) / 256);
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(k_residual, dim3(grid), dim3(256), 0, s, q, top1, n, E, q_residual);
    MS_HIP(hipGetLastError());
    const int32_t *cap_dev = nullptr;
    long long room = 0;
    int cmax = 1;
    rc = caps_to_device(caps.data(), T, E, 1, ws, &cap_dev, &room, &cmax, s);
    if (rc) return rc;
    int32_t src = solver_run(q_residual, T, E, 1, cmax, o, second, nullptr, nullptr, stats, ws, s, cap_dev, room);
    if (src != MAXSCORE_OK && src != MAXSCORE_ERR_NOT_CONVERGED) return src;
    hipLaunchKernelGGL(k_pair, dim3((T + 255) / 256), dim3(256), 0, s, top1, second, T, assign);
    MS_HIP(hipGetLastError());
    rc = assign_total_run(q, assign, T, E, 2, ws + L.state_off, total, flow, s);
    if (rc) return rc;
    return src;
}

}  // namespace maxscore
