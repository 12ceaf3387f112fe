// Drives the host side of the C ABI (api.cpp linked with host_stubs.cpp) under the sanitizers: error paths first,
// then calls that pass validation and reach the (stubbed) launchers, for every entry point that api.cpp defines.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "maxscore.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main()
{
    void *one = (void *)256;                 // an aligned non-null value that the stubs never dereference
    const int T = 300, d = 64, E = 12, k = 3, C = 80;
    const size_t ws = maxscore_workspace_bytes(T, d, E, k, C);
    CHECK(ws > 0 && ws % 256 == 0);
    CHECK(maxscore_workspace_bytes(T, d, E, E + 1, C) == 0);
    CHECK(maxscore_workspace_bytes(0, d, E, k, C) == 0);
    CHECK(maxscore_workspace_bytes(T, d, 5000, k, C) == 0);
    maxscore_stats st;
    maxscore_opts o = {1.0f, 20, 100, 12, MAXSCORE_ASSIGN_EXACT, 0u, nullptr, 0};
    // a4
    CHECK(maxscore_assign_i32(nullptr, T, E, k, C, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_NULL);
    CHECK(maxscore_assign_i32((int32_t *)one, T, E, E + 1, C, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_SHAPE);
    // more demand than capacity: solved on a padded copy of the rewards, which needs the larger workspace that
    // maxscore_workspace_bytes reports for that capacity; refused only when E + k padding experts do not fit
    const size_t ws10 = maxscore_workspace_bytes(T, d, E, k, 10);
    CHECK(ws10 > ws);
    CHECK(maxscore_assign_i32((int32_t *)one, T, E, k, 10, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_WORKSPACE);
    CHECK(maxscore_assign_i32((int32_t *)one, T, E, k, 10, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws10, nullptr) == MAXSCORE_OK);
    {
        const size_t wsb = maxscore_workspace_bytes(T, 0, 1000, 30, 1);
        CHECK(wsb > 0);
        CHECK(maxscore_assign_i32((int32_t *)one, T, 1000, 30, 1, &o, (int32_t *)one, nullptr, nullptr, &st, one, wsb, nullptr) == MAXSCORE_ERR_OVERSUBSCRIBED);
    }
    const size_t ws0 = maxscore_workspace_bytes(T, 0, E, k, C);     // without the scratch of the projection
    CHECK(ws0 > 0 && ws0 <= ws);
    CHECK(maxscore_assign_i32((int32_t *)one, T, E, k, C, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws0 - 1, nullptr) == MAXSCORE_ERR_WORKSPACE);
    CHECK(maxscore_assign_i32((int32_t *)one, T, E, k, C, &o, (int32_t *)one, nullptr, nullptr, &st, (void *)260, ws, nullptr) == MAXSCORE_ERR_WORKSPACE);
    CHECK(maxscore_assign_i32((int32_t *)one, T, E, k, C, nullptr, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_OK);
    // capacity vector (a host array that the call reads)
    std::vector<int32_t> caps(E, C);
    CHECK(maxscore_assign_caps_i32((int32_t *)one, T, E, k, caps.data(), &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_OK);
    caps[3] = -1;
    CHECK(maxscore_assign_caps_i32((int32_t *)one, T, E, k, caps.data(), &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_SHAPE);
    caps.assign(E, 1);
    CHECK(maxscore_assign_caps_i32((int32_t *)one, T, E, k, caps.data(), &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_OVERSUBSCRIBED);
    CHECK(maxscore_assign_kvec_i32((int32_t *)one, T, E, k, nullptr, C, nullptr, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_NULL);
    CHECK(maxscore_assign_kvec_i32((int32_t *)one, T, E, k, (int32_t *)one, C, nullptr, &o, (int32_t *)one, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_OK);
    // a1, a2, a5, a6
    CHECK(maxscore_router_logits(one, one, nullptr, 7, T, d, E, (float *)one, nullptr, 0, nullptr) == MAXSCORE_ERR_DTYPE);
    CHECK(maxscore_router_logits(one, one, nullptr, MAXSCORE_DTYPE_BF16, T, d, E, (float *)one, one, ws, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_softtopk((float *)one, T, E, k, -1.0f, 20, (float *)one, (int32_t *)one, nullptr) == MAXSCORE_ERR_SHAPE);
    CHECK(maxscore_softtopk((float *)one, T, E, k, 1.0f, 20, (float *)one, (int32_t *)one, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_gates((float *)one, nullptr, T, E, k, (float *)one, nullptr) == MAXSCORE_ERR_NULL);
    CHECK(maxscore_dispatch((int32_t *)one, (float *)one, T, E, k, (int32_t *)one, (int32_t *)one, nullptr, (int32_t *)one, one, ws, nullptr) == MAXSCORE_ERR_NULL);
    CHECK(maxscore_dispatch((int32_t *)one, (float *)one, T, E, k, (int32_t *)one, (int32_t *)one, (float *)one, (int32_t *)one, one, ws, nullptr) == MAXSCORE_OK);
    // routing entries: both kinds of assignment take short capacity (empty slots)
    float *f = (float *)one;
    int32_t *i = (int32_t *)one;
    CHECK(maxscore_route_scores(f, T, E, k, C, &o, i, i, f, i, i, f, i, nullptr, &st, one, ws, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_route_logits(f, T, E, k, 10, &o, f, i, i, f, i, i, f, i, nullptr, &st, one, ws10, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_route_logits(f, T, 1000, 30, 1, &o, f, i, i, f, i, i, f, i, nullptr, &st, one, maxscore_workspace_bytes(T, 0, 1000, 30, 1), nullptr) == MAXSCORE_ERR_OVERSUBSCRIBED);
    o.assignment = MAXSCORE_ASSIGN_ITER;
    CHECK(maxscore_route_logits(f, T, E, k, 10, &o, f, i, i, f, i, i, f, i, nullptr, &st, one, ws, nullptr) == MAXSCORE_OK);
    o.assignment = 5;
    CHECK(maxscore_route_logits(f, T, E, k, C, &o, f, i, i, f, i, i, f, i, nullptr, &st, one, ws, nullptr) == MAXSCORE_ERR_SHAPE);
    o.assignment = MAXSCORE_ASSIGN_EXACT;
    const size_t wsx = maxscore_workspace_bytes(T, d, E, k, C);
    CHECK(maxscore_route_xw(one, one, nullptr, MAXSCORE_DTYPE_BF16, T, d, E, k, C, &o, f, f, i, i, f, i, i, f, i, nullptr, &st, one, wsx, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_route_xw(one, one, nullptr, MAXSCORE_DTYPE_BF16, T, d, E, k, C, &o, nullptr, f, i, i, f, i, i, f, i, nullptr, &st, one, wsx, nullptr) == MAXSCORE_ERR_NULL);
    // the rest of the entry points, one accepted call each
    CHECK(maxscore_scores_op(f, T, E, k, MAXSCORE_OP_SOFTKMAX, 20, f, i, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_scores_op(f, T, E, k, 9, 20, f, i, nullptr) == MAXSCORE_ERR_SHAPE);
    CHECK(maxscore_aux_loss(f, i, T, E, 0.01f, f, f, f, one, ws, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_gates_backward(f, f, i, f, nullptr, T, E, k, f, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_assign_iter_i32(i, T, E, k, C, -1, i, nullptr, nullptr, nullptr, one, ws, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_assign_top1_residual_i32(i, T, E, C, &o, i, i, nullptr, nullptr, nullptr, &st, one, ws, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_assign_top1_sinkhorn(f, T, E, C, 0.05f, 10, i, nullptr, nullptr, one, ws, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_assign_top1_sinkhorn(f, T, E, C, 0.0f, 10, i, nullptr, nullptr, one, ws, nullptr) == MAXSCORE_ERR_SHAPE);
    CHECK(maxscore_dispatch_tokens(one, MAXSCORE_DTYPE_BF16, i, i, T, d, E, C, one, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_combine(one, MAXSCORE_DTYPE_FP32, i, i, f, T, d, E, k, C, f, nullptr) == MAXSCORE_OK);
    CHECK(maxscore_copy_bytes(one, one, 10, nullptr) == MAXSCORE_ERR_SHAPE);
    CHECK(maxscore_copy_bytes(one, one, 32, nullptr) == MAXSCORE_OK);
    maxscore_set_kernel_timing(1);
    maxscore_set_kernel_timing(0);
    for (int code = -9; code <= 0; ++code) CHECK(maxscore_status_string(code)[0] != 0);
    std::puts("host boundary under sanitizers: ok");
    return 0;
}
