/* A C-only client of the planner library: no Python, no torch.  It puts the hand example of the
 * recurrence (one GPU type, four operators costing 3, 1, 1, 3, two single-device groups, M = 4) on
 * the GPU through the HIP runtime's C interface, builds the tables, plans one two-stage candidate
 * and prints "splits b0 b1 b2 bottleneck iter_time status".  Expected: "0 2 4 4 20 0"
 * (D[2][4] = min(max(3, 5), max(4, 4), max(5, 3)) = 4, iteration time 8 + 3 * 4 = 20).
 * Built with:  hipcc -x c plan_tiny.c -I<include> -L<dir> -l:libharp_hip.so  (or gcc with the HIP
 * include path and -lamdhip64). */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "harp.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_HARP(x) do { int r_ = (x); if (r_ != HARP_OK) { fprintf(stderr, "%s: %d %s\n", #x, r_, harp_last_error(ctx)); return 3; } } while (0)

static void *to_device(const void *src, size_t bytes)
{
    void *d = NULL;
    if (hipMalloc(&d, bytes) != hipSuccess) return NULL;
    if (hipMemcpy(d, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return d;
}

int main(void)
{
    harp_ctx *ctx = NULL;
    if (harp_create(&ctx, 0) != HARP_OK) { fprintf(stderr, "harp_create failed\n"); return 1; }
    enum { L = 4, S_MAX = 2 };
    const int64_t fwd[L] = {3, 1, 1, 3}, zero[L] = {0, 0, 0, 0};
    const int32_t group_type[2] = {0, 0}, group_ndev[2] = {1, 1}, tp_degrees[1] = {1};
    const int64_t mem[1] = {1ll << 40}, bw[4] = {1, 1, 1, 1};
    harp_problem p;
    p.L = L; p.T = 1; p.G = 2; p.M = 4; p.ar_count = 4; p.flags = 0; p.n_tp = 1;
    p.tp_degrees = tp_degrees;
    p.fwd_us = (const int64_t *)to_device(fwd, sizeof fwd);
    p.bwd_us = (const int64_t *)to_device(zero, sizeof zero);
    p.param_bytes = (const int64_t *)to_device(zero, sizeof zero);
    p.stash_bytes = (const int64_t *)to_device(zero, sizeof zero);
    p.act_bytes = (const int64_t *)to_device(zero, sizeof zero);
    p.group_type = (const int32_t *)to_device(group_type, sizeof group_type);
    p.group_ndev = (const int32_t *)to_device(group_ndev, sizeof group_ndev);
    p.type_mem_bytes = (const int64_t *)to_device(mem, sizeof mem);
    p.bw_bytes_per_us = (const int64_t *)to_device(bw, sizeof bw);
    if (!p.fwd_us || !p.bwd_us || !p.param_bytes || !p.stash_bytes || !p.act_bytes || !p.group_type ||
        !p.group_ndev || !p.type_mem_bytes || !p.bw_bytes_per_us) { fprintf(stderr, "device copies failed\n"); return 2; }

    const size_t table_bytes = harp_tables_bytes(&p);
    void *table_buf = NULL;
    CHECK_HIP(hipMalloc(&table_buf, table_bytes));
    harp_tables *tables = NULL;
    CHECK_HARP(harp_build_segment_costs(ctx, &p, table_buf, table_bytes, &tables, NULL));
    CHECK_HARP(harp_tables_finalize(ctx, tables));

    const int32_t cand_S[1] = {2}, cand_group[S_MAX] = {0, 1}, cand_tp[S_MAX] = {1, 1};
    harp_candidates cands;
    cands.C = 1; cands.S_max = S_MAX;
    cands.cand_S = (const int32_t *)to_device(cand_S, sizeof cand_S);
    cands.cand_group = (const int32_t *)to_device(cand_group, sizeof cand_group);
    cands.cand_tp = (const int32_t *)to_device(cand_tp, sizeof cand_tp);
    harp_plans out;
    CHECK_HIP(hipMalloc((void **)&out.splits, sizeof(int32_t) * (S_MAX + 1)));
    CHECK_HIP(hipMalloc((void **)&out.dev_first, sizeof(int32_t) * S_MAX));
    CHECK_HIP(hipMalloc((void **)&out.bottleneck, sizeof(int64_t)));
    CHECK_HIP(hipMalloc((void **)&out.iter_time, sizeof(int64_t)));
    CHECK_HIP(hipMalloc((void **)&out.status, sizeof(int32_t)));
    const size_t ws_bytes = harp_plan_workspace_bytes(ctx, tables, &cands);
    void *ws = NULL;
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_HARP(harp_plan_batch(ctx, tables, &cands, &out, ws, ws_bytes, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    int32_t splits[S_MAX + 1], status;
    int64_t bottleneck, iter_time;
    CHECK_HIP(hipMemcpy(splits, out.splits, sizeof splits, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(&bottleneck, out.bottleneck, sizeof bottleneck, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(&iter_time, out.iter_time, sizeof iter_time, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(&status, out.status, sizeof status, hipMemcpyDeviceToHost));
    printf("%d %d %d %lld %lld %d\n", splits[0], splits[1], splits[2], (long long)bottleneck, (long long)iter_time, status);
    harp_tables_release(tables);
    harp_destroy(ctx);
    return (splits[0] == 0 && splits[1] == 2 && splits[2] == 4 && bottleneck == 4 && iter_time == 20 && status == 0) ? 0 : 4;
}
