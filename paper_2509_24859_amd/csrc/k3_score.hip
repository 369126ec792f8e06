// Stand-alone scorer and batch selection for gfx950.
//
// k3_score: iteration time of caller-chosen partitions under the cost model of the paper's
// section 5.2.2 (eq. gpipe_cost_model), one wavefront per candidate, lanes over stages.
// k4_argmin: final selection of section 5.2.3 (the min over evaluated candidates), lowest
// candidate index on ties.  Both are O(C S) bytes of streaming work.
#include "harp_internal.h"
#include "plan_common.h"

namespace harp {

namespace {

__global__ __launch_bounds__(64) void k3_score(TablesDev tb, CandDev cd, const int32_t *splits,
                                               int64_t *bottleneck, int64_t *iter_time,
                                               int32_t *status) {
    __shared__ SlotInfo slots;
    const int S_max = cd.S_max;
    for (int c = blockIdx.x; c < cd.C; c += gridDim.x) {
        __syncthreads();
        const int S = cd.cand_S[c];
        int st = load_and_check_slots(tb, S, S_max, cd.cand_group + int64_t(c) * S_max,
                                      cd.cand_tp + int64_t(c) * S_max, slots);
        int64_t bott = kInf, iter = kInf;
        if (st == HARP_CAND_OK)
            st = wave_score_partition(tb, S, slots.g, slots.k, splits + int64_t(c) * (S_max + 1),
                                      threadIdx.x, bott, iter);
        if (threadIdx.x == 0) {
            bottleneck[c] = bott;
            iter_time[c] = iter;
            status[c] = st;
        }
    }
}

constexpr int kArgminThreads = 1024;

__global__ __launch_bounds__(kArgminThreads) void k4_argmin(int32_t C, const int64_t *iter_time,
                                                            const int32_t *status,
                                                            int64_t *best_time, int32_t *best_index) {
    __shared__ int64_t val_s[kArgminThreads / 64];
    __shared__ int32_t idx_s[kArgminThreads / 64];
    int64_t best = kInf;
    int32_t bi = INT32_MAX;
    // eight independent loads per trip: one workgroup has to cover the whole batch, so the loop
    // is bound by memory latency, not by arithmetic
    constexpr int kUnroll = 8;
    int c = threadIdx.x;
    for (; c + (kUnroll - 1) * kArgminThreads < C; c += kUnroll * kArgminThreads) {
        int32_t st[kUnroll];
        int64_t v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            st[u] = status[c + u * kArgminThreads];
            v[u] = iter_time[c + u * kArgminThreads];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)     // c rises within a thread: first minimum kept
            if (st[u] == HARP_CAND_OK && v[u] < best) { best = v[u]; bi = c + u * kArgminThreads; }
    }
    for (; c < C; c += kArgminThreads) {
        if (status[c] != HARP_CAND_OK) continue;
        const int64_t v = iter_time[c];
        if (v < best) { best = v; bi = c; }
    }
    auto fold = [&](int64_t ov, int32_t oi) {
        if (ov < best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    };
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) fold(__shfl_xor(best, d, 64), __shfl_xor(bi, d, 64));
    if ((threadIdx.x & 63) == 0) { val_s[threadIdx.x >> 6] = best; idx_s[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kArgminThreads / 64; ++w) fold(val_s[w], idx_s[w]);
        *best_time = best;
        *best_index = (bi == INT32_MAX) ? -1 : bi;
    }
}

}  // namespace

void launch_score(const TablesDev &tb, const CandDev &cd, const int32_t *splits,
                  int64_t *bottleneck, int64_t *iter_time, int32_t *status, hipStream_t st) {
    if (cd.C == 0) return;
    const int groups = cd.C < (1 << 20) ? cd.C : (1 << 20);
    hipLaunchKernelGGL(k3_score, dim3(groups), dim3(64), 0, st, tb, cd, splits, bottleneck,
                       iter_time, status);
}

void launch_argmin(int32_t C, const int64_t *iter_time, const int32_t *status, int64_t *best_time,
                   int32_t *best_index, hipStream_t st) {
    hipLaunchKernelGGL(k4_argmin, dim3(1), dim3(kArgminThreads), 0, st, C, iter_time, status,
                       best_time, best_index);
}

}  // namespace harp
