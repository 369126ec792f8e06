// Device helpers shared by the planner and scorer kernels: candidate checking, the per-stage cost
// terms in int64, and the iteration-time score of a given partition.
#pragma once

#include "harp_internal.h"

namespace harp {

// Slot list of the candidate a workgroup is working on (LDS).
struct SlotInfo {
    uint16_t g[kMaxStages];          // device group of slot s
    uint8_t k[kMaxStages];           // index of the slot's degree in tp_degrees
    int32_t dev_first[kMaxStages];   // first global device id of slot s
};

// Checks a candidate and fills `sl`.  Called by every thread of the workgroup with uniform
// arguments; returns the same HARP_CAND_OK / HARP_CAND_INVALID to all of them.
__device__ __forceinline__ int load_and_check_slots(const TablesDev &tb, int S, int S_max,
                                                     const int32_t *grp, const int32_t *tpv,
                                                     SlotInfo &sl) {
    if (S < 1 || S > S_max) return HARP_CAND_INVALID;
    int bad = 0;
    for (int s = threadIdx.x; s < S; s += blockDim.x) {
        const int g = grp[s], tp = tpv[s];
        int k = -1;
        for (int q = 0; q < tb.n_tp; ++q)
            if (tb.tp[q] == tp) k = q;
        if (g < 0 || g >= tb.G || k < 0) bad = 1;
        else { sl.g[s] = (uint16_t)g; sl.k[s] = (uint8_t)k; }
    }
    if (__syncthreads_or(bad)) return HARP_CAND_INVALID;
    for (int s = threadIdx.x; s < S; s += blockDim.x) {
        const int g = sl.g[s];
        if (s == 0 || sl.g[s - 1] != g) {          // first slot of a run of group g
            for (int q = 0; q + 1 < s; ++q)
                if (sl.g[q] == g) bad = 1;          // the group was left and entered again
            int64_t used = 0;
            const int32_t base = tb.group_base[g];
            for (int q = s; q < S && sl.g[q] == g; ++q) {
                sl.dev_first[q] = base + (int32_t)used;
                used += tb.tp[sl.k[q]];
            }
            if (used > tb.group_ndev[g]) bad = 1;
        }
    }
    if (__syncthreads_or(bad)) return HARP_CAND_INVALID;
    return HARP_CAND_OK;
}

// Largest cap t_max the capped entry points accept: below 2^47 us like every time of an accepted
// problem, and small enough that a sum of at most 3 L terms plus (M - 1) caps stays inside int64.
__device__ __forceinline__ bool cap_out_of_range(const TablesDev &tb, int64_t cap) {
    const int64_t by_sum = INT64_MAX / (3 * int64_t(tb.L) + int64_t(tb.M));
    const int64_t limit = by_sum < kTimeLimit - 1 ? by_sum : kTimeLimit - 1;
    return cap > limit;
}

// All threads of the workgroup: outputs of a candidate without a plan.
__device__ __forceinline__ void write_failed(const PlansDev &out, int c, int S_max, int status) {
    int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
    int32_t *df = out.dev_first + int64_t(c) * S_max;
    for (int s = threadIdx.x; s <= S_max; s += blockDim.x) sp[s] = -1;
    for (int s = threadIdx.x; s < S_max; s += blockDim.x) df[s] = -1;
    if (threadIdx.x == 0) {
        out.bottleneck[c] = kInf;
        out.iter_time[c] = kInf;
        out.status[c] = status;
    }
}

// One wavefront (all 64 lanes): outputs of a candidate without a plan.
__device__ __forceinline__ void write_failed_wave(const PlansDev &out, int c, int S_max, int status, int lane) {
    int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
    int32_t *df = out.dev_first + int64_t(c) * S_max;
    for (int s = lane; s <= S_max; s += 64) sp[s] = -1;
    for (int s = lane; s < S_max; s += 64) df[s] = -1;
    if (lane == 0) {
        out.bottleneck[c] = kInf;
        out.iter_time[c] = kInf;
        out.status[c] = status;
    }
}

// One wavefront (all 64 lanes, uniform arguments): the cost model of the paper's section 5.2.2
// for the partition sp[0..S]:  sum_s (t_s + 2 c_s) + (M - 1) max_s max(t_s, c_s), after checking
// that the cuts rise strictly from 0 to L and that every stage fits in memory (eq. mem_cons).
// Every lane receives the same status, bottleneck and iteration time.
__device__ __forceinline__ int wave_score_partition(const TablesDev &tb, int S, const uint16_t *slot_g,
                                                    const uint8_t *slot_k, const int32_t *sp, int lane,
                                                    int64_t &bottleneck, int64_t &iter_time) {
    const int L = tb.L;
    int invalid = 0;
    if (lane == 0 && (sp[0] != 0 || sp[S] != L)) invalid = 1;
    for (int s = lane; s < S; s += 64)
        if (sp[s + 1] <= sp[s]) invalid = 1;
    bottleneck = kInf;
    iter_time = kInf;
    if (__any(invalid)) return HARP_CAND_INVALID;
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    int64_t worst = 0, single = 0;
    int unfit = 0;
    for (int s = lane; s < S; s += 64) {
        const int g = slot_g[s], k = slot_k[s];
        const int64_t tp = tb.tp[k];
        const int t = tb.group_type[g];
        const int j = sp[s], i = sp[s + 1];
        const int64_t n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
        const int64_t need = (PP[i] - PP[j]) + n_inflight * (PS[i] - PS[j]);
        if (need > tp * tb.type_mem[t]) unfit = 1;
        const int64_t *pf = tb.PF(t), *pr = tb.PR(g, k);
        const int64_t time = (pf[i] - pf[j] + tp - 1) / tp + (pr[i] - pr[j]);
        int64_t cut = 0;
        if (s < S - 1) {
            const int64_t link = tb.bw[int64_t(g) * tb.G + slot_g[s + 1]];
            cut = (tb.act_bytes[i - 1] + link - 1) / link;
        }
        const int64_t m = time > cut ? time : cut;
        worst = worst > m ? worst : m;
        single += time + 2 * cut;
    }
    if (__any(unfit)) return HARP_CAND_INFEASIBLE;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int64_t ow = __shfl_xor(worst, d, 64);
        single += __shfl_xor(single, d, 64);
        worst = worst > ow ? worst : ow;
    }
    bottleneck = worst;
    iter_time = single + int64_t(tb.M - 1) * worst;
    return HARP_CAND_OK;
}

}  // namespace harp
