// Stand-alone scorer and batch selection for gfx950.
//
// k3_score: iteration time of caller-chosen partitions under the cost model of the paper's
// section 5.2.2 (eq. gpipe_cost_model), one wavefront per candidate, lanes over stages.
// k3_score_fast is the same for tables with the 32-bit rows and at most 64 stages: the work is a
// few gathers per candidate, so the kernel is a chain of memory round trips, and this form has
// three of them where the general one has seven (everything whose address depends on nothing is
// loaded first, for the next candidate while the current one is worked; the slot list is checked in
// registers; stage and transfer times come from the fused 32-bit rows, without divisions).
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

constexpr int kScoreWaves = 4;       // independent wavefronts per workgroup of k3_score_fast

__global__ __launch_bounds__(kScoreWaves * 64) void k3_score_fast(TablesDev tb, CandDev cd, const int32_t *splits,
                                                                  int64_t *bottleneck, int64_t *iter_time,
                                                                  int32_t *status, uint32_t shift_packed) {
    const int lane = threadIdx.x & 63;
    const int wave_id = blockIdx.x * kScoreWaves + (threadIdx.x >> 6), n_waves = gridDim.x * kScoreWaves;
    const int S_max = cd.S_max, L = tb.L;
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    // what a candidate's work starts from: its stage count and, lane s, slot s and the cuts s, s + 1
    struct First { int S, g, tp, j, i; };
    auto load_first = [&](int c) -> First {
        First f{0, -1, 0, 0, 0};
        if (c < cd.C) {
            f.S = cd.cand_S[c];
            if (lane < S_max) {
                f.g = cd.cand_group[int64_t(c) * S_max + lane];
                f.tp = cd.cand_tp[int64_t(c) * S_max + lane];
                f.j = splits[int64_t(c) * (S_max + 1) + lane];
                f.i = splits[int64_t(c) * (S_max + 1) + lane + 1];
            }
        }
        return f;
    };
    First next = load_first(wave_id);
    for (int c = wave_id; c < cd.C; c += n_waves) {
        const First f = next;
        next = load_first(c + n_waves);
        const int S = __builtin_amdgcn_readfirstlane(f.S);
        const int g = f.g, j = f.j, i = f.i;
        int st = HARP_CAND_OK;
        int64_t bott = kInf, iter = kInf;
        const bool mine = lane < S;
        int k = -1;
        for (int q = 0; q < tb.n_tp; ++q)
            if (tb.tp[q] == f.tp) k = q;
        // Second round trip: everything the checks and the score read, requested at once with indices
        // forced into range (a candidate that fails a check ignores what comes back).
        const int g_next = __shfl_down(g, 1, 64);
        const bool slot_ok = g >= 0 && g < tb.G && k >= 0;
        const int gs = slot_ok ? g : 0, ks = slot_ok ? k : 0;
        const int gn = (g_next >= 0 && g_next < tb.G) ? g_next : 0;
        const int is = i < 0 ? 0 : (i > L ? L : i), js = j < 0 ? 0 : (j > L ? L : j);
        const int ndev = tb.group_ndev[gs];
        const int type = tb.group_type[gs];
        const uint32_t *p = tb.P32 + (int64_t(gs) * tb.n_tp + ks) * tb.pitch32;
        const uint32_t pi = p[is], pj = p[js];
        const uint32_t cut_here = tb.CM[(int64_t(gs) * tb.G + gn) * tb.pitch32 + is];
        // the running sums at a stage's lower cut are those at the upper cut of the stage before it
        // (cut 0, where they are 0, for the first): when the cuts are not a partition the candidate is
        // refused and the difference is not used
        const int64_t pp_i = PP[is], ps_i = PS[is];
        const int64_t pp_up = __shfl_up(pp_i, 1, 64), ps_up = __shfl_up(ps_i, 1, 64);
        const int64_t dpp = pp_i - (lane > 0 ? pp_up : 0), dps = ps_i - (lane > 0 ? ps_up : 0);
        if (S < 1 || S > S_max) {
            st = HARP_CAND_INVALID;
        } else if (__any(mine && !slot_ok)) {
            st = HARP_CAND_INVALID;
        } else {
            // runs of slots on one group: a group must not be entered twice, nor give more devices than it has
            const int g_prev = __shfl_up(g, 1, 64);
            const bool start = mine && (lane == 0 || g_prev != g);
            const unsigned long long starts = __ballot(start);
            int bad = 0;
            for (unsigned long long m = starts; m != 0; m &= m - 1) {
                const int q = __ffsll((long long)m) - 1;
                const int gq = __builtin_amdgcn_readlane(g, q);
                if (start && q < lane && gq == g) bad = 1;
            }
            long long upto = mine ? f.tp : 0;              // devices of slots 0 .. lane
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const long long o = __shfl_up(upto, d, 64);
                if (lane >= d) upto += o;
            }
            const unsigned long long later = lane < 63 ? starts >> (lane + 1) : 0ull;
            const int end = later != 0 ? lane + __ffsll((long long)later) - 1 : S - 1;    // last slot of this run
            const long long upto_end = __shfl(upto, end, 64);
            const long long before = __shfl_up(upto, 1, 64);
            if (start && upto_end - (lane > 0 ? before : 0) > ndev) bad = 1;
            if (__any(bad)) st = HARP_CAND_INVALID;
        }
        if (st == HARP_CAND_OK) {
            // the cuts rise strictly from 0 to L
            int invalid = (lane == 0 && j != 0) || (lane == S - 1 && i != L) || (mine && i <= j);
            if (__any(invalid)) st = HARP_CAND_INVALID;
        }
        if (st == HARP_CAND_OK) {
            uint32_t time = 0, cu = 0;
            int unfit = 0;
            if (mine) {
                const int shift = int((shift_packed >> (4 * k)) & 15u);
                if (lane < S - 1) cu = cut_here;
                const int64_t n_inflight = (S - lane) < tb.M ? (S - lane) : tb.M;
                if (dpp + n_inflight * dps > int64_t(f.tp) * tb.type_mem[type]) unfit = 1;
                time = (pi + (1u << shift) - 1u - pj) >> shift;
            }
            if (__any(unfit)) {
                st = HARP_CAND_INFEASIBLE;
            } else {
                uint32_t worst = time > cu ? time : cu;
                int64_t single = int64_t(time) + 2 * int64_t(cu);
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const uint32_t ow = __shfl_xor(worst, d, 64);
                    single += __shfl_xor(single, d, 64);
                    worst = worst > ow ? worst : ow;
                }
                bott = int64_t(worst);
                iter = single + int64_t(tb.M - 1) * int64_t(worst);
            }
        }
        if (lane == 0) {
            bottleneck[c] = bott;
            iter_time[c] = iter;
            status[c] = st;
        }
    }
}

// H-1F1B counterpart of k3_score (paper section 4.1: eq. Ni with the integer form of eq. dp_ni's
// increment): warm-up counts of caller-chosen partitions under the cap t_max[c], the memory
// constraint with those counts, and sum + (M - 1) t_max.  One wavefront per candidate: lanes
// compute the per-stage terms, lane 0 accumulates the counts from the last stage backwards.
__global__ __launch_bounds__(64) void k3_score_h1f1b(TablesDev tb, CandDev cd, const int32_t *splits,
                                                     const int64_t *t_max, int32_t *warmup,
                                                     int64_t *bottleneck, int64_t *iter_time, int32_t *status) {
    __shared__ SlotInfo slots;
    __shared__ int32_t count[kMaxStages];
    const int S_max = cd.S_max, L = tb.L, lane = threadIdx.x;
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    for (int c = blockIdx.x; c < cd.C; c += gridDim.x) {
        __syncthreads();
        const int S = cd.cand_S[c];
        const int32_t *sp = splits + int64_t(c) * (S_max + 1);
        int32_t *wu = warmup + int64_t(c) * S_max;
        const int64_t cap = t_max[c];
        int st = load_and_check_slots(tb, S, S_max, cd.cand_group + int64_t(c) * S_max,
                                      cd.cand_tp + int64_t(c) * S_max, slots);
        if (st == HARP_CAND_OK) {
            int invalid = (lane == 0 && (sp[0] != 0 || sp[S] != L)) ? 1 : 0;
            for (int s = lane; s < S; s += 64)
                if (sp[s + 1] <= sp[s]) invalid = 1;
            if (__any(invalid)) st = HARP_CAND_INVALID;
        }
        if (st == HARP_CAND_OK && cap_out_of_range(tb, cap)) st = HARP_CAND_INVALID;
        int64_t worst = 0, sum = 0;
        if (st == HARP_CAND_OK) {
            int over = cap < 0 ? 1 : 0;
            for (int s = lane; s < S; s += 64) {
                const int g = slots.g[s], k = slots.k[s];
                const int64_t tp = tb.tp[k];
                const int j = sp[s], i = sp[s + 1];
                const int64_t *pf = tb.PF(tb.group_type[g]), *pr = tb.PR(g, k);
                const int64_t time = (pf[i] - pf[j] + tp - 1) / tp + (pr[i] - pr[j]);
                int64_t cut = 0;
                if (s < S - 1) {
                    const int64_t link = tb.bw[int64_t(g) * tb.G + slots.g[s + 1]];
                    cut = (tb.act_bytes[i - 1] + link - 1) / link;
                }
                if (time > cap || cut > cap) over = 1;
                const int64_t x = 2 * cut - (cap >> 6);
                count[s] = 1 + (x > 0 ? 1 : 0) + (x > cap ? 1 : 0);     // delta; cut <= cap bounds the quotient by 2
                const int64_t m = time > cut ? time : cut;
                worst = worst > m ? worst : m;
                sum += time + 2 * cut;
            }
            if (__any(over)) st = HARP_CAND_INFEASIBLE;
        }
        __syncthreads();
        if (st == HARP_CAND_OK) {
            if (lane == 0) {
                int64_t n = 0;
                for (int s = S - 1; s >= 0; --s) {
                    n += count[s];
                    n = n < tb.M ? n : tb.M;
                    count[s] = int32_t(n);
                }
            }
            __syncthreads();
            int unfit = 0;
            for (int s = lane; s < S; s += 64) {
                const int j = sp[s], i = sp[s + 1];
                const int64_t need = (PP[i] - PP[j]) + int64_t(count[s]) * (PS[i] - PS[j]);
                if (need > int64_t(tb.tp[slots.k[s]]) * tb.type_mem[tb.group_type[slots.g[s]]]) unfit = 1;
            }
            if (__any(unfit)) st = HARP_CAND_INFEASIBLE;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const int64_t ow = __shfl_xor(worst, d, 64);
            sum += __shfl_xor(sum, d, 64);
            worst = worst > ow ? worst : ow;
        }
        for (int s = lane; s < S_max; s += 64) wu[s] = (st == HARP_CAND_OK && s < S) ? count[s] : -1;
        if (lane == 0) {
            bottleneck[c] = st == HARP_CAND_OK ? worst : kInf;
            iter_time[c] = st == HARP_CAND_OK ? sum + int64_t(tb.M - 1) * cap : kInf;
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

// Large batches: the same selection by many workgroups and two atomics.  The least time first (signed
// 64-bit minimum), then the lowest index that attains it (unsigned 32-bit minimum: the initial
// 0xFFFFFFFF reads back as -1 when no candidate qualifies).
constexpr int kArgminWideThreads = 256;
constexpr int kArgminWideItems = 8;
constexpr int kArgminWideFrom = 1 << 15;      // batches below this take the one-workgroup kernel

__global__ void k4_argmin_open(int64_t *best_time, int32_t *best_index) {
    if (threadIdx.x == 0) { *best_time = kInf; *best_index = -1; }
}

__global__ __launch_bounds__(kArgminWideThreads) void k4_argmin_time(int32_t C, const int64_t *iter_time,
                                                                      const int32_t *status, int64_t *best_time) {
    int64_t best = kInf;
    const int stride = gridDim.x * kArgminWideThreads;
    int c = blockIdx.x * kArgminWideThreads + threadIdx.x;
    for (; c + (kArgminWideItems - 1) * stride < C; c += kArgminWideItems * stride) {
        int32_t st[kArgminWideItems];
        int64_t v[kArgminWideItems];
#pragma unroll
        for (int u = 0; u < kArgminWideItems; ++u) { st[u] = status[c + u * stride]; v[u] = iter_time[c + u * stride]; }
#pragma unroll
        for (int u = 0; u < kArgminWideItems; ++u)
            if (st[u] == HARP_CAND_OK && v[u] < best) best = v[u];
    }
    for (; c < C; c += stride)
        if (status[c] == HARP_CAND_OK && iter_time[c] < best) best = iter_time[c];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int64_t o = __shfl_xor(best, d, 64);
        best = o < best ? o : best;
    }
    if ((threadIdx.x & 63) == 0 && best != kInf) atomicMin(reinterpret_cast<long long *>(best_time), (long long)best);
}

__global__ __launch_bounds__(kArgminWideThreads) void k4_argmin_index(int32_t C, const int64_t *iter_time,
                                                                       const int32_t *status, const int64_t *best_time,
                                                                       int32_t *best_index) {
    const int64_t want = *best_time;
    if (want == kInf) return;                 // no candidate qualifies: the index stays -1
    uint32_t bi = 0xFFFFFFFFu;
    const int stride = gridDim.x * kArgminWideThreads;
    for (int c = blockIdx.x * kArgminWideThreads + threadIdx.x; c < C; c += stride)
        if (iter_time[c] == want && status[c] == HARP_CAND_OK && uint32_t(c) < bi) bi = uint32_t(c);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(bi, d, 64);
        bi = o < bi ? o : bi;
    }
    if ((threadIdx.x & 63) == 0 && bi != 0xFFFFFFFFu) atomicMin(reinterpret_cast<unsigned int *>(best_index), bi);
}

}  // namespace

// fast32: the tables have the 32-bit rows and the caller has not asked for the int64 kernels.
void launch_score(const TablesDev &tb, const CandDev &cd, const int32_t *splits,
                  int64_t *bottleneck, int64_t *iter_time, int32_t *status, bool fast32, int n_cu,
                  hipStream_t st) {
    if (cd.C == 0) return;
    if (fast32 && cd.S_max <= 64) {
        uint32_t shift_packed = 0;
        for (int k = 0; k < tb.n_tp; ++k) shift_packed |= uint32_t(tb.tp_shift[k] & 15) << (4 * k);
        int groups = n_cu * (32 / kScoreWaves);                  // as many wavefronts as the chip holds
        const int want = (cd.C + kScoreWaves - 1) / kScoreWaves;
        if (groups > want) groups = want;
        hipLaunchKernelGGL(k3_score_fast, dim3(groups), dim3(kScoreWaves * 64), 0, st, tb, cd, splits, bottleneck,
                           iter_time, status, shift_packed);
        return;
    }
    const int groups = cd.C < (1 << 20) ? cd.C : (1 << 20);
    hipLaunchKernelGGL(k3_score, dim3(groups), dim3(64), 0, st, tb, cd, splits, bottleneck,
                       iter_time, status);
}

void launch_score_h1f1b(const TablesDev &tb, const CandDev &cd, const int32_t *splits, const int64_t *t_max,
                        int32_t *warmup, int64_t *bottleneck, int64_t *iter_time, int32_t *status,
                        hipStream_t st) {
    if (cd.C == 0) return;
    const int groups = cd.C < (1 << 20) ? cd.C : (1 << 20);
    hipLaunchKernelGGL(k3_score_h1f1b, dim3(groups), dim3(64), 0, st, tb, cd, splits, t_max, warmup,
                       bottleneck, iter_time, status);
}

void launch_argmin(int32_t C, const int64_t *iter_time, const int32_t *status, int64_t *best_time,
                   int32_t *best_index, hipStream_t st) {
    if (C < kArgminWideFrom) {
        hipLaunchKernelGGL(k4_argmin, dim3(1), dim3(kArgminThreads), 0, st, C, iter_time, status,
                           best_time, best_index);
        return;
    }
    int groups = (C + kArgminWideThreads * kArgminWideItems - 1) / (kArgminWideThreads * kArgminWideItems);
    if (groups > 2048) groups = 2048;
    hipLaunchKernelGGL(k4_argmin_open, dim3(1), dim3(64), 0, st, best_time, best_index);
    hipLaunchKernelGGL(k4_argmin_time, dim3(groups), dim3(kArgminWideThreads), 0, st, C, iter_time, status, best_time);
    hipLaunchKernelGGL(k4_argmin_index, dim3(groups), dim3(kArgminWideThreads), 0, st, C, iter_time, status,
                       best_time, best_index);
}

}  // namespace harp
