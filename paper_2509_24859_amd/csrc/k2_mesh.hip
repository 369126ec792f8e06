// Submesh choice inside the recurrence (paper section 5.2.3, eq. dp_general's third index).
//
// A candidate is an order of device groups and a stage count S.  With O_k = devices of the first k
// groups of the order, the state (s, i, d) means: the first s stages hold the first i operators and
// use exactly the first d devices.  A stage placed at device offset d runs on the group k with
// O_k <= d < O_{k+1} and takes tp of its devices (an allowed degree, d + tp <= O_{k+1}); when that
// exhausts the group, the next stage is on the next group and the cut crosses the inter-group
// link, otherwise the intra-group link.  All devices of all listed groups are used: the answer is
// the state (S, L, O_K).  Min-max form with the classic 1F1B counts, as on the hot path:
//   D[s+1][i][d + tp] = min over (j, tp) of max(D[s][j][d], time, comm),
// ties resolved by the lowest previous cut j, then the smallest degree.
//
// Mapping: one workgroup per ordering at a time (drawn from a shared counter); within a stage one
// lane per target cell (i, d'), the cells of a wave on consecutive i of one d' so that reads of the
// previous row and of the table rows are contiguous.  For every degree the lane scans the previous
// cuts downwards and stops once the stage time alone exceeds the best value found (the stage time
// never decreases as j moves down) or the stage no longer fits in memory (monotone as well); the
// stop is strict and the update accepts equal values at a lower j, which keeps the lowest j.  The
// three-index table does not fit in LDS (L x devices entries per stage): the two live rows and the
// back-pointers sit in a per-workgroup slice of the caller's workspace, L2-resident at the sizes
// of interest.  Two forms of every pass: one on the int64 rows (any degrees, any time width, values
// int64), and one on the fused 32-bit rows and the cut table for tables that have them
// (mesh_pass_fast, mesh_h1_pass_fast in mesh_passes.h), chosen per launch.
#include "mesh_passes.h"

namespace harp {

using namespace meshdp;

namespace {

// kExact = false: the min-max plan of every ordering.  kExact = true: the optimum of the
// iteration-time model (section 5.2.2) over every slicing and partition: the capped least-sum
// table is walked over the caps exactly as the exact search of the hot path walks them (first at
// t_S, then down from ceil(T / B), skipping caps that the sums rule out; equal totals keep the lower
// cap), which returns what the increasing sweep over every distinct stage cost returns.
template <bool kExact, bool kFast>
__device__ __forceinline__ void mesh_body(const TablesDev &tb, const OrdDev &od, const PlansDev &out,
                                          int32_t *stage_group, int32_t *stage_tp, int32_t *n_passes,
                                          unsigned char *ws, size_t per_group, int64_t n_dev, int *ticket) {
    __shared__ int32_t offs[kMaxOrderGroups + 1];     // O_0 .. O_K
    __shared__ uint16_t order[kMaxOrderGroups];      // group ids are below 4096
    __shared__ uint16_t group_at[kMeshGroupTable];    // group index (in the order) of every device offset
    __shared__ int32_t cuts[kMaxStages + 1], kept_cuts[kMaxStages + 1];
    __shared__ uint16_t slot_g[kMaxStages], kept_g[kMaxStages];
    __shared__ uint8_t slot_k[kMaxStages], kept_k[kMaxStages];
    __shared__ int32_t slot_first[kMaxStages], kept_first[kMaxStages];
    __shared__ int64_t scored[2];
    __shared__ int shared_int[2];
    const int L = tb.L, S_max = od.S_max;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x;
    const MeshSlice m = mesh_slice(ws, per_group, L, n_dev);
    const int64_t m_cap = tb.M;

    // all threads: thread 0 backtracks into cuts/slot_*, the first wave scores them
    auto backtrack_and_score = [&](int K, int S, int64_t &bott, int64_t &total) {
        if (tid == 0) mesh_backtrack<kFast>(tb, m, offs, order, K, S, n_dev, cuts, slot_g, slot_k, slot_first);
        __syncthreads();
        if (wave == 0) {
            int64_t b, t;
            wave_score_partition(tb, S, slot_g, slot_k, cuts, lane, b, t);
            if (lane == 0) { scored[0] = b; scored[1] = t; }
        }
        __syncthreads();
        bott = scored[0];
        total = scored[1];
    };
    // one pass over the stages, in the form the launch chose (the fast form keeps a row of memory sums in LDS)
    extern __shared__ __align__(16) unsigned char mesh_lds[];
    int64_t *Q = reinterpret_cast<int64_t *>(mesh_lds);
    auto run_pass = [&](auto capped, int K, int S, int64_t cap) -> int64_t {
        constexpr bool kCapped = decltype(capped)::value;
        if constexpr (kFast) return mesh_pass_fast<kCapped>(tb, m, offs, order, group_at, Q, K, S, n_dev, cap);
        else return mesh_pass<kCapped>(tb, m, offs, order, group_at, K, S, n_dev, cap);
    };
    auto keep = [&](int S) {
        for (int s = tid; s <= S; s += nthreads) kept_cuts[s] = cuts[s];
        for (int s = tid; s < S; s += nthreads) {
            kept_g[s] = slot_g[s]; kept_k[s] = slot_k[s]; kept_first[s] = slot_first[s];
        }
    };

    for (;;) {
        __syncthreads();
        if (tid == 0) shared_int[0] = atomicAdd(ticket, 1);
        __syncthreads();
        const int c = shared_int[0];
        if (c >= od.C) break;
        const int S = od.ord_S[c], K = od.ord_G[c];
        const int32_t *og = od.ord_group + int64_t(c) * od.G_max;
        int32_t *sg = stage_group + int64_t(c) * S_max, *stp = stage_tp + int64_t(c) * S_max;
        auto fail = [&](int status) {
            write_failed(out, c, S_max, status);
            for (int s = tid; s < S_max; s += nthreads) { sg[s] = -1; stp[s] = -1; }
            if (tid == 0 && n_passes) n_passes[c] = 0;
        };
        // the ordering itself: counts in range, group ids in range and distinct
        int bad = (S < 1 || S > S_max || K < 1 || K > od.G_max) ? 1 : 0;
        if (!bad)
            for (int k = tid; k < K; k += nthreads) {
                const int g = og[k];
                if (g < 0 || g >= tb.G) { bad = 1; continue; }
                for (int q = 0; q < k; ++q)
                    if (og[q] == g) bad = 1;
                order[k] = uint16_t(g);
            }
        if (__syncthreads_or(bad)) { fail(HARP_CAND_INVALID); continue; }
        if (tid == 0) {
            int64_t o = 0;
            offs[0] = 0;
            for (int k = 0; k < K; ++k) { o += tb.group_ndev[order[k]]; offs[k + 1] = int32_t(o); }
        }
        __syncthreads();
        const int Dtot = offs[K];
        if (S > L || S < K || S > Dtot) { fail(HARP_CAND_INFEASIBLE); continue; }
        if (Dtot <= kMeshGroupTable) {
            for (int k = 0; k < K; ++k)
                for (int d = offs[k] + tid; d < offs[k + 1]; d += nthreads) group_at[d] = uint16_t(k);
        }

        if (run_pass(std::false_type(), K, S, 0) == kInf) { fail(HARP_CAND_INFEASIBLE); continue; }
        int64_t t_S, best_T;
        backtrack_and_score(K, S, t_S, best_T);
        int64_t best_b = t_S;
        keep(S);
        int passes = 0;
        if (kExact) {
            int64_t cap = t_S;
            while (S >= 2) {
                const int64_t sum = run_pass(std::true_type(), K, S, cap);
                if (sum == kInf) break;              // cannot happen at or above t_S
                int64_t b, T;
                backtrack_and_score(K, S, b, T);
                ++passes;
                if (T < best_T || (T == best_T && b <= best_b)) {   // equal totals: the lower cap; equal caps: the capped plan
                    best_T = T;
                    best_b = b;
                    keep(S);
                }
                if (passes >= (1 << 20) || b > cap) break;           // cannot happen: the cap falls with every pass
                int64_t next_cap;
                if (passes == 1) {
                    next_cap = (best_T + m_cap - 1) / m_cap;
                } else {
                    next_cap = b - 1;
                    if (m_cap > 1) {
                        const int64_t bound = (best_T - sum) / (m_cap - 1);
                        next_cap = next_cap < bound ? next_cap : bound;
                    }
                }
                if (next_cap <= t_S) break;
                cap = next_cap;
            }
        }
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = tid; s <= S_max; s += nthreads) sp[s] = s <= S ? kept_cuts[s] : -1;
        for (int s = tid; s < S_max; s += nthreads) {
            sg[s] = s < S ? int32_t(kept_g[s]) : -1;
            stp[s] = s < S ? tb.tp[kept_k[s]] : -1;
            df[s] = s < S ? kept_first[s] : -1;
        }
        if (tid == 0) {
            out.bottleneck[c] = best_b;
            out.iter_time[c] = best_T;
            out.status[c] = HARP_CAND_OK;
            if (n_passes) n_passes[c] = passes;
        }
    }
}

template <bool kExact, bool kFast>
__global__ __launch_bounds__(kMeshMaxThreads) void k2_mesh(TablesDev tb, OrdDev od, PlansDev out,
                                                           int32_t *stage_group, int32_t *stage_tp,
                                                           int32_t *n_passes, unsigned char *ws,
                                                           size_t per_group, int64_t n_dev, int *ticket) {
    mesh_body<kExact, kFast>(tb, od, out, stage_group, stage_tp, n_passes, ws, per_group, n_dev, ticket);
}

template <bool kFast>
__device__ __forceinline__ void mesh_h1_body(const TablesDev &tb, const OrdDev &od, const int64_t *t_max,
                                             const PlansDev &out, int32_t *stage_group, int32_t *stage_tp,
                                             int32_t *warmup, unsigned char *ws, size_t per_group, int64_t n_dev,
                                             int *ticket) {
    __shared__ int32_t offs[kMaxOrderGroups + 1];
    __shared__ uint16_t order[kMaxOrderGroups];
    __shared__ uint16_t group_at[kMeshGroupTable];
    extern __shared__ __align__(16) unsigned char mesh_lds[];      // fast form: PP and PS, L + 1 entries each
    int64_t *sums_lds = reinterpret_cast<int64_t *>(mesh_lds);
    __shared__ int32_t cuts[kMaxStages + 1], count[kMaxStages];
    __shared__ uint16_t slot_g[kMaxStages];
    __shared__ uint8_t slot_k[kMaxStages];
    __shared__ int32_t slot_first[kMaxStages];
    __shared__ int shared_int[2];
    const int L = tb.L, S_max = od.S_max;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x;
    const MeshSlice m = mesh_slice(ws, per_group, L, n_dev);
    const int64_t m_cap = tb.M;

    for (;;) {
        __syncthreads();
        if (tid == 0) shared_int[0] = atomicAdd(ticket, 1);
        __syncthreads();
        const int c = shared_int[0];
        if (c >= od.C) break;
        const int S = od.ord_S[c], K = od.ord_G[c];
        const int64_t cap = t_max[c];
        const int32_t *og = od.ord_group + int64_t(c) * od.G_max;
        int32_t *sg = stage_group + int64_t(c) * S_max, *stp = stage_tp + int64_t(c) * S_max;
        int32_t *wu = warmup + int64_t(c) * S_max;
        auto fail = [&](int status) {
            write_failed(out, c, S_max, status);
            for (int s = tid; s < S_max; s += nthreads) { sg[s] = -1; stp[s] = -1; wu[s] = -1; }
        };
        int bad = (S < 1 || S > S_max || K < 1 || K > od.G_max) ? 1 : 0;
        if (!bad)
            for (int k = tid; k < K; k += nthreads) {
                const int g = og[k];
                if (g < 0 || g >= tb.G) { bad = 1; continue; }
                for (int q = 0; q < k; ++q)
                    if (og[q] == g) bad = 1;
                order[k] = uint16_t(g);
            }
        if (__syncthreads_or(bad)) { fail(HARP_CAND_INVALID); continue; }
        if (cap_out_of_range(tb, cap)) { fail(HARP_CAND_INVALID); continue; }
        if (tid == 0) {
            int64_t o = 0;
            offs[0] = 0;
            for (int k = 0; k < K; ++k) { o += tb.group_ndev[order[k]]; offs[k + 1] = int32_t(o); }
        }
        __syncthreads();
        const int Dtot = offs[K];
        if (S > L || S < K || S > Dtot || cap < 0) { fail(HARP_CAND_INFEASIBLE); continue; }
        if (Dtot <= kMeshGroupTable) {
            for (int k = 0; k < K; ++k)
                for (int d = offs[k] + tid; d < offs[k + 1]; d += nthreads) group_at[d] = uint16_t(k);
        }
        int64_t sum;
        if constexpr (kFast) sum = mesh_h1_pass_fast(tb, m, offs, order, group_at, sums_lds, K, S, n_dev, cap);
        else sum = mesh_h1_pass(tb, m, offs, order, group_at, K, S, n_dev, cap);
        if (sum == kInf) { fail(HARP_CAND_INFEASIBLE); continue; }
        if (tid == 0) mesh_h1_backtrack<kFast>(tb, m, offs, order, K, S, n_dev, cap, cuts, slot_g, slot_k, slot_first, count);
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = tid; s <= S_max; s += nthreads) sp[s] = s <= S ? cuts[s] : -1;
        for (int s = tid; s < S_max; s += nthreads) {
            sg[s] = s < S ? int32_t(slot_g[s]) : -1;
            stp[s] = s < S ? tb.tp[slot_k[s]] : -1;
            df[s] = s < S ? slot_first[s] : -1;
            wu[s] = s < S ? count[s] : -1;
        }
        if (wave == 0) {
            int64_t bott, iter;
            wave_score_partition(tb, S, slot_g, slot_k, cuts, lane, bott, iter);   // the plan's own bottleneck
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = sum + (m_cap - 1) * cap;
                out.status[c] = HARP_CAND_OK;
            }
        }
    }
}

template <bool kFast>
__global__ __launch_bounds__(kMeshMaxThreads) void k2_mesh_h1f1b(TablesDev tb, OrdDev od, const int64_t *t_max,
                                                                 PlansDev out, int32_t *stage_group,
                                                                 int32_t *stage_tp, int32_t *warmup,
                                                                 unsigned char *ws, size_t per_group,
                                                                 int64_t n_dev, int *ticket) {
    mesh_h1_body<kFast>(tb, od, t_max, out, stage_group, stage_tp, warmup, ws, per_group, n_dev, ticket);
}

__global__ void k2_mesh_clear(int *ticket) {
    if (threadIdx.x < 4) ticket[threadIdx.x] = 0;
}

}  // namespace

// A stage has up to L x devices target cells: small tables get many small workgroups (more
// orderings in flight), large ones few large workgroups (more lanes per ordering).
int plan_mesh_threads(int L, int64_t total_devices, int C, int n_cu) {
    if (int64_t(L + 1) * (total_devices + 1) >= 16384) return kMeshMaxThreads;
    // a batch too small to fill the chip with 256-thread workgroups gets more lanes per ordering
    if (C <= 2 * n_cu) return kMeshMaxThreads;
    if (C <= 4 * n_cu) return 512;
    return 256;
}

// Per-workgroup slice: two rows of the table, the back-pointers, and (first slice only) the ticket.
size_t plan_mesh_ws_per_group(int L, int S_max, int64_t total_devices) {
    const size_t row = size_t(total_devices + 1) * size_t(L + 1);
    size_t b = 2 * row * sizeof(int64_t) + 2 * row * sizeof(int32_t) + size_t(S_max) * row * sizeof(uint32_t);
    return (b + 255) & ~size_t(255);
}

void launch_plan_mesh(const TablesDev &tb, const OrdDev &od, const PlansDev &out, int32_t *stage_group,
                      int32_t *stage_tp, int32_t *n_passes, bool exact, bool fast32, void *ws, int n_groups,
                      int threads, int64_t total_devices, hipStream_t st) {
    // layout: 256 bytes for the ticket, then the slices
    int *ticket = static_cast<int *>(ws);
    unsigned char *slices = static_cast<unsigned char *>(ws) + 256;
    const size_t per_group = plan_mesh_ws_per_group(tb.L, od.S_max, total_devices);
    const dim3 grid(n_groups), block(threads);
    fast32 = fast32 && tb.L <= kMeshFastMaxL;      // the fast form keeps L + 1 memory sums in LDS
    const size_t lds = fast32 ? size_t(tb.L + 1) * sizeof(int64_t) : 0;
    hipLaunchKernelGGL(k2_mesh_clear, dim3(1), dim3(64), 0, st, ticket);
#define HARP_MESH_LAUNCH(E, F)                                                                            \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(k2_mesh<E, F>), grid, block, lds, st, tb, od, out, stage_group, stage_tp, \
                       n_passes, slices, per_group, total_devices, ticket)
    if (exact && fast32) HARP_MESH_LAUNCH(true, true);
    else if (exact) HARP_MESH_LAUNCH(true, false);
    else if (fast32) HARP_MESH_LAUNCH(false, true);
    else HARP_MESH_LAUNCH(false, false);
#undef HARP_MESH_LAUNCH
}

void launch_plan_mesh_h1f1b(const TablesDev &tb, const OrdDev &od, const int64_t *t_max, const PlansDev &out,
                            int32_t *stage_group, int32_t *stage_tp, int32_t *warmup, bool fast32, void *ws,
                            int n_groups, int threads, int64_t total_devices, hipStream_t st) {
    int *ticket = static_cast<int *>(ws);
    unsigned char *slices = static_cast<unsigned char *>(ws) + 256;
    const size_t per_group = plan_mesh_ws_per_group(tb.L, od.S_max, total_devices);
    const dim3 grid(n_groups), block(threads);
    fast32 = fast32 && tb.L <= kMeshFastMaxL;      // the fast form keeps 2 (L + 1) running sums in LDS
    const size_t lds = fast32 ? 2 * size_t(tb.L + 1) * sizeof(int64_t) : 0;
    hipLaunchKernelGGL(k2_mesh_clear, dim3(1), dim3(64), 0, st, ticket);
    if (fast32)
        hipLaunchKernelGGL(HIP_KERNEL_NAME(k2_mesh_h1f1b<true>), grid, block, lds, st, tb, od, t_max, out, stage_group,
                           stage_tp, warmup, slices, per_group, total_devices, ticket);
    else
        hipLaunchKernelGGL(HIP_KERNEL_NAME(k2_mesh_h1f1b<false>), grid, block, 0, st, tb, od, t_max, out,
                           stage_group, stage_tp, warmup, slices, per_group, total_devices, ticket);
}

}  // namespace harp
