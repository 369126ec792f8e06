// The search over the cap around the full recurrence (paper section 5.2.4 (2), (3)): the kernels of
// harp_plan_mesh_h1f1b_sweep_batch (orderings) and harp_plan_h1f1b_sweep_batch (candidates with a fixed
// slicing).  The passes themselves are in mesh_passes.h.
#include "mesh_passes.h"

namespace harp {

using namespace meshdp;

namespace {

// The smallest candidate cap above b (section 5.2.4 (2)).  Candidate caps are stage times of
// (group, degree) rows over every operator range, and transfer times of the inner cuts on some
// links; which rows and links is up to the caller (row_of(r, g, q) and link_of(r, g, h) return
// false for entries to skip).  A stage time grows with its end cut, so per (row, start cut) the
// first time above b is found by a binary search, or, when the caller lends a position array
// (pos, one entry per (row, start cut), filled by a call with fresh = true), by moving the
// position kept from the previous call forward: within one sweep b only rises, so the positions
// only advance and a call costs about one table read per entry.  Transfer times are looked at one
// by one.  Every thread takes part; kInf when there is none.
template <bool kFast, typename RowFn, typename LinkFn>
__device__ __forceinline__ int64_t next_cap_over(const TablesDev &tb, int n_rows, RowFn row_of, int n_links,
                                                 LinkFn link_of, int64_t b, unsigned long long *slot,
                                                 uint16_t *pos, bool fresh) {
    const int L = tb.L, tid = threadIdx.x, nthreads = blockDim.x;
    __syncthreads();
    if (tid == 0) *slot = ~0ull;
    __syncthreads();
    unsigned long long least = ~0ull;
    for (int x = tid; x < n_rows * L; x += nthreads) {
        const int j = x % L, r = x / L;
        int g, q;
        if (!row_of(r, g, q)) continue;
        const int64_t tp = tb.tp[q];
        const int shift = tb.tp_shift[q];
        const uint32_t *p32 = kFast ? tb.P32 + (int64_t(g) * tb.n_tp + q) * tb.pitch32 : nullptr;
        const int64_t *pf = tb.PF(tb.group_type[g]), *pr = tb.PR(g, q);
        auto time_to = [&](int i) -> int64_t {
            if (kFast) return int64_t((p32[i] + uint32_t(tp) - 1u - p32[j]) >> shift);
            const int64_t work = pf[i] - pf[j];
            return (shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp) + (pr[i] - pr[j]);
        };
        int i;                                        // first end cut whose time is above b; L + 1: none
        if (pos && !fresh) {
            i = pos[x];
            while (i <= L && time_to(i) <= b) ++i;
        } else if (time_to(L) <= b) {
            i = L + 1;
        } else {
            int lo = j + 1, hi = L;                   // time_to(hi) > b
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (time_to(mid) > b) hi = mid; else lo = mid + 1;
            }
            i = hi;
        }
        if (pos) pos[x] = uint16_t(i);
        if (i <= L) {
            const unsigned long long v = (unsigned long long)time_to(i);
            least = v < least ? v : least;
        }
    }
    if (L >= 2) {
        for (int x = tid; x < n_links * (L - 1); x += nthreads) {
            const int i = 1 + x % (L - 1), r = x / (L - 1);
            int g, h;
            if (!link_of(r, g, h)) continue;
            int64_t v;
            if (kFast) {
                v = tb.CM[(int64_t(g) * tb.G + h) * tb.pitch32 + i];
            } else {
                const int64_t link = tb.bw[int64_t(g) * tb.G + h];
                v = (tb.act_bytes[i - 1] + link - 1) / link;
            }
            if (v > b && (unsigned long long)v < least) least = (unsigned long long)v;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t lo = __shfl_xor(uint32_t(least), d, 64), hi = __shfl_xor(uint32_t(least >> 32), d, 64);
        const unsigned long long o = ((unsigned long long)hi << 32) | lo;
        least = o < least ? o : least;
    }
    if ((tid & 63) == 0 && least != ~0ull) atomicMin(slot, least);
    __syncthreads();
    const unsigned long long v = *slot;
    return v == ~0ull ? kInf : int64_t(v);
}

// Candidate caps of an ordering: the stage times of every listed group and usable degree, and the
// transfer times on the links the ordering can use (inside a group, and to the group after it).
template <bool kFast>
__device__ __forceinline__ int64_t mesh_next_cap(const TablesDev &tb, const uint16_t *order, int K, int64_t b,
                                                 unsigned long long *slot, uint16_t *pos, bool fresh) {
    auto row_of = [&](int r, int &g, int &q) -> bool {
        q = r % tb.n_tp;
        g = order[r / tb.n_tp];
        return tb.tp[q] <= tb.group_ndev[g];
    };
    auto link_of = [&](int r, int &g, int &h) -> bool {
        const int k = r >> 1;
        if ((r & 1) && k + 1 >= K) return false;
        g = order[k];
        h = (r & 1) ? order[k + 1] : g;
        return true;
    };
    return next_cap_over<kFast>(tb, K * tb.n_tp, row_of, 2 * K, link_of, b, slot, pos, fresh);
}

// Candidate caps of a fixed slicing: the stage times of the slots (group and degree of every stage
// given) and the transfer times on the links between consecutive slots.
template <bool kFast>
__device__ __forceinline__ int64_t mesh_next_cap_slots(const TablesDev &tb, int S, const uint16_t *stage_g,
                                                       const uint8_t *stage_q, int64_t b, unsigned long long *slot,
                                                       uint16_t *pos, bool fresh) {
    auto row_of = [&](int r, int &g, int &q) -> bool {
        g = stage_g[r];
        q = stage_q[r];
        return true;
    };
    auto link_of = [&](int r, int &g, int &h) -> bool {
        g = stage_g[r];
        h = stage_g[r + 1];
        return true;
    };
    return next_cap_over<kFast>(tb, S, row_of, S - 1, link_of, b, slot, pos, fresh);
}

// The search around the full recurrence (section 5.2.4 (2)), with the caps of one ordering shared
// by several workgroups (the batched evaluation of 5.2.4 (3)).  The k-th candidate value at or
// above t_S has index k whoever tries it.
//  lower:  one workgroup per ordering checks it, runs the classic min-max pass for the lower end
//          t_S (no cap below it admits a plan, and H-1F1B's counts are never below the classic
//          ones) and tries t_S itself, which has a plan for most orderings;
//  climb:  for the others, W walkers per ordering walk the caps upwards from index 1, walker j
//          running the H-1F1B pass on the indices congruent to j until one has a plan; the lowest
//          such index is kept as an atomic minimum, and a walker stops once it is above it;
//  open:   the walker with the lowest index hands its plan over; it fixes t_E = ceil(T / B);
//  rest:   W walkers per ordering walk ALL later caps up to t_E (finding the next cap costs a few
//          percent of a pass) and run the H-1F1B pass on their own indices, keeping their best plan;
//  pick:   per ordering the smallest T = least sum + (B - 1) cap over the kept plans, the lower cap
//          on equal T; that is what trying the caps one after the other returns.
// The limit max_caps cuts the sweep at the same cap for every W.
struct SweepHead {
    int64_t T, cap;
    int32_t tried, state;    // state: kSweepNone, kSweepPlan, or kSweepFailed + a candidate status
    int32_t pad[2];
};
constexpr int kSweepNone = 0, kSweepPlan = 1, kSweepFailed = 16;

// One kept plan: head | cuts [S_max + 1] | first device [S_max] | count [S_max] (int32) | group
// [S_max] (uint16) | degree index [S_max] (uint8), rounded up to 16 bytes.
__host__ __device__ inline size_t sweep_slot_bytes(int S_max) {
    const size_t b = sizeof(SweepHead) + 4 * size_t(3 * S_max + 1) + 2 * size_t(S_max) + size_t(S_max);
    return (b + 15) & ~size_t(15);
}
struct SweepSlot {
    SweepHead *head;
    int32_t *cuts, *first, *count;
    uint16_t *g;
    uint8_t *k;
};
__device__ __forceinline__ SweepSlot sweep_slot(unsigned char *slots, int S_max, int W, int c, int j) {
    unsigned char *base = slots + (size_t(c) * size_t(W + 1) + size_t(j)) * sweep_slot_bytes(S_max);
    SweepSlot t;
    t.head = reinterpret_cast<SweepHead *>(base);
    t.cuts = reinterpret_cast<int32_t *>(base + sizeof(SweepHead));
    t.first = t.cuts + (S_max + 1);
    t.count = t.first + S_max;
    t.g = reinterpret_cast<uint16_t *>(t.count + S_max);
    t.k = reinterpret_cast<uint8_t *>(t.g + S_max);
    return t;
}

// kRest = false: the first launch (ticket over orderings).  kRest = true: the second (ticket over
// ordering x W).
// kForced: the batch holds candidates with a fixed slicing (od.ord_S = their stage counts, slot
// lists in cand_group / cand_tp): every stage's group and degree are given, so each stage has one
// device offset and one degree, and the candidate values are those of the slots and of the links
// between consecutive slots.
// kPhase: kSweepLower (one item per ordering: validity and t_S), kSweepClimb, kSweepRest (W items per
// ordering each).  Ws is the number of walker slots per ordering in the workspace (the largest W of
// the phases); slot Ws holds the opening.
constexpr int kSweepLower = 0, kSweepClimb = 1, kSweepRest = 2;
template <bool kFast, int kPhase, bool kForced>
__device__ __forceinline__ void mesh_sweep_body(const TablesDev &tb, const OrdDev &od, const int32_t *cand_group,
                                                const int32_t *cand_tp, int max_caps, int W, int Ws,
                                                unsigned char *slots, int *first_idx, int64_t *lower,
                                                unsigned char *ws, size_t per_group, int64_t n_dev, int *ticket,
                                                size_t pos_bytes) {
    constexpr bool kRest = kPhase == kSweepRest;
    // fast form: PP and PS (or Q), L + 1 entries each; then pos_bytes of cap positions
    extern __shared__ __align__(16) unsigned char mesh_lds[];
    int64_t *sums_lds = reinterpret_cast<int64_t *>(mesh_lds);
    uint16_t *pos_lds = reinterpret_cast<uint16_t *>(mesh_lds + (kFast ? 2 * size_t(tb.L + 1) * sizeof(int64_t) : 0));
    __shared__ int32_t offs[kMaxOrderGroups + 1];
    __shared__ uint16_t order[kMaxOrderGroups];
    __shared__ uint16_t group_at[kMeshGroupTable];
    __shared__ int32_t cuts[kMaxStages + 1], count[kMaxStages];
    __shared__ uint16_t slot_g[kMaxStages];
    __shared__ uint8_t slot_k[kMaxStages];
    __shared__ int32_t slot_first[kMaxStages];
    __shared__ int shared_int[2];
    __shared__ unsigned long long next_slot;
    __shared__ uint8_t forced_q[kForced ? kMaxStages : 1];          // degree index of every stage
    __shared__ uint16_t forced_g[kForced ? kMaxStages : 1];         // group of every stage
    __shared__ int32_t forced_off[kForced ? kMaxStages + 1 : 1];    // device offset of every stage
    const int L = tb.L, S_max = od.S_max;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const MeshSlice m = mesh_slice(ws, per_group, L, n_dev);
    const int64_t m_cap = tb.M;
    const int n_items = od.C * W;
    const uint8_t *fq = kForced ? forced_q : nullptr;
    const int32_t *fo = kForced ? forced_off : nullptr;

    for (;;) {
        __syncthreads();
        if (tid == 0) shared_int[0] = atomicAdd(ticket, 1);
        __syncthreads();
        const int item = shared_int[0];
        if (item >= n_items) break;
        const int c = item / W, j = item - c * W;
        const SweepSlot opening = sweep_slot(slots, S_max, Ws, c, Ws);
        const SweepSlot mine = kPhase == kSweepLower ? opening : sweep_slot(slots, S_max, Ws, c, j);
        auto leave = [&](int state, int tried) {
            if (tid == 0) { mine.head->T = kInf; mine.head->cap = kInf; mine.head->tried = tried; mine.head->state = state; }
        };
        int64_t cap = 0, t_E = kInf;
        int tried = 0;
        if (kPhase == kSweepClimb) {
            // the first launch found this ordering malformed or without any plan: nothing to climb
            if (opening.head->state != kSweepNone) { leave(kSweepNone, 0); continue; }
        }
        if (kRest) {
            // what the first launch found for this ordering (written before this kernel started)
            if (opening.head->state != kSweepPlan) { leave(kSweepNone, opening.head->tried); continue; }
            cap = opening.head->cap;
            tried = opening.head->tried;
            t_E = (opening.head->T + m_cap - 1) / m_cap;
        }
        const int S = od.ord_S[c];
        int K;
        if constexpr (kForced) {
            // the slot list: stages in range, groups and degrees known, slots of a group adjacent and
            // within the group's devices; the groups in order of appearance are the ordering
            int bad = (S < 1 || S > S_max) ? 1 : 0;
            if (tid == 0 && !bad) {
                const int32_t *grp = cand_group + int64_t(c) * S_max, *tpv = cand_tp + int64_t(c) * S_max;
                int k = -1, used = 0;
                forced_off[0] = 0;
                for (int st = 0; st < S && !bad; ++st) {
                    const int g = grp[st];
                    int q = -1;
                    for (int x = 0; x < tb.n_tp; ++x)
                        if (tb.tp[x] == tpv[st]) q = x;
                    if (g < 0 || g >= tb.G || q < 0) { bad = 1; break; }
                    if (k < 0 || order[k] != g) {                  // first slot of a run of group g
                        for (int x = 0; x <= k; ++x)
                            if (order[x] == g) bad = 1;            // the group was left and entered again
                        if (k >= 0) offs[k + 1] = forced_off[st];
                        ++k;
                        order[k] = uint16_t(g);
                        used = 0;
                    }
                    used += tpv[st];
                    if (used > tb.group_ndev[g]) bad = 1;
                    forced_q[st] = uint8_t(q);
                    forced_g[st] = uint16_t(g);
                    forced_off[st + 1] = forced_off[st] + tpv[st];
                }
                offs[0] = 0;
                if (!bad) offs[k + 1] = forced_off[S];
                shared_int[1] = k + 1;
            }
            if (__syncthreads_or(bad)) { leave(kSweepFailed + HARP_CAND_INVALID, 0); continue; }
            K = shared_int[1];
        } else {
            K = od.ord_G[c];
            const int32_t *og = od.ord_group + int64_t(c) * od.G_max;
            int bad = (S < 1 || S > S_max || K < 1 || K > od.G_max) ? 1 : 0;
            if (!bad)
                for (int k = tid; k < K; k += nthreads) {
                    const int g = og[k];
                    if (g < 0 || g >= tb.G) { bad = 1; continue; }
                    for (int q = 0; q < k; ++q)
                        if (og[q] == g) bad = 1;
                    order[k] = uint16_t(g);
                }
            if (__syncthreads_or(bad)) { leave(kSweepFailed + HARP_CAND_INVALID, 0); continue; }
            if (tid == 0) {
                int64_t o = 0;
                offs[0] = 0;
                for (int k = 0; k < K; ++k) { o += tb.group_ndev[order[k]]; offs[k + 1] = int32_t(o); }
            }
            __syncthreads();
        }
        const int Dtot = offs[K];
        if (S > L || S < K || S > Dtot) { leave(kSweepFailed + HARP_CAND_INFEASIBLE, 0); continue; }
        if (Dtot <= kMeshGroupTable) {
            for (int k = 0; k < K; ++k)
                for (int d = offs[k] + tid; d < offs[k + 1]; d += nthreads) group_at[d] = uint16_t(k);
        }
        auto h1_pass = [&](int64_t at) -> int64_t {
            if constexpr (kFast) return mesh_h1_pass_fast(tb, m, offs, order, group_at, sums_lds, K, S, n_dev, at, fq, fo);
            else return mesh_h1_pass(tb, m, offs, order, group_at, K, S, n_dev, at, fq, fo);
        };
        // positions of the candidate values, kept between calls when this item's rows fit in the array
        const int cap_rows = kForced ? S : K * tb.n_tp;
        uint16_t *pos = (L < 65535 && size_t(cap_rows) * size_t(L) * sizeof(uint16_t) <= pos_bytes) ? pos_lds : nullptr;
        bool fresh = true;
        auto next_cap = [&](int64_t after) -> int64_t {
            const bool first_call = fresh;
            fresh = false;
            if constexpr (kForced) return mesh_next_cap_slots<kFast>(tb, S, forced_g, forced_q, after, &next_slot, pos, first_call);
            else return mesh_next_cap<kFast>(tb, order, K, after, &next_slot, pos, first_call);
        };
        // thread 0 backtracks the pass just run; everyone copies the plan to this item's slot
        auto keep = [&](int64_t at, int64_t T) {
            if (tid == 0)
                mesh_h1_backtrack<kFast>(tb, m, offs, order, K, S, n_dev, at, cuts, slot_g, slot_k, slot_first, count);
            __syncthreads();
            for (int s = tid; s <= S; s += nthreads) mine.cuts[s] = cuts[s];
            for (int s = tid; s < S; s += nthreads) {
                mine.g[s] = slot_g[s]; mine.k[s] = slot_k[s]; mine.first[s] = slot_first[s]; mine.count[s] = count[s];
            }
            if (tid == 0) { mine.head->T = T; mine.head->cap = at; }
        };
        if constexpr (kPhase == kSweepLower) {
            // validity (checked above), the lower end of the sweep, and the cap of index 0 (t_S itself),
            // which has a plan for most orderings: then the climb has nothing left to do
            int64_t t_S;
            if constexpr (kFast) t_S = mesh_pass_fast<false>(tb, m, offs, order, group_at, sums_lds, K, S, n_dev, 0, fq, fo);
            else t_S = mesh_pass<false>(tb, m, offs, order, group_at, K, S, n_dev, 0, fq, fo);
            if (t_S == kInf) { leave(kSweepFailed + HARP_CAND_INFEASIBLE, 0); continue; }
            const int64_t sum = h1_pass(t_S);
            if (sum != kInf) {
                keep(t_S, sum + (m_cap - 1) * t_S);
                if (tid == 0) { mine.head->tried = 1; mine.head->state = kSweepPlan; }
            } else {
                if (tid == 0) lower[c] = t_S;
                leave(kSweepNone, 1);
            }
        } else if constexpr (kPhase == kSweepClimb) {
            // the climb from t_S (index 0, tried without a plan by the first launch) to the first cap
            // with a plan, shared by the W walkers of the ordering: each walks every cap and tries
            // those whose index is congruent to its own; the lowest index found so far (first_idx, an
            // atomic minimum) tells the others where to stop.  Every index below the final minimum
            // has been tried by its walker and has no plan.
            cap = lower[c];
            tried = 1;
            int state = kSweepFailed + HARP_CAND_INFEASIBLE;
            for (int idx = 1;; ++idx) {
                if (tried >= max_caps) break;
                const int64_t nb = next_cap(cap);
                if (nb == kInf) break;
                cap = nb;
                __syncthreads();
                if (tid == 0) shared_int[1] = atomicAdd(&first_idx[c], 0);
                __syncthreads();
                if (idx > shared_int[1]) { state = kSweepNone; break; }        // a lower cap already has a plan
                tried = idx + 1;
                if ((idx - 1) % W != j) continue;
                const int64_t sum = h1_pass(cap);
                if (sum == kInf) continue;
                keep(cap, sum + (m_cap - 1) * cap);
                if (tid == 0) atomicMin(&first_idx[c], idx);
                state = kSweepPlan;
                break;
            }
            if (state != kSweepPlan) { leave(state, tried); continue; }
            if (tid == 0) { mine.head->tried = tried; mine.head->state = kSweepPlan; }
        } else {
            int64_t best_T = kInf;
            for (int step = 0; tried < max_caps; ++step) {
                const int64_t nb = next_cap(cap);
                if (nb == kInf || nb > t_E) break;
                cap = nb;
                ++tried;
                if (step % W != j) continue;
                const int64_t sum = h1_pass(cap);
                if (sum == kInf) continue;
                const int64_t T = sum + (m_cap - 1) * cap;
                if (T < best_T) {                      // caps rise, so the lower cap keeps an equal T
                    best_T = T;
                    keep(cap, T);
                }
            }
            if (best_T == kInf) { leave(kSweepNone, tried); continue; }
            if (tid == 0) { mine.head->tried = tried; mine.head->state = kSweepPlan; }
        }
    }
}

template <bool kFast, int kPhase, bool kForced>
__global__ __launch_bounds__(kMeshMaxThreads) void k2_mesh_h1f1b_sweep(TablesDev tb, OrdDev od,
                                                                       const int32_t *cand_group,
                                                                       const int32_t *cand_tp, int max_caps, int W,
                                                                       int Ws, unsigned char *slots, int *first_idx,
                                                                       int64_t *lower, unsigned char *ws,
                                                                       size_t per_group, int64_t n_dev, int *ticket,
                                                                       size_t pos_bytes) {
    mesh_sweep_body<kFast, kPhase, kForced>(tb, od, cand_group, cand_tp, max_caps, W, Ws, slots, first_idx, lower, ws,
                                            per_group, n_dev, ticket, pos_bytes);
}

// After the climb, one wavefront per ordering that the climb had to work on: the walker that found
// the lowest cap with a plan (index first_idx, walker (first_idx - 1) mod W) hands its plan over as
// the opening of the sweep; without one, the opening carries walker 0's verdict and count of caps
// tried.
__global__ __launch_bounds__(256) void k2_mesh_sweep_open(OrdDev od, int W, int Ws, unsigned char *slots,
                                                          const int *first_idx) {
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (c >= od.C) return;
    const int S_max = od.S_max;
    const SweepSlot opening = sweep_slot(slots, S_max, Ws, c, Ws);
    if (opening.head->state != kSweepNone) return;        // malformed, or no plan even with the classic counts
    const int f = first_idx[c];
    const SweepSlot from = sweep_slot(slots, S_max, Ws, c, f == INT32_MAX ? 0 : (f - 1) % W);
    if (f != INT32_MAX) {
        for (int s = lane; s <= S_max; s += 64) opening.cuts[s] = from.cuts[s];
        for (int s = lane; s < S_max; s += 64) {
            opening.first[s] = from.first[s]; opening.count[s] = from.count[s];
            opening.g[s] = from.g[s]; opening.k[s] = from.k[s];
        }
    }
    if (lane == 0) {
        opening.head->T = from.head->T;
        opening.head->cap = from.head->cap;
        opening.head->tried = f == INT32_MAX ? from.head->tried : f + 1;
        opening.head->state = from.head->state;
    }
}

__global__ void k2_mesh_sweep_clear(int *ticket, int *first_idx, int C) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < 4) ticket[c] = 0;                    // one ticket per launch of the search
    if (c < C) first_idx[c] = INT32_MAX;
}

// One wavefront per ordering: the best of its W + 1 kept plans goes to the outputs.
__global__ __launch_bounds__(256) void k2_mesh_sweep_pick(TablesDev tb, OrdDev od, int W, int Ws, unsigned char *slots,
                                                          PlansDev out, int32_t *stage_group, int32_t *stage_tp,
                                                          int32_t *warmup, int64_t *t_max_out, int32_t *n_caps) {
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (c >= od.C) return;
    const int S_max = od.S_max;
    int32_t *sp = out.splits + int64_t(c) * (S_max + 1), *df = out.dev_first + int64_t(c) * S_max;
    // a batch of candidates (fixed slicing) has no slicing to report
    int32_t *sg = stage_group ? stage_group + int64_t(c) * S_max : nullptr;
    int32_t *stp = stage_tp ? stage_tp + int64_t(c) * S_max : nullptr;
    int32_t *wu = warmup + int64_t(c) * S_max;
    const SweepSlot opening = sweep_slot(slots, S_max, Ws, c, Ws);
    if (opening.head->state != kSweepPlan) {
        for (int s = lane; s <= S_max; s += 64) sp[s] = -1;
        for (int s = lane; s < S_max; s += 64) {
            df[s] = -1; wu[s] = -1;
            if (sg) sg[s] = -1;
            if (stp) stp[s] = -1;
        }
        if (lane == 0) {
            out.bottleneck[c] = kInf;
            out.iter_time[c] = kInf;
            out.status[c] = opening.head->state - kSweepFailed;
            t_max_out[c] = kInf;
            if (n_caps) n_caps[c] = opening.head->tried;
        }
        return;
    }
    int best = Ws;
    int64_t best_T = opening.head->T, best_cap = opening.head->cap;
    for (int j = 0; j < W; ++j) {
        const SweepHead *h = sweep_slot(slots, S_max, Ws, c, j).head;
        if (h->state == kSweepPlan && (h->T < best_T || (h->T == best_T && h->cap < best_cap))) {
            best = j; best_T = h->T; best_cap = h->cap;
        }
    }
    const SweepSlot b = sweep_slot(slots, S_max, Ws, c, best);
    const int S = od.ord_S[c];
    for (int s = lane; s <= S_max; s += 64) sp[s] = s <= S ? b.cuts[s] : -1;
    for (int s = lane; s < S_max; s += 64) {
        if (sg) sg[s] = s < S ? int32_t(b.g[s]) : -1;
        if (stp) stp[s] = s < S ? tb.tp[b.k[s]] : -1;
        df[s] = s < S ? b.first[s] : -1;
        wu[s] = s < S ? b.count[s] : -1;
    }
    int64_t bott, iter;
    wave_score_partition(tb, S, b.g, b.k, b.cuts, lane, bott, iter);      // the plan's own bottleneck
    if (lane == 0) {
        out.bottleneck[c] = bott;
        out.iter_time[c] = best_T;
        out.status[c] = HARP_CAND_OK;
        t_max_out[c] = best_cap;
        if (n_caps) n_caps[c] = sweep_slot(slots, S_max, Ws, c, 0).head->tried;
    }
}


}  // namespace

// cand_group / cand_tp not null: the batch holds candidates with a fixed slicing (od.ord_S = their
// stage counts), and stage_group / stage_tp may be null.  W_climb and W walkers per ordering in the
// climb and in the rest of the sweep.
void launch_plan_mesh_h1f1b_sweep(const TablesDev &tb, const OrdDev &od, const int32_t *cand_group,
                                  const int32_t *cand_tp, int max_caps, const PlansDev &out,
                                  int32_t *stage_group, int32_t *stage_tp, int32_t *warmup, int64_t *t_max_out,
                                  int32_t *n_caps, bool fast32, void *ws, int n_groups, int threads, int W_climb,
                                  int W, int64_t total_devices, hipStream_t st) {
    // layout: 256 bytes for the tickets | n_groups slices | (Ws + 1) kept plans per ordering | t_S per
    // ordering | index of the first cap with a plan per ordering
    int *ticket = static_cast<int *>(ws);
    unsigned char *slices = static_cast<unsigned char *>(ws) + 256;
    const size_t per_group = plan_mesh_ws_per_group(tb.L, od.S_max, total_devices);
    const int Ws = W_climb > W ? W_climb : W;
    unsigned char *slots = slices + size_t(n_groups) * per_group;
    int64_t *lower = reinterpret_cast<int64_t *>(slots + size_t(od.C) * size_t(Ws + 1) * sweep_slot_bytes(od.S_max));
    int *first_idx = reinterpret_cast<int *>(lower + od.C);
    fast32 = fast32 && tb.L <= kMeshFastMaxL;
    const bool forced = cand_group != nullptr;
    // cap positions: one uint16 per (row, start cut), kept in LDS when the largest item's rows fit
    // beside the static arrays in a workgroup's 64 KiB
    const size_t sums = fast32 ? 2 * size_t(tb.L + 1) * sizeof(int64_t) : 0;
    const size_t rows_max = forced ? size_t(od.S_max) : size_t(tb.G) * size_t(tb.n_tp);
    size_t pos_bytes = (rows_max * size_t(tb.L) * sizeof(uint16_t) + 15) & ~size_t(15);
    if (sums + pos_bytes > (size_t(40) << 10)) pos_bytes = 0;
    const size_t lds = sums + pos_bytes;
    const dim3 block(threads);
    auto grid_for = [&](long long items) { return dim3(unsigned(items < n_groups ? items : n_groups)); };
    hipLaunchKernelGGL(k2_mesh_sweep_clear, dim3((od.C + 255) / 256), dim3(256), 0, st, ticket, first_idx, od.C);
#define HARP_SWEEP_PHASE(F, P, X, WALKERS, TICKET)                                                               \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(k2_mesh_h1f1b_sweep<F, P, X>), grid_for((long long)od.C * (WALKERS)), block,  \
                       lds, st, tb, od, cand_group, cand_tp, max_caps, WALKERS, Ws, slots, first_idx, lower, slices, \
                       per_group, total_devices, ticket + (TICKET), pos_bytes)
#define HARP_SWEEP_LAUNCH(F, X)                                                                                  \
    HARP_SWEEP_PHASE(F, kSweepLower, X, 1, 0);                                                                    \
    HARP_SWEEP_PHASE(F, kSweepClimb, X, W_climb, 1);                                                              \
    hipLaunchKernelGGL(k2_mesh_sweep_open, dim3((od.C + 3) / 4), dim3(256), 0, st, od, W_climb, Ws, slots,        \
                       first_idx);                                                                                \
    HARP_SWEEP_PHASE(F, kSweepRest, X, W, 2)
    if (fast32 && forced) { HARP_SWEEP_LAUNCH(true, true); }
    else if (fast32) { HARP_SWEEP_LAUNCH(true, false); }
    else if (forced) { HARP_SWEEP_LAUNCH(false, true); }
    else { HARP_SWEEP_LAUNCH(false, false); }
#undef HARP_SWEEP_LAUNCH
#undef HARP_SWEEP_PHASE
    hipLaunchKernelGGL(k2_mesh_sweep_pick, dim3((od.C + 3) / 4), dim3(256), 0, st, tb, od, W, Ws, slots, out,
                       stage_group, stage_tp, warmup, t_max_out, n_caps);
}

size_t plan_mesh_sweep_slot_bytes(int S_max) { return sweep_slot_bytes(S_max); }

}  // namespace harp
