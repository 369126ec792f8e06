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
// (mesh_pass_fast, mesh_h1_pass_fast), chosen per launch.
#include <type_traits>

#include "harp_internal.h"
#include "fast_common.h"
#include "plan_common.h"

namespace harp {

namespace {

constexpr int kMeshMaxThreads = 1024;   // workgroup size is chosen per launch: 256 or 1024

struct MeshSlice {
    int64_t *D0, *D1;    // [devices + 1][L + 1]
    int32_t *N0, *N1;    // [devices + 1][L + 1]: warm-up counts (H-1F1B form only)
    uint32_t *arg;       // [S_max][devices + 1][L + 1]: j | degree index << 16
};

__device__ __forceinline__ MeshSlice mesh_slice(unsigned char *ws, size_t per_group, int L, int64_t n_dev) {
    unsigned char *mine = ws + size_t(blockIdx.x) * per_group;
    const size_t row = size_t(n_dev + 1) * size_t(L + 1);
    MeshSlice m;
    m.D0 = reinterpret_cast<int64_t *>(mine);
    m.D1 = m.D0 + row;
    m.N0 = reinterpret_cast<int32_t *>(m.D1 + row);
    m.N1 = m.N0 + row;
    m.arg = reinterpret_cast<uint32_t *>(m.N1 + row);
    return m;
}

// One pass over all stages for the ordering in (offs, order), every thread of the workgroup taking
// part.  kCapped = false: min-max form.  kCapped = true: least sum of (t + 2c) over transitions
// whose stage and transfer times are at most cap.  Returns the value of the state (S, L, all
// devices); back-pointers are left in the slice.
constexpr int kMeshGroupTable = 2048;   // device offsets whose group index is kept in LDS

// This form works from the int64 rows (any degrees, any time width), with a division per transfer
// time; mesh_pass_fast below is the form for tables that have the 32-bit rows.
template <bool kCapped>
__device__ __forceinline__ int64_t mesh_pass(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                             const uint16_t *order, const uint16_t *group_at, int K, int S,
                                             int64_t n_dev, int64_t cap, const uint8_t *forced = nullptr,
                                             const int32_t *forced_off = nullptr) {
    const int L = tb.L, W = L + 1, tid = threadIdx.x, nthreads = blockDim.x;
    const int Dtot = offs[K];
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    int64_t *Dp = m.D0, *Dn = m.D1;
    __syncthreads();                                 // the previous pass is done with the rows
    for (int x = tid; x < (Dtot + 1) * W; x += nthreads) Dp[x] = kInf;
    __syncthreads();
    if (tid == 0) Dp[0] = 0;                         // no stage, no operator, no device
    for (int s = 0; s < S; ++s) {
        __syncthreads();                             // row s is complete
        const bool last = (s == S - 1);
        const int64_t n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
        // targets: i in [i_lo, i_hi], d' in [d_lo, d_hi]; every later stage needs an operator and a device
        const int i_lo = last ? L : s + 1, i_hi = L - (S - 1 - s);
        // a fixed slicing (forced) leaves one device offset per stage
        const int d_lo = forced ? forced_off[s + 1] : (last ? Dtot : s + 1);
        const int d_hi = forced ? forced_off[s + 1] : (last ? Dtot : Dtot - (S - 1 - s));
        const int n_i = i_hi - i_lo + 1, n_d = d_hi - d_lo + 1;
        uint32_t *arg_s = m.arg + size_t(s) * size_t(n_dev + 1) * W;
        for (int x = tid; x < n_i * n_d; x += nthreads) {
            const int i = i_lo + x % n_i, d2 = d_lo + x / n_i;
            int64_t best = kInf;
            int best_j = 0x7FFF, best_q = 0;
            // the group whose devices end at or after d2: the stage [d2 - tp, d2) must lie inside one group
            int k = 0;
            if (Dtot <= kMeshGroupTable) k = group_at[d2 - 1];     // the group of the stage's last device
            else while (offs[k + 1] < d2) ++k;                     // offs[k] < d2 <= offs[k + 1]
            const int g = order[k];
            const int t = tb.group_type[g];
            const int64_t *pf = tb.PF(t);
            const int64_t mem_dev = tb.type_mem[t];
            const int g_next = last ? g : (d2 == offs[k + 1] ? order[k + 1 < K ? k + 1 : k] : g);
            int64_t cut = 0;
            if (!last) {
                const int64_t link = tb.bw[int64_t(g) * tb.G + g_next];
                cut = (tb.act_bytes[i - 1] + link - 1) / link;
            }
            const int64_t pfi = pf[i], ppi = PP[i], psi = PS[i];
            if (!kCapped || cut <= cap) {
                for (int q = 0; q < tb.n_tp; ++q) {
                    if (forced && q != forced[s]) continue;
                    const int64_t tp = tb.tp[q];
                    const int d = d2 - int(tp);
                    // the stage must stay inside group k, and s stages have used at least s devices
                    // (row s holds nothing else: entries outside the ranges written for it are stale)
                    if (d < offs[k] || d < s) continue;
                    const int shift = tb.tp_shift[q];
                    const int64_t *pr = tb.PR(g, q);
                    const int64_t pri = pr[i];
                    const int64_t capm = tp * mem_dev;
                    const int64_t *row = Dp + size_t(d) * W;
                    for (int j = i - 1; j >= s; --j) {
                        const int64_t work = pfi - pf[j];
                        const int64_t time = (shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp) + (pri - pr[j]);
                        // the stage time never decreases as j moves down: beyond the cap, or beyond the
                        // best value of the min-max form, no lower j can be taken or can match
                        if (time > (kCapped ? cap : best)) break;
                        if ((ppi - PP[j]) + n_inflight * (psi - PS[j]) > capm) break;   // nor fit in memory
                        const int64_t prev = row[j];
                        if (prev == kInf) continue;
                        int64_t val;
                        if (kCapped) {
                            val = prev + time + 2 * cut;
                        } else {
                            val = prev > time ? prev : time;
                            val = val > cut ? val : cut;
                        }
                        if (val < best || (val == best && j < best_j)) { best = val; best_j = j; best_q = q; }
                    }
                }
            }
            Dn[size_t(d2) * W + i] = best;
            arg_s[size_t(d2) * W + i] = uint32_t(best_j) | (uint32_t(best_q) << 16);
        }
        int64_t *tmp = Dp; Dp = Dn; Dn = tmp;
    }
    __syncthreads();
    return Dp[size_t(Dtot) * W + L];
}

// The same pass on the 32-bit rows, for tables that allow them (every degree a power of two, every
// time below 2^31 us) and L <= kMeshFastMaxL.  What changes is the cost of a transition, not the result:
//  * the memory test of eq. mem_cons becomes one comparison: with Q[j] = PP[j] + N_s PS[j], kept in
//    LDS for the stage, the stage [j, i) fits iff Q[j] >= Q[i] - tp * mem;
//  * the min-max values are times, so the live rows are uint32 (the least sums of the capped form
//    stay int64);
//  * the best (value, previous cut, degree index) is one 64-bit key and the tie rule (lowest cut,
//    then smallest degree) is an unsigned minimum: min-max key = value << 32 | j << 3 | q, capped
//    key = sum << 19 | j << 3 | q (a sum of at most 256 stage and transfer times stays below 2^42);
//  * four previous cuts per trip, all evaluated under predicates; entries below a stop cannot
//    update (their time exceeds the best value or the cap, or they do not fit), so only the last
//    entry of a trip decides whether the lane goes on.
constexpr int kMeshFastMaxL = 4096;

template <bool kCapped>
__device__ __forceinline__ int64_t mesh_pass_fast(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                                  const uint16_t *order, const uint16_t *group_at, int64_t *Q,
                                                  int K, int S, int64_t n_dev, int64_t cap,
                                                  const uint8_t *forced = nullptr,
                                                  const int32_t *forced_off = nullptr) {
    using ValT = typename std::conditional<kCapped, int64_t, uint32_t>::type;
    constexpr uint64_t kNoKey = ~0ull;
    const int L = tb.L, W = L + 1, tid = threadIdx.x, nthreads = blockDim.x;
    const int Dtot = offs[K];
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    ValT *Dp = reinterpret_cast<ValT *>(m.D0), *Dn = reinterpret_cast<ValT *>(m.D1);
    const ValT none = kCapped ? ValT(kInf) : ValT(fastdp::kInf32);
    if (kCapped && cap < 0) return kInf;             // no transition has a negative time (uniform exit)
    const uint32_t cap32 = cap > 0xFFFFFFFEll ? 0xFFFFFFFEu : uint32_t(cap);
    __syncthreads();                                 // the previous pass is done with the rows
    for (int x = tid; x < (Dtot + 1) * W; x += nthreads) Dp[x] = none;
    __syncthreads();
    if (tid == 0) Dp[0] = 0;                         // no stage, no operator, no device
    for (int s = 0; s < S; ++s) {
        __syncthreads();                             // row s is complete, the previous stage is done with Q
        const bool last = (s == S - 1);
        const int64_t n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
        for (int j = tid; j <= L; j += nthreads) Q[j] = PP[j] + n_inflight * PS[j];
        __syncthreads();
        const int i_lo = last ? L : s + 1, i_hi = L - (S - 1 - s);
        // a fixed slicing (forced) leaves one device offset per stage
        const int d_lo = forced ? forced_off[s + 1] : (last ? Dtot : s + 1);
        const int d_hi = forced ? forced_off[s + 1] : (last ? Dtot : Dtot - (S - 1 - s));
        const int n_i = i_hi - i_lo + 1, n_d = d_hi - d_lo + 1;
        uint32_t *arg_s = m.arg + size_t(s) * size_t(n_dev + 1) * W;
        for (int x = tid; x < n_i * n_d; x += nthreads) {
            const int i = i_lo + x % n_i, d2 = d_lo + x / n_i;
            int k = 0;
            if (Dtot <= kMeshGroupTable) k = group_at[d2 - 1];     // the group of the stage's last device
            else while (offs[k + 1] < d2) ++k;                     // offs[k] < d2 <= offs[k + 1]
            const int g = order[k];
            const int64_t mem_dev = tb.type_mem[tb.group_type[g]];
            const int g_next = last ? g : (d2 == offs[k + 1] ? order[k + 1 < K ? k + 1 : k] : g);
            const uint32_t cut = last ? 0u : tb.CM[(int64_t(g) * tb.G + g_next) * tb.pitch32 + i];
            const int64_t qi = Q[i];
            uint64_t best = kNoKey;
            if (!kCapped || cut <= cap32) {
                for (int q = 0; q < tb.n_tp; ++q) {
                    if (forced && q != forced[s]) continue;
                    const int tp = tb.tp[q];
                    const int d = d2 - tp;
                    // the stage must stay inside group k, and s stages have used at least s devices
                    // (row s holds nothing else: entries outside the ranges written for it are stale)
                    if (d < offs[k] || d < s) continue;
                    const int shift = tb.tp_shift[q];
                    const uint32_t *p32 = tb.P32 + (int64_t(g) * tb.n_tp + q) * tb.pitch32;
                    const uint32_t xi = p32[i] + uint32_t(tp) - 1u;
                    const int64_t th = qi - int64_t(tp) * mem_dev;
                    const ValT *row = Dp + size_t(d) * W;
                    int j = i - 1;
                    bool more = true;                 // i > s always
                    while (more) {
                        const int j1 = (j - 1) > s ? (j - 1) : s, j2 = (j - 2) > s ? (j - 2) : s,
                                  j3 = (j - 3) > s ? (j - 3) : s;
                        const uint32_t p0 = p32[j], p1 = p32[j1], p2 = p32[j2], p3 = p32[j3];
                        const ValT r0 = row[j], r1 = row[j1], r2 = row[j2], r3 = row[j3];
                        const int64_t q0 = Q[j], q1 = Q[j1], q2 = Q[j2], q3 = Q[j3];
                        uint32_t tj;
#define HARP_MESH_STEP(P, R, QV, JJ)                                                              \
    {                                                                                             \
        tj = (xi - (P)) >> shift;                                                                 \
        uint64_t key;                                                                             \
        bool ok = (QV) >= th;                                                                     \
        if (kCapped) {                                                                            \
            ok = ok & ((R) != none) & (tj <= cap32);                                              \
            key = ((uint64_t(R) + uint64_t(tj) + 2ull * cut) << 19) |                             \
                  uint64_t((uint32_t(JJ) << 3) | uint32_t(q));                                    \
        } else {                                                                                  \
            key = (uint64_t(fastdp::umax3(uint32_t(R), tj, cut)) << 32) |                         \
                  uint64_t((uint32_t(JJ) << 3) | uint32_t(q));                                    \
        }                                                                                         \
        best = (ok & (key < best)) ? key : best;                                                  \
    }
                        HARP_MESH_STEP(p0, r0, q0, j)
                        HARP_MESH_STEP(p1, r1, q1, j1)
                        HARP_MESH_STEP(p2, r2, q2, j2)
                        HARP_MESH_STEP(p3, r3, q3, j3)
#undef HARP_MESH_STEP
                        more = ((j - 3) > s) & (q3 >= th) & (tj <= (kCapped ? cap32 : uint32_t(best >> 32)));
                        j -= 4;
                    }
                }
            }
            ValT value;
            uint32_t jq;
            if (kCapped) {
                value = best == kNoKey ? none : ValT(best >> 19);
                jq = uint32_t(best) & 0x7FFFFu;
            } else {
                value = ValT(best >> 32);             // an unreached cell keeps all ones
                jq = uint32_t(best) & 0x7FFFFu;
            }
            Dn[size_t(d2) * W + i] = value;
            arg_s[size_t(d2) * W + i] = (jq >> 3) | ((jq & 7u) << 16);
        }
        ValT *tmp = Dp; Dp = Dn; Dn = tmp;
    }
    __syncthreads();
    const ValT v = Dp[size_t(Dtot) * W + L];
    return v == none ? kInf : int64_t(v);
}

// Thread 0: follows the back-pointers from (S, L, all devices).
__device__ __forceinline__ void mesh_backtrack(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                               const uint16_t *order, int K, int S, int64_t n_dev, int32_t *cuts,
                                               uint16_t *slot_g, uint8_t *slot_k, int32_t *slot_first) {
    const int L = tb.L, W = L + 1;
    int i = L, d = offs[K];
    cuts[S] = L;
    for (int s = S; s >= 1; --s) {
        const uint32_t a = m.arg[(size_t(s - 1) * size_t(n_dev + 1) + size_t(d)) * W + i];
        int j = int(a & 0xFFFFu);
        const int q = int(a >> 16) & 7;
        j = j < L ? j : L - 1;                      // a finite value only chains through cuts inside the row
        d -= tb.tp[q];
        d = d > 0 ? d : 0;
        int k = 0;
        while (k + 1 < K && offs[k + 1] <= d) ++k;
        cuts[s - 1] = j;
        slot_g[s - 1] = uint16_t(order[k]);
        slot_k[s - 1] = uint8_t(q);
        slot_first[s - 1] = tb.group_base[order[k]] + (d - offs[k]);
        i = j;
    }
}

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
        if (tid == 0) mesh_backtrack(tb, m, offs, order, K, S, n_dev, cuts, slot_g, slot_k, slot_first);
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

// c <= cap, so the quotient of eq. dp_ni is 0, 1 or 2 and needs no division.
__device__ __forceinline__ int mesh_delta(int64_t c, int64_t cap) {
    const int64_t x = 2 * c - (cap >> 6);
    return 1 + (x > 0 ? 1 : 0) + (x > cap ? 1 : 0);
}

// The paper's recurrence in full for one cap (section 5.2.3: eq. dp_general with its device index and
// the H-1F1B warm-up count of eq. dp_ni in the state), suffix direction.  State (s, i, e): the last s
// stages hold the operators from i on and use the last e devices; it keeps the least sum of (t + 2c)
// under the cap and the count of its first stage as determined by the continuation that attained
// it.  One lane per target cell (i, e); per degree an upward scan of the end cuts j, which stops at
// the cap (the stage time grows with j) or when the stage no longer fits even with a count of one.
// Ties: lowest end cut, then smallest degree.  Returns the value of (S, 0, all devices).
__device__ __forceinline__ int64_t mesh_h1_pass(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                                const uint16_t *order, const uint16_t *group_at, int K, int S,
                                                int64_t n_dev, int64_t cap, const uint8_t *forced = nullptr,
                                                const int32_t *forced_off = nullptr) {
    const int L = tb.L, W = L + 1, tid = threadIdx.x, nthreads = blockDim.x;
    const int Dtot = offs[K];
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    int64_t *Gp = m.D0, *Gn = m.D1;
    int32_t *Np = m.N0, *Nn = m.N1;
    __syncthreads();
    for (int x = tid; x < (Dtot + 1) * W; x += nthreads) { Gp[x] = kInf; Np[x] = 0; }
    __syncthreads();
    if (tid == 0) Gp[L] = 0;                         // no stages left: no operators, no devices (e = 0, i = L)
    for (int s = 1; s <= S; ++s) {
        __syncthreads();                             // row s - 1 is complete
        const bool whole = (s == S);
        const int i_lo = whole ? 0 : S - s, i_hi = whole ? 0 : L - s;
        // a fixed slicing (forced) leaves one device count for the last s stages
        const int e_lo = forced ? Dtot - forced_off[S - s] : (whole ? Dtot : s);
        const int e_hi = forced ? Dtot - forced_off[S - s] : (whole ? Dtot : Dtot - (S - s));
        const int j_hi = L - (s - 1);
        const int n_i = i_hi - i_lo + 1, n_e = e_hi - e_lo + 1;
        uint32_t *arg_s = m.arg + size_t(s - 1) * size_t(n_dev + 1) * W;
        for (int x = tid; x < n_i * n_e; x += nthreads) {
            const int i = i_lo + x % n_i, e = e_lo + x / n_i;
            const int d0 = Dtot - e;                 // first device of the stage this step places
            int k = 0;
            if (Dtot <= kMeshGroupTable) k = group_at[d0];
            else while (offs[k + 1] <= d0) ++k;
            const int g = order[k];
            const int t = tb.group_type[g];
            const int64_t *pf = tb.PF(t);
            const int64_t mem_dev = tb.type_mem[t];
            const int64_t pfi = pf[i], ppi = PP[i], psi = PS[i];
            int64_t best = kInf;
            int best_j = 0x7FFFFFFF, best_q = 0, best_n = 0;
            for (int q = 0; q < tb.n_tp; ++q) {
                if (forced && q != forced[S - s]) continue;
                const int64_t tp = tb.tp[q];
                const int e0 = e - int(tp);
                // the stage stays inside group k; the stages behind it have used at least one device
                // each (row s - 1 holds nothing else), and none at all exactly when there are none
                if (d0 + int(tp) > offs[k + 1] || e0 < s - 1 || (s == 1) != (e0 == 0)) continue;
                const int g_next = (s == 1) ? g : (d0 + int(tp) == offs[k + 1] ? order[k + 1 < K ? k + 1 : k] : g);
                const int shift = tb.tp_shift[q];
                const int64_t *pr = tb.PR(g, q);
                const int64_t link = tb.bw[int64_t(g) * tb.G + g_next];
                const int64_t pri = pr[i];
                const int64_t capm = tp * mem_dev;
                const int64_t *rowG = Gp + size_t(e0) * W;
                const int32_t *rowN = Np + size_t(e0) * W;
                for (int j = i + 1; j <= j_hi; ++j) {
                    const int64_t work = pf[j] - pfi;
                    const int64_t time = (shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp) + (pr[j] - pri);
                    if (time > cap) break;                                   // constraint (i); grows with j
                    const int64_t dpp = PP[j] - ppi, dps = PS[j] - psi;
                    if (dpp + dps > capm) break;                             // no count fits from here on
                    const int64_t rest = rowG[j];
                    if (rest == kInf) continue;
                    int64_t cut = 0;
                    if (s > 1) cut = (tb.act_bytes[j - 1] + link - 1) / link;
                    if (cut > cap) continue;                                 // constraint (ii)
                    int64_t n = mesh_delta(cut, cap) + rowN[j];              // eq. dp_ni
                    n = n < tb.M ? n : tb.M;
                    if (dpp + n * dps > capm) continue;                      // constraint (iii), eq. mem_cons
                    const int64_t val = rest + time + 2 * cut;
                    if (val < best || (val == best && j < best_j)) { best = val; best_j = j; best_q = q; best_n = int(n); }
                }
            }
            Gn[size_t(e) * W + i] = best;
            Nn[size_t(e) * W + i] = best_n;
            arg_s[size_t(e) * W + i] = uint32_t(best_j & 0xFFFF) | (uint32_t(best_q) << 16);
        }
        int64_t *tg = Gp; Gp = Gn; Gn = tg;
        int32_t *tn = Np; Np = Nn; Nn = tn;
    }
    __syncthreads();
    return Gp[size_t(Dtot) * W];
}

// The same pass on the 32-bit rows (tables that have them, L <= kMeshFastMaxL).  The running sums PP and
// PS sit in LDS for the whole pass.  A state's least sum and its count share one 64-bit word,
// sum << 10 | count: a count grows by at most 3 per stage (eq. delta_i under constraint (ii)) and
// there are at most 256 stages, so it stays below 1024, and a sum stays below 2^42.  The quotient
// of eq. dp_ni is read off two thresholds on the transfer time: 2c - e > 0 iff c > e >> 1, and
// 2c - e > cap iff c > (cap + e) >> 1, with e = cap >> 6.  The best (sum, end cut, degree index) is
// one key, sum << 19 | j << 3 | q; four end cuts per trip under predicates, the last one deciding
// whether the lane goes on (the stage time and the memory need with a count of one both grow with j).
__device__ __forceinline__ int64_t mesh_h1_pass_fast(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                                     const uint16_t *order, const uint16_t *group_at,
                                                     int64_t *PPl, int K, int S, int64_t n_dev, int64_t cap,
                                                     const uint8_t *forced = nullptr,
                                                     const int32_t *forced_off = nullptr) {
    constexpr uint64_t kNone = ~0ull;
    const int L = tb.L, W = L + 1, tid = threadIdx.x, nthreads = blockDim.x;
    const int Dtot = offs[K];
    int64_t *PSl = PPl + W;
    uint64_t *Gp = reinterpret_cast<uint64_t *>(m.D0), *Gn = reinterpret_cast<uint64_t *>(m.D1);
    const uint32_t cap32 = cap > 0xFFFFFFFEll ? 0xFFFFFFFEu : uint32_t(cap);
    const uint64_t e6 = uint64_t(cap) >> 6;
    const uint64_t th1_64 = e6 >> 1, th2_64 = (uint64_t(cap) + e6) >> 1;
    const uint32_t th1 = th1_64 > 0xFFFFFFFFull ? 0xFFFFFFFFu : uint32_t(th1_64);
    const uint32_t th2 = th2_64 > 0xFFFFFFFFull ? 0xFFFFFFFFu : uint32_t(th2_64);
    const uint32_t m_cap = uint32_t(tb.M);
    __syncthreads();
    {
        const int64_t *PP = tb.PP(), *PS = tb.PS();
        for (int j = tid; j <= L; j += nthreads) { PPl[j] = PP[j]; PSl[j] = PS[j]; }
    }
    for (int x = tid; x < (Dtot + 1) * W; x += nthreads) Gp[x] = kNone;
    __syncthreads();
    if (tid == 0) Gp[L] = 0;                         // no stages left: no operators, no devices, count 0
    for (int s = 1; s <= S; ++s) {
        __syncthreads();                             // row s - 1 is complete
        const bool whole = (s == S);
        const int i_lo = whole ? 0 : S - s, i_hi = whole ? 0 : L - s;
        // a fixed slicing (forced) leaves one device count for the last s stages
        const int e_lo = forced ? Dtot - forced_off[S - s] : (whole ? Dtot : s);
        const int e_hi = forced ? Dtot - forced_off[S - s] : (whole ? Dtot : Dtot - (S - s));
        const int j_hi = L - (s - 1);
        const int n_i = i_hi - i_lo + 1, n_e = e_hi - e_lo + 1;
        uint32_t *arg_s = m.arg + size_t(s - 1) * size_t(n_dev + 1) * W;
        for (int x = tid; x < n_i * n_e; x += nthreads) {
            const int i = i_lo + x % n_i, e = e_lo + x / n_i;
            const int d0 = Dtot - e;                 // first device of the stage this step places
            int k = 0;
            if (Dtot <= kMeshGroupTable) k = group_at[d0];
            else while (offs[k + 1] <= d0) ++k;
            const int g = order[k];
            const int64_t mem_dev = tb.type_mem[tb.group_type[g]];
            const int64_t ppi = PPl[i], psi = PSl[i];
            uint64_t best = kNone;
            uint32_t best_n = 0;
            for (int q = 0; q < tb.n_tp; ++q) {
                if (forced && q != forced[S - s]) continue;
                const int tp = tb.tp[q];
                const int e0 = e - tp;
                // the stage stays inside group k; the stages behind it have used at least one device
                // each (row s - 1 holds nothing else), and none at all exactly when there are none
                if (d0 + tp > offs[k + 1] || e0 < s - 1 || (s == 1) != (e0 == 0)) continue;
                const int g_next = (s == 1) ? g : (d0 + tp == offs[k + 1] ? order[k + 1 < K ? k + 1 : k] : g);
                const int shift = tb.tp_shift[q];
                const uint32_t *p32 = tb.P32 + (int64_t(g) * tb.n_tp + q) * tb.pitch32;
                const uint32_t *cm = tb.CM + (int64_t(g) * tb.G + g_next) * tb.pitch32;
                const uint32_t xi = p32[i] - uint32_t(tp) + 1u;       // time = (P[j] + tp - 1 - P[i]) >> shift
                const int64_t capm = int64_t(tp) * mem_dev;
                const uint64_t *row = Gp + size_t(e0) * W;
                int j = i + 1;
                bool more = true;                     // i < j_hi always
                while (more) {
                    const int j1 = (j + 1) < j_hi ? (j + 1) : j_hi, j2 = (j + 2) < j_hi ? (j + 2) : j_hi,
                              j3 = (j + 3) < j_hi ? (j + 3) : j_hi;
                    const uint32_t p0 = p32[j], p1 = p32[j1], p2 = p32[j2], p3 = p32[j3];
                    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
                    if (s > 1) { c0 = cm[j]; c1 = cm[j1]; c2 = cm[j2]; c3 = cm[j3]; }
                    const uint64_t r0 = row[j], r1 = row[j1], r2 = row[j2], r3 = row[j3];
                    const int64_t a0 = PPl[j], a1 = PPl[j1], a2 = PPl[j2], a3 = PPl[j3];
                    const int64_t b0 = PSl[j], b1 = PSl[j1], b2 = PSl[j2], b3 = PSl[j3];
                    bool live;
#define HARP_MESH_H1_STEP(P, CUT, R, A, B, JJ)                                                    \
    {                                                                                             \
        const uint32_t tj = ((P) - xi) >> shift;                                                  \
        const int64_t dpp = (A) - ppi, dps = (B) - psi;                                           \
        live = (tj <= cap32) & (dpp + dps <= capm);          /* constraint (i); a count of one */ \
        uint32_t n = 1u + ((CUT) > th1 ? 1u : 0u) + ((CUT) > th2 ? 1u : 0u) + (uint32_t(R) & 1023u); \
        n = n < m_cap ? n : m_cap;                                                     /* eq. dp_ni */ \
        const bool ok = live & ((R) != kNone) & ((CUT) <= cap32) & (dpp + int64_t(n) * dps <= capm); \
        const uint64_t key = ((((R) >> 10) + uint64_t(tj) + 2ull * (CUT)) << 19) |                \
                             uint64_t((uint32_t(JJ) << 3) | uint32_t(q));                         \
        const bool upd = ok & (key < best);                                                       \
        best = upd ? key : best;                                                                  \
        best_n = upd ? n : best_n;                                                                \
    }
                    HARP_MESH_H1_STEP(p0, c0, r0, a0, b0, j)
                    HARP_MESH_H1_STEP(p1, c1, r1, a1, b1, j1)
                    HARP_MESH_H1_STEP(p2, c2, r2, a2, b2, j2)
                    HARP_MESH_H1_STEP(p3, c3, r3, a3, b3, j3)
#undef HARP_MESH_H1_STEP
                    more = ((j + 3) < j_hi) & live;
                    j += 4;
                }
            }
            Gn[size_t(e) * W + i] = best == kNone ? kNone : (((best >> 19) << 10) | uint64_t(best_n));
            const uint32_t jq = uint32_t(best) & 0x7FFFFu;
            arg_s[size_t(e) * W + i] = (jq >> 3) | ((jq & 7u) << 16);
        }
        uint64_t *tg = Gp; Gp = Gn; Gn = tg;
    }
    __syncthreads();
    const uint64_t v = Gp[size_t(Dtot) * W];
    return v == kNone ? kInf : int64_t(v >> 10);
}

// Thread 0: follows the back-pointers of the H-1F1B form from (S, 0, all devices) and recomputes the
// counts by eq. Ni along the plan, from the last stage backwards.
__device__ __forceinline__ void mesh_h1_backtrack(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                                  const uint16_t *order, int K, int S, int64_t n_dev, int64_t cap,
                                                  int32_t *cuts, uint16_t *slot_g, uint8_t *slot_k,
                                                  int32_t *slot_first, int32_t *count) {
    const int L = tb.L, W = L + 1, Dtot = offs[K];
    const int64_t m_cap = tb.M;
    int i = 0, e = Dtot;
    for (int slot = 0; slot < S; ++slot) {
        const int s = S - slot;
        const uint32_t a = m.arg[(size_t(s - 1) * size_t(n_dev + 1) + size_t(e)) * W + i];
        int j = int(a & 0xFFFFu);
        const int q = int(a >> 16) & 7;
        j = j <= L ? j : L;                     // a finite sum only chains through cuts inside the row
        const int d0 = Dtot - e;
        int k = 0;
        while (k + 1 < K && offs[k + 1] <= d0) ++k;
        cuts[slot] = i;
        slot_g[slot] = order[k];
        slot_k[slot] = uint8_t(q);
        slot_first[slot] = tb.group_base[order[k]] + (d0 - offs[k]);
        i = j;
        e -= tb.tp[q];
        e = e > 0 ? e : 0;
    }
    cuts[S] = L;
    int64_t n = 0;
    for (int slot = S - 1; slot >= 0; --slot) {
        int64_t cut = 0;
        if (slot < S - 1) {
            const int64_t link = tb.bw[int64_t(slot_g[slot]) * tb.G + slot_g[slot + 1]];
            cut = (tb.act_bytes[cuts[slot + 1] - 1] + link - 1) / link;
        }
        n += mesh_delta(cut, cap);
        n = n < m_cap ? n : m_cap;
        count[slot] = int32_t(n);
    }
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
        if (tid == 0) mesh_h1_backtrack(tb, m, offs, order, K, S, n_dev, cap, cuts, slot_g, slot_k, slot_first, count);
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
                mesh_h1_backtrack(tb, m, offs, order, K, S, n_dev, at, cuts, slot_g, slot_k, slot_first, count);
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

__global__ void k2_mesh_sweep_clear(int *first_idx, int C) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
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
    hipLaunchKernelGGL(k2_mesh_clear, dim3(1), dim3(64), 0, st, ticket);
    hipLaunchKernelGGL(k2_mesh_sweep_clear, dim3((od.C + 255) / 256), dim3(256), 0, st, first_idx, od.C);
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
