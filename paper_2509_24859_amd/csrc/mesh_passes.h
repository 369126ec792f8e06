// Passes of the submesh planner (paper section 5.2.3, eq. dp_general with its device index): device
// functions shared by the kernels that plan a batch of orderings once (k2_mesh.hip) and by the search
// over the cap (k2_sweep.hip).  Every function is called by all threads of a workgroup.
#pragma once

#include <type_traits>

#include "harp_internal.h"
#include "fast_common.h"
#include "plan_common.h"

namespace harp {
namespace meshdp {

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
constexpr int kMeshFastMaxL = 4096;     // and below 8192, so that a cut fits the 13 bits of a packed back-pointer

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
        uint16_t *arg_s = reinterpret_cast<uint16_t *>(m.arg) + size_t(s) * size_t(n_dev + 1) * W;   // packed form
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
            arg_s[size_t(d2) * W + i] = uint16_t(((jq >> 3) & 0x1FFFu) | ((jq & 7u) << 13));
        }
        ValT *tmp = Dp; Dp = Dn; Dn = tmp;
    }
    __syncthreads();
    const ValT v = Dp[size_t(Dtot) * W + L];
    return v == none ? kInf : int64_t(v);
}

// Thread 0: follows the back-pointers from (S, L, all devices).
// kPacked: the back-pointers were written by a 32-bit pass (uint16: cut | degree index << 13, which
// holds every cut of a sequence the 32-bit rows exist for), otherwise by an int64 pass (uint32:
// cut | degree index << 16).
template <bool kPacked>
__device__ __forceinline__ void mesh_backtrack(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                               const uint16_t *order, int K, int S, int64_t n_dev, int32_t *cuts,
                                               uint16_t *slot_g, uint8_t *slot_k, int32_t *slot_first) {
    const int L = tb.L, W = L + 1;
    int i = L, d = offs[K];
    cuts[S] = L;
    for (int s = S; s >= 1; --s) {
        const size_t at = (size_t(s - 1) * size_t(n_dev + 1) + size_t(d)) * W + i;
        const uint32_t a = kPacked ? reinterpret_cast<const uint16_t *>(m.arg)[at] : m.arg[at];
        int j = int(a & (kPacked ? 0x1FFFu : 0xFFFFu));
        const int q = int(a >> (kPacked ? 13 : 16)) & 7;
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
        uint16_t *arg_s = reinterpret_cast<uint16_t *>(m.arg) + size_t(s - 1) * size_t(n_dev + 1) * W;   // packed form
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
            arg_s[size_t(e) * W + i] = uint16_t(((jq >> 3) & 0x1FFFu) | ((jq & 7u) << 13));
        }
        uint64_t *tg = Gp; Gp = Gn; Gn = tg;
    }
    __syncthreads();
    const uint64_t v = Gp[size_t(Dtot) * W];
    return v == kNone ? kInf : int64_t(v >> 10);
}

// Thread 0: follows the back-pointers of the H-1F1B form from (S, 0, all devices) and recomputes the
// counts by eq. Ni along the plan, from the last stage backwards.
template <bool kPacked>
__device__ __forceinline__ void mesh_h1_backtrack(const TablesDev &tb, const MeshSlice &m, const int32_t *offs,
                                                  const uint16_t *order, int K, int S, int64_t n_dev, int64_t cap,
                                                  int32_t *cuts, uint16_t *slot_g, uint8_t *slot_k,
                                                  int32_t *slot_first, int32_t *count) {
    const int L = tb.L, W = L + 1, Dtot = offs[K];
    const int64_t m_cap = tb.M;
    int i = 0, e = Dtot;
    for (int slot = 0; slot < S; ++slot) {
        const int s = S - slot;
        const size_t at = (size_t(s - 1) * size_t(n_dev + 1) + size_t(e)) * W + i;
        const uint32_t a = kPacked ? reinterpret_cast<const uint16_t *>(m.arg)[at] : m.arg[at];
        int j = int(a & (kPacked ? 0x1FFFu : 0xFFFFu));
        const int q = int(a >> (kPacked ? 13 : 16)) & 7;
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

}  // namespace meshdp
}  // namespace harp
