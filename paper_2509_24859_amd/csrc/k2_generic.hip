// Generic planner-search kernel for gfx950: the dense min-max recurrence in int64.
//
// Paper section 5.2.3 (eq. dp_general with the submesh of every stage fixed by the candidate,
// constraints (i)-(iii)) evaluated exactly as stated: for every stage s and every end cut i, all
// previous cuts j that can matter are tried.  One workgroup works on one candidate at a time; one lane
// owns one DP cell of the current stage and walks j downwards from i - 1 until the stage no longer
// fits in memory or its time alone rules every lower j out, keeping the lowest j among equal values
// (no reachability bands, no feasibility index, no 32-bit rows: k2_generic shares none of the fast
// kernel's pruning).  Rows of D and the back-pointers live in a
// per-workgroup slice of the caller's workspace (L2-resident at the sizes of interest).  This path
// accepts any degree (division when it is not a power of two) and any L up to 65535; the 32-bit
// path in k2_fast.hip is the fast one.
//
// k2_banded, k2_banded_exact and k2_banded_h1f1b are the planners of this path when the batch's
// feasibility index fits its limits (it does unless L, the in-flight counts and the degree list are
// all large): same int64 arithmetic, but they run behind the pre-pass of k2_fast.hip, which needs
// nothing but the memory sums, and so work on the reachability bands only and read each cell's
// range of fitting cuts from the index instead of evaluating eq. mem_cons per transition.  The rows
// k2_banded keeps in LDS are a third of the unbanded kernel's per candidate, so several times as
// many candidates are in flight per CU.
#include "harp_internal.h"
#include "fast_common.h"
#include "plan_common.h"

namespace harp {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

// Per-workgroup slice of the workspace: two DP rows and the back-pointers.
struct GenericSlice {
    int64_t *D0, *D1;
    uint16_t *arg;      // [S_max][L+1], row s = stage s
};

__device__ __forceinline__ GenericSlice generic_slice(unsigned char *ws, size_t ws_per_group, int L) {
    unsigned char *mine = ws + size_t(blockIdx.x) * ws_per_group;
    GenericSlice g;
    g.D0 = reinterpret_cast<int64_t *>(mine);
    g.D1 = g.D0 + (L + 1);
    g.arg = reinterpret_cast<uint16_t *>(g.D1 + (L + 1));
    return g;
}

// One pass of the recurrence over all stages of the candidate in `slots`, every thread of the
// workgroup taking part.  kCapped = false: the min-max form, D[s+1][i] = min_j max(D[s][j], time,
// comm).  kCapped = true: the least-sum form under a cap on every stage and transfer time
// (section 5.2.3 with constraints (i), (ii)), D[s+1][i] = min_j D[s][j] + time + 2 comm over
// time <= cap, cells with comm > cap unreachable.  Both keep the lowest j among equal values.
// Returns the row that holds D[S][.].
// Sequences of up to kGenericLdsL operators keep the six rows a stage reads (the two memory sums, the
// stage's compute and all-reduce sums, the two DP rows) in LDS; longer ones read them from global
// memory (L2).  Same arithmetic either way.
constexpr int kGenericLdsL = 1279;      // 6 x 1280 x 8 B = 60 KB

size_t generic_lds_bytes(int L) { return L <= kGenericLdsL ? size_t(6) * (L + 1) * sizeof(int64_t) : 0; }

template <bool kCapped>
__device__ __forceinline__ const int64_t *generic_pass(const TablesDev &tb, const SlotInfo &slots, int S,
                                                       const GenericSlice &w, int64_t time_cap) {
    extern __shared__ __align__(16) unsigned char generic_lds[];
    const int L = tb.L;
    const bool rows_in_lds = L <= kGenericLdsL;
    int64_t *stage = reinterpret_cast<int64_t *>(generic_lds);       // [6][L + 1] when rows_in_lds
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    int64_t *Dp = w.D0, *Dn = w.D1;
    __syncthreads();                          // an earlier pass is done with the rows
    if (rows_in_lds) {
        for (int i = threadIdx.x; i <= L; i += kThreads) { stage[i] = PP[i]; stage[(L + 1) + i] = PS[i]; }
        PP = stage;
        PS = stage + (L + 1);
        Dp = stage + 4 * (L + 1);
        Dn = stage + 5 * (L + 1);
    }
    for (int i = threadIdx.x; i <= L; i += kThreads) Dp[i] = (i == 0) ? 0 : kInf;
    __syncthreads();
    for (int s = 0; s < S; ++s) {
        const int g = slots.g[s], k = slots.k[s];
        const int64_t tp = tb.tp[k];
        const int shift = tb.tp_shift[k];
        const int t = tb.group_type[g];
        const int64_t *pf = tb.PF(t), *pr = tb.PR(g, k);
        if (rows_in_lds) {
            int64_t *spf = stage + 2 * (L + 1), *spr = stage + 3 * (L + 1);
            for (int i = threadIdx.x; i <= L; i += kThreads) { spf[i] = pf[i]; spr[i] = pr[i]; }
            __syncthreads();                  // (the barrier that ended the previous stage lets these be overwritten)
            pf = spf;
            pr = spr;
        }
        const int64_t n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
        const int64_t cap = tp * tb.type_mem[t];
        const bool last = (s == S - 1);
        const int64_t link = last ? 1 : tb.bw[int64_t(g) * tb.G + slots.g[s + 1]];
        const int i_lo = last ? L : s + 1, i_hi = L - (S - 1 - s);
        uint16_t *arg_row = w.arg + size_t(s) * (L + 1);
        for (int i = i_lo + int(threadIdx.x); i <= i_hi; i += kThreads) {
            const int64_t cut = last ? 0 : (tb.act_bytes[i - 1] + link - 1) / link;
            const int64_t pfi = pf[i], pri = pr[i], ppi = PP[i], psi = PS[i];
            int64_t best = kInf;
            int best_j = 0;
            if (!kCapped || cut <= time_cap) {
                // previous cuts from i - 1 downwards.  Both the memory need and the stage time never
                // decrease as j moves down, so once a cut does not fit, or its time alone is above
                // the cap (capped form) or above the best value so far (min-max form: strictly, an
                // equal value at a lower j still has to be seen), no lower j can be taken or can
                // match, and the scan stops.
                for (int j = i - 1; j >= s; --j) {
                    const int64_t need = (ppi - PP[j]) + n_inflight * (psi - PS[j]);
                    if (need > cap) break;
                    const int64_t work = pfi - pf[j];
                    const int64_t comp = shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp;
                    const int64_t time = comp + (pri - pr[j]);
                    if (time > (kCapped ? time_cap : best)) break;
                    const int64_t dj = Dp[j];
                    if (dj == kInf) continue;
                    if (kCapped) {
                        if (dj + time <= best) { best = dj + time; best_j = j; }   // j falls: the lower j keeps a tie
                    } else {
                        int64_t val = time > dj ? time : dj;
                        val = val > cut ? val : cut;
                        if (val <= best) { best = val; best_j = j; }
                    }
                }
            }
            Dn[i] = (kCapped && best != kInf) ? best + 2 * cut : best;
            arg_row[i] = (uint16_t)best_j;
        }
        __syncthreads();
        int64_t *tmp = Dp; Dp = Dn; Dn = tmp;
    }
    return Dp;
}

// Thread 0: follows the back-pointers from (S, L) into cuts[0..S].
__device__ __forceinline__ void generic_backtrack(const GenericSlice &w, int S, int L, int32_t *cuts) {
    int b = L;
    cuts[S] = L;
    for (int s = S - 1; s >= 0; --s) {
        b = w.arg[size_t(s) * (L + 1) + b];
        cuts[s] = b;
    }
}

__global__ __launch_bounds__(kThreads) void k2_generic(TablesDev tb, CandDev cd, PlansDev out,
                                                        unsigned char *ws, size_t ws_per_group) {
    __shared__ SlotInfo slots;
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GenericSlice w = generic_slice(ws, ws_per_group, L);

    for (int c = blockIdx.x; c < cd.C; c += gridDim.x) {
        __syncthreads();   // previous candidate's tail is done with the shared state
        const int S = cd.cand_S[c];
        const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
        int status = load_and_check_slots(tb, S, S_max, grp, tpv, slots);
        if (status == HARP_CAND_OK && S > L) status = HARP_CAND_INFEASIBLE;
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            continue;
        }
        const int64_t *Dp = generic_pass<false>(tb, slots, S, w, 0);
        if (Dp[L] == kInf) {          // uniform: every thread reads the same cell
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            continue;
        }
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        if (threadIdx.x == 0) generic_backtrack(w, S, L, sp);
        for (int s = S + 1 + threadIdx.x; s <= S_max; s += kThreads) sp[s] = -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = threadIdx.x; s < S_max; s += kThreads) df[s] = s < S ? slots.dev_first[s] : -1;
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
        if (wave == 0) {
            int64_t bott, iter;
            const int st = wave_score_partition(tb, S, slots.g, slots.k, sp, lane, bott, iter);
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = iter;
                out.status[c] = st;
            }
        }
    }
}

// ---------------------------------------------------------------------------------- k2_banded

constexpr int kBandedThreads = 128;
constexpr int kBandedLdsL = 2047;       // 4 rows x 2048 x 8 B = 64 KB: stage sums and DP rows in LDS up to here

size_t banded_lds_bytes(int L) { return L <= kBandedLdsL ? size_t(4) * (L + 1) * sizeof(int64_t) : 0; }

// One pass of the recurrence of one live candidate over its bands, in either form of generic_pass
// (kCapped = false: min-max; true: least sum under the cap time_cap): row s + 1 has the cells
// B[s+1] .. F[s+1], cell i tries the previous cuts max(lo(i), B[s]) .. min(i - 1, F[s]) downwards,
// lo(i) from the feasibility index.  The scan stops as in the unbanded kernel once the stage time
// alone exceeds the best value (min-max form: strictly; the update is non-strict, so the lowest j
// among equal values is kept) or the cap (capped form).  The bands come from eq. mem_cons alone, so
// they bound the plans of every cap.  The last stage has the single cell L: its previous cuts are
// spread over the threads and reduced.  Returns D[S][L] to every thread; back-pointers are in w.arg.
template <bool kCapped>
__device__ __forceinline__ int64_t banded_pass(const TablesDev &tb, const SlotInfo &slots, int S,
                                               const uint32_t *band, const uint16_t *lo_tab, int lo_pitch,
                                               const GenericSlice &w, int64_t time_cap, int64_t *red_v,
                                               int *red_j) {
    const int nthreads = blockDim.x;
    extern __shared__ __align__(16) unsigned char generic_lds[];
    const int L = tb.L;
    const bool rows_in_lds = L <= kBandedLdsL;
    int64_t *stage = reinterpret_cast<int64_t *>(generic_lds);       // [4][L + 1] when rows_in_lds
    int64_t *Dp = w.D0, *Dn = w.D1;
    if (rows_in_lds) {
        Dp = stage + 2 * (L + 1);
        Dn = stage + 3 * (L + 1);
    }
    __syncthreads();                          // an earlier pass is done with the rows
    if (threadIdx.x == 0) Dp[0] = 0;          // row 0 is the single cut 0 (its band)
    const int rows_per_n = tb.T * tb.n_tp;
    for (int s = 0; s < S; ++s) {
        const int g = slots.g[s], k = slots.k[s];
        const int64_t tp = tb.tp[k];
        const int shift = tb.tp_shift[k];
        const int t = tb.group_type[g];
        const int64_t *pf = tb.PF(t), *pr = tb.PR(g, k);
        const uint32_t b0 = band[s], b1 = band[s + 1];
        const int jl = fastdp::band_lo(b0), jh = fastdp::band_hi(b0);      // previous cuts: row s
        const int il = fastdp::band_lo(b1), ih = fastdp::band_hi(b1);      // cells: row s + 1
        __syncthreads();                      // row s is complete, the previous stage's sums are free
        if (rows_in_lds) {
            int64_t *spf = stage, *spr = stage + (L + 1);
            for (int i = jl + int(threadIdx.x); i <= ih; i += nthreads) { spf[i] = pf[i]; spr[i] = pr[i]; }
            __syncthreads();
            pf = spf;
            pr = spr;
        }
        const int n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
        const uint16_t *lo_row = lo_tab + (size_t(n_inflight - 1) * rows_per_n + size_t(t) * tb.n_tp + k) * lo_pitch;
        const bool last = (s == S - 1);
        uint16_t *arg_row = w.arg + size_t(s) * (L + 1);
        if (!last) {
            const int64_t link = tb.bw[int64_t(g) * tb.G + slots.g[s + 1]];
            for (int i = il + int(threadIdx.x); i <= ih; i += nthreads) {
                const int64_t cut = (tb.act_bytes[i - 1] + link - 1) / link;
                const int64_t pfi = pf[i] + tp - 1, pri = pr[i];
                const int lo_i = lo_row[i];
                const int lo = lo_i > jl ? lo_i : jl;
                const int hi = (i - 1) < jh ? (i - 1) : jh;
                int64_t best = kInf;
                int best_j = i - 1;
                if (!kCapped || cut <= time_cap) {
                    for (int j = hi; j >= lo; --j) {
                        const int64_t work = pfi - pf[j];
                        const int64_t comp = shift >= 0 ? work >> shift : work / tp;
                        const int64_t time = comp + (pri - pr[j]);
                        if (time > (kCapped ? time_cap : best)) break;
                        const int64_t dj = Dp[j];
                        if (dj == kInf) continue;                 // an unreachable cut
                        if (kCapped) {
                            if (dj + time <= best) { best = dj + time; best_j = j; }   // j falls: the lower j keeps a tie
                        } else {
                            int64_t val = time > dj ? time : dj;
                            val = val > cut ? val : cut;
                            if (val <= best) { best = val; best_j = j; }
                        }
                    }
                }
                Dn[i] = (kCapped && best != kInf) ? best + 2 * cut : best;
                arg_row[i] = (uint16_t)best_j;
            }
        } else {
            // cell L: threads over the previous cuts, then the least value and the lowest cut among equals
            const int64_t pfi = pf[L] + tp - 1, pri = pr[L];
            const int lo_i = lo_row[L];
            const int lo = lo_i > jl ? lo_i : jl;
            const int hi = (L - 1) < jh ? (L - 1) : jh;
            int64_t best = kInf;
            int best_j = INT32_MAX;
            for (int j = lo + int(threadIdx.x); j <= hi; j += nthreads) {
                const int64_t work = pfi - pf[j];
                const int64_t comp = shift >= 0 ? work >> shift : work / tp;
                const int64_t time = comp + (pri - pr[j]);
                const int64_t dj = Dp[j];
                if (dj == kInf || (kCapped && time > time_cap)) continue;
                const int64_t val = kCapped ? dj + time : (time > dj ? time : dj);
                if (val < best) { best = val; best_j = j; }      // j rises within a thread
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const int64_t ov = __shfl_xor(best, d, 64);
                const int oj = __shfl_xor(best_j, d, 64);
                if (ov < best || (ov == best && oj < best_j)) { best = ov; best_j = oj; }
            }
            if ((threadIdx.x & 63) == 0) { red_v[threadIdx.x >> 6] = best; red_j[threadIdx.x >> 6] = best_j; }
            __syncthreads();
            if (threadIdx.x == 0) {
                for (int q = 1; q < nthreads / 64; ++q)
                    if (red_v[q] < best || (red_v[q] == best && red_j[q] < best_j)) { best = red_v[q]; best_j = red_j[q]; }
                red_v[0] = best;
                arg_row[L] = (uint16_t)(best == kInf ? L - 1 : best_j);
            }
            __syncthreads();
            return red_v[0];
        }
        int64_t *tmp = Dp; Dp = Dn; Dn = tmp;
    }
    return kInf;          // S >= 1: the last stage returns above
}

__global__ __launch_bounds__(kBandedThreads) void k2_banded(TablesDev tb, CandDev cd, PlansDev out, int *counts,
                                                             const int32_t *live_list, const uint32_t *dead_list,
                                                             const uint32_t *bands, const uint16_t *lo_tab,
                                                             int lo_pitch, unsigned char *ws, size_t ws_per_group) {
    __shared__ SlotInfo slots;
    __shared__ uint32_t band[kMaxStages + 1];
    __shared__ int64_t red_v[kBandedThreads / 64];
    __shared__ int red_j[kBandedThreads / 64];
    __shared__ int ticket;
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GenericSlice w = generic_slice(ws, ws_per_group, L);
    const int n_live = counts[0], n_dead = counts[1];

    // candidates differ in stages and band widths: workgroups draw them from a shared counter
    for (;;) {
        __syncthreads();   // previous candidate's tail is done with the shared state
        if (threadIdx.x == 0) ticket = atomicAdd(&counts[5], 1);
        __syncthreads();
        const int n = ticket;
        if (n >= n_live) break;
        const int c = live_list[n];
        const int S = cd.cand_S[c];
        const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
        // the pre-pass has checked the slot list; this fills the slot arrays and the first devices
        const int status = load_and_check_slots(tb, S, S_max, grp, tpv, slots);
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            continue;
        }
        for (int s = threadIdx.x; s <= S; s += kBandedThreads) band[s] = bands[int64_t(c) * (S_max + 1) + s];
        __syncthreads();
        if (banded_pass<false>(tb, slots, S, band, lo_tab, lo_pitch, w, 0, red_v, red_j) == kInf) {
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);      // the bands were bounds only
            continue;
        }
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        if (threadIdx.x == 0) generic_backtrack(w, S, L, sp);
        for (int s = S + 1 + threadIdx.x; s <= S_max; s += kBandedThreads) sp[s] = -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = threadIdx.x; s < S_max; s += kBandedThreads) df[s] = s < S ? slots.dev_first[s] : -1;
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
        if (wave == 0) {
            int64_t bott, iter;
            const int st = wave_score_partition(tb, S, slots.g, slots.k, sp, lane, bott, iter);
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = iter;
                out.status[c] = st;
            }
        }
    }
    // candidates the pre-pass rejected: no plan to report
    for (int n = blockIdx.x; n < n_dead; n += gridDim.x) {
        const uint32_t e = dead_list[n];
        write_failed(out, int(e & ((1u << fastdp::kDeadStatusShift) - 1u)), S_max, int(e >> fastdp::kDeadStatusShift));
    }
}

// The exact search (sweep over the cap of section 5.2.4 (2)) in int64, for tables without the
// 32-bit rows: the min-max pass gives t_S, then capped least-sum passes walk the caps exactly as
// the 32-bit kernel does (first at t_S, then down from ceil(T / B), skipping caps that the sums
// rule out; equal totals keep the lower cap).
__global__ __launch_bounds__(kThreads) void k2_generic_exact(TablesDev tb, CandDev cd, PlansDev out,
                                                              int32_t *n_passes, unsigned char *ws,
                                                              size_t ws_per_group) {
    __shared__ SlotInfo slots;
    __shared__ int32_t trial[kMaxStages + 1], kept[kMaxStages + 1];
    __shared__ int64_t scored[2];
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GenericSlice w = generic_slice(ws, ws_per_group, L);
    const int64_t m_cap = tb.M;

    // all threads: bottleneck and total of the cuts in trial[], by the cost model itself
    auto score_trial = [&](int S, int64_t &bott, int64_t &total) {
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
        if (wave == 0) {
            int64_t b, t;
            wave_score_partition(tb, S, slots.g, slots.k, trial, lane, b, t);
            if (lane == 0) { scored[0] = b; scored[1] = t; }
        }
        __syncthreads();
        bott = scored[0];
        total = scored[1];
    };

    for (int c = blockIdx.x; c < cd.C; c += gridDim.x) {
        __syncthreads();
        const int S = cd.cand_S[c];
        const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
        int status = load_and_check_slots(tb, S, S_max, grp, tpv, slots);
        if (status == HARP_CAND_OK && S > L) status = HARP_CAND_INFEASIBLE;
        if (status == HARP_CAND_OK && generic_pass<false>(tb, slots, S, w, 0)[L] == kInf)
            status = HARP_CAND_INFEASIBLE;
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            if (threadIdx.x == 0 && n_passes) n_passes[c] = 0;
            continue;
        }
        if (threadIdx.x == 0) generic_backtrack(w, S, L, trial);
        int64_t t_S, best_T, best_b;
        score_trial(S, t_S, best_T);
        best_b = t_S;
        for (int s = threadIdx.x; s <= S; s += kThreads) kept[s] = trial[s];
        int passes = 0;
        int64_t cap = t_S;
        while (S >= 2) {
            const int64_t sum = generic_pass<true>(tb, slots, S, w, cap)[L];
            if (sum == kInf) break;   // cannot happen at or above t_S
            if (threadIdx.x == 0) generic_backtrack(w, S, L, trial);
            int64_t b, T;
            score_trial(S, b, T);
            ++passes;
            if (T < best_T || (T == best_T && b <= best_b)) {   // equal totals: the lower cap; equal caps: the capped plan
                best_T = T;
                best_b = b;
                for (int s = threadIdx.x; s <= S; s += kThreads) kept[s] = trial[s];
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
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        for (int s = threadIdx.x; s <= S_max; s += kThreads) sp[s] = s <= S ? kept[s] : -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = threadIdx.x; s < S_max; s += kThreads) df[s] = s < S ? slots.dev_first[s] : -1;
        if (threadIdx.x == 0) {
            out.bottleneck[c] = best_b;
            out.iter_time[c] = best_T;
            out.status[c] = HARP_CAND_OK;
            if (n_passes) n_passes[c] = passes;
        }
    }
}

// The same search behind the pre-pass: the min-max pass and every capped pass run over the
// candidate's reachability bands with their ranges of previous cuts from the feasibility index
// (banded_pass); the walk over the caps is the one above.
__global__ __launch_bounds__(kBandedThreads) void k2_banded_exact(TablesDev tb, CandDev cd, PlansDev out,
                                                                   int32_t *n_passes, int *counts,
                                                                   const int32_t *live_list, const uint32_t *dead_list,
                                                                   const uint32_t *bands, const uint16_t *lo_tab,
                                                                   int lo_pitch, unsigned char *ws, size_t ws_per_group) {
    __shared__ SlotInfo slots;
    __shared__ uint32_t band[kMaxStages + 1];
    __shared__ int32_t trial[kMaxStages + 1], kept[kMaxStages + 1];
    __shared__ int64_t scored[2];
    __shared__ int64_t red_v[kBandedThreads / 64];
    __shared__ int red_j[kBandedThreads / 64];
    __shared__ int ticket;
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GenericSlice w = generic_slice(ws, ws_per_group, L);
    const int64_t m_cap = tb.M;
    const int n_live = counts[0], n_dead = counts[1];

    // all threads: bottleneck and total of the cuts in trial[], by the cost model itself
    auto score_trial = [&](int S, int64_t &bott, int64_t &total) {
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
        if (wave == 0) {
            int64_t b, t;
            wave_score_partition(tb, S, slots.g, slots.k, trial, lane, b, t);
            if (lane == 0) { scored[0] = b; scored[1] = t; }
        }
        __syncthreads();
        bott = scored[0];
        total = scored[1];
    };

    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) ticket = atomicAdd(&counts[5], 1);
        __syncthreads();
        const int n = ticket;
        if (n >= n_live) break;
        const int c = live_list[n];
        const int S = cd.cand_S[c];
        const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
        int status = load_and_check_slots(tb, S, S_max, grp, tpv, slots);
        for (int s = threadIdx.x; s <= S && status == HARP_CAND_OK; s += kBandedThreads)
            band[s] = bands[int64_t(c) * (S_max + 1) + s];
        __syncthreads();
        if (status == HARP_CAND_OK &&
            banded_pass<false>(tb, slots, S, band, lo_tab, lo_pitch, w, 0, red_v, red_j) == kInf)
            status = HARP_CAND_INFEASIBLE;
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            if (threadIdx.x == 0 && n_passes) n_passes[c] = 0;
            continue;
        }
        if (threadIdx.x == 0) generic_backtrack(w, S, L, trial);
        int64_t t_S, best_T, best_b;
        score_trial(S, t_S, best_T);
        best_b = t_S;
        for (int s = threadIdx.x; s <= S; s += kBandedThreads) kept[s] = trial[s];
        int passes = 0;
        int64_t cap = t_S;
        while (S >= 2) {
            const int64_t sum = banded_pass<true>(tb, slots, S, band, lo_tab, lo_pitch, w, cap, red_v, red_j);
            if (sum == kInf) break;   // cannot happen at or above t_S
            if (threadIdx.x == 0) generic_backtrack(w, S, L, trial);
            int64_t b, T;
            score_trial(S, b, T);
            ++passes;
            if (T < best_T || (T == best_T && b <= best_b)) {   // equal totals: the lower cap; equal caps: the capped plan
                best_T = T;
                best_b = b;
                for (int s = threadIdx.x; s <= S; s += kBandedThreads) kept[s] = trial[s];
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
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        for (int s = threadIdx.x; s <= S_max; s += kBandedThreads) sp[s] = s <= S ? kept[s] : -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = threadIdx.x; s < S_max; s += kBandedThreads) df[s] = s < S ? slots.dev_first[s] : -1;
        if (threadIdx.x == 0) {
            out.bottleneck[c] = best_b;
            out.iter_time[c] = best_T;
            out.status[c] = HARP_CAND_OK;
            if (n_passes) n_passes[c] = passes;
        }
    }
    // candidates the pre-pass rejected: no plan to report
    for (int n = blockIdx.x; n < n_dead; n += gridDim.x) {
        const uint32_t e = dead_list[n];
        const int c = int(e & ((1u << fastdp::kDeadStatusShift) - 1u));
        write_failed(out, c, S_max, int(e >> fastdp::kDeadStatusShift));
        if (threadIdx.x == 0 && n_passes) n_passes[c] = 0;
    }
}

// The capped suffix recurrence with H-1F1B warm-up counts (paper sections 4.1, 5.2.3: eq.
// dp_general, eq. dp_ni, eq. mem_cons) in int64, for tables without the 32-bit rows.  Slice of the
// workspace: two rows of suffix sums, two of counts, the row handed to the slot in front (sum plus
// twice the cut's transfer time; count the stage in front would have), back-pointers.
struct H1Slice {
    int64_t *G0, *G1, *H;
    int32_t *N0, *N1, *NN;
    uint16_t *arg;      // [S_max][L+1], row = slot
};

__device__ __forceinline__ H1Slice h1_slice(unsigned char *ws, size_t ws_per_group, int L) {
    unsigned char *mine = ws + size_t(blockIdx.x) * ws_per_group;
    H1Slice g;
    g.G0 = reinterpret_cast<int64_t *>(mine);
    g.G1 = g.G0 + (L + 1);
    g.H = g.G1 + (L + 1);
    g.N0 = reinterpret_cast<int32_t *>(g.H + (L + 1));
    g.N1 = g.N0 + (L + 1);
    g.NN = g.N1 + (L + 1);
    g.arg = reinterpret_cast<uint16_t *>(g.NN + (L + 1));
    return g;
}

__global__ __launch_bounds__(kThreads) void k2_generic_h1f1b(TablesDev tb, CandDev cd, const int64_t *t_max,
                                                              PlansDev out, int32_t *warmup,
                                                              unsigned char *ws, size_t ws_per_group) {
    __shared__ SlotInfo slots;
    __shared__ int32_t trial[kMaxStages + 1], count[kMaxStages];
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const H1Slice w = h1_slice(ws, ws_per_group, L);
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    const int64_t m_cap = tb.M;

    for (int c = blockIdx.x; c < cd.C; c += gridDim.x) {
        __syncthreads();
        const int S = cd.cand_S[c];
        const int64_t cap_t = t_max[c];
        const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
        int32_t *wu = warmup + int64_t(c) * S_max;
        int status = load_and_check_slots(tb, S, S_max, grp, tpv, slots);
        if (status == HARP_CAND_OK && cap_out_of_range(tb, cap_t)) status = HARP_CAND_INVALID;
        if (status == HARP_CAND_OK && (S > L || cap_t < 0)) status = HARP_CAND_INFEASIBLE;
        const int64_t *Gp = w.G0;
        if (status == HARP_CAND_OK) {
            for (int i = threadIdx.x; i <= L; i += kThreads) { w.G0[i] = (i == L) ? 0 : kInf; w.N0[i] = 0; }
            int64_t *Gn = w.G1;
            int32_t *Np = w.N0, *Nn = w.N1;
            int64_t *Gcur = w.G0;
            for (int slot = S - 1; slot >= 0; --slot) {
                const int s = S - slot;                     // stages from this slot to the end
                const int g = slots.g[slot], k = slots.k[slot];
                const int64_t tp = tb.tp[k];
                const int shift = tb.tp_shift[k];
                const int t = tb.group_type[g];
                const int64_t *pf = tb.PF(t), *pr = tb.PR(g, k);
                const int64_t capm = tp * tb.type_mem[t];
                const bool last = (slot == S - 1);
                const int64_t link = last ? 1 : tb.bw[int64_t(g) * tb.G + slots.g[slot + 1]];
                const int j_lo = slot + 1, j_hi = L - (s - 1);
                __syncthreads();                            // the previous slot's rows are complete
                // the row handed over by the slots behind, made ready for this slot's transitions
                for (int j = j_lo + threadIdx.x; j <= j_hi; j += kThreads) {
                    const int64_t cut = last ? 0 : (tb.act_bytes[j - 1] + link - 1) / link;
                    const int64_t rest = Gcur[j];
                    w.H[j] = (rest == kInf || cut > cap_t) ? kInf : rest + 2 * cut;
                    const int64_t x = 2 * cut - (cap_t >> 6);
                    const int64_t n = 1 + (x > 0 ? 1 : 0) + (x > cap_t ? 1 : 0) + Np[j];
                    w.NN[j] = int32_t(n < m_cap ? n : m_cap);
                }
                __syncthreads();
                const int i_lo = slot, i_hi = slot == 0 ? 0 : L - s;
                uint16_t *arg_row = w.arg + size_t(slot) * (L + 1);
                for (int i = i_lo + wave; i <= i_hi; i += kWaves) {
                    const int64_t pfi = pf[i], pri = pr[i], ppi = PP[i], psi = PS[i];
                    int64_t best = kInf;
                    int best_j = INT32_MAX, best_n = 0;
                    // end cuts in runs of 64 upwards; the stage time and its memory need with a count of
                    // one both grow with j, so once the highest cut of a run is above the cap or does
                    // not fit, no higher cut can be taken
                    for (int base = (i + 1 > j_lo ? i + 1 : j_lo); base <= j_hi; base += 64) {
                        const int j = base + lane;
                        if (j <= j_hi) {
                            const int64_t h = w.H[j];
                            const int64_t work = pf[j] - pfi;
                            const int64_t comp = shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp;
                            const int64_t time = comp + (pr[j] - pri);
                            const int n = w.NN[j];
                            if (h != kInf && time <= cap_t && (PP[j] - ppi) + int64_t(n) * (PS[j] - psi) <= capm &&
                                h + time < best) {
                                best = h + time; best_j = j; best_n = n;       // j rises within a lane
                            }
                        }
                        const int high = base + 63 < j_hi ? base + 63 : j_hi;
                        if (high == j_hi) break;
                        const int64_t work_h = pf[high] - pfi;
                        const int64_t time_h = (shift >= 0 ? (work_h + tp - 1) >> shift : (work_h + tp - 1) / tp) +
                                               (pr[high] - pri);
                        if (time_h > cap_t || (PP[high] - ppi) + (PS[high] - psi) > capm) break;
                    }
#pragma unroll
                    for (int d = 32; d >= 1; d >>= 1) {
                        const int64_t ov = __shfl_xor(best, d, 64);
                        const int oj = __shfl_xor(best_j, d, 64);
                        const int on = __shfl_xor(best_n, d, 64);
                        if (ov < best || (ov == best && oj < best_j)) { best = ov; best_j = oj; best_n = on; }
                    }
                    if (lane == 0) {
                        Gn[i] = best;
                        Nn[i] = best_n;
                        arg_row[i] = (uint16_t)(best == kInf ? 0 : best_j);
                    }
                }
                // cells of the next slot read Gn over [slot, ...]: everything it may touch is written
                // above, except starts this slot cannot use
                for (int i = i_hi + 1 + threadIdx.x; i <= L; i += kThreads) { Gn[i] = kInf; Nn[i] = 0; }
                int64_t *tg = Gcur; Gcur = Gn; Gn = tg;
                int32_t *tn = Np; Np = Nn; Nn = tn;
            }
            __syncthreads();
            Gp = Gcur;
            if (Gp[0] == kInf) status = HARP_CAND_INFEASIBLE;
        }
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            for (int s = threadIdx.x; s < S_max; s += kThreads) wu[s] = -1;
            continue;
        }
        const int64_t sum = Gp[0];
        if (threadIdx.x == 0) {
            int b = 0;
            for (int slot = 0; slot < S; ++slot) { trial[slot] = b; b = w.arg[size_t(slot) * (L + 1) + b]; }
            trial[S] = b;
            // counts by eq. Ni along the plan, from the last stage backwards
            int64_t n = 0;
            for (int slot = S - 1; slot >= 0; --slot) {
                int64_t cut = 0;
                if (slot < S - 1) {
                    const int64_t link = tb.bw[int64_t(slots.g[slot]) * tb.G + slots.g[slot + 1]];
                    cut = (tb.act_bytes[trial[slot + 1] - 1] + link - 1) / link;
                }
                const int64_t x = 2 * cut - (cap_t >> 6);
                n += 1 + (x > 0 ? 1 : 0) + (x > cap_t ? 1 : 0);
                n = n < m_cap ? n : m_cap;
                count[slot] = int32_t(n);
            }
        }
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        for (int s = threadIdx.x; s <= S_max; s += kThreads) sp[s] = s <= S ? trial[s] : -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = threadIdx.x; s < S_max; s += kThreads) {
            df[s] = s < S ? slots.dev_first[s] : -1;
            wu[s] = s < S ? count[s] : -1;
        }
        if (wave == 0) {
            int64_t bott, iter;
            wave_score_partition(tb, S, slots.g, slots.k, trial, lane, bott, iter);   // the plan's own bottleneck
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = sum + (m_cap - 1) * cap_t;
                out.status[c] = HARP_CAND_OK;
            }
        }
    }
}

}  // namespace

// The same recurrence behind the pre-pass.  The bands of the classic counts bound it from outside
// (H-1F1B's counts are never below the classic ones, so a stage that does not fit with the classic
// count does not fit at all): slot `slot` has the start cuts B[slot] .. F[slot], and a start cut i
// takes the end cuts max(i + 1, B[slot+1]) .. min(hi(i), F[slot+1]) upwards, hi(i) the highest end
// cut that fits with the classic count, from the feasibility index.  One lane per start cut; the
// scan stops at the cap (the stage time grows with the end cut).
__global__ __launch_bounds__(kBandedThreads) void k2_banded_h1f1b(TablesDev tb, CandDev cd, const int64_t *t_max,
                                                                   PlansDev out, int32_t *warmup, int *counts,
                                                                   const int32_t *live_list, const uint32_t *dead_list,
                                                                   const uint32_t *bands, const uint16_t *hi_tab,
                                                                   int idx_pitch, unsigned char *ws,
                                                                   size_t ws_per_group) {
    __shared__ SlotInfo slots;
    __shared__ uint32_t band[kMaxStages + 1];
    __shared__ int32_t trial[kMaxStages + 1], count[kMaxStages];
    __shared__ int ticket;
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const H1Slice w = h1_slice(ws, ws_per_group, L);
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    const int64_t m_cap = tb.M;
    const int n_live = counts[0], n_dead = counts[1];
    const int rows_per_n = tb.T * tb.n_tp;

    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) ticket = atomicAdd(&counts[5], 1);
        __syncthreads();
        const int n = ticket;
        if (n >= n_live) break;
        const int c = live_list[n];
        const int S = cd.cand_S[c];
        const int64_t cap_t = t_max[c];
        const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
        int32_t *wu = warmup + int64_t(c) * S_max;
        int status = load_and_check_slots(tb, S, S_max, grp, tpv, slots);
        if (status == HARP_CAND_OK && cap_out_of_range(tb, cap_t)) status = HARP_CAND_INVALID;
        if (status == HARP_CAND_OK && cap_t < 0) status = HARP_CAND_INFEASIBLE;
        const int64_t *Gp = w.G0;
        if (status == HARP_CAND_OK) {
            for (int s = threadIdx.x; s <= S; s += kBandedThreads) band[s] = bands[int64_t(c) * (S_max + 1) + s];
            if (threadIdx.x == 0) { w.G0[L] = 0; w.N0[L] = 0; }      // row S is the single cut L
            int64_t *Gn = w.G1;
            int32_t *Np = w.N0, *Nn = w.N1;
            int64_t *Gcur = w.G0;
            for (int slot = S - 1; slot >= 0; --slot) {
                const int g = slots.g[slot], k = slots.k[slot];
                const int64_t tp = tb.tp[k];
                const int shift = tb.tp_shift[k];
                const int t = tb.group_type[g];
                const int64_t *pf = tb.PF(t), *pr = tb.PR(g, k);
                const int64_t capm = tp * tb.type_mem[t];
                const bool last = (slot == S - 1);
                const int64_t link = last ? 1 : tb.bw[int64_t(g) * tb.G + slots.g[slot + 1]];
                __syncthreads();                            // the previous slot's rows and the bands are complete
                const uint32_t b0 = band[slot], b1 = band[slot + 1];
                const int il = fastdp::band_lo(b0), ih = fastdp::band_hi(b0);      // start cuts of this slot
                const int jl = fastdp::band_lo(b1), jh = fastdp::band_hi(b1);      // its end cuts
                const int n_classic = int((S - slot) < m_cap ? (S - slot) : m_cap);
                const uint16_t *hi_row = hi_tab + (size_t(n_classic - 1) * rows_per_n + size_t(t) * tb.n_tp + k) * idx_pitch;
                // the row handed over by the slots behind, made ready for this slot's transitions
                for (int j = jl + int(threadIdx.x); j <= jh; j += kBandedThreads) {
                    const int64_t cut = last ? 0 : (tb.act_bytes[j - 1] + link - 1) / link;
                    const int64_t rest = Gcur[j];
                    w.H[j] = (rest == kInf || cut > cap_t) ? kInf : rest + 2 * cut;
                    const int64_t x = 2 * cut - (cap_t >> 6);
                    const int64_t nn = 1 + (x > 0 ? 1 : 0) + (x > cap_t ? 1 : 0) + Np[j];
                    w.NN[j] = int32_t(nn < m_cap ? nn : m_cap);
                }
                __syncthreads();
                uint16_t *arg_row = w.arg + size_t(slot) * (L + 1);
                for (int i = il + int(threadIdx.x); i <= ih; i += kBandedThreads) {
                    const int64_t pfi = pf[i], pri = pr[i], ppi = PP[i], psi = PS[i];
                    const int reach = hi_row[i];
                    const int first = (i + 1) > jl ? (i + 1) : jl;
                    const int end = reach < jh ? reach : jh;
                    int64_t best = kInf;
                    int best_j = 0, best_n = 0;
                    for (int j = first; j <= end; ++j) {
                        const int64_t work = pf[j] - pfi;
                        const int64_t comp = shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp;
                        const int64_t time = comp + (pr[j] - pri);
                        if (time > cap_t) break;
                        const int64_t h = w.H[j];
                        const int nn = w.NN[j];
                        if (h != kInf && (PP[j] - ppi) + int64_t(nn) * (PS[j] - psi) <= capm && h + time < best) {
                            best = h + time; best_j = j; best_n = nn;          // j rises: the lowest end cut keeps a tie
                        }
                    }
                    Gn[i] = best;
                    Nn[i] = best_n;
                    arg_row[i] = (uint16_t)best_j;
                }
                int64_t *tg = Gcur; Gcur = Gn; Gn = tg;
                int32_t *tn = Np; Np = Nn; Nn = tn;
            }
            __syncthreads();
            Gp = Gcur;
            if (Gp[0] == kInf) status = HARP_CAND_INFEASIBLE;
        }
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            for (int s = threadIdx.x; s < S_max; s += kBandedThreads) wu[s] = -1;
            continue;
        }
        const int64_t sum = Gp[0];
        if (threadIdx.x == 0) {
            int b = 0;
            for (int slot = 0; slot < S; ++slot) { trial[slot] = b; b = w.arg[size_t(slot) * (L + 1) + b]; }
            trial[S] = b;
            // counts by eq. Ni along the plan, from the last stage backwards
            int64_t nn = 0;
            for (int slot = S - 1; slot >= 0; --slot) {
                int64_t cut = 0;
                if (slot < S - 1) {
                    const int64_t link = tb.bw[int64_t(slots.g[slot]) * tb.G + slots.g[slot + 1]];
                    cut = (tb.act_bytes[trial[slot + 1] - 1] + link - 1) / link;
                }
                const int64_t x = 2 * cut - (cap_t >> 6);
                nn += 1 + (x > 0 ? 1 : 0) + (x > cap_t ? 1 : 0);
                nn = nn < m_cap ? nn : m_cap;
                count[slot] = int32_t(nn);
            }
        }
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        for (int s = threadIdx.x; s <= S_max; s += kBandedThreads) sp[s] = s <= S ? trial[s] : -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = threadIdx.x; s < S_max; s += kBandedThreads) {
            df[s] = s < S ? slots.dev_first[s] : -1;
            wu[s] = s < S ? count[s] : -1;
        }
        if (wave == 0) {
            int64_t bott, iter;
            wave_score_partition(tb, S, slots.g, slots.k, trial, lane, bott, iter);   // the plan's own bottleneck
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = sum + (m_cap - 1) * cap_t;
                out.status[c] = HARP_CAND_OK;
            }
        }
    }
    // candidates the pre-pass rejected: no plan; a cap outside the accepted range is the caller's mistake first
    for (int n = blockIdx.x; n < n_dead; n += gridDim.x) {
        const uint32_t e = dead_list[n];
        const int c = int(e & ((1u << fastdp::kDeadStatusShift) - 1u));
        int status = int(e >> fastdp::kDeadStatusShift);
        if (status == HARP_CAND_INFEASIBLE && cap_out_of_range(tb, t_max[c])) status = HARP_CAND_INVALID;
        write_failed(out, c, S_max, status);
        for (int s = threadIdx.x; s < S_max; s += kBandedThreads) warmup[int64_t(c) * S_max + s] = -1;
    }
}

size_t plan_generic_h1f1b_ws_per_group(int L, int S_max) {
    size_t b = size_t(3) * (L + 1) * sizeof(int64_t) + size_t(3) * (L + 1) * sizeof(int32_t) +
               size_t(S_max) * (L + 1) * sizeof(uint16_t);
    return (b + 255) & ~size_t(255);
}

void launch_plan_generic_h1f1b(const TablesDev &tb, const CandDev &cd, const int64_t *t_max, const PlansDev &out,
                               int32_t *warmup, void *ws, int n_groups, bool banded, hipStream_t st) {
    if (banded) {
        const fastdp::FastWorkspace w = fastdp::carve(ws, fastdp::fast_shape(tb, cd), 0);
        launch_plan_prepass(tb, cd, ws, 0, st);
        const long long idx_rows = (long long)fastdp::lo_n_max(tb.L, cd.S_max, tb.M) * tb.T * tb.n_tp;
        const int idx_pitch = int(fastdp::lo_pitch(tb.L));
        hipLaunchKernelGGL(k2_banded_h1f1b, dim3(n_groups), dim3(kBandedThreads), 0, st, tb, cd, t_max, out, warmup,
                           w.counts, w.live_list, w.dead_list, w.bands, w.lo_tab + idx_rows * idx_pitch, idx_pitch,
                           static_cast<unsigned char *>(ws) + w.total, plan_generic_h1f1b_ws_per_group(tb.L, cd.S_max));
        return;
    }
    hipLaunchKernelGGL(k2_generic_h1f1b, dim3(n_groups), dim3(kThreads), 0, st, tb, cd, t_max, out, warmup,
                       static_cast<unsigned char *>(ws), plan_generic_h1f1b_ws_per_group(tb.L, cd.S_max));
}

size_t plan_generic_ws_per_group(int L, int S_max) {
    size_t b = size_t(2) * (L + 1) * sizeof(int64_t) + size_t(S_max) * (L + 1) * sizeof(uint16_t);
    return (b + 255) & ~size_t(255);
}

// banded: the workspace starts with the pre-pass area (plan_fast_ws_bytes with no slices) and the
// workgroups' slices follow it.
void launch_plan_generic(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                         int n_groups, bool banded, hipStream_t st) {
    if (!banded) {
        hipLaunchKernelGGL(k2_generic, dim3(n_groups), dim3(kThreads), generic_lds_bytes(tb.L), st, tb, cd, out,
                           static_cast<unsigned char *>(ws), plan_generic_ws_per_group(tb.L, cd.S_max));
        return;
    }
    const fastdp::FastWorkspace w = fastdp::carve(ws, fastdp::fast_shape(tb, cd), 0);
    launch_plan_prepass(tb, cd, ws, 0, st);
    hipLaunchKernelGGL(k2_banded, dim3(n_groups), dim3(kBandedThreads), banded_lds_bytes(tb.L), st, tb, cd, out,
                       w.counts, w.live_list, w.dead_list, w.bands, w.lo_tab, int(fastdp::lo_pitch(tb.L)),
                       static_cast<unsigned char *>(ws) + w.total, plan_generic_ws_per_group(tb.L, cd.S_max));
}

void launch_plan_generic_exact(const TablesDev &tb, const CandDev &cd, const PlansDev &out, int32_t *n_passes,
                               void *ws, int n_groups, bool banded, hipStream_t st) {
    if (banded) {
        const fastdp::FastWorkspace w = fastdp::carve(ws, fastdp::fast_shape(tb, cd), 0);
        launch_plan_prepass(tb, cd, ws, 0, st);
        hipLaunchKernelGGL(k2_banded_exact, dim3(n_groups), dim3(kBandedThreads), banded_lds_bytes(tb.L), st, tb, cd,
                           out, n_passes, w.counts, w.live_list, w.dead_list, w.bands, w.lo_tab,
                           int(fastdp::lo_pitch(tb.L)), static_cast<unsigned char *>(ws) + w.total,
                           plan_generic_ws_per_group(tb.L, cd.S_max));
        return;
    }
    hipLaunchKernelGGL(k2_generic_exact, dim3(n_groups), dim3(kThreads), generic_lds_bytes(tb.L), st, tb, cd, out, n_passes,
                       static_cast<unsigned char *>(ws), plan_generic_ws_per_group(tb.L, cd.S_max));
}

}  // namespace harp
