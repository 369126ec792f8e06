// The capped recurrence with H-1F1B warm-up counts (paper sections 4.1 and 5.2.3), 32-bit path.
//
// Under H-1F1B the last stage launches one forward microbatch during warm-up and every earlier
// stage launches delta more than the stage after it (eq. Ni), with delta in {1, 2, 3} growing with
// the transfer time of the cut between them relative to the cap t_max (eq. dp_ni; integer form:
// slack = t_max / 64 rounded down, delta = 1 if 2c <= slack, 2 if 2c - slack <= t_max, else 3).
// A stage's memory need depends on its count (eq. mem_cons), and the count depends on everything
// behind the stage, so the recurrence runs in the paper's own suffix direction (eq. dp_general):
// the state "the last stages, from slot sigma on, start at operator i" holds the least sum of
// (t + 2c) under the cap and carries the warm-up count of its first stage as determined by the
// continuation that attained the least sum.  Counts never exceed the number of microbatches.
//
// Mapping: one wavefront per live candidate at a time (64-thread workgroups), one lane per cell
// of the current slot's reachability band (the bands of the pre-pass were computed with the classic
// 1F1B counts, which are never larger than H-1F1B's, so they remain outer bounds), rows in LDS that
// hold the cuts one slot touches; a candidate whose widest slot does not fit the wavefront's LDS
// share is queued for a second launch with one 256-thread workgroup per candidate and rows over the
// whole sequence, which is also the form the 64-bit instantiation has.
// The row handed from slot sigma+1 to slot sigma is stored ready for use: entry j holds the
// suffix sum plus twice the transfer time of the cut at j (infinity when that transfer exceeds the
// cap) and the count the stage in front of j would have, so a transition is one stage time, one
// memory test and one add.  Scans run upwards in j with a strict comparison, which keeps the lowest j
// among equal sums; the stage time grows with j and stops the scan at the cap, and the scan ends at
// the highest end cut that fits with the slot's classic count (from the pre-pass's feasibility
// index: a larger count cannot fit where the classic one does not).
//
// Sums are 32-bit while they stay below 2^31 - 1 - cap, so that a stored sum plus any admissible
// stage time cannot reach infinity (2^31); a candidate for which some cell would exceed that is
// queued and redone by the instantiation with 64-bit sums.
#include "fast_common.h"
#include "harp_internal.h"
#include "plan_common.h"

namespace harp {

using namespace fastdp;

namespace {

constexpr int kTail = 4;     // spare entries behind a row: a group of four may overrun the band

template <typename SumT> struct H1Traits;
template <> struct H1Traits<uint32_t> {
    static constexpr uint32_t inf = 0x80000000u;
    struct alignas(8) Entry { uint32_t h, nn; };
};
template <> struct H1Traits<uint64_t> {
    static constexpr uint64_t inf = uint64_t(1) << 62;
    struct alignas(16) Entry { uint64_t h; uint32_t nn; uint32_t unused; };
};

struct alignas(16) MemPair { int64_t pp, ps; };

// c <= cap, so the quotient of eq. dp_ni is 0, 1 or 2 and needs no division.
__device__ __forceinline__ uint32_t h1f1b_delta(uint32_t c, int64_t cap) {
    const int64_t x = 2 * int64_t(c) - (cap >> 6);
    return 1u + (x > 0 ? 1u : 0u) + (x > cap ? 1u : 0u);
}

// LDS in front of the rows: per-slot constants, two scalars, band and trial cuts, two flags, the
// wavefronts' ranges of finite sums, index-row offsets, the plan's deltas, slot lists
__host__ __device__ inline size_t h1f1b_small_bytes(int S_max) {
    const size_t b = size_t(S_max) * sizeof(StageConst) + 16 + size_t(S_max + 1) * 8 + 8 + 64 + size_t(S_max) * 11;
    return (b + 15) & ~size_t(15);
}
// bytes per cut of the rows in LDS when every row is sized for one slot: one row of memory sums, two
// of entries, one of times
__host__ __device__ inline size_t h1f1b_cut_bytes(size_t entry) { return sizeof(MemPair) + 2 * entry + 4; }

// counts: [0] live, [1] dead, [2] queued for 64-bit sums, [6] and [7] tickets of the 32- and 64-bit
// kernels, [10] candidates queued for rows over the whole sequence, [11] next item of that list.
// Both queues sit in the unused tail of the dead list, the 64-bit one from its front, the other from
// its back.
//
// kMode 0: a workgroup per candidate, LDS rows with an entry for every cut.  kMode 1: a wavefront
// per candidate (64-thread workgroups), LDS rows that hold the cuts one slot touches (a slot's cells
// and continuations: B[slot] .. F[slot+1]), sized for the candidate's widest slot; a candidate that
// does not fit is queued.  kMode 2: as 0, on the candidates queued by 1.
template <typename SumT, int kMode>
__device__ __forceinline__ void h1f1b_body(const TablesDev &tb, const CandDev &cd, const int64_t *t_max,
                                           const PlansDev &out, int32_t *warmup, int *counts,
                                           const int32_t *live_list, uint32_t *dead_list,
                                           const uint32_t *bands, const uint16_t *hi_tab, int idx_pitch,
                                           unsigned char *arg_base, size_t arg_per_group, int row_len,
                                           int arg_pitch) {
    using Entry = typename H1Traits<SumT>::Entry;
    constexpr SumT kInfSum = H1Traits<SumT>::inf;
    constexpr bool kWide = sizeof(SumT) == 8;
    constexpr bool kBandRows = kMode == 1;
    extern __shared__ __align__(16) unsigned char lds_raw[];

    const int L = tb.L, S_max = cd.S_max;
    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = uniform(tid >> 6);
    StageConst *sc = reinterpret_cast<StageConst *>(lds_raw);                          // [S_max]
    uint64_t *scal = reinterpret_cast<uint64_t *>(sc + S_max);                         // [2]
    uint32_t *band = reinterpret_cast<uint32_t *>(scal + 2);                           // [S_max + 1]
    int32_t *trial = reinterpret_cast<int32_t *>(band + S_max + 1);                    // [S_max + 1]
    uint32_t *flags = reinterpret_cast<uint32_t *>(trial + S_max + 1);                 // [2]: ticket, overflow
    // element offset of each slot's row of the feasibility index: the highest end cut that fits with the
    // classic count of the slot, an outer bound for H-1F1B's (its counts are never below the classic ones)
    int32_t *fin_w = reinterpret_cast<int32_t *>(flags + 2);                           // [2][4][2]: per slot parity and wavefront, lowest and highest cell with a finite sum
    uint32_t *hi_off = reinterpret_cast<uint32_t *>(fin_w + 16);                       // [S_max]
    uint32_t *deltas = hi_off + S_max;                                                 // [S_max]
    uint16_t *slot_g = reinterpret_cast<uint16_t *>(deltas + S_max);                   // [S_max]
    uint8_t *slot_k = reinterpret_cast<uint8_t *>(slot_g + S_max);                     // [S_max]
    // Rows of row_len entries.  Whole-sequence form: one row of memory sums, two of entries, two of
    // times; entry x of a row is cut x.  Slot-sized form: a row's entry 0 is the lowest cut of the
    // slot it serves, and the memory sums and times of the slot in front take the place of this
    // slot's once its cells are done (one wavefront: its LDS operations execute in order).
    MemPair *mem0 = reinterpret_cast<MemPair *>(lds_raw + h1f1b_small_bytes(S_max));
    MemPair *mem1 = mem0;
    Entry *rows0 = reinterpret_cast<Entry *>(mem1 + row_len);
    Entry *rows1 = rows0 + row_len;
    uint32_t *prow0 = reinterpret_cast<uint32_t *>(rows1 + row_len);
    uint32_t *prow1 = kBandRows ? prow0 : prow0 + row_len;
    uint16_t *arg = reinterpret_cast<uint16_t *>(arg_base + size_t(blockIdx.x) * arg_per_group);
    const int n_dead = counts[1];
    const int n_items = kWide ? counts[2] : kMode == 2 ? counts[10] : counts[0];
    int *next_item = counts + (kWide ? 7 : kMode == 2 ? 11 : 6);
    const int64_t m_cap = tb.M;
    const int64_t *PP = tb.PP(), *PS = tb.PS();

    // the running sums of parameter and stash bytes are the same for every candidate
    if (!kBandRows) {
        for (int j = tid; j <= L; j += nthreads) mem0[j] = MemPair{PP[j], PS[j]};
        for (int j = L + 1 + tid; j < row_len; j += nthreads) mem0[j] = MemPair{0, 0};
        for (int j = L + 1 + tid; j < row_len; j += nthreads) { prow0[j] = 0; prow1[j] = 0; }
    }

    for (;;) {
        __syncthreads();   // the previous candidate's tail has finished with LDS
        if (tid == 0) { flags[0] = (uint32_t)atomicAdd(next_item, 1); flags[1] = 0; }
        __syncthreads();
        const int n = uniform((int)flags[0]);
        if (n >= n_items) break;
        const int c = kWide ? int(dead_list[n_dead + n]) : kMode == 2 ? int(dead_list[cd.C - 1 - n]) : live_list[n];
        const int S = cd.cand_S[c];
        const int64_t cap64 = t_max[c];
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        int32_t *wu = warmup + int64_t(c) * S_max;
        if (cap64 < 0 || cap_out_of_range(tb, cap64)) {   // no time fits under a negative cap; too large a cap is refused
            write_failed(out, c, S_max, cap64 < 0 ? HARP_CAND_INFEASIBLE : HARP_CAND_INVALID);
            for (int s = tid; s < S_max; s += nthreads) wu[s] = -1;
            continue;
        }
        const uint32_t tcap = (uint32_t)(cap64 > 0x7FFFFFFFll ? 0x7FFFFFFFll : cap64);   // no time here is larger
        {
            const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
            const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
            for (int s = tid; s < S; s += nthreads) {
                const int g = grp[s], k = tp_index(tb, tpv[s]);
                const int g_next = s + 1 < S ? grp[s + 1] : g;
                slot_g[s] = (uint16_t)g;
                slot_k[s] = (uint8_t)k;
                sc[s].cap = int64_t(tb.tp[k]) * tb.type_mem[tb.group_type[g]];
                sc[s].p_row = uint32_t((int64_t(g) * tb.n_tp + k) * tb.pitch32);
                sc[s].cm_row_shift = uint32_t((int64_t(g) * tb.G + g_next) * tb.pitch32) |
                                     (uint32_t(tb.tp_shift[k]) << 27);
                int32_t first = tb.group_base[g];
                for (int q = s - 1; q >= 0 && grp[q] == g; --q) first += tpv[q];
                df[s] = first;
                const int n_classic = int((S - s) < m_cap ? (S - s) : m_cap);
                hi_off[s] = uint32_t((int64_t(n_classic - 1) * tb.T * tb.n_tp + int64_t(tb.group_type[g]) * tb.n_tp + k) *
                                     idx_pitch);
            }
            for (int s = S + tid; s < S_max; s += nthreads) df[s] = -1;
            for (int s = tid; s <= S; s += nthreads) band[s] = bands[int64_t(c) * (S_max + 1) + s];
        }
        // stored sums stay this small, so that adding an admissible stage time cannot reach infinity
        const uint64_t limit = kWide ? uint64_t(kInfSum) - 1 : uint64_t(kInfSum) - 1 - tcap;
        __syncthreads();          // slot constants and bands are in LDS
        if (kBandRows) {
            // a slot touches its cells and its continuations, B[slot] .. F[slot+1], and up to kTail
            // entries behind them
            int span = 0;
            for (int s = tid; s < S; s += nthreads) {
                const int w = band_hi(band[s + 1]) - (s == 0 ? 0 : band_lo(band[s])) + 1;
                span = w > span ? w : span;
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const int o = __shfl_xor(span, d, 64);
                span = o > span ? o : span;
            }
            if (uniform(span) + kTail > row_len) {
                if (tid == 0) dead_list[cd.C - 1 - atomicAdd(&counts[10], 1)] = uint32_t(c);
                continue;
            }
        }
        // prologue: behind the last stage no operators are left and nothing is launched yet (the last
        // stage itself adds delta(0) = 1); the fused time row of the last slot over its cells and its
        // single continuation
        {
            const int il0 = (S == 1) ? 0 : band_lo((uint32_t)uniform((int)band[S - 1]));
            Entry *row_S = rows0 - (kBandRows ? L : 0);
            if (tid == 0) { row_S[L].h = 0; row_S[L].nn = 1; }
            if (tid >= 1 && tid <= kTail) row_S[L + tid].h = kInfSum;
            const uint32_t *p32 = tb.P32 + (uint32_t)uniform((int)sc[S - 1].p_row);
            uint32_t *pr = prow0 - (kBandRows ? il0 : 0);
            for (int x = il0 + tid; x <= L; x += nthreads) pr[x] = p32[x];
            if (kBandRows) {
                MemPair *mm = mem0 - il0;
                for (int x = il0 + tid; x <= L + kTail - 1; x += nthreads)
                    mm[x] = x <= L ? MemPair{PP[x], PS[x]} : MemPair{0, 0};
            }
        }
        lds_barrier();
        int cur = 0, pcur = 0;
        const int wave_first = wave * 64;
        // Continuations with a finite sum lie in [fin_lo, fin_hi]: scans are clamped to that range,
        // which changes no value, and a row without a finite sum ends the candidate - no plan - at
        // once.  Every wavefront keeps the range of its own cells (one ballot per round of cells); a
        // workgroup's wavefronts exchange theirs through LDS at the barrier that ends a slot.
        int fin_lo = L, fin_hi = L;
        auto end_of_slot = [&](int slot, int new_lo, int new_hi) -> bool {      // true: no continuation is left
            if (!kBandRows && lane == 0) {
                fin_w[((slot & 1) * 4 + wave) * 2] = new_lo;
                fin_w[((slot & 1) * 4 + wave) * 2 + 1] = new_hi;
            }
            lds_barrier();
            if (slot == 0) return false;
            if (kBandRows) {
                // lane 0 has a cell in every round that any lane has one in: its copy is complete
                fin_lo = uniform(new_lo);
                fin_hi = uniform(new_hi);
            } else {
                int lo = INT32_MAX, hi = -1;
                for (int w = 0; w < int(nthreads >> 6); ++w) {
                    const int wl = fin_w[((slot & 1) * 4 + w) * 2], wh = fin_w[((slot & 1) * 4 + w) * 2 + 1];
                    lo = wl < lo ? wl : lo;
                    hi = wh > hi ? wh : hi;
                }
                fin_lo = uniform(lo);
                fin_hi = uniform(hi);
            }
            if (fin_hi < 0 && tid == 0) scal[0] = uint64_t(kInfSum);
            return fin_hi < 0;
        };
        for (int slot = S - 1; slot >= 0; --slot) {
            const uint32_t b0 = (uint32_t)uniform((int)band[slot]);
            const uint32_t b1 = (uint32_t)uniform((int)band[slot + 1]);
            const int il = slot == 0 ? 0 : band_lo(b0), ih = slot == 0 ? 0 : band_hi(b0);   // cells
            const int jl = band_lo(b1), jh = band_hi(b1);                                     // continuations
            const int jl_f = fin_lo > jl ? fin_lo : jl;
            const int jh_f = fin_hi < jh ? fin_hi : jh;
            int new_lo = INT32_MAX, new_hi = -1;        // this wavefront's cells with a finite sum
            // what the slot in front will read of its own time row: its cells and this slot's cells
            const int nl = slot >= 2 ? band_lo((uint32_t)uniform((int)band[slot - 1])) : 0;
            const bool stage_next = slot >= 1;
            // a wave whose lanes own neither a cell nor a staged entry only keeps the barrier
            if (il + wave_first > ih && (!stage_next || nl + wave_first > ih)) {
                if (end_of_slot(slot, INT32_MAX, -1)) break;
                cur ^= 1;
                pcur ^= 1;
                continue;
            }
            const uint32_t rsv = (uint32_t)uniform((int)sc[slot].cm_row_shift);
            const int shift = int(rsv >> 27);
            const uint32_t tp = 1u << shift;
            const int64_t capm = uniform64(sc[slot].cap);
            const uint16_t *hi_row = hi_tab + (uint32_t)uniform((int)hi_off[slot]);
            // rows of this slot start at its lowest cell il, the row of continuations at jl, the rows
            // staged for the slot in front at nl
            const uint32_t *pr_cur = (pcur ? prow1 : prow0) - (kBandRows ? il : 0);
            uint32_t *pr_next = (pcur ? prow0 : prow1) - (kBandRows ? nl : 0);
            const MemPair *mem = (pcur ? mem1 : mem0) - (kBandRows ? il : 0);
            MemPair *mem_next = (pcur ? mem0 : mem1) - (kBandRows ? nl : 0);
            const Entry *prev = (cur ? rows1 : rows0) - (kBandRows ? jl : 0);
            Entry *next = (cur ? rows0 : rows1) - (kBandRows ? il : 0);
            // the cut in front of this slot's stage (between slot - 1 and slot)
            const uint32_t *cm_front = stage_next ? tb.CM + ((uint32_t)uniform((int)sc[slot - 1].cm_row_shift) & kRowMask)
                                                  : nullptr;
            const uint32_t *p32_n = stage_next ? tb.P32 + (uint32_t)uniform((int)sc[slot - 1].p_row) : nullptr;
            // requests for the slot in front: entry xn of its time row, and this lane's own cut time
            const int xn = nl + tid;
            uint32_t p_n = 0, cf_first = 0;
            if (stage_next && xn <= ih) p_n = p32_n[xn];
            if (stage_next && il + tid <= ih) cf_first = cm_front[il + tid];

            bool first_trip = true;
            for (int i = il + tid; i <= ih; i += nthreads) {
                const MemPair mi = mem[i];
                const uint32_t xi = pr_cur[i];
                SumT best = kInfSum;
                uint32_t best_n = 0;
                int best_j = 0;
                int j = (i + 1) > jl_f ? (i + 1) : jl_f;
                // end cuts beyond the classic count's reach cannot fit with a larger count either
                const int reach = hi_row[i];
                const int end = reach < jh_f ? reach : jh_f;
                bool more = j <= end;
                while (more) {
                    uint32_t tj = 0;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        // entries behind the band (up to kTail behind L) hold an infinite sum; what
                        // the other rows hold there is never used
                        const Entry e = prev[j + u];
                        const MemPair mj = mem[j + u];
                        tj = (pr_cur[j + u] + tp - 1 - xi) >> shift;
                        const int64_t dpp = mj.pp - mi.pp, dps = mj.ps - mi.ps;
                        const bool fits = dpp + int64_t(e.nn) * dps <= capm;
                        const SumT v = e.h + tj;
                        const bool upd = fits & (tj <= tcap) & (v < best) & ((j + u) <= end);
                        best = upd ? v : best;
                        best_n = upd ? e.nn : best_n;
                        best_j = upd ? (j + u) : best_j;
                    }
                    more = ((j + 4) <= end) & (tj <= tcap);
                    j += 4;
                }
                arg[slot * arg_pitch + i] = (uint16_t)best_j;
                if (stage_next) {
                    const uint32_t cf = first_trip ? cf_first : cm_front[i];
                    const uint64_t total = uint64_t(best) + 2ull * cf;
                    const bool reach = (best < kInfSum) & (cf <= tcap);
                    if (reach & (total > limit)) flags[1] = 1;        // needs 64-bit sums
                    const bool finite = reach & (total <= limit);
                    next[i].h = finite ? SumT(total) : kInfSum;
                    {
                        // lanes hold consecutive cells from i - lane on: the lowest and the highest lane with
                        // a finite sum bound this round's cells
                        const unsigned long long fm = __ballot(finite);
                        if (fm != 0) {
                            const int base = uniform(i - lane);
                            const int lo_r = base + __ffsll((long long)fm) - 1, hi_r = base + 63 - __clzll((long long)fm);
                            new_lo = lo_r < new_lo ? lo_r : new_lo;
                            new_hi = hi_r > new_hi ? hi_r : new_hi;
                        }
                    }
                    const uint32_t nn = h1f1b_delta(cf, cap64) + best_n;
                    next[i].nn = nn < uint32_t(m_cap) ? nn : uint32_t(m_cap);
                } else {
                    scal[0] = uint64_t(best);
                }
                first_trip = false;
            }
            if (stage_next) {
                if (tid < kTail) next[ih + 1 + tid].h = kInfSum;     // behind the band
                if (xn <= ih) pr_next[xn] = p_n;
                for (int x = xn + nthreads; x <= ih; x += nthreads) pr_next[x] = p32_n[x];
                if (kBandRows) {
                    for (int x = xn; x <= ih + kTail - 1; x += nthreads)
                        mem_next[x] = x <= L ? MemPair{PP[x], PS[x]} : MemPair{0, 0};
                }
            }
            if (end_of_slot(slot, new_lo, new_hi)) break;
            cur ^= 1;
            pcur ^= 1;
        }
        __syncthreads();
        if (!kWide && uniform((int)flags[1]) != 0) {
            if (tid == 0) dead_list[n_dead + atomicAdd(&counts[2], 1)] = uint32_t(c);
            continue;
        }
        const uint64_t sum = (uint64_t)uniform64((int64_t)scal[0]);
        if (sum >= uint64_t(kInfSum)) {
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            for (int s = tid; s < S_max; s += nthreads) wu[s] = -1;
            continue;
        }
        if (tid == 0) {
            int b = 0;
            for (int slot = 0; slot < S; ++slot) {
                trial[slot] = b;
                b = arg[slot * arg_pitch + b];
                b = b <= L ? b : L;      // a finite sum only chains through cuts inside the row
            }
            trial[S] = b;
        }
        __syncthreads();
        // one lane per stage: the plan's own bottleneck, and the counts by eq. Ni along the plan
        if (wave == 0) {
            uint32_t w = 0;
            for (int s = lane; s < S; s += 64) {
                const int j = trial[s], i = trial[s + 1];
                const uint32_t rsl = sc[s].cm_row_shift;
                const int shift = int(rsl >> 27);
                const uint32_t *p = tb.P32 + sc[s].p_row;
                const uint32_t t = (p[i] + (1u << shift) - 1u - p[j]) >> shift;
                const uint32_t cu = s < S - 1 ? tb.CM[(rsl & kRowMask) + uint32_t(i)] : 0u;
                const uint32_t m = t > cu ? t : cu;
                w = w > m ? w : m;
                deltas[s] = s < S - 1 ? h1f1b_delta(cu, cap64) : 1u;
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const uint32_t ow = __shfl_xor(w, d, 64);
                w = w > ow ? w : ow;
            }
            if (lane == 0) {
                out.bottleneck[c] = int64_t(w);
                out.iter_time[c] = int64_t(sum) + (m_cap - 1) * cap64;
                out.status[c] = HARP_CAND_OK;
            }
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t nrun = 0;
            for (int s = S - 1; s >= 0; --s) {
                nrun += deltas[s];
                nrun = nrun < uint32_t(m_cap) ? nrun : uint32_t(m_cap);
                wu[s] = int32_t(nrun);
            }
        }
        for (int s = tid; s <= S_max; s += nthreads) sp[s] = s <= S ? trial[s] : -1;
        for (int s = S + tid; s < S_max; s += nthreads) wu[s] = -1;
    }
    // candidates the pre-pass rejected: no plan to report
    if (!kWide && kMode != 2) {
        for (int n = blockIdx.x; n < n_dead; n += gridDim.x) {
            const uint32_t e = dead_list[n];
            const int c = int(e & ((1u << kDeadStatusShift) - 1u));
            const int st = cap_out_of_range(tb, t_max[c]) ? HARP_CAND_INVALID : int(e >> kDeadStatusShift);
            write_failed(out, c, S_max, st);
            for (int s = tid; s < S_max; s += nthreads) warmup[int64_t(c) * S_max + s] = -1;
        }
    }
}

#define HARP_H1F1B_KERNEL(NAME, BOUNDS, SUM, MODE)                                                                  \
    __global__ BOUNDS void NAME(TablesDev tb, CandDev cd, const int64_t *t_max, PlansDev out, int32_t *warmup,     \
                                int *counts, const int32_t *live_list, uint32_t *dead_list, const uint32_t *bands, \
                                const uint16_t *hi_tab, int idx_pitch, unsigned char *arg_base,                    \
                                size_t arg_per_group, int row_len, int arg_pitch) {                                \
        h1f1b_body<SUM, MODE>(tb, cd, t_max, out, warmup, counts, live_list, dead_list, bands, hi_tab, idx_pitch,  \
                              arg_base, arg_per_group, row_len, arg_pitch);                                        \
    }
HARP_H1F1B_KERNEL(k2_h1f1b, __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(5, 5))), uint32_t, 1)
HARP_H1F1B_KERNEL(k2_h1f1b_rows, __launch_bounds__(kFastThreads) __attribute__((amdgpu_waves_per_eu(8, 8))), uint32_t, 2)
HARP_H1F1B_KERNEL(k2_h1f1b_wide, __launch_bounds__(kFastThreads), uint64_t, 0)
#undef HARP_H1F1B_KERNEL

int h1f1b_row_len(int L) { return (L + 1 + kTail + 7) / 8 * 8; }

// whole-sequence rows: one of memory sums, two of entries, two of times
size_t h1f1b_lds_bytes(int L, int S_max, size_t entry) {
    return h1f1b_small_bytes(S_max) + size_t(h1f1b_row_len(L)) * (sizeof(MemPair) + 2 * entry + 8);
}

}  // namespace

// Runs the pre-pass itself (launch_plan_fast's first two kernels are shared through
// launch_plan_prepass) and then the three instantiations.  n_groups: resident 256-thread workgroups;
// n_slices: back-pointer slices in the workspace (the wavefront-per-candidate launch runs at most
// that many).
void launch_plan_h1f1b(const TablesDev &tb, const CandDev &cd, const int64_t *t_max, const PlansDev &out,
                       int32_t *warmup, void *ws, int n_groups, int n_slices, int n_cu, hipStream_t st) {
    const FastWorkspace w = carve(ws, fast_shape(tb, cd), n_groups);
    launch_plan_prepass(tb, cd, ws, n_groups, st);
    const int row_len = h1f1b_row_len(tb.L);
    const int idx_pitch = int(lo_pitch(tb.L));
    const uint16_t *hi_tab = w.lo_tab + (long long)lo_n_max(tb.L, cd.S_max, tb.M) * tb.T * tb.n_tp * idx_pitch;
    const size_t per_group = fast_arg_per_group(tb.L, cd.S_max);
    const int arg_pitch = fast_row_len(tb.L);
    // Wavefronts per CU of the first launch and the row entries their LDS share leaves: as many
    // wavefronts as hold rows for the whole sequence, between 14 and 24 (measured on the 512-operator
    // workload, where such rows would leave 7: 10 per CU 8.9 ms, 12 7.7, 14 7.6, 16 7.9, 20 10.4 - the
    // smaller the share, the more candidates leave for the second launch; on the 160-operator one,
    // where 22 fit: 16 per CU 2.2 ms, 20 2.0).
    const size_t small = h1f1b_small_bytes(cd.S_max);
    int per_cu = int((size_t(160) << 10) / (small + size_t(row_len) * h1f1b_cut_bytes(8) + 128));
    per_cu = per_cu < 14 ? 14 : (per_cu > 24 ? 24 : per_cu);
    const size_t share = ((size_t(160) << 10) / per_cu - 128) & ~size_t(15);
    int entries = share > small + h1f1b_cut_bytes(8) * 16 ? int((share - small) / h1f1b_cut_bytes(8)) & ~1 : 16;
    if (entries > row_len) entries = row_len;
    int n_waves = per_cu * n_cu;
    if (n_waves > n_slices) n_waves = n_slices;
    if (n_waves > cd.C) n_waves = cd.C;
    if (n_waves < 1) n_waves = 1;
    hipLaunchKernelGGL(k2_h1f1b, dim3(n_waves), dim3(64), small + size_t(entries) * h1f1b_cut_bytes(8), st, tb, cd,
                       t_max, out, warmup, w.counts, w.live_list, w.dead_list, w.bands, hi_tab, idx_pitch, w.arg,
                       per_group, entries, arg_pitch);
    if (entries < row_len)
        hipLaunchKernelGGL(k2_h1f1b_rows, dim3(n_groups), dim3(kFastThreads), h1f1b_lds_bytes(tb.L, cd.S_max, 8),
                           st, tb, cd, t_max, out, warmup, w.counts, w.live_list, w.dead_list, w.bands, hi_tab,
                           idx_pitch, w.arg, per_group, row_len, arg_pitch);
    hipLaunchKernelGGL(k2_h1f1b_wide, dim3(n_groups), dim3(kFastThreads), h1f1b_lds_bytes(tb.L, cd.S_max, 16), st,
                       tb, cd, t_max, out, warmup, w.counts, w.live_list, w.dead_list, w.bands, hi_tab, idx_pitch,
                       w.arg, per_group, row_len, arg_pitch);
}

}  // namespace harp
