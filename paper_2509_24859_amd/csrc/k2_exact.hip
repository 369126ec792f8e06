// Exact optimum of the iteration-time model for every candidate: the t_max sweep of the paper's
// section 5.2.4 (2) on top of the capped recurrence of section 5.2.3.
//
// For a cap t_max on every stage and transfer time (constraints (i), (ii)) and the memory limit
// (constraint (iii), eq. mem_cons), the capped recurrence finds the partition with the least
//   sum_s (t_s + 2 c_s);
// the iteration time of eq. gpipe_cost_model is that sum plus (B - 1) t_max, and the optimum over
// all partitions is the least such total over the caps between t_S, the smallest feasible cap (what
// the min-max planner found), and t_E = ceil(T(t_S) / B), beyond which no cap can win.
//
// Only caps that are the bottleneck of their own least-sum plan can attain the optimum (a plan
// whose bottleneck is below the cap is found again, with a smaller total, at that bottleneck), so
// the sweep is walked instead of enumerated.  The first pass runs at t_S and gives a total T that
// is usually close to the optimum.  The walk then starts at ceil(T / B) and moves down: run the
// capped recurrence at the cap, read the bottleneck b of the plan it returns, score it, continue
// at b - 1; every cap in between returns the same plan and a larger total.  Sums only grow as the
// cap shrinks, so once a pass has returned the sum s, a lower cap can match the best total T only
// with a bottleneck of at most (T - s) / (B - 1): the walk jumps to that cap when it is below
// b - 1, and ends when the next cap would be t_S or less.  Among equal totals the lower cap is
// kept, the choice an increasing sweep makes by accepting only strictly smaller totals.  The
// result is bit for bit what the increasing sweep over every distinct stage cost returns; it
// takes a handful of passes instead of hundreds.
//
// One pass is the band-limited, LDS-resident stage loop of the min-max kernel with three changes:
// a cell's value is the least sum (previous row + stage time, plus twice the cell's transfer time),
// previous cuts whose stage time exceeds the cap are excluded (the stage time never decreases as
// the previous cut moves down, so the downward scan stops there), and a cell whose own transfer
// time exceeds the cap is unreachable.
//
// Sums are 32-bit whenever the candidate allows it.  The min-max plan is admissible at every cap of
// the walk, so no least-sum plan costs more than that plan's own sum U, and a cell whose value
// exceeds U lies on none of them: such values are replaced by infinity, which changes no result
// and keeps every finite value at or below U.  With U < 2^31 and infinity = 2^31, a value plus a
// stage time (below 2^31 on these tables) never wraps and infinity plus any time never passes for
// a sum.  Candidates with U >= 2^31 (iterations of more than half an hour) are queued and redone
// by the same kernel instantiated with 64-bit sums.
//
// Three launches.  k2_exact works a candidate per wavefront (64-thread workgroups, 20 per CU): a
// DP row is 77 cuts wide on the 512-operator workload, so a 256-thread workgroup per candidate left
// three wavefronts in four idle at every stage's barrier.  Its two LDS rows hold the cuts of one
// stage only (row s starts at B[s], sized for the candidate's widest stage), and what is left of the
// wavefront's LDS share keeps one-byte back-pointers, as in the min-max kernel.  A candidate whose
// widest stage does not fit the share is queued for k2_exact_rows, the workgroup-per-candidate form
// with rows over the whole sequence (launched only when L makes such a candidate possible), and the
// candidates that need 64-bit sums for k2_exact_wide.
#include "fast_common.h"
#include "harp_internal.h"
#include "plan_common.h"

namespace harp {

using namespace fastdp;

namespace {

template <typename SumT> struct SumTraits;
template <> struct SumTraits<uint32_t> {
    static constexpr uint32_t inf = 0x80000000u;
    struct alignas(8) Entry { uint32_t d, p; };
};
template <> struct SumTraits<uint64_t> {
    static constexpr uint64_t inf = uint64_t(1) << 62;
    struct alignas(16) Entry { uint64_t d; uint32_t p; uint32_t unused; };
};

constexpr int64_t kNarrowLimit = int64_t(1) << 31;   // sums below this run in 32 bits

// One-byte back-pointers of the wavefront-per-candidate kernel, as in the min-max kernel: the distance
// from the cut below the cell to the chosen previous cut, kArgEscape when it does not fit (the cut
// itself then sits in the 16-bit slice).  A stage's word in aoff is where the back-pointer of cut 0
// of its row would sit, biased to stay positive, with a flag when the stage's back-pointers are in
// the LDS arena rather than in the one-byte slice.
constexpr int kArgEscape = 255;
constexpr uint32_t kArgBias = 1u << 16;
constexpr uint32_t kArgInLds = 1u << 31;

// LDS in front of the rows: per-stage constants, two scalars, band, trial and kept cuts, back-pointer
// offsets, index-row offsets, slot lists
__host__ __device__ inline size_t exact_small_bytes(int S_max) {
    const size_t b = size_t(S_max) * sizeof(StageConst) + 16 + size_t(S_max + 1) * 16 + size_t(S_max) * 7;
    return (b + 15) & ~size_t(15);
}

// counts: [0] live candidates, [1] dead candidates, [2] candidates queued for 64-bit sums,
// [3], [4] next item of the 32- and 64-bit kernels' work lists, [10] candidates queued for rows over
// the whole sequence, [11] next item of that list.
// Both queues sit in the unused tail of the dead list (live + dead = C entries in all): the 64-bit
// one grows from its front, the other from its back.
//
// kMode 0: a workgroup per candidate, LDS rows with an entry for every cut.  kMode 1: a wavefront
// per candidate (the launch has 64-thread workgroups), LDS rows that hold the cuts of one stage
// (row s starts at B[s]); a candidate whose widest stage does not fit them is queued.  kMode 2: as
// 0, on the candidates queued by 1.
template <typename SumT, int kMode>
__device__ __forceinline__ void exact_body(const TablesDev &tb, const CandDev &cd, const PlansDev &out,
                                           int32_t *n_passes, int *counts, const int32_t *live_list,
                                           uint32_t *dead_list, const uint32_t *bands, const uint16_t *lo_tab,
                                           int lo_pitch, unsigned char *arg_base, size_t arg_per_group,
                                           size_t arg_u8_off, int row_len, int lds_row_entries) {
    using Pair = typename SumTraits<SumT>::Entry;
    constexpr SumT kInfSum = SumTraits<SumT>::inf;
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
    int32_t *kept = trial + S_max + 1;                                                 // [S_max + 1]
    uint32_t *aoff = reinterpret_cast<uint32_t *>(kept + S_max + 1);                   // [S_max + 1]
    // element offset of each stage's row of the feasibility index (lowest fitting previous cut per cut)
    uint32_t *lo_off = aoff + S_max + 1;                                               // [S_max]
    uint16_t *slot_g = reinterpret_cast<uint16_t *>(lo_off + S_max);                   // [S_max]
    uint8_t *slot_k = reinterpret_cast<uint8_t *>(slot_g + S_max);                     // [S_max]
    // two rows, kPad entries in front of a row's lowest cut: of lds_row_entries entries each, or (a
    // wavefront per candidate) of what the candidate's widest stage needs, the rest of the 2 *
    // lds_row_entries entries being the arena of one-byte back-pointers
    Pair *buf0 = reinterpret_cast<Pair *>(lds_raw + exact_small_bytes(S_max)) + kPad;
    Pair *buf1 = buf0 + lds_row_entries;
    uint8_t *arena = nullptr;
    uint32_t arena_bytes = 0;
    uint16_t *arg = reinterpret_cast<uint16_t *>(arg_base + size_t(blockIdx.x) * arg_per_group);
    uint8_t *arg8 = reinterpret_cast<uint8_t *>(arg) + arg_u8_off;     // the slice's one-byte entries
    const int n_dead = counts[1];
    const int n_items = kWide ? counts[2] : kMode == 2 ? counts[10] : counts[0];
    const int64_t m_cap = tb.M;

    // candidates differ widely in passes, so workgroups draw them from a shared counter
    int *next_item = counts + (kWide ? 4 : kMode == 2 ? 11 : 3);
    for (;;) {
        __syncthreads();   // the previous candidate's tail has finished with LDS
        if (tid == 0) scal[0] = (uint64_t)atomicAdd(next_item, 1);
        __syncthreads();
        const int n = uniform((int)scal[0]);
        if (n >= n_items) break;
        const int c = kWide ? int(dead_list[n_dead + n]) : kMode == 2 ? int(dead_list[cd.C - 1 - n]) : live_list[n];
        const int S = cd.cand_S[c];
        // the min-max planner has run on this batch: candidates it found no plan for stay as they are,
        // and a single stage has only one partition
        if (out.status[c] != HARP_CAND_OK || S < 2) {
            if (tid == 0 && n_passes) n_passes[c] = 0;
            continue;
        }
        const int64_t t_S = out.bottleneck[c];
        const int64_t T_S = out.iter_time[c];
        const int64_t limit = T_S - (m_cap - 1) * t_S;      // the min-max plan's own sum
        if (!kWide && limit >= kNarrowLimit) {
            if (tid == 0) dead_list[n_dead + atomicAdd(&counts[2], 1)] = uint32_t(c);
            continue;
        }
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
                const int n_inflight = int((S - s) < m_cap ? (S - s) : m_cap);
                lo_off[s] = uint32_t((int64_t(n_inflight - 1) * tb.T * tb.n_tp + int64_t(tb.group_type[g]) * tb.n_tp + k) *
                                     lo_pitch);
            }
            for (int s = tid; s <= S; s += nthreads) band[s] = bands[int64_t(c) * (S_max + 1) + s];
        }
        __syncthreads();
        if (kBandRows) {
            // stage s reads the cuts B[s] .. F[s+1] of its rows
            int span = 0;
            for (int s = tid; s < S; s += nthreads) {
                const int w = band_hi(band[s + 1]) - band_lo(band[s]) + 1;
                span = w > span ? w : span;
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const int o = __shfl_xor(span, d, 64);
                span = o > span ? o : span;
            }
            const int row_entries = (uniform(span) + kPad + 1) & ~1;
            if (row_entries > lds_row_entries) {
                if (tid == 0) dead_list[cd.C - 1 - atomicAdd(&counts[10], 1)] = uint32_t(c);
                continue;
            }
            buf1 = buf0 + row_entries;
            arena = reinterpret_cast<uint8_t *>(buf0 - kPad + 2 * row_entries);
            arena_bytes = uint32_t(2 * (lds_row_entries - row_entries)) * uint32_t(sizeof(Pair));
            // where the back-pointers of each stage start: running sum of the widths of rows 1 .. S-1
            // (the last row has the single cell L); stages that fit the arena are flagged
            uint32_t carry = 0;
            for (int s0 = 0; s0 <= S; s0 += 64) {
                const int s = s0 + lane;
                uint32_t b = 0, wdt = 0;
                if (s <= S) b = band[s];
                if (s >= 1 && s < S) wdt = uint32_t(band_hi(b) - band_lo(b) + 1);
                uint32_t inc = wdt;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const uint32_t o = __shfl_up(inc, d, 64);
                    if (lane >= d) inc += o;
                }
                if (s >= 1 && s <= S) {
                    const uint32_t begin = carry + inc - wdt;
                    uint32_t word = begin + kArgBias - uint32_t(band_lo(b));
                    if (s < S && begin + wdt <= arena_bytes) word |= kArgInLds;
                    aoff[s - 1] = word;
                }
                carry += __shfl(inc, 63, 64);
            }
            __syncthreads();
        }

        int64_t t_cap64 = t_S;                  // the first pass: least sum at the smallest feasible cap
        int64_t best_T = kInf, best_b = kInf;
        int passes = 0;
        for (;;) {
            const uint32_t tcap = (uint32_t)uniform((int)(uint32_t)t_cap64);
            // ---- one capped pass
            uint32_t cut_i = 0;
            int lo_i = 0;
            {
                const uint32_t *p32 = tb.P32 + (uint32_t)uniform((int)sc[0].p_row);
                const uint32_t *cm = tb.CM + ((uint32_t)uniform((int)sc[0].cm_row_shift) & kRowMask);
                const uint16_t *lo0 = lo_tab + (uint32_t)uniform((int)lo_off[0]);
                const uint32_t b1 = (uint32_t)uniform((int)band[1]);
                Pair *rows = buf0;              // row 0 starts at cut 0 = B[0]
                for (int j = tid; j <= band_hi(b1); j += nthreads) rows[j].p = p32[j];
                if (band_lo(b1) + tid <= band_hi(b1)) { cut_i = cm[band_lo(b1) + tid]; lo_i = lo0[band_lo(b1) + tid]; }
                // below cut 0: never a predecessor; the time read there must stay small
                if (tid < 3) { rows[-1 - tid].d = kInfSum; rows[-1 - tid].p = 0xFFFFFFFFu; }
                if (tid == 0) rows[0].d = 0;
            }
            lds_barrier();

            int cur = 0;
            const int wave_first = wave * 64;
            // Cuts of the previous row with a finite sum lie in [fin_lo, fin_hi] (a wavefront per
            // candidate keeps track; the workgroup forms use the whole band).  Under a cap most of a
            // band is out of reach - its cells are infinite - and a scan that starts above fin_hi or
            // runs below fin_lo would only read infinite sums: clamping the scans to the finite range
            // changes no value and ends them at once for cells the cap has cut off.
            int fin_lo = 0, fin_hi = 0;
            for (int s = 0; s < S - 1; ++s) {
                const uint32_t b1 = (uint32_t)uniform((int)band[s + 1]);
                const uint32_t b2 = (uint32_t)uniform((int)band[s + 2]);
                const int il = band_lo(b1), ih = band_hi(b1);     // cells: row s + 1
                const int top_n = band_hi(b2);                    // stage s+1 reads its rows up to here
                if (il + wave_first > top_n && wave != 0) {
                    lds_barrier();
                    cur ^= 1;
                    continue;
                }
                const uint32_t rs = (uint32_t)uniform((int)sc[s].cm_row_shift);
                const int shift = int(rs >> 27);
                const uint32_t tp = 1u << shift;
                const uint32_t b0 = (uint32_t)uniform((int)band[s]);
                const int jl = band_lo(b0), jh = band_hi(b0);     // predecessors: row s
                const int jl_f = kBandRows && fin_lo > jl ? fin_lo : jl;
                const int jh_f = kBandRows && fin_hi < jh ? fin_hi : jh;
                int new_lo = INT32_MAX, new_hi = -1;               // cells of row s + 1 with a finite sum (wavefront form)
                const uint32_t *cm_s = tb.CM + (rs & kRowMask);
                const uint16_t *lo_s = lo_tab + (uint32_t)uniform((int)lo_off[s]);
                const uint16_t *lo_n_row = lo_tab + (uint32_t)uniform((int)lo_off[s + 1]);
                const Pair *prev = (cur ? buf1 : buf0) - (kBandRows ? jl : 0);
                Pair *next = (cur ? buf0 : buf1) - (kBandRows ? il : 0);
                const uint32_t *p32_n = tb.P32 + (uint32_t)uniform((int)sc[s + 1].p_row);
                const uint32_t *cm_n = tb.CM + ((uint32_t)uniform((int)sc[s + 1].cm_row_shift) & kRowMask);
                const bool next_has_cut = s + 2 < S;
                const uint32_t a_word = kBandRows ? (uint32_t)uniform((int)aoff[s]) : 0u;
                const bool arg_in_lds = (a_word & kArgInLds) != 0;
                const uint32_t a0 = (a_word & ~kArgInLds) - kArgBias;       // + cut = index of the cut's back-pointer
                auto put_arg = [&](int i, int best_j) {
                    if (kBandRows) {
                        const int rel = i - 1 - best_j;
                        const uint32_t at = a0 + uint32_t(i);
                        const uint8_t code = (uint8_t)(rel < kArgEscape ? rel : kArgEscape);
                        if (arg_in_lds) arena[at] = code;
                        else arg8[at] = code;
                        if (rel >= kArgEscape) arg[at] = (uint16_t)best_j;
                    } else {
                        arg[s * row_len + i] = (uint16_t)best_j;
                    }
                };

                const int jn = il + tid;
                uint32_t p_n = 0, cut_n = 0;
                int lo_n = 0;
                if (jn <= top_n) p_n = p32_n[jn];
                if (band_lo(b2) + tid <= top_n) {       // the first cell this thread has in row s + 2
                    if (next_has_cut) cut_n = cm_n[band_lo(b2) + tid];
                    lo_n = lo_n_row[band_lo(b2) + tid];
                }

                // One cell: least sum over the previous cuts that fit in memory (from the feasibility
                // index: cuts lo .. i - 1) and under the cap, scanned downwards four per trip.  The
                // stage time never decreases as j moves down, so the last entry of a trip decides
                // whether the lane goes on.  Equal sums keep the lowest j.
                auto cell = [&](int i, uint32_t cut, int lo_idx) -> int {
                    const int lo = lo_idx > jl_f ? lo_idx : jl_f;
                    const uint32_t xi = prev[i].p + tp - 1;
                    SumT best = kInfSum;
                    int best_j = 0;
                    int j = (i - 1) < jh_f ? (i - 1) : jh_f;
                    bool more = (j >= lo) & (cut <= tcap);
                    while (more) {
                        const Pair *pe = prev + (j - 3);
                        const Pair e3 = pe[0], e2 = pe[1], e1 = pe[2], e0 = pe[3];
                        uint32_t tj;
#define HARP_STEP(E, K)                                                        \
    {                                                                          \
        tj = (xi - (E).p) >> shift;                                            \
        const SumT v = (E).d + tj;                                             \
        const bool upd = (j - (K) >= lo) & (tj <= tcap) & (v <= best);         \
        best = upd ? v : best;                                                 \
        best_j = upd ? j - (K) : best_j;                                       \
    }
                        HARP_STEP(e0, 0)
                        HARP_STEP(e1, 1)
                        HARP_STEP(e2, 2)
                        HARP_STEP(e3, 3)
#undef HARP_STEP
                        more = ((j - 3) > lo) & (tj <= tcap);
                        j -= 4;
                    }
                    const uint64_t total = uint64_t(best) + 2ull * cut;
                    const bool finite = !(best >= kInfSum || total > uint64_t(limit));
                    next[i].d = finite ? SumT(total) : kInfSum;
                    if (kBandRows) {
                        // lanes hold consecutive cells from i - tid on: the lowest and the highest lane with
                        // a finite sum bound this round's cells
                        const unsigned long long fm = __ballot(finite);
                        if (fm != 0) {
                            const int base = uniform(i - tid);
                            const int lo_r = base + __ffsll((long long)fm) - 1, hi_r = base + 63 - __clzll((long long)fm);
                            new_lo = lo_r < new_lo ? lo_r : new_lo;
                            new_hi = hi_r > new_hi ? hi_r : new_hi;
                        }
                    }
                    return best >= kInfSum ? i - 1 : best_j;        // no previous cut: any value, a short one
                };
                const int i0 = il + tid;
                int first_j = 0;
                if (i0 <= ih) first_j = cell(i0, cut_i, lo_i);
                for (int i = i0 + nthreads; i <= ih; i += nthreads)
                    put_arg(i, cell(i, cm_s[i], lo_s[i]));
                if (tid < 3) {                                  // below the band of row s + 1
                    next[il - 1 - tid].d = kInfSum;
                    next[il - 1 - tid].p = 0xFFFFFFFFu;
                }

                if (jn <= top_n) next[jn].p = p_n;
                for (int j = jn + nthreads; j <= top_n; j += nthreads) next[j].p = p32_n[j];
                asm volatile("" : "+v"(cut_n));
                cut_i = cut_n;
                lo_i = lo_n;
                if (i0 <= ih) put_arg(i0, first_j);
                if (kBandRows) {
                    // lane 0 has a cell in every round that any lane has one in: its copy is complete
                    fin_hi = uniform(new_hi);
                    fin_lo = fin_hi < 0 ? L + 1 : uniform(new_lo);     // no finite cell: an empty range
                }
                lds_barrier();
                cur ^= 1;
            }
            // the last stage has the single cell i = L: lanes over j, lexicographic reduction
            if (wave == 0) {
                const int s = S - 1;
                const int shift = int((uint32_t)uniform((int)sc[s].cm_row_shift) >> 27);
                const uint32_t tp = 1u << shift;
                const uint32_t b0 = (uint32_t)uniform((int)band[s]);
                const Pair *prev = (cur ? buf1 : buf0) - (kBandRows ? band_lo(b0) : 0);
                const uint32_t xi = prev[L].p + tp - 1;
                int hi = (L - 1) < band_hi(b0) ? (L - 1) : band_hi(b0);
                const int lo_L = uniform((int)lo_tab[size_t((uint32_t)uniform((int)lo_off[s])) + L]);
                int lo = lo_L > band_lo(b0) ? lo_L : band_lo(b0);
                if (kBandRows && S > 1) {
                    hi = fin_hi < hi ? fin_hi : hi;
                    lo = fin_lo > lo ? fin_lo : lo;
                }
                unsigned long long best = kInfSum;
                int best_j = INT32_MAX;
                for (int j = lo + lane; j <= hi; j += 64) {
                    const uint32_t tj = (xi - prev[j].p) >> shift;
                    const unsigned long long v = (unsigned long long)prev[j].d + tj;
                    if (tj <= tcap && v < best) { best = v; best_j = j; }   // j rises within a lane
                }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const unsigned long long ov = __shfl_xor(best, d, 64);
                    const int oj = __shfl_xor(best_j, d, 64);
                    if (ov < best || (ov == best && oj < best_j)) { best = ov; best_j = oj; }
                }
                if (lane == 0) {
                    if (kBandRows) trial[S - 1] = best_j;
                    else arg[(S - 1) * row_len + L] = (uint16_t)best_j;
                    scal[0] = best;
                }
            }
            __syncthreads();          // back-pointers of every wave are visible to thread 0
            const int64_t sum = uniform64((int64_t)scal[0]);
            if (sum >= int64_t(kInfSum)) break;   // no plan under this cap (cannot happen at or above t_S)
            if (tid == 0) {
                trial[S] = L;
                if (kBandRows) {
                    int b = trial[S - 1];
                    for (int s = S - 2; s >= 0; --s) {
                        // a finite sum only chains through cuts inside the rows; the clamp keeps the index
                        // inside the stage's back-pointers whatever the cut
                        const uint32_t bw = band[s + 1];
                        b = b < band_lo(bw) ? band_lo(bw) : (b > band_hi(bw) ? band_hi(bw) : b);
                        const uint32_t word = aoff[s];
                        const uint32_t at = (word & ~kArgInLds) - kArgBias + uint32_t(b);
                        const int rel = (word & kArgInLds) ? arena[at] : arg8[at];
                        b = rel == kArgEscape ? int(arg[at]) : b - 1 - rel;
                        trial[s] = b;
                    }
                } else {
                    int b = L;
                    for (int s = S - 1; s >= 0; --s) {
                        b = arg[s * row_len + b];
                        b = b < L ? b : L;      // a finite sum only chains through cuts inside the row
                        trial[s] = b;
                    }
                }
            }
            __syncthreads();
            // the plan's bottleneck, one lane per stage
            if (wave == 0) {
                uint32_t w = 0;
                for (int s = lane; s < S; s += 64) {
                    const int j = trial[s], i = trial[s + 1];
                    const uint32_t rs = sc[s].cm_row_shift;
                    const int shift = int(rs >> 27);
                    const uint32_t *p = tb.P32 + sc[s].p_row;
                    const uint32_t t = (p[i] + (1u << shift) - 1u - p[j]) >> shift;
                    const uint32_t cu = s < S - 1 ? tb.CM[(rs & kRowMask) + uint32_t(i)] : 0u;
                    const uint32_t m = t > cu ? t : cu;
                    w = w > m ? w : m;
                }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const uint32_t ow = __shfl_xor(w, d, 64);
                    w = w > ow ? w : ow;
                }
                if (lane == 0) scal[1] = w;
            }
            __syncthreads();
            const int64_t b = uniform64((int64_t)scal[1]);
            const int64_t T = sum + (m_cap - 1) * b;
            ++passes;
            if (T < best_T || (T == best_T && b < best_b)) {     // equal totals: the lower cap
                best_T = T;
                best_b = b;
                for (int s = tid; s <= S; s += nthreads) kept[s] = trial[s];
            }
            if (passes >= (1 << 20) || b > t_cap64) break;       // cannot happen: the cap falls with every pass
            int64_t next_cap;
            if (passes == 1) {
                // every plan costs at least B times its bottleneck (the bottleneck is one of the
                // terms of the sum), so nothing above t_E = ceil(T / B) can beat the total T in hand
                next_cap = (best_T + m_cap - 1) / m_cap;
                if (next_cap > 0x7FFFFFFFll) next_cap = 0x7FFFFFFFll;   // no time on these tables is larger
            } else {
                next_cap = b - 1;
            }
            // Sums only grow as the cap shrinks, so a plan found at or below a cap that returned
            // the sum `sum` costs at least sum + (B - 1) b' with its own bottleneck b': it can match
            // the best total only if b' <= (best_T - sum) / (B - 1).  Caps above that are skipped.
            if (passes > 1 && m_cap > 1) {
                const int64_t bound = (best_T - sum) / (m_cap - 1);
                next_cap = next_cap < bound ? next_cap : bound;
            }
            if (next_cap <= t_S) break;         // the plan at t_S is already in hand
            t_cap64 = next_cap;
        }
        __syncthreads();
        if (tid == 0 && n_passes) n_passes[c] = passes;
        if (best_T == kInf) {
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            continue;
        }
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        for (int s = tid; s <= S; s += nthreads) sp[s] = kept[s];
        __syncthreads();
        if (wave == 0) {
            int64_t bott, iter;
            const int st = wave_score_partition(tb, S, slot_g, slot_k, sp, lane, bott, iter);
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = iter;
                out.status[c] = st;
            }
        }
    }
    // candidates the pre-pass rejected keep the outputs the min-max kernel wrote
    if (!kWide && n_passes) {
        for (int n = blockIdx.x * nthreads + tid; n < n_dead; n += gridDim.x * nthreads)
            n_passes[dead_list[n] & ((1u << kDeadStatusShift) - 1u)] = 0;
    }
}

#define HARP_EXACT_KERNEL(NAME, BOUNDS, SUM, MODE)                                                                  \
    __global__ BOUNDS void NAME(TablesDev tb, CandDev cd, PlansDev out, int32_t *n_passes, int *counts,            \
                                const int32_t *live_list, uint32_t *dead_list, const uint32_t *bands,             \
                                const uint16_t *lo_tab, int lo_pitch, unsigned char *arg_base,                    \
                                size_t arg_per_group, size_t arg_u8_off, int row_len, int lds_row_entries) {      \
        exact_body<SUM, MODE>(tb, cd, out, n_passes, counts, live_list, dead_list, bands, lo_tab, lo_pitch,       \
                              arg_base, arg_per_group, arg_u8_off, row_len, lds_row_entries);                     \
    }
HARP_EXACT_KERNEL(k2_exact, __launch_bounds__(64), uint32_t, 1)
HARP_EXACT_KERNEL(k2_exact_rows, __launch_bounds__(kFastThreads) __attribute__((amdgpu_waves_per_eu(8, 8))), uint32_t, 2)
HARP_EXACT_KERNEL(k2_exact_wide, __launch_bounds__(kFastThreads), uint64_t, 0)
#undef HARP_EXACT_KERNEL

}  // namespace

// Runs after launch_plan_fast on the same stream and workspace: the live list, the bands and the
// min-max results in `out` are its inputs.  n_groups: resident 256-thread workgroups; n_slices:
// back-pointer slices in the workspace (the wavefront-per-candidate launch runs at most that many).
void launch_plan_exact(const TablesDev &tb, const CandDev &cd, const PlansDev &out, int32_t *n_passes,
                       void *ws, int n_groups, int n_slices, int n_cu, hipStream_t st) {
    const FastWorkspace w = carve(ws, fast_shape(tb, cd), n_groups);
    const int full_row = fast_row_len(tb.L);
    const size_t small = exact_small_bytes(cd.S_max);
    // Wavefronts per CU of the first launch (its registers allow five per SIMD; 16 to 24 per CU
    // measure the same, 28 and more are slower because more candidates leave for the second launch)
    // and the row entries their LDS share leaves.
    const int per_cu = 20;
    size_t share = ((size_t(160) << 10) / per_cu - 128) & ~size_t(15);
    int entries = share > small + 2 * 8 * (kPad + 8) ? int((share - small) / 16) : kPad + 8;
    if (entries > full_row) entries = full_row;
    int n_waves = per_cu * n_cu;
    if (n_waves > n_slices) n_waves = n_slices;
    if (n_waves > cd.C) n_waves = cd.C;
    if (n_waves < 1) n_waves = 1;
    const int lo_p = int(lo_pitch(tb.L));
    const size_t per_group = fast_arg_per_group(tb.L, cd.S_max);
    const size_t u8_off = fast_arg_u16_bytes(tb.L, cd.S_max);
    hipLaunchKernelGGL(k2_exact, dim3(n_waves), dim3(64), small + size_t(entries) * 16, st, tb, cd, out, n_passes,
                       w.counts, w.live_list, w.dead_list, w.bands, w.lo_tab, lo_p, w.arg, per_group, u8_off,
                       full_row, entries);
    if (entries < full_row)
        hipLaunchKernelGGL(k2_exact_rows, dim3(n_groups), dim3(kFastThreads), small + size_t(full_row) * 16, st,
                           tb, cd, out, n_passes, w.counts, w.live_list, w.dead_list, w.bands, w.lo_tab, lo_p,
                           w.arg, per_group, u8_off, full_row, full_row);
    hipLaunchKernelGGL(k2_exact_wide, dim3(n_groups), dim3(kFastThreads), small + size_t(full_row) * 32, st, tb,
                       cd, out, n_passes, w.counts, w.live_list, w.dead_list, w.bands, w.lo_tab, lo_p, w.arg,
                       per_group, u8_off, full_row, full_row);
}

}  // namespace harp
