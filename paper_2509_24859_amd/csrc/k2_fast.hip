// Fast planner-search kernels for gfx950: reachability bands, 32-bit times, bounded scans, rows in LDS.
//
// Same recurrence as the generic kernel (paper section 5.2.3, eq. dp_general with the submesh of
// each stage fixed by the candidate; constraints (i)-(iii)), same results bit for bit, but the
// work is cut down with facts that hold for every valid problem (all costs and byte counts are
// non-negative, which the table build has verified):
//
//  * eq. mem_cons is monotone: a longer stage never needs less memory.  Hence (a) the fitting
//    previous cuts of cell (s, i) are exactly j >= lo(s, i); (b) the largest cut any plan can reach
//    after s stages, F[s], obeys F[s+1] <= max{ i : stage s over [F[s], i) fits }; (c) the smallest
//    cut from which the remaining stages can still hold the remaining operators, B[s], obeys
//    B[s] >= lo(s, B[s+1]).  Cells outside [B[s], F[s]] are either unreachable or cannot be
//    completed, so no optimal plan passes through them and no cell that lies on a complete plan has
//    them as a fitting predecessor: the DP is run on the band only.  A band that comes out empty,
//    B[0] > 0, or F[S] < L proves the candidate infeasible before any DP work.  (The bands are
//    bounds, not exact sets: a candidate whose band is non-empty can still turn out infeasible,
//    which the DP then reports.)  k2_band computes the two chains with one thread per candidate.
//  * the stage time time(s; j, i) never decreases when j moves down.  Scanning j downwards from
//    i-1, once time(s; j, i) exceeds the best value found so far no lower j can match or beat it,
//    and the scan stops.  The stop uses a strict comparison and the update a non-strict one, so
//    the lowest j among equal values is kept, as the recurrence demands.  Nothing is assumed
//    about the previous DP row (it is not monotone when transfer times dominate); in the worst
//    case the scan covers the whole band.
//
// With tp a power of two and every time below 2^31 us (both checked by the table build), the
// stage time is one subtraction and one shift on the fused 32-bit row
//   P[j] = PF[type][j] + tp * PR[g][tp][j]:   time(s; j, i) = (P[i] + tp - 1 - P[j]) >> log2 tp,
// because ceil(a / tp) + b = ceil((a + tp b) / tp) for integers.  Transfer times come from the
// per-link cut table built beside the rows.
//
// Mapping of k2_fast: one workgroup per live candidate at a time (persistent workgroups draw
// from the list k2_band compacted through a shared counter), one lane per DP cell of the current stage's band (more trips
// when the band is wider than the workgroup), lanes of a wave on consecutive cells so that LDS
// reads of (D[j], P[j]) pairs are stride-1 or broadcast.  The previous DP row and the slot's P row
// sit interleaved in LDS so that one 8-byte read feeds a transition.  What stage s+1 needs from
// global memory (its slot's P row, the memory row, the cell's own cut time) is requested at the
// top of stage s, lands in registers while stage s scans, and is committed to the other LDS buffer
// before the single LDS-only barrier that ends the stage.  Values that are the same for the whole
// workgroup are moved to scalar registers so that addressing runs on the scalar unit.  The lone
// cell of the last stage is reduced across a wavefront with a lexicographic (value, j) minimum.
// Back-pointers go to a per-workgroup slice of the caller's workspace as uint16.
#include "harp_internal.h"
#include "fast_common.h"
#include "plan_common.h"

namespace harp {

using namespace fastdp;

namespace {


// Pre-pass, one thread per candidate: checks the slot list and computes the reachability band
// [B[s], F[s]] of every DP row from the memory constraint alone (two chains of binary searches
// over the running sums).  Candidates that pass go to the live list; malformed ones and those
// proven infeasible go to the dead list with their status.
//
// Every probe of the searches is a dependent load and every candidate walks its slot list twice,
// so everything the loops touch is staged in LDS first: the running sums PP and PS, the memory
// cap of every (group, degree), and the workgroup's slot lists, read from global memory once,
// coalesced, and stored slot-major so that the per-thread walks are conflict-free.  Bands are
// written slot-major as well ([s][c]), which keeps the writes of a wave contiguous.
constexpr int kBandCapTable = 1024;     // caps kept in LDS when G * n_tp is at most this
constexpr uint16_t kBadSlot = 0xFFFFu;

int band_threads(int S_max) { return S_max <= 64 ? 256 : (S_max <= 128 ? 128 : 64); }

__global__ __launch_bounds__(256) void k2_band(TablesDev tb, CandDev cd, int *counts, int32_t *live_list,
                                               uint32_t *dead_list, uint32_t *bands, int caps_in_lds) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int L = tb.L, S_max = cd.S_max, C = cd.C;
    const int nthreads = blockDim.x, pitch = nthreads + 2;
    int64_t *PP = reinterpret_cast<int64_t *>(lds_raw);      // [L + 1]
    int64_t *PS = PP + (L + 1);                              // [L + 1]
    int64_t *caps = PS + (L + 1);                            // [G * n_tp] when caps_in_lds
    uint16_t *slots = reinterpret_cast<uint16_t *>(caps + (caps_in_lds ? tb.G * tb.n_tp : 0));  // [S_max][pitch]
    const int c0 = blockIdx.x * nthreads;
    {
        const int64_t *gp = tb.PP(), *gs = tb.PS();
        for (int i = threadIdx.x; i <= L; i += nthreads) { PP[i] = gp[i]; PS[i] = gs[i]; }
        if (caps_in_lds)
            for (int q = threadIdx.x; q < tb.G * tb.n_tp; q += nthreads) {
                const int g = q / tb.n_tp, k = q - g * tb.n_tp;
                caps[q] = int64_t(tb.tp[k]) * tb.type_mem[tb.group_type[g]];
            }
        // slot lists of this workgroup's candidates: (group << 3) | degree index, or kBadSlot
        const int n_here = (C - c0) < nthreads ? (C - c0) : nthreads;
        const int32_t *grp = cd.cand_group + int64_t(c0) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c0) * S_max;
        for (int idx = threadIdx.x; idx < n_here * S_max; idx += nthreads) {
            const int cl = idx / S_max, s = idx - cl * S_max;
            const int g = grp[idx];
            const int k = tp_index(tb, tpv[idx]);
            slots[s * pitch + cl] = (g < 0 || g >= tb.G || k < 0) ? kBadSlot : (uint16_t)((g << 3) | k);
        }
    }
    __syncthreads();
    const int cl = threadIdx.x, c = c0 + cl;
    if (c >= C) return;
    const int S = cd.cand_S[c];
    const int R = L - S + 1;
    auto cap_of = [&](int g, int k) -> int64_t {
        return caps_in_lds ? caps[g * tb.n_tp + k] : int64_t(tb.tp[k]) * tb.type_mem[tb.group_type[g]];
    };

    int status = HARP_CAND_OK;
    bool feasible = S <= L;
    if (S < 1 || S > S_max) status = HARP_CAND_INVALID;
    // one walk over the slots: well-formedness, and the forward chain
    // F[s+1] = largest cut that stage s can reach from F[s]
    int64_t used = 0;
    unsigned long long seen = 0;                      // groups already entered, when G <= 64
    int prev_g = -1, F = 0;
    if (status == HARP_CAND_OK) bands[c] = 0;
    for (int s = 0; status == HARP_CAND_OK && s < S; ++s) {
        const uint16_t code = slots[s * pitch + cl];
        if (code == kBadSlot) { status = HARP_CAND_INVALID; break; }
        const int g = code >> 3, k = code & 7;
        if (g != prev_g) {                            // first slot of a run of group g
            if (tb.G <= 64) {
                if ((seen >> g) & 1ull) status = HARP_CAND_INVALID;   // the group was left and entered again
                seen |= 1ull << g;
            } else {
                for (int q = 0; q + 1 < s; ++q)
                    if ((slots[q * pitch + cl] >> 3) == g) status = HARP_CAND_INVALID;
            }
            used = 0;
            prev_g = g;
        }
        used += tb.tp[k];
        if (used > tb.group_ndev[g]) status = HARP_CAND_INVALID;
        if (feasible) {
            const int64_t n = (S - s) < tb.M ? (S - s) : tb.M;
            const int64_t cap = cap_of(g, k);
            const int64_t q0 = PP[F] + n * PS[F];
            const int top = (s == S - 1) ? L : s + R;
            int a = F, b = top;                               // need(F, a) <= cap always holds
            if ((PP[b] + n * PS[b]) - q0 <= cap) a = b;
            while (b - a > 1) {
                const int m = (a + b) >> 1;
                if ((PP[m] + n * PS[m]) - q0 <= cap) a = m; else b = m;
            }
            F = a;
            if (F < s + 1 || (s == S - 1 && F != L)) feasible = false;
            else bands[int64_t(s + 1) * C + c] = uint32_t(F) << 16;
        }
    }
    // backward chain: B[s] = smallest cut from which stage s can reach B[s+1]
    if (status == HARP_CAND_OK && feasible) {
        int B = L;
        bands[int64_t(S) * C + c] |= uint32_t(L);
        for (int s = S - 1; s >= 0; --s) {
            const uint16_t code = slots[s * pitch + cl];
            const int64_t n = (S - s) < tb.M ? (S - s) : tb.M;
            const int64_t cap = cap_of(code >> 3, code & 7);
            const int64_t qb = PP[B] + n * PS[B];
            int a = s, b = B;                                 // need(b, B) <= cap holds at b = B
            if (qb - (PP[a] + n * PS[a]) <= cap) b = a;
            while (b - a > 1) {
                const int m = (a + b) >> 1;
                if (qb - (PP[m] + n * PS[m]) <= cap) b = m; else a = m;
            }
            B = b;
            uint32_t *w = bands + int64_t(s) * C + c;
            const int hi = band_hi(*w);
            if (hi < B || (s == 0 && B != 0)) { feasible = false; break; }
            *w = uint32_t(B) | (uint32_t(hi) << 16);
        }
    }
    if (status == HARP_CAND_OK && !feasible) status = HARP_CAND_INFEASIBLE;

    // append to the live or the dead list with one atomic per wave and list: lanes rank themselves
    const int lane = threadIdx.x & 63;
    const bool alive = status == HARP_CAND_OK;
    const unsigned long long here = __ballot(1), live_m = __ballot(alive), dead_m = here & ~live_m;
    const int leader = __ffsll((long long)here) - 1;
    int base_live = 0, base_dead = 0;
    if (lane == leader) {
        if (live_m) base_live = atomicAdd(&counts[0], __popcll(live_m));
        if (dead_m) base_dead = atomicAdd(&counts[1], __popcll(dead_m));
    }
    base_live = __shfl(base_live, leader, 64);
    base_dead = __shfl(base_dead, leader, 64);
    const unsigned long long below = (1ull << lane) - 1ull;
    if (alive) live_list[base_live + __popcll(live_m & below)] = c;
    else dead_list[base_dead + __popcll(dead_m & below)] = uint32_t(c) | (uint32_t(status) << kDeadStatusShift);
}

__global__ void k2_clear_count(int *counts) {
    if (threadIdx.x < 8) counts[threadIdx.x] = 0;
}

__global__ __launch_bounds__(kFastThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k2_fast(TablesDev tb, CandDev cd, PlansDev out, int *counts, const int32_t *live_list,
             const uint32_t *dead_list, const uint32_t *bands, unsigned char *arg_base, size_t arg_per_group,
             int row_len) {
    extern __shared__ __align__(16) unsigned char lds_raw[];

    const int L = tb.L, S_max = cd.S_max;
    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = uniform(tid >> 6);
    // every LDS row has kPad spare entries in front, so that the group of four previous cuts
    // ending at any j >= 0 can be read at fixed offsets without clamping
    int64_t *Qb = reinterpret_cast<int64_t *>(lds_raw) + kPad;                        // [2][row_len]
    Pair *rows = reinterpret_cast<Pair *>(lds_raw + size_t(row_len) * 16) + kPad;     // [2][row_len]
    StageConst *sc = reinterpret_cast<StageConst *>(lds_raw + size_t(row_len) * 32);  // [S_max]
    uint32_t *ticket = reinterpret_cast<uint32_t *>(sc + S_max);                       // [1]
    uint32_t *band = ticket + 1;                                                       // [S_max + 1]
    uint16_t *slot_g = reinterpret_cast<uint16_t *>(band + S_max + 1);                 // [S_max]
    uint8_t *slot_k = reinterpret_cast<uint8_t *>(slot_g + S_max);                     // [S_max]
    uint16_t *arg = reinterpret_cast<uint16_t *>(arg_base + size_t(blockIdx.x) * arg_per_group);
    const int64_t *PP = tb.PP(), *PS = tb.PS();
    const int n_live = counts[0], n_dead = counts[1];
    int *next_item = counts + 5;
    const int64_t m_cap = tb.M;

    // candidates differ in stages and band widths, so workgroups draw them from a shared counter
    for (;;) {
        __syncthreads();   // the previous candidate's tail has finished with LDS
        if (tid == 0) *ticket = (uint32_t)atomicAdd(next_item, 1);
        __syncthreads();
        const int n = uniform((int)*ticket);
        if (n >= n_live) break;
        const int c = live_list[n];
        const int S = cd.cand_S[c];
        {
            const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
            const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
            int32_t *df = out.dev_first + int64_t(c) * S_max;
            for (int s = tid; s < S; s += nthreads) {
                const int g = grp[s], k = tp_index(tb, tpv[s]);
                const int g_next = s + 1 < S ? grp[s + 1] : g;
                slot_g[s] = (uint16_t)g;
                slot_k[s] = (uint8_t)k;
                sc[s].cap = int64_t(tb.tp[k]) * tb.type_mem[tb.group_type[g]];
                sc[s].p_row = uint32_t((int64_t(g) * tb.n_tp + k) * tb.pitch32);
                sc[s].cm_row_shift = uint32_t((int64_t(g) * tb.G + g_next) * tb.pitch32) |
                                     (uint32_t(tb.tp_shift[k]) << 27);
                // first device of the slot: its group's base plus the degrees of the group's
                // earlier slots (they are adjacent; the pre-pass has checked that)
                int32_t first = tb.group_base[g];
                for (int q = s - 1; q >= 0 && grp[q] == g; --q) first += tpv[q];
                df[s] = first;
            }
            for (int s = S + tid; s < S_max; s += nthreads) df[s] = -1;
            for (int s = tid; s <= S; s += nthreads) band[s] = bands[int64_t(s) * cd.C + c];
        }
        __syncthreads();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        bool dead = false;
        if (S >= 2) {
            // prologue: rows of stage 0 over [0, F[1]] and the thread's own cut time of stage 0
            uint32_t cut_i = 0;
            {
                const uint32_t *p32 = tb.P32 + (uint32_t)uniform((int)sc[0].p_row);
                const uint32_t *cm = tb.CM + ((uint32_t)uniform((int)sc[0].cm_row_shift) & kRowMask);
                const int64_t n0 = S < m_cap ? S : m_cap;
                const uint32_t b1 = (uint32_t)uniform((int)band[1]);
                for (int j = tid; j <= band_hi(b1); j += nthreads) {
                    rows[j].p = p32[j];
                    Qb[j] = PP[j] + n0 * PS[j];
                }
                if (band_lo(b1) + tid <= band_hi(b1)) cut_i = cm[band_lo(b1) + tid];
                if (tid < 3) rows[-1 - tid].d = kInf32;   // below cut 0: never a predecessor
                if (tid == 0) rows[0].d = 0;
            }
            lds_barrier();

            int cur = 0;
            const int wave_first = wave * 64;
            for (int s = 0; s < S - 1; ++s) {
                const uint32_t b1 = (uint32_t)uniform((int)band[s + 1]);
                const uint32_t b2 = (uint32_t)uniform((int)band[s + 2]);
                const int il = band_lo(b1), ih = band_hi(b1);     // cells: row s + 1
                const int top_n = band_hi(b2);                    // stage s+1 reads its rows up to here
                // a wave whose lanes own neither a cell nor a staged entry only keeps the barrier
                if (il + wave_first > top_n && wave != 0) {
                    lds_barrier();
                    cur ^= 1;
                    continue;
                }
                const uint32_t rs = (uint32_t)uniform((int)sc[s].cm_row_shift);
                const int shift = int(rs >> 27);
                const uint32_t tp = 1u << shift;
                const int64_t cap = uniform64(sc[s].cap);
                const uint32_t b0 = (uint32_t)uniform((int)band[s]);
                const int jl = band_lo(b0), jh = band_hi(b0);     // predecessors: row s
                const uint32_t *cm_s = tb.CM + (rs & kRowMask);
                const Pair *prev = rows + cur * row_len;
                Pair *next = rows + (cur ^ 1) * row_len;
                const int64_t *Q = Qb + cur * row_len;
                int64_t *Qn = Qb + (cur ^ 1) * row_len;
                const uint32_t *p32_n = tb.P32 + (uint32_t)uniform((int)sc[s + 1].p_row);
                const uint32_t *cm_n = tb.CM + ((uint32_t)uniform((int)sc[s + 1].cm_row_shift) & kRowMask);
                const bool next_has_cut = s + 2 < S;

                // requests for stage s+1: entry jn of its rows, and this thread's own cut time
                const int jn = il + tid;
                uint32_t p_n = 0, cut_n = 0;
                int64_t pp_n = 0, ps_n = 0;
                if (jn <= top_n) { p_n = p32_n[jn]; pp_n = PP[jn]; ps_n = PS[jn]; }
                if (next_has_cut && band_lo(b2) + tid <= top_n) cut_n = cm_n[band_lo(b2) + tid];

                // One DP cell: scan the fitting previous cuts of the band downwards, four per trip.
                // Fitting cuts are j >= lo with Q[lo] >= Q[i] - cap (memory need is monotone in
                // j), so an entry counts while its Q passes the threshold, a plain predicate;
                // entries below the band hold D = infinity and never win.  Entries below a stop
                // cannot update (their time exceeds the best value), so only the last entry of a
                // trip decides whether the lane goes on.  Returns the back-pointer.
                auto cell = [&](int i, uint32_t cut) -> int {
                    const int64_t th = Q[i] - cap;
                    const uint32_t xi = prev[i].p + tp - 1;
                    uint32_t best = kInf32;
                    int best_j = 0;
                    int j = (i - 1) < jh ? (i - 1) : jh;
                    bool more = j >= jl;
                    while (more) {
                        const Pair *pe = prev + (j - 3);
                        const int64_t *pq = Q + (j - 3);
                        const Pair e3 = pe[0], e2 = pe[1], e1 = pe[2], e0 = pe[3];
                        const int64_t q3 = pq[0], q2 = pq[1], q1 = pq[2], q0 = pq[3];
                        uint32_t tj;
#define HARP_STEP(E, QV, JJ)                                                   \
    {                                                                          \
        tj = (xi - (E).p) >> shift;                                            \
        const uint32_t v = umax3((E).d, tj, cut);                              \
        const bool upd = ((QV) >= th) & (v <= best);                           \
        best = upd ? v : best;                                                 \
        best_j = upd ? (JJ) : best_j;                                          \
    }
                        HARP_STEP(e0, q0, j)
                        HARP_STEP(e1, q1, j - 1)
                        HARP_STEP(e2, q2, j - 2)
                        HARP_STEP(e3, q3, j - 3)
#undef HARP_STEP
                        more = ((j - 3) > jl) & (q3 >= th) & (tj <= best);
                        j -= 4;
                    }
                    next[i].d = best;
                    return best_j;
                };
                const int i0 = il + tid;
                int first_j = 0;
                if (i0 <= ih) first_j = cell(i0, cut_i);
                // a band wider than the workgroup takes more trips; their cut times come straight
                // from the table
                for (int i = i0 + nthreads; i <= ih; i += nthreads)
                    arg[s * row_len + i] = (uint16_t)cell(i, cm_s[i]);
                if (tid < 3) next[il - 1 - tid].d = kInf32;     // below the band of row s + 1

                // commit the staged entries of stage s+1, then let the back-pointer go
                const int64_t n1 = (S - s - 1) < m_cap ? (S - s - 1) : m_cap;
                if (jn <= top_n) {
                    next[jn].p = p_n;
                    Qn[jn] = pp_n + n1 * ps_n;
                }
                for (int j = jn + nthreads; j <= top_n; j += nthreads) {
                    next[j].p = p32_n[j];
                    Qn[j] = PP[j] + n1 * PS[j];
                }
                // the cut time requested above must have landed before the next stage issues its own
                // requests: vector memory returns in order, so a wait placed at its first use inside
                // the next scan would also wait for those
                asm volatile("" : "+v"(cut_n));
                cut_i = cut_n;
                if (i0 <= ih) arg[s * row_len + i0] = (uint16_t)first_j;
                lds_barrier();
                cur ^= 1;
            }
            // the last stage has the single cell i = L: lanes over j, lexicographic reduction
            {
                const int s = S - 1;
                if (wave == 0) {
                    const int shift = int((uint32_t)uniform((int)sc[s].cm_row_shift) >> 27);
                    const uint32_t tp = 1u << shift;
                    const int64_t cap = uniform64(sc[s].cap);
                    const uint32_t b0 = (uint32_t)uniform((int)band[s]);
                    const Pair *prev = rows + cur * row_len;
                    const int64_t *Q = Qb + cur * row_len;
                    const int64_t th = Q[L] - cap;
                    const uint32_t xi = prev[L].p + tp - 1;
                    const int hi = (L - 1) < band_hi(b0) ? (L - 1) : band_hi(b0);
                    uint32_t best = kInf32;
                    int best_j = INT32_MAX;
                    for (int j = band_lo(b0) + lane; j <= hi; j += 64) {
                        if (Q[j] < th) continue;
                        const Pair e = prev[j];
                        const uint32_t tj = (xi - e.p) >> shift;
                        const uint32_t v = e.d > tj ? e.d : tj;
                        if (v < best) { best = v; best_j = j; }   // j rises within a lane
                    }
#pragma unroll
                    for (int d = 32; d >= 1; d >>= 1) {
                        const uint32_t ov = __shfl_xor(best, d, 64);
                        const int oj = __shfl_xor(best_j, d, 64);
                        if (ov < best || (ov == best && oj < best_j)) { best = ov; best_j = oj; }
                    }
                    if (lane == 0) arg[s * row_len + L] = (uint16_t)(best == kInf32 ? 0xFFFFu : best_j);
                }
                __syncthreads();          // back-pointers of every wave are visible to thread 0
                if (arg[s * row_len + L] == 0xFFFFu) dead = true;   // L <= 1024, so no cut has this value
            }
            if (!dead && tid == 0) {
                int b = L;
                sp[S] = L;
                for (int s = S - 1; s >= 0; --s) { b = arg[s * row_len + b]; sp[s] = b; }
            }
        } else if (tid == 0) {
            sp[0] = 0;    // one stage holds every operator; the pre-pass has checked that it fits
            sp[1] = L;
        }
        if (dead) {
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            continue;
        }
        for (int s = S + 1 + tid; s <= S_max; s += nthreads) sp[s] = -1;
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
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
    // candidates the pre-pass rejected: no plan to report
    for (int n = blockIdx.x; n < n_dead; n += gridDim.x) {
        const uint32_t e = dead_list[n];
        write_failed(out, int(e & ((1u << kDeadStatusShift) - 1u)), S_max, int(e >> kDeadStatusShift));
    }
}


}  // namespace

size_t plan_fast_ws_bytes(int L, int S_max, int C, int n_groups) {
    return carve(nullptr, L, S_max, C, n_groups).total;
}

// Workgroups that can be resident at once: bounded by threads (2048 per CU) and LDS (160 KiB).
int plan_fast_groups(int L, int S_max, int n_cu) {
    const int by_threads = 2048 / kFastThreads;
    int by_lds = int((size_t(160) << 10) / (fast_lds_bytes(L, S_max) + 64));
    int per_cu = by_threads < by_lds ? by_threads : by_lds;
    if (per_cu < 1) per_cu = 1;
    return per_cu * n_cu;
}

// Pre-pass shared by every 32-bit planner entry point: clears the counters, checks the slot lists,
// computes the reachability bands and compacts the live and dead lists.
void launch_plan_prepass(const TablesDev &tb, const CandDev &cd, void *ws, int n_groups, hipStream_t st) {
    const FastWorkspace w = carve(ws, tb.L, cd.S_max, cd.C, n_groups);
    hipLaunchKernelGGL(k2_clear_count, dim3(1), dim3(64), 0, st, w.counts);
    const int caps_in_lds = tb.G * tb.n_tp <= kBandCapTable ? 1 : 0;
    const int bt = band_threads(cd.S_max);
    const size_t band_lds = size_t(tb.L + 1) * 16 + (caps_in_lds ? size_t(tb.G) * tb.n_tp * 8 : 0) +
                            size_t(cd.S_max) * (bt + 2) * 2;
    hipLaunchKernelGGL(k2_band, dim3((cd.C + bt - 1) / bt), dim3(bt), band_lds, st, tb, cd, w.counts,
                       w.live_list, w.dead_list, w.bands, caps_in_lds);
}

void launch_plan_fast(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                      int n_groups, hipStream_t st) {
    const FastWorkspace w = carve(ws, tb.L, cd.S_max, cd.C, n_groups);
    launch_plan_prepass(tb, cd, ws, n_groups, st);
    hipLaunchKernelGGL(k2_fast, dim3(n_groups), dim3(kFastThreads), fast_lds_bytes(tb.L, cd.S_max), st, tb,
                       cd, out, w.counts, w.live_list, w.dead_list, w.bands, w.arg,
                       fast_arg_per_group(tb.L, cd.S_max), fast_row_len(tb.L));
}

}  // namespace harp
