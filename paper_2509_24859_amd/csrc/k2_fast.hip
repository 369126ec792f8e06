// Fast planner-search kernels for gfx950: reachability bands, a feasibility index, 32-bit times,
// bounded scans, one wavefront per candidate with its rows in LDS.
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
//  * lo(s, i) depends on the stage only through its in-flight count n = min(S - s, M) and the memory
//    of its submesh, tp devices of one GPU type.  The pre-pass therefore also writes a feasibility
//    index of stage ranges per (count, GPU type, degree) into the workspace, once per call (the
//    precomputed index of feasible stage-mesh pairs of section 5.2.4 (1), reduced to what this
//    device model needs: one lower limit per end cut and one upper limit per start cut): row
//    (n, type, k), entry i = the lowest j such that operators [j, i) fit, and in a second table
//    entry j = the highest i such that they do.  A DP cell then knows its range of previous cuts
//    from one 16-bit load, the recurrence itself touches no byte count at all, and each link of
//    the band chains above is one lookup.
//  * the stage time time(s; j, i) never decreases when j moves down.  Scanning j downwards from
//    i-1, once time(s; j, i) exceeds the best value found so far no lower j can match or beat it,
//    and the scan stops.  The stop uses a strict comparison and the update a non-strict one, so
//    the lowest j among equal values is kept, as the recurrence demands.  Nothing is assumed
//    about the previous DP row (it is not monotone when transfer times dominate); in the worst
//    case the scan covers the whole range.
//
// With tp a power of two and every time below 2^31 us (both checked by the table build), the
// stage time is one subtraction and one shift on the fused 32-bit row
//   P[j] = PF[type][j] + tp * PR[g][tp][j]:   time(s; j, i) = (P[i] + tp - 1 - P[j]) >> log2 tp,
// because ceil(a / tp) + b = ceil((a + tp b) / tp) for integers.  Transfer times come from the
// per-link cut table built beside the rows.
//
// Mapping of k2_fast: one wavefront per live candidate at a time (persistent wavefronts draw from
// the list k2_band compacted through a shared counter; the wavefronts of a workgroup share nothing
// and never meet at a barrier), one lane per DP cell of the current stage's band, 64 cells per
// chunk.  The DP row and the stage's fused time row sit interleaved in LDS, one 8-byte entry per
// cut, in a single buffer: chunks are taken from the top of the band downwards and a cell only
// reads cuts below itself, so writing the new row over the old one never destroys a value that is
// still needed, and the time row of the next stage replaces the current one once the stage is done
// (its entries were requested from global memory before the stage's scans and wait in registers).
// Previous cuts are scanned four per trip; a trip keeps the least of its four values and its own
// position, and the lowest cut inside the winning trip is found once per cell afterwards.
// The buffer is band-relative: the entry of cut j of stage s sits at offset j - B[s], and the buffer
// is sized for the candidate's widest stage, not for L; a candidate whose widest stage does not fit
// the wavefront's share of LDS is queued for a second pass with a share sized for L.
// Back-pointers are one byte each (distance to the previous cut; 255 refers to a 16-bit entry in
// the wavefront's slice of the workspace): in an LDS arena while the candidate's rows fit there, so
// that the backtrack of most candidates never leaves the CU, in the slice beyond that.
#include "harp_internal.h"
#include "fast_common.h"
#include "plan_common.h"

namespace harp {

using namespace fastdp;

namespace {


// Feasibility index, one workgroup per row (n, GPU type t, degree index k): for every cut i the
// lowest j such that operators [j, i) fit, lo, and for every cut j the highest i such that [j, i)
// fit, hi; "fit" is (PP[i] - PP[j]) + n (PS[i] - PS[j]) <= tp_k * type_mem[t] (eq. mem_cons with n
// micro-batches in flight).  The need is monotone in both ends, so each entry is one binary
// search over Q = PP + n PS, which the workgroup keeps in LDS.
__global__ __launch_bounds__(256) void k2_index(TablesDev tb, uint16_t *lo_tab, uint16_t *hi_tab, int pitch,
                                                int n_rows) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    int64_t *Q = reinterpret_cast<int64_t *>(lds_raw);       // [L + 1]
    const int L = tb.L, rows_per_n = tb.T * tb.n_tp;
    const int64_t *gp = tb.PP(), *gs = tb.PS();
    for (int row = blockIdx.x; row < n_rows; row += gridDim.x) {
        const int n = row / rows_per_n + 1;
        const int tk = row - (n - 1) * rows_per_n;
        const int t = tk / tb.n_tp, k = tk - t * tb.n_tp;
        const int64_t cap = int64_t(tb.tp[k]) * tb.type_mem[t];
        __syncthreads();
        for (int i = threadIdx.x; i <= L; i += blockDim.x) Q[i] = gp[i] + int64_t(n) * gs[i];
        __syncthreads();
        uint16_t *lo = lo_tab + size_t(row) * pitch, *hi = hi_tab + size_t(row) * pitch;
        for (int i = threadIdx.x; i <= L; i += blockDim.x) {
            const int64_t q = Q[i];
            int a = -1, b = i;                  // Q[b] >= q - cap holds at b = i; Q[a] < q - cap (a = -1: none)
            while (b - a > 1) {
                const int m = (a + b) >> 1;
                if (Q[m] >= q - cap) b = m; else a = m;
            }
            lo[i] = (uint16_t)b;
            a = i, b = L + 1;                   // Q[a] - q <= cap holds at a = i; Q[b] - q > cap (b = L + 1: none)
            while (b - a > 1) {
                const int m = (a + b) >> 1;
                if (Q[m] - q <= cap) a = m; else b = m;
            }
            hi[i] = (uint16_t)a;
        }
    }
}

// Pre-pass, one thread per candidate: checks the slot list and computes the reachability band
// [B[s], F[s]] of every DP row from the memory constraint alone.  With the feasibility index in
// place each link of the two chains is one lookup:
//   F[s+1] = min(hi(n_s, type_s, k_s)[F[s]], top_s),     B[s] = max(lo(n_s, type_s, k_s)[B[s+1]], s),
// top_s being the last cut that leaves one operator to every later stage.  Candidates that pass go
// to the live list; malformed ones and those proven infeasible go to the dead list with their
// status.
//
// Every candidate walks its slot list twice, so the workgroup's slot lists are read from global
// memory once, coalesced, and kept in LDS slot-major (conflict-free per-thread walks).  The two
// chains leave their limits in LDS tiles as well, and the workgroup writes the bands of its
// candidates as one contiguous run, candidate-major ([c][s]): the wavefront that later plans
// candidate c reads its row with one coalesced load.
constexpr int kBandTypeTable = 2048;    // GPU type and size of every group kept in LDS when G is at most this
constexpr uint16_t kBadSlot = 0xFFFFu;

int band_threads(int S_max) { return S_max <= 64 ? 256 : (S_max <= 128 ? 128 : 64); }

__global__ __launch_bounds__(256) void k2_band(TablesDev tb, CandDev cd, int *counts, int32_t *live_list,
                                               uint32_t *dead_list, uint32_t *bands, int types_in_lds,
                                               const uint16_t *lo_tab, const uint16_t *hi_tab, int idx_pitch) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int L = tb.L, S_max = cd.S_max, C = cd.C;
    const int nthreads = blockDim.x, pitch = nthreads + 2;
    // slot codes, replaced stage by stage by the lower band limits B[s]; and the upper limits F[s]
    uint16_t *slots = reinterpret_cast<uint16_t *>(lds_raw);        // [S_max + 1][pitch]
    uint16_t *ftile = slots + (S_max + 1) * pitch;                  // [S_max + 1][pitch]
    int32_t *gtype = reinterpret_cast<int32_t *>(ftile + (S_max + 1) * pitch);   // [G] when types_in_lds
    int32_t *gndev = gtype + tb.G;                                               // [G] when types_in_lds
    const int c0 = blockIdx.x * nthreads;
    const int n_here = (C - c0) < nthreads ? (C - c0) : nthreads;
    {
        if (types_in_lds)
            for (int g = threadIdx.x; g < tb.G; g += nthreads) {
                gtype[g] = tb.group_type[g];
                gndev[g] = tb.group_ndev[g];
            }
        // slot lists of this workgroup's candidates: (group << 3) | degree index, or kBadSlot
        const int32_t *grp = cd.cand_group + int64_t(c0) * S_max;
        const int32_t *tpv = cd.cand_tp + int64_t(c0) * S_max;
        // four loads in flight per thread: the loop is bound by their latency
        const int n_slots = n_here * S_max;
        for (int idx0 = threadIdx.x; idx0 < n_slots; idx0 += 4 * nthreads) {
            int g4[4], t4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = idx0 + u * nthreads;
                g4[u] = idx < n_slots ? grp[idx] : 0;
                t4[u] = idx < n_slots ? tpv[idx] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = idx0 + u * nthreads;
                if (idx < n_slots) {
                    const int cl = idx / S_max, s = idx - cl * S_max;
                    const int g = g4[u], k = tp_index(tb, t4[u]);
                    slots[s * pitch + cl] = (g < 0 || g >= tb.G || k < 0) ? kBadSlot : (uint16_t)((g << 3) | k);
                }
            }
        }
    }
    __syncthreads();
    const int cl = threadIdx.x, c = c0 + cl;
    const bool mine = c < C;
    const int S = mine ? cd.cand_S[c] : 0;
    const int R = L - S + 1;
    // row of the index for a stage with n micro-batches in flight on degree index k of group g
    auto index_row = [&](int n, int g, int k) -> size_t {
        const int t = types_in_lds ? gtype[g] : tb.group_type[g];
        return size_t(((n - 1) * tb.T + t) * tb.n_tp + k) * idx_pitch;
    };

    int status = HARP_CAND_OK;
    bool feasible = S <= L;
    if (S < 1 || S > S_max) status = HARP_CAND_INVALID;
    // one walk over the slots: well-formedness, and the forward chain
    // F[s+1] = largest cut that stage s can reach from F[s]
    int64_t used = 0;
    unsigned long long seen = 0;                      // groups already entered, when G <= 64
    int prev_g = -1, F = 0;
    ftile[cl] = 0;
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
        if (used > (types_in_lds ? gndev[g] : tb.group_ndev[g])) status = HARP_CAND_INVALID;
        if (feasible) {
            const int n = (S - s) < tb.M ? (S - s) : tb.M;
            const int reach = hi_tab[index_row(n, g, k) + F];
            const int top = (s == S - 1) ? L : s + R;
            F = reach < top ? reach : top;
            if (F < s + 1 || (s == S - 1 && F != L)) feasible = false;
            else ftile[(s + 1) * pitch + cl] = (uint16_t)F;
        }
    }
    // backward chain: B[s] = smallest cut from which stage s can reach B[s+1]; B[s] takes the place of
    // the slot code of stage s, which is no longer needed
    if (status == HARP_CAND_OK && feasible) {
        int B = L;
        slots[S * pitch + cl] = (uint16_t)L;
        for (int s = S - 1; s >= 0; --s) {
            const uint16_t code = slots[s * pitch + cl];
            const int n = (S - s) < tb.M ? (S - s) : tb.M;
            const int from = lo_tab[index_row(n, code >> 3, code & 7) + B];
            B = from > s ? from : s;
            const int hi = ftile[s * pitch + cl];
            if (hi < B || (s == 0 && B != 0)) { feasible = false; break; }
            slots[s * pitch + cl] = (uint16_t)B;
        }
    }
    if (status == HARP_CAND_OK && !feasible) status = HARP_CAND_INFEASIBLE;

    // append to the live or the dead list with one atomic per wave and list: lanes rank themselves
    const int lane = threadIdx.x & 63;
    const bool alive = mine && status == HARP_CAND_OK;
    const unsigned long long here = __ballot(mine), live_m = __ballot(alive), dead_m = here & ~live_m;
    const int leader = __ffsll((long long)here) - 1;
    int base_live = 0, base_dead = 0;
    if (here != 0) {
        if (lane == leader) {
            if (live_m) base_live = atomicAdd(&counts[0], __popcll(live_m));
            if (dead_m) base_dead = atomicAdd(&counts[1], __popcll(dead_m));
        }
        base_live = __shfl(base_live, leader, 64);
        base_dead = __shfl(base_dead, leader, 64);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (alive) live_list[base_live + __popcll(live_m & below)] = c;
        else if (mine) dead_list[base_dead + __popcll(dead_m & below)] = uint32_t(c) | (uint32_t(status) << kDeadStatusShift);
    }
    // the bands of the workgroup's candidates leave LDS as one contiguous run of rows (rows of
    // candidates without bands carry whatever the tiles held: nobody reads them)
    __syncthreads();
    uint32_t *dst = bands + int64_t(c0) * (S_max + 1);
    for (int e = threadIdx.x; e < n_here * (S_max + 1); e += nthreads) {
        const int cand = e / (S_max + 1), s = e - cand * (S_max + 1);
        dst[e] = uint32_t(slots[s * pitch + cand]) | (uint32_t(ftile[s * pitch + cand]) << 16);
    }
}

__global__ void k2_clear_count(int *counts) {
    if (threadIdx.x < 32) counts[threadIdx.x] = 0;
}

__global__ void k2_clear_work(unsigned long long *work) {
    if (threadIdx.x < 4) work[threadIdx.x] = 0;
}

// ---------------------------------------------------------------------------------- k2_fast

constexpr int kPrefetchChunks = 2;      // chunks of the next stage's time row held in registers
constexpr int kArgEscape = 255;         // one-byte back-pointer: distance too long, see the slice
constexpr uint32_t kArgBias = 1u << 16;     // keeps (stage offset - lowest cut of the row) positive
constexpr uint32_t kArgInLds = 1u << 31;    // flag on that word: the stage's back-pointers are in the LDS arena

// wavefront-scope ordering of LDS traffic: one wavefront's LDS operations execute in order, so
// this only keeps the compiler from moving accesses across the phases of a stage
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint32_t umin2(uint32_t a, uint32_t b) { return a < b ? a : b; }

struct FastArgs {
    const uint32_t *bands;        // [C][S_max + 1]
    const uint16_t *lo_tab;       // feasibility index
    unsigned char *arg_base;      // back-pointer slices
    size_t arg_per_wave;
    size_t arg_u8_off;            // where a slice's one-byte entries start
    unsigned long long *work;     // [4] transitions, cells, trips, candidates (counting build only)
    int lo_pitch, lds_per_wave;
    int wide_pass;                // 1: the pass over the candidates the first pass found too wide for its LDS share
    uint32_t shift_packed;        // log2 of degree k in bits 4k .. 4k+3
};

// per-wavefront LDS slice: band [S_max+1] | slot [S_max] | aoff [S_max+1] | cuts [S_max+1] | row entries
// of the candidate's widest stage | arena (the rest)
__host__ __device__ inline size_t fast_wave_small_bytes(int S_max) {
    return (size_t(S_max + 1) * 12 + size_t(S_max) * 4 + 15) & ~size_t(15);
}
// bytes of row entries for a stage that reads `span` cuts: kPad spare entries in front, so that the
// group of four previous cuts ending at any cut of the stage can be read without clamping
__host__ __device__ inline size_t fast_row_bytes(int span) {
    return (size_t(span + kPad) * sizeof(Pair) + 15) & ~size_t(15);
}

template <bool kCount>
__global__ __launch_bounds__(kFastWaves * 64) void k2_fast(TablesDev tb, CandDev cd, PlansDev out, int *counts,
                                                            const int32_t *live_list,
                                                            uint32_t *dead_list, FastArgs fa) {
    extern __shared__ __align__(16) unsigned char lds_raw[];

    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63;
    const int wave = uniform(threadIdx.x >> 6);
    const int wave_id = blockIdx.x * kFastWaves + wave, n_waves = gridDim.x * kFastWaves;
    unsigned char *mine = lds_raw + size_t(wave) * fa.lds_per_wave;
    uint32_t *band = reinterpret_cast<uint32_t *>(mine);                               // [S_max + 1]
    uint32_t *slot = band + (S_max + 1);                                               // [S_max]
    uint32_t *aoff = slot + S_max;                                                     // [S_max + 1]
    int32_t *cuts = reinterpret_cast<int32_t *>(aoff + (S_max + 1));                   // [S_max + 1]
    const int small_bytes = int(fast_wave_small_bytes(S_max));
    // row entries: entry of cut j of the stage whose lowest cut is `base` sits at rows0[j - base]
    Pair *rows0 = reinterpret_cast<Pair *>(mine + small_bytes) + kPad;
    uint16_t *slice = reinterpret_cast<uint16_t *>(fa.arg_base + size_t(wave_id) * fa.arg_per_wave);
    uint8_t *slice8 = reinterpret_cast<uint8_t *>(slice) + fa.arg_u8_off;
    // first pass: the live list; second pass: the candidates the first one queued behind the dead list
    const int n_dead = counts[1];
    const int n_live = fa.wide_pass ? counts[8] : counts[0];
    int *next_item = counts + (fa.wide_pass ? 9 : 5);
    const int m_cap = tb.M;
    const int rows_per_n = tb.T * tb.n_tp;
    unsigned long long n_trans = 0, n_cells = 0, n_trips = 0, n_cands = 0;

    // scalars of one stage, from the packed slot word  g | k << 12 | type << 16
    struct Stage {
        const uint32_t *p_row, *cm_row;
        const uint16_t *lo;
        int shift;
    };
    auto stage_of = [&](int s, int S) -> Stage {
        const uint32_t w = (uint32_t)uniform((int)slot[s]);
        const uint32_t wn = (uint32_t)uniform((int)slot[s + 1 < S ? s + 1 : s]);
        const int g = int(w & 0xFFFu), k = int((w >> 12) & 7u), t = int(w >> 16);
        const int gn = int(wn & 0xFFFu);
        const int n = (S - s) < m_cap ? (S - s) : m_cap;
        Stage st;
        st.p_row = tb.P32 + (int64_t(g) * tb.n_tp + k) * tb.pitch32;
        st.cm_row = tb.CM + (int64_t(g) * tb.G + gn) * tb.pitch32;
        st.lo = fa.lo_tab + (int64_t(n - 1) * rows_per_n + t * tb.n_tp + k) * fa.lo_pitch;
        st.shift = int((fa.shift_packed >> (4 * k)) & 15u);
        return st;
    };

    // candidates differ in stages and band widths, so wavefronts draw them from a shared counter
    for (;;) {
        // Every lane takes part in the draw (only the first adds one).  A draw under `if (lane == 0)`
        // would sit right behind the lane-0 stores that end the previous candidate; the compiler
        // joins two such branches, and the other lanes then reach the broadcast below on their own,
        // ahead of lane 0 and without a ticket.
        wave_sync();
        const int n = uniform(atomicAdd(next_item, lane == 0 ? 1 : 0));
        if (n >= n_live) break;
        const int c = uniform(fa.wide_pass ? int(dead_list[n_dead + n]) : live_list[n]);
        const int S = uniform(cd.cand_S[c]);
        wave_sync();              // the previous candidate's tail has finished with LDS
        {
            const int32_t *grp = cd.cand_group + int64_t(c) * S_max;
            const int32_t *tpv = cd.cand_tp + int64_t(c) * S_max;
            int32_t *df = out.dev_first + int64_t(c) * S_max;
            const uint32_t *bd = fa.bands + int64_t(c) * (S_max + 1);
            for (int s = lane; s < S; s += 64) {
                const int g = grp[s], k = tp_index(tb, tpv[s]);
                slot[s] = uint32_t(g) | (uint32_t(k) << 12) | (uint32_t(tb.group_type[g]) << 16);
                // first device of the slot: its group's base plus the degrees of the group's
                // earlier slots (they are adjacent; the pre-pass has checked that)
                int32_t first = tb.group_base[g];
                for (int q = s - 1; q >= 0 && grp[q] == g; --q) first += tpv[q];
                df[s] = first;
            }
            for (int s = S + lane; s < S_max; s += 64) df[s] = -1;
            // bands, and where the back-pointers of each stage start: running sum of the widths of
            // rows 1 .. S-1 (the last row has the single cell L, kept in a register)
            uint32_t carry = 0;
            for (int s0 = 0; s0 <= S; s0 += 64) {
                const int s = s0 + lane;
                uint32_t b = 0, wdt = 0;
                if (s <= S) { b = bd[s]; band[s] = b; }
                if (s >= 1 && s < S) wdt = uint32_t(band_hi(b) - band_lo(b) + 1);
                uint32_t inc = wdt;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const uint32_t o = __shfl_up(inc, d, 64);
                    if (lane >= d) inc += o;
                }
                // aoff[s - 1] = where the back-pointer of cut 0 of row s would sit (stage s - 1 writes
                // row s): the stage's offset less the row's lowest cut, biased to stay positive
                if (s >= 1 && s <= S) aoff[s - 1] = carry + inc - wdt + kArgBias - uint32_t(band_lo(b));
                carry += __shfl(inc, 63, 64);
            }
        }
        wave_sync();
        // LDS of this candidate: row entries for its widest stage (stage s reads the cuts B[s] .. F[s+1]),
        // the rest of the wavefront's share for back-pointers.  A candidate whose widest stage does
        // not fit the share is queued for the second pass, which runs with a share sized for L.
        int span = 0;
        for (int s = lane; s < S; s += 64) {
            const int w = band_hi(band[s + 1]) - band_lo(band[s]) + 1;
            span = w > span ? w : span;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const int o = __shfl_xor(span, d, 64);
            span = o > span ? o : span;
        }
        span = uniform(span);
        const int row_bytes = int(fast_row_bytes(span));
        if (small_bytes + row_bytes > fa.lds_per_wave) {
            if (lane == 0) dead_list[n_dead + atomicAdd(&counts[8], 1)] = uint32_t(c);
            continue;
        }
        uint8_t *arena = reinterpret_cast<uint8_t *>(mine) + small_bytes + row_bytes;
        const uint32_t arena_bytes = uint32_t(fa.lds_per_wave - small_bytes - row_bytes);
        // stages whose back-pointers fit the arena (offset + width within it) are flagged once
        for (int s = lane; s + 1 < S; s += 64) {
            const uint32_t end = aoff[s] - kArgBias + uint32_t(band_hi(band[s + 1])) + 1u;
            if (end <= arena_bytes) aoff[s] |= kArgInLds;
        }
        wave_sync();
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        uint32_t final_v = 0;
        if (S >= 2) {
            // prologue: time row of stage 0 over [0, F[1]]; row 0 of the DP is the single cut 0
            Stage cur = stage_of(0, S);
            {
                const int top = band_hi((uint32_t)uniform((int)band[1]));
                for (int j = lane; j <= top; j += 64) rows0[j].p = cur.p_row[j];
                if (lane == 0) rows0[0].d = 0;
            }
            // first work item: the top chunk of stage 0
            uint32_t cut_c = 0;
            int lo_c = 0;
            {
                const uint32_t b1 = (uint32_t)uniform((int)band[1]);
                const int il = band_lo(b1), ih = band_hi(b1);
                const int i = il + ((ih - il) & ~63) + lane;
                if (i <= ih) { cut_c = cur.cm_row[i]; lo_c = cur.lo[i]; }
            }
            wave_sync();

            for (int s = 0; s < S - 1; ++s) {
                const uint32_t b0 = (uint32_t)uniform((int)band[s]);
                const uint32_t b1 = (uint32_t)uniform((int)band[s + 1]);
                const uint32_t b2 = (uint32_t)uniform((int)band[s + 2]);
                const int jl = band_lo(b0), jh = band_hi(b0);     // predecessors: row s
                const int il = band_lo(b1), ih = band_hi(b1);     // cells: row s + 1
                const int top_n = band_hi(b2);                    // stage s+1 reads its time row up to here
                const int shift = cur.shift;
                const uint32_t tp = 1u << shift;
                const Stage nxt = stage_of(s + 1, S);
                const bool nxt_is_last = s + 2 == S;
                const uint32_t a_word = (uint32_t)uniform((int)aoff[s]);
                const bool arg_in_lds = (a_word & kArgInLds) != 0;
                const uint32_t a0 = (a_word & ~kArgInLds) - kArgBias;       // + cut = index of the cut's back-pointer
                Pair *rows = rows0 - jl;          // this stage's entries: cut j at rows[j], from B[s] on

                // requests for the time row of stage s+1: entries [il, top_n], first chunks in registers
                uint32_t pn[kPrefetchChunks];
#pragma unroll
                for (int q = 0; q < kPrefetchChunks; ++q) {
                    pn[q] = 0u;
                    if (il + q * 64 <= top_n) {       // most stages are a chunk or two wide
                        const int j = il + q * 64 + lane;
                        if (j <= top_n) pn[q] = nxt.p_row[j];
                    }
                }

                for (int q = (ih - il) >> 6; q >= 0; --q) {
                    const int i = il + q * 64 + lane;
                    // requests for the next work item: the chunk below, or the top chunk of the next stage
                    uint32_t cut_n = 0;
                    int lo_n = 0;
                    if (q > 0) {
                        cut_n = cur.cm_row[i - 64];
                        lo_n = cur.lo[i - 64];
                    } else if (!nxt_is_last) {
                        const int i2l = band_lo(b2);
                        const int i2 = i2l + ((top_n - i2l) & ~63) + lane;
                        if (i2 <= top_n) { cut_n = nxt.cm_row[i2]; lo_n = nxt.lo[i2]; }
                    }

                    // One DP cell: the previous cuts that fit are lo .. hi; four per trip, downwards.
                    // A trip keeps the least of its four values; ties between trips go to the lower
                    // one.  Entries below a stop cannot match the best value (their stage time alone
                    // exceeds it), so only the last entry of a trip decides whether the lane goes on.
                    uint32_t best = kInf32;
                    int best_j = 0;
                    if (i <= ih) {
                        const int hi = (i - 1) < jh ? (i - 1) : jh;
                        const int lo = lo_c > jl ? lo_c : jl;
                        const uint32_t xi = rows[i].p + tp - 1;
                        const uint32_t cut = cut_c;
                        int bt = hi;
                        int j = hi;
                        while (j - 3 >= lo) {
                            const Pair *pe = rows + (j - 3);
                            const Pair e3 = pe[0], e2 = pe[1], e1 = pe[2], e0 = pe[3];
                            const uint32_t t3 = (xi - e3.p) >> shift;
                            const uint32_t v0 = umax3(e0.d, (xi - e0.p) >> shift, cut);
                            const uint32_t v1 = umax3(e1.d, (xi - e1.p) >> shift, cut);
                            const uint32_t v2 = umax3(e2.d, (xi - e2.p) >> shift, cut);
                            const uint32_t v3 = umax3(e3.d, t3, cut);
                            const uint32_t m = umin2(umin2(v0, v1), umin2(v2, v3));
                            const bool upd = m <= best;
                            best = upd ? m : best;
                            bt = upd ? j : bt;
                            if (kCount) { n_trans += 4; ++n_trips; }
                            j = t3 > best ? lo - 1 : j - 4;
                        }
                        // what is left of the range: at most three cuts, j .. lo
                        {
                            const Pair *pe = rows + (j - 3);
                            const Pair e2 = pe[1], e1 = pe[2], e0 = pe[3];
                            const uint32_t v0 = j >= lo ? umax3(e0.d, (xi - e0.p) >> shift, cut) : kInf32;
                            const uint32_t v1 = j - 1 >= lo ? umax3(e1.d, (xi - e1.p) >> shift, cut) : kInf32;
                            const uint32_t v2 = j - 2 >= lo ? umax3(e2.d, (xi - e2.p) >> shift, cut) : kInf32;
                            const uint32_t m = umin2(umin2(v0, v1), v2);
                            const bool upd = (m <= best) & (j >= lo);
                            best = upd ? m : best;
                            bt = upd ? j : bt;
                            if (kCount) { n_trans += j >= lo ? uint32_t(j - lo + 1) : 0u; n_trips += j >= lo; ++n_cells; }
                        }
                        // the lowest cut of the winning trip that attains the best value
                        {
                            const Pair *pw = rows + (bt - 3);
                            const Pair w3 = pw[0], w2 = pw[1], w1 = pw[2];
                            const uint32_t u1 = umax3(w1.d, (xi - w1.p) >> shift, cut);
                            const uint32_t u2 = umax3(w2.d, (xi - w2.p) >> shift, cut);
                            const uint32_t u3 = umax3(w3.d, (xi - w3.p) >> shift, cut);
                            best_j = bt;
                            best_j = ((u1 == best) & (bt - 1 >= lo)) ? bt - 1 : best_j;
                            best_j = ((u2 == best) & (bt - 2 >= lo)) ? bt - 2 : best_j;
                            best_j = ((u3 == best) & (bt - 3 >= lo)) ? bt - 3 : best_j;
                            best_j = best == kInf32 ? i - 1 : best_j;      // no previous cut fits: any value
                        }
                    }
                    wave_sync();      // every lane has read what it needs of the old row
                    if (i <= ih) {
                        rows[i].d = best;
                        const int rel = i - 1 - best_j;
                        const uint32_t at = a0 + uint32_t(i);
                        // one byte per cell, in LDS while the candidate's rows fit the arena
                        const uint8_t code = (uint8_t)(rel < kArgEscape ? rel : kArgEscape);
                        if (arg_in_lds) arena[at] = code;
                        else slice8[at] = code;
                        if (rel >= kArgEscape) slice[at] = (uint16_t)best_j;
                    }
                    wave_sync();
                    cut_c = cut_n;
                    lo_c = lo_n;
                }

                // The time row of stage s+1 takes the place of this stage's, and the entries move down
                // to start at B[s+1]: chunk by chunk upwards, every lane reading its old DP value before
                // any lane writes (a chunk lands at or below its old place and never on a chunk that is
                // still to be read).
                Pair *rows_n = rows0 - il;
#pragma unroll
                for (int q = 0; q < kPrefetchChunks; ++q) {
                    if (il + q * 64 > top_n) break;
                    const int j = il + q * 64 + lane;
                    uint32_t d_keep = 0;
                    if (j <= ih) d_keep = rows[j].d;
                    wave_sync();
                    if (j <= top_n) rows_n[j] = Pair{d_keep, pn[q]};
                    wave_sync();
                }
                for (int j0 = il + kPrefetchChunks * 64; j0 <= top_n; j0 += 64) {
                    const int j = j0 + lane;
                    uint32_t d_keep = 0, p_new = 0;
                    if (j <= ih) d_keep = rows[j].d;
                    if (j <= top_n) p_new = nxt.p_row[j];
                    wave_sync();
                    if (j <= top_n) rows_n[j] = Pair{d_keep, p_new};
                    wave_sync();
                }
                cur = nxt;
            }
            // the last stage has the single cell i = L: lanes over j, lexicographic reduction
            int last_j;
            {
                const int s = S - 1;
                const uint32_t b0 = (uint32_t)uniform((int)band[s]);
                const int shift = cur.shift;
                const Pair *rows = rows0 - band_lo(b0);
                const uint32_t xi = rows[L].p + (1u << shift) - 1;
                const int lo_L = uniform((int)cur.lo[L]);
                const int lo = lo_L > band_lo(b0) ? lo_L : band_lo(b0);
                const int hi = (L - 1) < band_hi(b0) ? (L - 1) : band_hi(b0);
                uint32_t best = kInf32;
                int best_j = INT32_MAX;
                for (int j = lo + lane; j <= hi; j += 64) {
                    const Pair e = rows[j];
                    const uint32_t tj = (xi - e.p) >> shift;
                    const uint32_t v = e.d > tj ? e.d : tj;
                    if (v < best) { best = v; best_j = j; }   // j rises within a lane
                    if (kCount) ++n_trans;
                }
                if (kCount && lane == 0) { ++n_cells; ++n_cands; }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const uint32_t ov = __shfl_xor(best, d, 64);
                    const int oj = __shfl_xor(best_j, d, 64);
                    if (ov < best || (ov == best && oj < best_j)) { best = ov; best_j = oj; }
                }
                final_v = (uint32_t)uniform((int)best);
                last_j = uniform(best_j);
            }
            if (final_v == kInf32) {          // the bands were bounds: the recurrence found no plan
                write_failed_wave(out, c, S_max, HARP_CAND_INFEASIBLE, lane);
                continue;
            }
            // backtrack along the back-pointers
            if (lane == 0) {
                int b = last_j;
                cuts[S] = L;
                cuts[S - 1] = b;
                for (int s = S - 2; s >= 0; --s) {
                    const uint32_t a_word = aoff[s];
                    const uint32_t at = (a_word & ~kArgInLds) - kArgBias + uint32_t(b);
                    int rel;
                    if (a_word & kArgInLds) rel = arena[at];
                    else rel = slice8[at];
                    b = rel == kArgEscape ? int(slice[at]) : b - 1 - rel;
                    cuts[s] = b;
                }
            }
            wave_sync();
        } else {
            // one stage holds every operator; the pre-pass has checked that it fits
            if (lane == 0) { cuts[0] = 0; cuts[1] = L; }
            if (kCount && lane == 0) ++n_cands;
            wave_sync();
        }
        for (int s = lane; s <= S_max; s += 64) sp[s] = s <= S ? cuts[s] : -1;
        // score of the plan (section 5.2.2): sum of (t + 2c) + (M - 1) bottleneck, lanes over stages
        {
            uint32_t worst = 0;
            int64_t single = 0;
            for (int s = lane; s < S; s += 64) {
                const uint32_t w = slot[s], wn = slot[s + 1 < S ? s + 1 : s];
                const int g = int(w & 0xFFFu), k = int((w >> 12) & 7u), gn = int(wn & 0xFFFu);
                const int shift = int((fa.shift_packed >> (4 * k)) & 15u);
                const uint32_t *p = tb.P32 + (int64_t(g) * tb.n_tp + k) * tb.pitch32;
                const int j = cuts[s], i = cuts[s + 1];
                const uint32_t t = (p[i] + (1u << shift) - 1u - p[j]) >> shift;
                const uint32_t cu = s < S - 1 ? tb.CM[(int64_t(g) * tb.G + gn) * tb.pitch32 + i] : 0u;
                const uint32_t m = t > cu ? t : cu;
                worst = worst > m ? worst : m;
                single += int64_t(t) + 2 * int64_t(cu);
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const uint32_t ow = __shfl_xor(worst, d, 64);
                single += __shfl_xor(single, d, 64);
                worst = worst > ow ? worst : ow;
            }
            if (lane == 0) {
                out.bottleneck[c] = int64_t(worst);
                out.iter_time[c] = single + int64_t(m_cap - 1) * int64_t(worst);
                out.status[c] = HARP_CAND_OK;
            }
        }
    }
    // candidates the pre-pass rejected: no plan to report
    for (int n = wave_id; n < n_dead && !fa.wide_pass; n += n_waves) {
        const uint32_t e = dead_list[n];
        write_failed_wave(out, int(e & ((1u << kDeadStatusShift) - 1u)), S_max, int(e >> kDeadStatusShift), lane);
    }
    if (kCount) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            n_trans += __shfl_xor(n_trans, d, 64);
            n_cells += __shfl_xor(n_cells, d, 64);
            n_trips += __shfl_xor(n_trips, d, 64);
            n_cands += __shfl_xor(n_cands, d, 64);
        }
        if (lane == 0) {
            atomicAdd(&fa.work[0], n_trans);
            atomicAdd(&fa.work[1], n_cells);
            atomicAdd(&fa.work[2], n_trips);
            atomicAdd(&fa.work[3], n_cands);
        }
    }
}

struct FastLaunch {
    int waves_per_cu, lds_per_wave;
    bool second_pass;        // some candidate of this shape may not fit the first pass's share
    int wide_waves_per_cu, wide_lds_per_wave;
};

// LDS split.  A wavefront's share holds its small per-candidate arrays, the row entries of the
// candidate's widest stage and, in what is left, one-byte back-pointers.  Measured on the
// 512-operator workload with rows sized for L: 16 resident wavefronts per CU plan the batch in
// 6.1 ms, 24 in 5.2 ms, 28 in 5.3 ms, so the first pass runs 24 per CU (six per SIMD); a candidate
// whose widest stage does not fit that share goes to a second pass whose share is sized for a
// stage over the whole sequence (launched only when L makes that possible).
FastLaunch fast_launch_shape(int L, int S_max) {
    const size_t lds_cu = size_t(160) << 10;
    const size_t small = fast_wave_small_bytes(S_max);
    const size_t widest = small + fast_row_bytes(L + 1);
    FastLaunch f;
    int waves = 24;
    while (waves > kFastWaves && (small + fast_row_bytes(8)) * waves > lds_cu) waves -= kFastWaves;
    f.waves_per_cu = waves;
    f.lds_per_wave = int((lds_cu / waves - 128) & ~size_t(15));     // a little under an even split: allocation granules
    f.second_pass = widest > size_t(f.lds_per_wave);
    int wide = 24;
    while (wide > kFastWaves && (widest + 128) * wide > lds_cu) wide -= kFastWaves;
    f.wide_waves_per_cu = wide;
    f.wide_lds_per_wave = int((lds_cu / wide - 128) & ~size_t(15));
    if (size_t(f.wide_lds_per_wave) < widest) f.wide_lds_per_wave = int(widest);
    return f;
}

}  // namespace

size_t plan_fast_ws_bytes(const TablesDev &tb, int S_max, int C, int n_slices) {
    const FastShape f{tb.L, S_max, C, tb.M, tb.T, tb.n_tp};
    return carve(nullptr, f, n_slices).total;
}

size_t plan_fast_index_bytes(const TablesDev &tb, int S_max) {
    return lo_table_bytes(tb.L, S_max, tb.M, tb.T, tb.n_tp);
}

void launch_clear_work(unsigned long long *work, hipStream_t st) {
    hipLaunchKernelGGL(k2_clear_work, dim3(1), dim3(64), 0, st, work);
}

// Wavefronts of k2_fast that can be resident at once.
int plan_fast_waves(int L, int S_max, int n_cu) {
    return fast_launch_shape(L, S_max).waves_per_cu * n_cu;
}

// Workgroups of the other 32-bit kernels that can be resident at once: bounded by threads (2048
// per CU) and LDS (160 KiB).
int plan_fast_groups(int L, int S_max, int n_cu) {
    const int by_threads = 2048 / kFastThreads;
    int by_lds = int((size_t(160) << 10) / (fast_lds_bytes(L, S_max) + 64));
    int per_cu = by_threads < by_lds ? by_threads : by_lds;
    if (per_cu < 1) per_cu = 1;
    return per_cu * n_cu;
}

// Pre-pass shared by every 32-bit planner entry point: clears the counters, checks the slot lists,
// computes the reachability bands, compacts the live and dead lists, and writes the feasibility
// index.
void launch_plan_prepass(const TablesDev &tb, const CandDev &cd, void *ws, int n_slices, hipStream_t st) {
    const FastWorkspace w = carve(ws, fast_shape(tb, cd), n_slices);
    hipLaunchKernelGGL(k2_clear_count, dim3(1), dim3(64), 0, st, w.counts);
    const long long idx_rows = (long long)lo_n_max(tb.L, cd.S_max, tb.M) * tb.T * tb.n_tp;
    const int idx_pitch = int(lo_pitch(tb.L));
    hipLaunchKernelGGL(k2_index, dim3(unsigned(idx_rows < 65536 ? idx_rows : 65536)), dim3(256),
                       size_t(tb.L + 1) * 8, st, tb, w.lo_tab, w.lo_tab + idx_rows * idx_pitch, idx_pitch,
                       int(idx_rows));
    const int types_in_lds = tb.G <= kBandTypeTable ? 1 : 0;
    const int bt = band_threads(cd.S_max);
    const size_t band_lds = size_t(cd.S_max + 1) * (bt + 2) * 2 * 2 + (types_in_lds ? size_t(tb.G) * 8 : 0);
    hipLaunchKernelGGL(k2_band, dim3((cd.C + bt - 1) / bt), dim3(bt), band_lds, st, tb, cd, w.counts,
                       w.live_list, w.dead_list, w.bands, types_in_lds, w.lo_tab,
                       w.lo_tab + idx_rows * idx_pitch, idx_pitch);
}

// n_slices: back-pointer slices in the workspace; k2_fast runs with at most that many wavefronts.
void launch_plan_fast(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                      int n_slices, int n_cu, unsigned long long *work, hipStream_t st) {
    const FastWorkspace w = carve(ws, fast_shape(tb, cd), n_slices);
    launch_plan_prepass(tb, cd, ws, n_slices, st);
    const FastLaunch shape = fast_launch_shape(tb.L, cd.S_max);
    FastArgs fa;
    fa.bands = w.bands;
    fa.lo_tab = w.lo_tab;
    fa.arg_base = w.arg;
    fa.arg_per_wave = fast_arg_per_group(tb.L, cd.S_max);
    fa.arg_u8_off = fast_arg_u16_bytes(tb.L, cd.S_max);
    fa.work = work;
    fa.lo_pitch = int(lo_pitch(tb.L));
    fa.shift_packed = 0;
    for (int k = 0; k < tb.n_tp; ++k) fa.shift_packed |= uint32_t(tb.tp_shift[k] & 15) << (4 * k);
    for (int pass = 0; pass < (shape.second_pass ? 2 : 1); ++pass) {
        const int per_cu = pass ? shape.wide_waves_per_cu : shape.waves_per_cu;
        fa.lds_per_wave = pass ? shape.wide_lds_per_wave : shape.lds_per_wave;
        fa.wide_pass = pass;
        // whole workgroups only: every wavefront of the grid owns a slice (n_slices >= kFastWaves)
        int n_groups = per_cu * n_cu / kFastWaves;
        if (n_groups > n_slices / kFastWaves) n_groups = n_slices / kFastWaves;
        if (n_groups > (cd.C + kFastWaves - 1) / kFastWaves) n_groups = (cd.C + kFastWaves - 1) / kFastWaves;
        if (n_groups < 1) n_groups = 1;
        const size_t lds = size_t(kFastWaves) * fa.lds_per_wave;
        if (work)
            hipLaunchKernelGGL(k2_fast<true>, dim3(n_groups), dim3(kFastWaves * 64), lds, st, tb, cd, out, w.counts,
                               w.live_list, w.dead_list, fa);
        else
            hipLaunchKernelGGL(k2_fast<false>, dim3(n_groups), dim3(kFastWaves * 64), lds, st, tb, cd, out, w.counts,
                               w.live_list, w.dead_list, fa);
    }
}

}  // namespace harp
