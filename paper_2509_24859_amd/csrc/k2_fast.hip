// Fast planner-search kernel for gfx950: 32-bit times, bounded scans, rows in LDS.
//
// Same recurrence as the generic kernel (paper section 5.2.3, eq. dp_general with the submesh of
// each stage fixed by the candidate; constraints (i)-(iii)), same results bit for bit, but the
// work per DP cell is cut down with two facts that hold for every valid problem (all costs and
// byte counts are non-negative, which the table build has verified):
//
//  * eq. mem_cons is monotone in the previous cut j: a longer stage never needs less memory.  So
//    the fitting cuts of cell (s, i) are exactly j >= lo(s, i), and lo is found by one binary
//    search over the running sum  Q[j] = PP[j] + N_s PS[j]  kept in LDS.
//  * the stage time time(s; j, i) never decreases when j moves down.  Scanning j downwards from
//    i-1, once time(s; j, i) exceeds the best value found so far no lower j can match or beat it,
//    and the scan stops.  The stop uses a strict comparison and the update a non-strict one, so
//    the lowest j among equal values is kept, as the recurrence demands.  Nothing is assumed
//    about the previous DP row (it is not monotone when transfer times dominate); in the worst
//    case the scan degenerates to the dense one.
//
// With tp a power of two and every time below 2^31 us (both checked by the table build), the
// stage time is one subtraction and one shift on the fused 32-bit row
//   P[j] = PF[type][j] + tp * PR[g][tp][j]:   time(s; j, i) = (P[i] + tp - 1 - P[j]) >> log2 tp,
// because ceil(a / tp) + b = ceil((a + tp b) / tp) for integers.  Transfer times come from the
// per-link cut table built beside the rows.
//
// Mapping: one workgroup per candidate at a time (persistent workgroups stride over the batch),
// one lane per DP cell of the current stage, lanes of a wave on consecutive cells so that LDS
// reads of (D[j], P[j]) pairs are stride-1 or broadcast.  The previous DP row and the slot's P row
// sit interleaved in LDS so that one 8-byte read feeds a transition.  The single cell of the last
// stage is reduced across a wavefront with a lexicographic (value, j) minimum.  Back-pointers go
// to a per-workgroup slice of the caller's workspace as uint16.
#include "harp_internal.h"
#include "plan_common.h"

namespace harp {

namespace {

constexpr uint32_t kInf32 = 0xFFFFFFFFu;
constexpr int kMaxThreads = 1024;

struct alignas(8) Pair {
    uint32_t d;   // previous DP row
    uint32_t p;   // fused time row of the stage's slot
};

__device__ __forceinline__ uint32_t umax3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t m = a > b ? a : b;
    return m > c ? m : c;
}

__global__ __launch_bounds__(kMaxThreads) void k2_fast(TablesDev tb, CandDev cd, PlansDev out,
                                                        unsigned char *ws, size_t ws_per_group,
                                                        int row_len) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ SlotInfo slots;
    __shared__ int fmax_s[2];

    const int L = tb.L, S_max = cd.S_max;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x;
    int64_t *Q = reinterpret_cast<int64_t *>(lds_raw);                    // [row_len]
    Pair *rows = reinterpret_cast<Pair *>(lds_raw + size_t(row_len) * 8); // [2][row_len]
    uint16_t *arg = reinterpret_cast<uint16_t *>(ws + size_t(blockIdx.x) * ws_per_group);
    const int64_t *PP = tb.PP(), *PS = tb.PS();

    for (int c = blockIdx.x; c < cd.C; c += gridDim.x) {
        __syncthreads();   // the previous candidate's tail has finished with LDS
        const int S = cd.cand_S[c];
        int status = load_and_check_slots(tb, S, S_max, cd.cand_group + int64_t(c) * S_max,
                                          cd.cand_tp + int64_t(c) * S_max, slots);
        if (status == HARP_CAND_OK && S > L) status = HARP_CAND_INFEASIBLE;
        if (status != HARP_CAND_OK) {
            write_failed(out, c, S_max, status);
            continue;
        }
        if (tid == 0) { rows[0].d = 0; fmax_s[0] = 0; }
        // fused time row of slot 0 into buffer 0
        {
            const uint32_t *p32 = tb.P32 + (int64_t(slots.g[0]) * tb.n_tp + slots.k[0]) * tb.pitch32;
            for (int j = tid; j <= L; j += nthreads) rows[j].p = p32[j];
        }
        __syncthreads();

        int cur = 0;
        bool dead = false;
        for (int s = 0; s < S; ++s) {
            const int g = slots.g[s], k = slots.k[s];
            const uint32_t tp = (uint32_t)tb.tp[k];
            const int shift = tb.tp_shift[k];
            const int t = tb.group_type[g];
            const int64_t n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
            const int64_t cap = int64_t(tp) * tb.type_mem[t];
            const bool last = (s == S - 1);
            const int i_lo = last ? L : s + 1, i_hi = L - (S - 1 - s);
            Pair *prev = rows + size_t(cur) * row_len;
            Pair *next = rows + size_t(cur ^ 1) * row_len;
            const int fmax_prev = fmax_s[cur];
            // memory row of this stage, and the next slot's time row into the other buffer
            for (int j = s + tid; j <= i_hi; j += nthreads) Q[j] = PP[j] + n_inflight * PS[j];
            if (!last) {
                const uint32_t *p32 = tb.P32 + (int64_t(slots.g[s + 1]) * tb.n_tp + slots.k[s + 1]) * tb.pitch32;
                for (int j = s + 1 + tid; j <= L; j += nthreads) next[j].p = p32[j];
            }
            if (tid == 0) fmax_s[cur ^ 1] = -1;
            __syncthreads();

            uint16_t *arg_row = arg + size_t(s) * row_len;
            if (!last) {
                const uint32_t *cm = tb.CM + (int64_t(g) * tb.G + slots.g[s + 1]) * tb.pitch32;
                for (int i0 = i_lo; i0 <= i_hi; i0 += nthreads) {
                    const int i = i0 + tid;
                    const bool live = i <= i_hi;
                    uint32_t best = kInf32;
                    int best_j = 0;
                    if (live) {
                        // fitting cuts: j >= lo, lo = first j in [s, i] with Q[j] >= Q[i] - cap
                        const int64_t th = Q[i] - cap;
                        int lo = s;
                        if (Q[s] < th) {
                            int a = s, b = i;           // Q[a] < th <= Q[b]
                            while (b - a > 1) {
                                const int m = (a + b) >> 1;
                                if (Q[m] < th) a = m; else b = m;
                            }
                            lo = b;
                        }
                        const int hi = (i - 1) < fmax_prev ? (i - 1) : fmax_prev;
                        const uint32_t cut = cm[i];
                        const uint32_t xi = prev[i].p + tp - 1;
                        for (int j = hi; j >= lo; --j) {
                            const Pair e = prev[j];
                            const uint32_t tj = (xi - e.p) >> shift;
                            const uint32_t v = umax3(e.d, tj, cut);
                            if (v <= best) { best = v; best_j = j; }
                            if (tj > best) break;
                        }
                        next[i].d = best;
                        arg_row[i] = (uint16_t)best_j;
                    }
                    const unsigned long long finite = __ballot(live && best != kInf32);
                    if (lane == 0 && finite) atomicMax(&fmax_s[cur ^ 1], i0 + wave * 64 + 63 - __clzll(finite));
                }
            } else if (wave == 0) {
                // the last stage has the single cell i = L: lanes over j, lexicographic reduction
                const int i = L;
                const int64_t th = Q[i] - cap;
                const uint32_t xi = prev[i].p + tp - 1;
                const int hi = (i - 1) < fmax_prev ? (i - 1) : fmax_prev;
                uint32_t best = kInf32;
                int best_j = INT32_MAX;
                for (int j = s + lane; j <= hi; j += 64) {
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
                if (lane == 0) {
                    next[i].d = best;
                    arg_row[i] = (uint16_t)(best == kInf32 ? 0 : best_j);
                    fmax_s[cur ^ 1] = best == kInf32 ? -1 : i;
                }
            }
            __syncthreads();
            cur ^= 1;
            if (fmax_s[cur] < 0) { dead = true; break; }   // uniform: no cell of this row is reachable
        }
        if (dead) {
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            continue;
        }
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        if (tid == 0) {
            int b = L;
            sp[S] = L;
            for (int s = S - 1; s >= 0; --s) { b = arg[size_t(s) * row_len + b]; sp[s] = b; }
        }
        for (int s = S + 1 + tid; s <= S_max; s += nthreads) sp[s] = -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = tid; s < S_max; s += nthreads) df[s] = s < S ? slots.dev_first[s] : -1;
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
        if (wave == 0) {
            int64_t bott, iter;
            const int st = wave_score_partition(tb, S, slots, sp, lane, bott, iter);
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = iter;
                out.status[c] = st;
            }
        }
    }
}

int fast_threads(int L) {
    int t = (L + 63) / 64 * 64;
    return t > kMaxThreads ? kMaxThreads : t;
}

int fast_row_len(int L) { return (L + 1 + 7) / 8 * 8; }

size_t fast_lds_bytes(int L) { return size_t(fast_row_len(L)) * (8 + 2 * sizeof(Pair)); }

}  // namespace

size_t plan_fast_ws_per_group(int L, int S_max) {
    size_t b = size_t(S_max) * fast_row_len(L) * sizeof(uint16_t);
    return (b + 255) & ~size_t(255);
}

// Workgroups that can be resident at once: bounded by threads (2048 per CU) and LDS (160 KiB).
int plan_fast_groups(int L, int n_cu) {
    const int by_threads = 2048 / fast_threads(L);
    const size_t lds = fast_lds_bytes(L) + sizeof(SlotInfo) + 64;
    int by_lds = int((size_t(160) << 10) / lds);
    int per_cu = by_threads < by_lds ? by_threads : by_lds;
    if (per_cu > 16) per_cu = 16;
    if (per_cu < 1) per_cu = 1;
    return per_cu * n_cu;
}

void launch_plan_fast(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                      int n_groups, hipStream_t st) {
    hipLaunchKernelGGL(k2_fast, dim3(n_groups), dim3(fast_threads(tb.L)), fast_lds_bytes(tb.L), st, tb,
                       cd, out, static_cast<unsigned char *>(ws), plan_fast_ws_per_group(tb.L, cd.S_max),
                       fast_row_len(tb.L));
}

}  // namespace harp
