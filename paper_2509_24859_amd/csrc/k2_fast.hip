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
// one lane per DP cell of the current stage (thread t owns cell i = s + 1 + t, so the problem must
// have L <= 1024), lanes of a wave on consecutive cells so that LDS reads of (D[j], P[j]) pairs
// are stride-1 or broadcast.  The previous DP row and the slot's P row sit interleaved in LDS so
// that one 8-byte read feeds a transition.  Everything stage s+1 needs from global memory (its
// slot's P row, the memory row, the cell's own cut time) is requested at the top of stage s, lands
// in registers while stage s scans, and is committed to the other LDS buffer before the single
// LDS-only barrier that ends the stage.  Values that are the same for the whole workgroup (slot
// constants, the reach of the previous row) are moved to scalar registers so that addressing runs
// on the scalar unit.  The lone cell of the last stage is reduced across a wavefront with a
// lexicographic (value, j) minimum.  Back-pointers go to a per-workgroup slice of the caller's
// workspace as uint16.
#include "harp_internal.h"
#include "plan_common.h"

namespace harp {

namespace {

constexpr uint32_t kInf32 = 0xFFFFFFFFu;
constexpr int kMaxThreads = 1024;
constexpr int kPad = 4;

struct alignas(8) Pair {
    uint32_t d;   // previous DP row
    uint32_t p;   // fused time row of the stage's slot
};

// Workgroup barrier that orders LDS traffic only.  Global loads and stores stay in flight across
// it (the stage loop never communicates through global memory), which keeps the round trips of the
// back-pointer stores and of the next stage's table rows off the per-stage critical path.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t umax3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t m = a > b ? a : b;
    return m > c ? m : c;
}

// A value every lane of the wave holds, moved to a scalar register.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ const T *uniform_ptr(const T *p);
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <typename T>
__device__ __forceinline__ const T *uniform_ptr(const T *p) {
    return reinterpret_cast<const T *>(uniform64(reinterpret_cast<int64_t>(p)));
}

// Per-slot constants of the candidate in flight, computed once per candidate so that the stage
// loop starts from LDS and never waits on a chain of dependent global loads.
struct alignas(16) StageConst {
    int64_t cap;            // tp * device memory of the slot's GPU type
    const uint32_t *p32;    // the slot's fused time row
    const uint32_t *cm;     // cut-time row of the link to the next slot
    int32_t shift;          // log2 tp
    int32_t pad;
};

__global__ __launch_bounds__(kMaxThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k2_fast(TablesDev tb, CandDev cd, PlansDev out, unsigned char *ws, size_t ws_per_group, int row_len) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ SlotInfo slots;
    __shared__ StageConst sc[kMaxStages];
    __shared__ int fmax_s[3];

    const int L = tb.L, S_max = cd.S_max;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x;
    // every LDS row has kPad spare entries in front, so that the group of four previous cuts
    // ending at any j >= 0 can be read at fixed offsets without clamping
    int64_t *Qb = reinterpret_cast<int64_t *>(lds_raw) + kPad;                        // [2][row_len]
    Pair *rows = reinterpret_cast<Pair *>(lds_raw + size_t(row_len) * 16) + kPad;     // [2][row_len]
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
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        bool dead = false;
        if (S >= 2) {
            const int R = L - S + 1;          // cells per stage; stage s touches rows s .. s+R
            for (int s = tid; s < S; s += nthreads) {
                const int g = slots.g[s], k = slots.k[s];
                sc[s].cap = int64_t(tb.tp[k]) * tb.type_mem[tb.group_type[g]];
                sc[s].p32 = tb.P32 + (int64_t(g) * tb.n_tp + k) * tb.pitch32;
                sc[s].cm = tb.CM + (int64_t(g) * tb.G + (s + 1 < S ? slots.g[s + 1] : g)) * tb.pitch32;
                sc[s].shift = tb.tp_shift[k];
            }
            __syncthreads();
            const bool live = tid < R;        // this thread owns a cell in every stage but the last
            const bool stages = tid <= R;     // this thread stages one entry of every row
            const int64_t m_cap = tb.M;

            // prologue: rows of stage 0 and the thread's own cut time of stage 0
            uint32_t cut_i = 0;
            {
                const uint32_t *p32 = uniform_ptr(sc[0].p32);
                const uint32_t *cm = uniform_ptr(sc[0].cm);
                const int64_t n0 = S < m_cap ? S : m_cap;
                if (stages) {
                    rows[tid].p = p32[tid];
                    Qb[tid] = PP[tid] + n0 * PS[tid];
                }
                if (live) cut_i = cm[tid + 1];
                if (tid < 3) rows[-1 - tid].d = kInf32;   // below cut 0: never a predecessor
                if (tid == 0) { rows[0].d = 0; fmax_s[0] = 0; fmax_s[1] = -1; }
            }
            lds_barrier();

            int cur = 0;
            int fmax_prev = 0;                // reach of the previous row, carried in a register
            int f_next = 1, f_reset = 2;      // rotating slots of fmax_s: target now, target next
            for (int s = 0; s < S - 1; ++s) {
                const int shift = uniform(sc[s].shift);
                const uint32_t tp = 1u << shift;
                const int64_t cap = uniform64(sc[s].cap);
                int *fmax_next = &fmax_s[f_next];
                const Pair *prev = rows + cur * row_len;
                Pair *next = rows + (cur ^ 1) * row_len;
                const int64_t *Q = Qb + cur * row_len;
                int64_t *Qn = Qb + (cur ^ 1) * row_len;
                if (tid == 0) fmax_s[f_reset] = -1;

                // requests for stage s+1: entry jn of its rows, and this thread's own cut time
                const int jn = s + 1 + tid;
                const bool next_has_cut = s + 2 < S;
                uint32_t p_n = 0, cut_n = 0;
                int64_t pp_n = 0, ps_n = 0;
                {
                    const uint32_t *p32 = uniform_ptr(sc[s + 1].p32);
                    const uint32_t *cm = uniform_ptr(sc[s + 1].cm);
                    if (stages) { p_n = p32[jn]; pp_n = PP[jn]; ps_n = PS[jn]; }
                    if (live && next_has_cut) cut_n = cm[jn + 1];
                }

                const int i = s + 1 + tid;
                uint32_t best = kInf32;
                int best_j = 0;
                if (live) {
                    // fitting cuts are j >= lo with Q[lo] >= Q[i] - cap (memory need is monotone
                    // in j), so the downward scan also stops at the first misfit
                    const int64_t th = Q[i] - cap;
                    const uint32_t xi = prev[i].p + tp - 1;
                    // Four previous cuts per trip, read at fixed offsets below j.  An entry counts
                    // while it fits in memory (monotone in j, so a plain predicate); entries below
                    // cut s hold D = infinity and never win.  Entries below a stop cannot update
                    // (their time exceeds the best value), so only the last entry of a trip
                    // decides whether the lane goes on.
                    int j = (i - 1) < fmax_prev ? (i - 1) : fmax_prev;
                    bool more = true;
                    while (more) {
                        const Pair *pe = prev + (j - 3);
                        const int64_t *pq = Q + (j - 3);
                        const Pair e3 = pe[0], e2 = pe[1], e1 = pe[2], e0 = pe[3];
                        const int64_t q3 = pq[0], q2 = pq[1], q1 = pq[2], q0 = pq[3];
                        uint32_t tj;
#define HARP_STEP(E, QV, JJ)                                                   \
    {                                                                          \
        tj = (xi - (E).p) >> shift;                                            \
        const uint32_t v = umax3((E).d, tj, cut_i);                            \
        const bool upd = ((QV) >= th) & (v <= best);                           \
        best = upd ? v : best;                                                 \
        best_j = upd ? (JJ) : best_j;                                          \
    }
                        HARP_STEP(e0, q0, j)
                        HARP_STEP(e1, q1, j - 1)
                        HARP_STEP(e2, q2, j - 2)
                        HARP_STEP(e3, q3, j - 3)
#undef HARP_STEP
                        more = ((j - 3) > s) & (q3 >= th) & (tj <= best);
                        j -= 4;
                    }
                    next[i].d = best;
                }
                if (tid < 3) next[s - tid].d = kInf32;     // cuts below s+1 for the next stage
                const unsigned long long finite = __ballot(best != kInf32);
                if (lane == 0 && finite) atomicMax(fmax_next, s + 1 + wave * 64 + 63 - __clzll(finite));

                // commit the staged entries of stage s+1, then let the back-pointer go
                if (stages) {
                    const int64_t n1 = (S - s - 1) < m_cap ? (S - s - 1) : m_cap;
                    next[jn].p = p_n;
                    Qn[jn] = pp_n + n1 * ps_n;
                }
                cut_i = cut_n;
                if (live) arg[s * row_len + i] = (uint16_t)best_j;
                lds_barrier();
                cur ^= 1;
                fmax_prev = uniform(*fmax_next);
                { const int t = 3 - f_next - f_reset; f_next = f_reset; f_reset = t; }
                if (fmax_prev < 0) { dead = true; break; }   // no cell of this row is reachable
            }
            if (!dead) {
                // the last stage has the single cell i = L: lanes over j, lexicographic reduction
                const int s = S - 1;
                if (wave == 0) {
                    const int shift = uniform(sc[s].shift);
                    const uint32_t tp = 1u << shift;
                    const int64_t cap = uniform64(sc[s].cap);
                    const Pair *prev = rows + cur * row_len;
                    const int64_t *Q = Qb + cur * row_len;
                    const int64_t th = Q[L] - cap;
                    const uint32_t xi = prev[L].p + tp - 1;
                    const int hi = (L - 1) < fmax_prev ? (L - 1) : fmax_prev;
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
                        arg[s * row_len + L] = (uint16_t)(best == kInf32 ? 0 : best_j);
                        fmax_s[f_next] = best == kInf32 ? -1 : L;
                    }
                }
                __syncthreads();          // back-pointers of every wave are visible to thread 0
                if (fmax_s[f_next] < 0) dead = true;
            }
            if (!dead && tid == 0) {
                int b = L;
                sp[S] = L;
                for (int s = S - 1; s >= 0; --s) { b = arg[s * row_len + b]; sp[s] = b; }
            }
        } else if (tid == 0) {
            sp[0] = 0;    // one stage holds every operator; the score below checks that it fits
            sp[1] = L;
        }
        if (dead) {
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            continue;
        }
        for (int s = S + 1 + tid; s <= S_max; s += nthreads) sp[s] = -1;
        int32_t *df = out.dev_first + int64_t(c) * S_max;
        for (int s = tid; s < S_max; s += nthreads) df[s] = s < S ? slots.dev_first[s] : -1;
        __syncthreads();              // the cuts written by thread 0 are read by the first wave
        int st = HARP_CAND_OK;
        if (wave == 0) {
            int64_t bott, iter;
            st = wave_score_partition(tb, S, slots, sp, lane, bott, iter);
            if (lane == 0) {
                out.bottleneck[c] = bott;
                out.iter_time[c] = iter;
                out.status[c] = st;
            }
        }
        if (S == 1) {                 // a single stage that does not fit: no plan to report
            if (__syncthreads_or(wave == 0 && st != HARP_CAND_OK)) {
                for (int s = tid; s <= S_max; s += nthreads) sp[s] = -1;
                for (int s = tid; s < S_max; s += nthreads) df[s] = -1;
            }
        }
    }
}

int fast_threads(int L) {
    int t = (L + 63) / 64 * 64;
    return t > kMaxThreads ? kMaxThreads : t;
}

int fast_row_len(int L) { return (L + 1 + kPad + 7) / 8 * 8; }

size_t fast_lds_bytes(int L) { return size_t(fast_row_len(L)) * (16 + 2 * sizeof(Pair)); }

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
    hipLaunchKernelGGL(k2_fast, dim3(n_groups), dim3(fast_threads(tb.L)), fast_lds_bytes(tb.L), st, tb, cd,
                       out, static_cast<unsigned char *>(ws), plan_fast_ws_per_group(tb.L, cd.S_max),
                       fast_row_len(tb.L));
}

}  // namespace harp
