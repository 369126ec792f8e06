// Generic planner-search kernel for gfx950: the dense min-max recurrence in int64.
//
// Paper section 5.2.3 (eq. dp_general with the submesh of every stage fixed by the candidate,
// constraints (i)-(iii)) evaluated exactly as stated: for every stage s and every end cut i, all
// previous cuts j are tried.  One workgroup works on one candidate at a time; one wavefront owns
// one DP cell and its 64 lanes stride over j, then reduce (value, j) lexicographically across the
// wave, which keeps the lowest j among equal values.  Rows of D and the back-pointers live in a
// per-workgroup slice of the caller's workspace (L2-resident at the sizes of interest).  This path
// accepts any degree (division when it is not a power of two) and any L up to 65535; the 32-bit
// path in k2_fast.hip is the fast one.
#include "harp_internal.h"
#include "plan_common.h"

namespace harp {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__global__ __launch_bounds__(kThreads) void k2_generic(TablesDev tb, CandDev cd, PlansDev out,
                                                        unsigned char *ws, size_t ws_per_group) {
    __shared__ SlotInfo slots;
    const int L = tb.L, S_max = cd.S_max;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char *mine = ws + size_t(blockIdx.x) * ws_per_group;
    int64_t *D0 = reinterpret_cast<int64_t *>(mine);
    int64_t *D1 = D0 + (L + 1);
    uint16_t *arg = reinterpret_cast<uint16_t *>(D1 + (L + 1));   // [S_max][L+1], row s = stage s
    const int64_t *PP = tb.PP(), *PS = tb.PS();

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
        for (int i = threadIdx.x; i <= L; i += kThreads) D0[i] = (i == 0) ? 0 : kInf;
        __syncthreads();
        int64_t *Dp = D0, *Dn = D1;
        for (int s = 0; s < S; ++s) {
            const int g = slots.g[s], k = slots.k[s];
            const int64_t tp = tb.tp[k];
            const int shift = tb.tp_shift[k];
            const int t = tb.group_type[g];
            const int64_t *pf = tb.PF(t), *pr = tb.PR(g, k);
            const int64_t n_inflight = (S - s) < tb.M ? (S - s) : tb.M;
            const int64_t cap = tp * tb.type_mem[t];
            const bool last = (s == S - 1);
            const int64_t link = last ? 1 : tb.bw[int64_t(g) * tb.G + slots.g[s + 1]];
            const int i_lo = last ? L : s + 1, i_hi = L - (S - 1 - s);
            uint16_t *arg_row = arg + size_t(s) * (L + 1);
            for (int i = i_lo + wave; i <= i_hi; i += kWaves) {
                const int64_t cut = last ? 0 : (tb.act_bytes[i - 1] + link - 1) / link;
                const int64_t pfi = pf[i], pri = pr[i], ppi = PP[i], psi = PS[i];
                int64_t best = kInf;
                int best_j = INT32_MAX;
                for (int j = s + lane; j < i; j += 64) {
                    const int64_t dj = Dp[j];
                    if (dj == kInf) continue;
                    const int64_t need = (ppi - PP[j]) + n_inflight * (psi - PS[j]);
                    if (need > cap) continue;
                    const int64_t work = pfi - pf[j];
                    const int64_t comp = shift >= 0 ? (work + tp - 1) >> shift : (work + tp - 1) / tp;
                    int64_t val = comp + (pri - pr[j]);
                    val = val > dj ? val : dj;
                    val = val > cut ? val : cut;
                    if (val < best) { best = val; best_j = j; }
                }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const int64_t ov = __shfl_xor(best, d, 64);
                    const int oj = __shfl_xor(best_j, d, 64);
                    if (ov < best || (ov == best && oj < best_j)) { best = ov; best_j = oj; }
                }
                if (lane == 0) {
                    Dn[i] = best;
                    arg_row[i] = (uint16_t)(best == kInf ? 0 : best_j);
                }
            }
            __syncthreads();
            int64_t *tmp = Dp; Dp = Dn; Dn = tmp;
        }
        if (Dp[L] == kInf) {          // uniform: every thread reads the same cell
            write_failed(out, c, S_max, HARP_CAND_INFEASIBLE);
            continue;
        }
        int32_t *sp = out.splits + int64_t(c) * (S_max + 1);
        if (threadIdx.x == 0) {
            int b = L;
            sp[S] = L;
            for (int s = S - 1; s >= 0; --s) { b = arg[size_t(s) * (L + 1) + b]; sp[s] = b; }
        }
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

}  // namespace

size_t plan_generic_ws_per_group(int L, int S_max) {
    size_t b = size_t(2) * (L + 1) * sizeof(int64_t) + size_t(S_max) * (L + 1) * sizeof(uint16_t);
    return (b + 255) & ~size_t(255);
}

void launch_plan_generic(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                         int n_groups, hipStream_t st) {
    hipLaunchKernelGGL(k2_generic, dim3(n_groups), dim3(kThreads), 0, st, tb, cd, out,
                       static_cast<unsigned char *>(ws), plan_generic_ws_per_group(tb.L, cd.S_max));
}

}  // namespace harp
