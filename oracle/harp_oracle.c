/*
 * CPU oracle for the inter-operator planner search of HARP (paper section 5.2).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded C written from the paper's statement of
 * the planning problem.  It shares no code with the HIP library and must never be reachable from
 * the product path: only the tests, the smoke check and the benchmark's cpu_baseline leg call it.
 *
 * What is computed, for every candidate (an ordered list of S slots, slot s = tp_s devices of
 * device group g_s):
 *
 *   - the stage partition 0 = b_0 < b_1 < ... < b_S = L of the operator sequence that minimises
 *     the largest per-stage cost  max_s max(time_s, comm_s)  subject to the per-device memory
 *     limit.  This is the smallest feasible bottleneck t_max of section 5.2.4 (2) for the DP of
 *     section 5.2.3 (eq. dp_general) with the submesh of each stage fixed by the candidate, and
 *     with constraints (i) stage time <= t_max, (ii) C(j) <= t_max and (iii) eq. mem_cons.
 *   - the iteration time of that plan under the cost model of section 5.2.2
 *     (eq. gpipe_cost_model):  sum_s (t_s + 2 c_s) + (B - 1) t_max,  B = number of microbatches.
 *
 * Readings where the paper leaves the model open (all integer, microseconds and bytes):
 *   t_s   = ceil(sum of (fwd+bwd) over the stage's operators on the group's GPU type / tp)
 *           + sum over the stage's operators of the tensor-parallel all-reduce time
 *             ceil(ar_count * 2 (tp-1) * act_bytes[l] / (tp * bw[g][g]))      (0 when tp == 1)
 *   c_s   = ceil(act_bytes[b_{s+1}-1] / bw[g_s][g_{s+1}])   for s < S-1, 0 for the last stage
 *   mem   : sum(param_bytes) + N_s * sum(stash_bytes) <= tp * type_mem_bytes, with the classic
 *           1F1B in-flight count N_s = min(S - s, B)  (section 2.1: stage i of S keeps S-i+1)
 *   ties  : the recurrence scans the previous cut j in increasing order and keeps the first j that
 *           attains the minimum, so the lowest j wins.
 *
 * Every loop below is the definition written out: no blocking, no pruning, no reordering.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_INF INT64_MAX

enum { ORACLE_OK = 0, ORACLE_BAD_ARG = -1, ORACLE_OVERFLOW = -5 };
enum { CAND_OK = 0, CAND_INFEASIBLE = 1, CAND_INVALID = 2 };

typedef struct {
    int32_t L, T, G, M, ar_count, n_tp;
    const int32_t *tp_degrees;      /* [n_tp] ascending, first is 1 */
    const int64_t *fwd_us, *bwd_us; /* [T][L] */
    const int64_t *param_bytes, *stash_bytes, *act_bytes; /* [L] */
    const int32_t *group_type, *group_ndev;               /* [G] */
    const int64_t *type_mem_bytes;                        /* [T] */
    const int64_t *bw;                                    /* [G][G] bytes per microsecond */
} oracle_problem;

typedef __int128 wide;

static const wide LIMIT63 = (((wide)1) << 63) - 1;
static const wide LIMIT47 = (((wide)1) << 47);

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

/* Tables of running sums, index i = 0..L, entry 0 is 0.
 *   PF[t][i]      sum_{l<i} fwd_us[t][l] + bwd_us[t][l]
 *   PP[i], PS[i]  sum_{l<i} param_bytes[l], stash_bytes[l]
 *   PR[g][k][i]   sum_{l<i} all-reduce time of operator l at degree tp_degrees[k] inside group g
 * Returns ORACLE_OVERFLOW when the inputs leave the range in which every later quantity is known
 * to fit in int64 (magnitude preconditions of the library), ORACLE_BAD_ARG for malformed input. */
int oracle_build_tables(const oracle_problem *p, int64_t *PF, int64_t *PP, int64_t *PS, int64_t *PR)
{
    const int L = p->L, T = p->T, G = p->G, K = p->n_tp;
    /* the tables themselves have no length limit beyond int32 comfort; planning is limited to
     * 65535 operators (see oracle_plan_batch) */
    if (L < 1 || L > (1 << 24) || T < 1 || G < 1 || p->M < 1 || K < 1 || K > 8 || p->ar_count < 0)
        return ORACLE_BAD_ARG;
    if (p->tp_degrees[0] != 1) return ORACLE_BAD_ARG;
    for (int k = 1; k < K; ++k)
        if (p->tp_degrees[k] <= p->tp_degrees[k - 1]) return ORACLE_BAD_ARG;
    for (int g = 0; g < G; ++g) {
        if (p->group_type[g] < 0 || p->group_type[g] >= T || p->group_ndev[g] < 1) return ORACLE_BAD_ARG;
        for (int h = 0; h < G; ++h)
            if (p->bw[g * G + h] < 1) return ORACLE_BAD_ARG;
    }
    for (int t = 0; t < T; ++t) {
        if (p->type_mem_bytes[t] < 0) return ORACLE_BAD_ARG;
        for (int l = 0; l < L; ++l)
            if (p->fwd_us[t * L + l] < 0 || p->bwd_us[t * L + l] < 0) return ORACLE_BAD_ARG;
    }
    for (int l = 0; l < L; ++l)
        if (p->param_bytes[l] < 0 || p->stash_bytes[l] < 0 || p->act_bytes[l] < 0) return ORACLE_BAD_ARG;

    const int64_t tp_max = p->tp_degrees[K - 1];
    wide worst = 0; /* largest stage time or transfer time any plan can see */

    for (int t = 0; t < T; ++t) {
        wide acc = 0;
        PF[t * (L + 1)] = 0;
        for (int l = 0; l < L; ++l) {
            acc += (wide)p->fwd_us[t * L + l] + (wide)p->bwd_us[t * L + l];
            if (acc > LIMIT63) return ORACLE_OVERFLOW;
            PF[t * (L + 1) + l + 1] = (int64_t)acc;
        }
    }
    {
        wide ap = 0, as = 0;
        PP[0] = 0; PS[0] = 0;
        for (int l = 0; l < L; ++l) {
            ap += p->param_bytes[l];
            as += p->stash_bytes[l];
            if (ap > LIMIT63 || as > LIMIT63) return ORACLE_OVERFLOW;
            PP[l + 1] = (int64_t)ap;
            PS[l + 1] = (int64_t)as;
        }
        /* memory need of any segment with any in-flight count, and the limit it is compared to */
        int64_t n_max = p->M < L ? p->M : L;
        if (ap + (wide)n_max * as > LIMIT63) return ORACLE_OVERFLOW;
        for (int t = 0; t < T; ++t)
            if ((wide)tp_max * p->type_mem_bytes[t] > LIMIT63) return ORACLE_OVERFLOW;
    }
    for (int g = 0; g < G; ++g) {
        const int64_t b = p->bw[g * G + g];
        for (int k = 0; k < K; ++k) {
            const int64_t tp = p->tp_degrees[k];
            int64_t *row = PR + ((size_t)(g * K + k)) * (L + 1);
            wide acc = 0;
            row[0] = 0;
            for (int l = 0; l < L; ++l) {
                if (tp > 1) {
                    wide num = (wide)p->ar_count * 2 * (tp - 1) * p->act_bytes[l];
                    wide den = (wide)tp * b;
                    if (num > LIMIT63 || den > LIMIT63) return ORACLE_OVERFLOW;
                    acc += (num + den - 1) / den;
                }
                if (acc > LIMIT63) return ORACLE_OVERFLOW;
                row[l + 1] = (int64_t)acc;
            }
            wide whole = (wide)PF[p->group_type[g] * (L + 1) + L] + acc;
            if (whole > worst) worst = whole;
        }
    }
    for (int l = 0; l < L; ++l)
        for (int gh = 0; gh < G * G; ++gh) {
            wide c = ((wide)p->act_bytes[l] + p->bw[gh] - 1) / p->bw[gh];
            if (c > worst) worst = c;
        }
    if (worst >= LIMIT47) return ORACLE_OVERFLOW;
    /* iteration time: at most L stage times, 2 (L-1) transfers and (M-1) bottlenecks */
    if (worst * ((wide)3 * L + p->M) > LIMIT63) return ORACLE_OVERFLOW;
    return ORACLE_OK;
}

typedef struct {
    const oracle_problem *p;
    const int64_t *PF, *PP, *PS, *PR;
} tables_view;

static int tp_index(const oracle_problem *p, int tp)
{
    for (int k = 0; k < p->n_tp; ++k)
        if (p->tp_degrees[k] == tp) return k;
    return -1;
}

/* Candidate well-formedness: stage count in range, groups in range, degrees allowed, slots of a
 * group adjacent, no group over-subscribed. */
static int candidate_valid(const oracle_problem *p, int S, int S_max, const int32_t *grp, const int32_t *tp)
{
    if (S < 1 || S > S_max) return 0;
    int ok = 1;
    int64_t *used = (int64_t *)calloc((size_t)p->G, sizeof(int64_t));
    char *closed = (char *)calloc((size_t)p->G, 1);
    for (int s = 0; s < S && ok; ++s) {
        int g = grp[s];
        if (g < 0 || g >= p->G || tp[s] < 1 || tp_index(p, tp[s]) < 0) { ok = 0; break; }
        if (closed[g]) { ok = 0; break; }
        used[g] += tp[s];
        if (used[g] > p->group_ndev[g]) { ok = 0; break; }
        if (s + 1 < S && grp[s + 1] != g) closed[g] = 1;
    }
    free(used);
    free(closed);
    return ok;
}

/* Stage time t_s of operators [j, i) on slot (g, tp). */
static int64_t stage_time(const tables_view *v, int g, int tp, int j, int i)
{
    const oracle_problem *p = v->p;
    const int L = p->L;
    const int64_t *pf = v->PF + (size_t)p->group_type[g] * (L + 1);
    const int64_t *pr = v->PR + ((size_t)(g * p->n_tp + tp_index(p, tp))) * (L + 1);
    return ceil_div(pf[i] - pf[j], tp) + (pr[i] - pr[j]);
}

/* Transfer time c_s of the cut placed before operator i, from group g to group h. */
static int64_t cut_time(const oracle_problem *p, int g, int h, int i)
{
    return ceil_div(p->act_bytes[i - 1], p->bw[g * p->G + h]);
}

/* eq. mem_cons with parameters and activations sharded evenly over the tp devices of the slot:
 * (params + n * stash) / tp <= device memory, compared without dividing. */
static int memory_fits(const tables_view *v, int g, int tp, int64_t n_inflight, int j, int i)
{
    const oracle_problem *p = v->p;
    int64_t need = (v->PP[i] - v->PP[j]) + n_inflight * (v->PS[i] - v->PS[j]);
    return need <= (int64_t)tp * p->type_mem_bytes[p->group_type[g]];
}

static void fill_failed(int S_max, int32_t *splits, int32_t *dev_first, int64_t *bott, int64_t *iter)
{
    for (int s = 0; s <= S_max; ++s) splits[s] = -1;
    for (int s = 0; s < S_max; ++s) dev_first[s] = -1;
    *bott = ORACLE_INF;
    *iter = ORACLE_INF;
}

/* First global device id of every slot: groups are numbered consecutively in group-id order and a
 * group's slots take its devices in slot order. */
static void slot_devices(const oracle_problem *p, int S, int S_max, const int32_t *grp, const int32_t *tp,
                         int32_t *dev_first)
{
    for (int s = 0; s < S_max; ++s) dev_first[s] = -1;
    for (int s = 0; s < S; ++s) {
        int32_t base = 0;
        for (int g = 0; g < grp[s]; ++g) base += p->group_ndev[g];
        for (int q = 0; q < s; ++q)
            if (grp[q] == grp[s]) base += tp[q];
        dev_first[s] = base;
    }
}

/* Cost model of section 5.2.2 for a given partition.  Returns the candidate status. */
static int score_partition(const tables_view *v, int S, const int32_t *grp, const int32_t *tp,
                           const int32_t *b, int64_t *bott, int64_t *iter)
{
    const oracle_problem *p = v->p;
    if (b[0] != 0 || b[S] != p->L) return CAND_INVALID;
    for (int s = 0; s < S; ++s)
        if (b[s + 1] <= b[s]) return CAND_INVALID;
    int64_t worst = 0, single = 0;
    for (int s = 0; s < S; ++s) {
        int64_t n = (S - s) < p->M ? (S - s) : p->M;
        if (!memory_fits(v, grp[s], tp[s], n, b[s], b[s + 1])) return CAND_INFEASIBLE;
        int64_t t = stage_time(v, grp[s], tp[s], b[s], b[s + 1]);
        int64_t c = (s == S - 1) ? 0 : cut_time(p, grp[s], grp[s + 1], b[s + 1]);
        worst = max64(worst, max64(t, c));
        single += t + 2 * c;
    }
    *bott = worst;
    *iter = single + (int64_t)(p->M - 1) * worst;
    return CAND_OK;
}

/* One candidate: min-max recurrence over stages, back-pointers, backtrack, score. */
static int plan_one(const tables_view *v, int S, int S_max, const int32_t *grp, const int32_t *tp,
                    int64_t *D_prev, int64_t *D_next, int32_t *arg,
                    int32_t *splits, int32_t *dev_first, int64_t *bott, int64_t *iter)
{
    const oracle_problem *p = v->p;
    const int L = p->L;
    fill_failed(S_max, splits, dev_first, bott, iter);
    if (!candidate_valid(p, S, S_max, grp, tp)) return CAND_INVALID;
    if (S > L) return CAND_INFEASIBLE;

    for (int i = 0; i <= L; ++i) D_prev[i] = ORACLE_INF;
    D_prev[0] = 0;
    for (int s = 0; s < S; ++s) {
        const int64_t n = (S - s) < p->M ? (S - s) : p->M;
        int32_t *arg_row = arg + (size_t)(s + 1) * (L + 1);
        for (int i = 0; i <= L; ++i) { D_next[i] = ORACLE_INF; arg_row[i] = -1; }
        /* stage s ends at cut i; the S-1-s later stages each need one operator */
        for (int i = s + 1; i <= L - (S - 1 - s); ++i) {
            if (s == S - 1 && i != L) continue;
            const int64_t c = (s == S - 1) ? 0 : cut_time(p, grp[s], grp[s + 1], i);
            int64_t best = ORACLE_INF;
            int32_t best_j = -1;
            for (int j = s; j < i; ++j) {
                if (D_prev[j] == ORACLE_INF) continue;
                if (!memory_fits(v, grp[s], tp[s], n, j, i)) continue;
                int64_t val = max64(D_prev[j], max64(stage_time(v, grp[s], tp[s], j, i), c));
                if (val < best) { best = val; best_j = j; }
            }
            D_next[i] = best;
            arg_row[i] = best_j;
        }
        int64_t *tmp = D_prev; D_prev = D_next; D_next = tmp;
    }
    if (D_prev[L] == ORACLE_INF) return CAND_INFEASIBLE;

    splits[S] = L;
    for (int s = S - 1; s >= 0; --s)
        splits[s] = arg[(size_t)(s + 1) * (L + 1) + splits[s + 1]];
    slot_devices(p, S, S_max, grp, tp, dev_first);
    int st = score_partition(v, S, grp, tp, splits, bott, iter);
    if (st != CAND_OK || *bott != D_prev[L]) abort(); /* the plan found must score to the DP value */
    return CAND_OK;
}

/* Plans candidates c_begin..c_end-1 of a batch; outputs are indexed by absolute candidate. */
int oracle_plan_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                      const int64_t *PR, int32_t C, int32_t S_max, const int32_t *cand_S,
                      const int32_t *cand_group, const int32_t *cand_tp, int32_t c_begin, int32_t c_end,
                      int32_t *splits, int32_t *dev_first, int64_t *bottleneck, int64_t *iter_time,
                      int32_t *status)
{
    if (C < 0 || S_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end) return ORACLE_BAD_ARG;
    if (p->L > 65535) return ORACLE_BAD_ARG; /* the library plans at most 65535 operators */
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    int64_t *D0 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
    int64_t *D1 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
    int32_t *arg = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S_max + 1) * (size_t)(L + 1));
    if (!D0 || !D1 || !arg) { free(D0); free(D1); free(arg); return ORACLE_BAD_ARG; }
    for (int32_t c = c_begin; c < c_end; ++c) {
        status[c] = plan_one(&v, cand_S[c], S_max, cand_group + (size_t)c * S_max, cand_tp + (size_t)c * S_max,
                             D0, D1, arg, splits + (size_t)c * (S_max + 1), dev_first + (size_t)c * S_max,
                             bottleneck + c, iter_time + c);
    }
    free(D0); free(D1); free(arg);
    return ORACLE_OK;
}

/* Scores caller-chosen partitions (eq. gpipe_cost_model); splits[c] holds b_0..b_S. */
int oracle_score_1f1b(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                      const int64_t *PR, int32_t C, int32_t S_max, const int32_t *cand_S,
                      const int32_t *cand_group, const int32_t *cand_tp, const int32_t *splits,
                      int64_t *bottleneck, int64_t *iter_time, int32_t *status)
{
    if (C < 0 || S_max < 1) return ORACLE_BAD_ARG;
    tables_view v = { p, PF, PP, PS, PR };
    for (int32_t c = 0; c < C; ++c) {
        const int32_t *grp = cand_group + (size_t)c * S_max, *tp = cand_tp + (size_t)c * S_max;
        bottleneck[c] = ORACLE_INF;
        iter_time[c] = ORACLE_INF;
        if (!candidate_valid(p, cand_S[c], S_max, grp, tp)) { status[c] = CAND_INVALID; continue; }
        int64_t b = ORACLE_INF, t = ORACLE_INF;
        status[c] = score_partition(&v, cand_S[c], grp, tp, splits + (size_t)c * (S_max + 1), &b, &t);
        if (status[c] == CAND_OK) { bottleneck[c] = b; iter_time[c] = t; }
    }
    return ORACLE_OK;
}

/* Final selection over the batch: smallest iteration time among feasible candidates, lowest
 * candidate index on ties; index -1 and time INF when none is feasible. */
int oracle_argmin_batch(int32_t C, const int64_t *iter_time, const int32_t *status,
                        int64_t *best_time, int32_t *best_index)
{
    *best_time = ORACLE_INF;
    *best_index = -1;
    for (int32_t c = 0; c < C; ++c)
        if (status[c] == CAND_OK && iter_time[c] < *best_time) { *best_time = iter_time[c]; *best_index = c; }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Exact optimum of the cost model for one candidate: the search of section 5.2.3 / 5.2.4 (2).
 *
 * For a fixed cap t_max the DP of eq. dp_general minimises the first term of eq.
 * gpipe_cost_model, sum_s (t_s + 2 c_s), over partitions whose every stage obeys (i) t_s <= t_max,
 * (ii) c_s <= t_max and (iii) eq. mem_cons; the latency under that cap is
 *   T(t_max) = F(S, L; t_max) + (B - 1) t_max,
 * and the answer is the minimum of T over the candidate caps.  Candidate caps are the distinct
 * stage costs max(t, c) of fitting stages; those below the smallest feasible cap t_S (the min-max
 * bottleneck) admit no plan, and those above t_E = ceil(T(t_S) / B) cannot win (section 5.2.4 (2)),
 * so the sweep runs over the caps in [t_S, t_E] in increasing order.  The first cap that attains
 * the minimum is kept (strict comparison), and inside a DP the lowest previous cut wins ties.
 */

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* capped DP; returns F(S, L) or INF and fills splits with the plan's cuts */
static int64_t capped_min_sum(const tables_view *v, int S, const int32_t *grp, const int32_t *tp,
                              int64_t cap, int64_t *F_prev, int64_t *F_next, int32_t *arg, int32_t *splits)
{
    const oracle_problem *p = v->p;
    const int L = p->L;
    for (int i = 0; i <= L; ++i) F_prev[i] = ORACLE_INF;
    F_prev[0] = 0;
    for (int s = 0; s < S; ++s) {
        const int64_t n = (S - s) < p->M ? (S - s) : p->M;
        int32_t *arg_row = arg + (size_t)(s + 1) * (L + 1);
        for (int i = 0; i <= L; ++i) { F_next[i] = ORACLE_INF; arg_row[i] = -1; }
        for (int i = s + 1; i <= L - (S - 1 - s); ++i) {
            if (s == S - 1 && i != L) continue;
            const int64_t c = (s == S - 1) ? 0 : cut_time(p, grp[s], grp[s + 1], i);
            if (c > cap) continue;                                    /* constraint (ii) */
            int64_t best = ORACLE_INF;
            int32_t best_j = -1;
            for (int j = s; j < i; ++j) {
                if (F_prev[j] == ORACLE_INF) continue;
                if (!memory_fits(v, grp[s], tp[s], n, j, i)) continue; /* constraint (iii) */
                const int64_t t = stage_time(v, grp[s], tp[s], j, i);
                if (t > cap) continue;                                /* constraint (i) */
                const int64_t val = F_prev[j] + t + 2 * c;
                if (val < best) { best = val; best_j = j; }
            }
            F_next[i] = best;
            arg_row[i] = best_j;
        }
        int64_t *tmp = F_prev; F_prev = F_next; F_next = tmp;
    }
    if (F_prev[L] == ORACLE_INF) return ORACLE_INF;
    splits[S] = L;
    for (int s = S - 1; s >= 0; --s)
        splits[s] = arg[(size_t)(s + 1) * (L + 1) + splits[s + 1]];
    return F_prev[L];
}

/* Exact search for candidates c_begin..c_end-1.  Outputs as oracle_plan_batch, with bottleneck =
 * the winning cap (which is the plan's own largest stage cost) and iter_time = the optimum of eq.
 * gpipe_cost_model; n_caps[c] = number of caps swept. */
int oracle_plan_exact_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                            const int64_t *PR, int32_t C, int32_t S_max, const int32_t *cand_S,
                            const int32_t *cand_group, const int32_t *cand_tp, int32_t c_begin, int32_t c_end,
                            int32_t *splits, int32_t *dev_first, int64_t *bottleneck, int64_t *iter_time,
                            int32_t *status, int32_t *n_caps)
{
    if (C < 0 || S_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end) return ORACLE_BAD_ARG;
    if (p->L > 65535) return ORACLE_BAD_ARG;
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    int64_t *D0 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
    int64_t *D1 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
    int32_t *arg = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S_max + 1) * (size_t)(L + 1));
    int32_t *trial = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S_max + 1));
    size_t caps_room = 1024;
    int64_t *caps = (int64_t *)malloc(sizeof(int64_t) * caps_room);
    if (!D0 || !D1 || !arg || !trial || !caps) return ORACLE_BAD_ARG;
    for (int32_t c = c_begin; c < c_end; ++c) {
        const int S = cand_S[c];
        const int32_t *grp = cand_group + (size_t)c * S_max, *tp = cand_tp + (size_t)c * S_max;
        int32_t *sp = splits + (size_t)c * (S_max + 1);
        n_caps[c] = 0;
        /* smallest feasible cap t_S and the latency of its plan: the min-max search above */
        status[c] = plan_one(&v, S, S_max, grp, tp, D0, D1, arg, sp, dev_first + (size_t)c * S_max,
                             bottleneck + c, iter_time + c);
        if (status[c] != CAND_OK) continue;
        const int64_t t_S = bottleneck[c];
        const int64_t t_E = ceil_div(iter_time[c], p->M);
        /* candidate caps: distinct costs of fitting stages inside [t_S, t_E] */
        size_t n = 0;
        for (int s = 0; s < S; ++s) {
            const int64_t nin = (S - s) < p->M ? (S - s) : p->M;
            for (int i = s + 1; i <= L - (S - 1 - s); ++i) {
                if (s == S - 1 && i != L) continue;
                const int64_t cc = (s == S - 1) ? 0 : cut_time(p, grp[s], grp[s + 1], i);
                for (int j = s; j < i; ++j) {
                    if (!memory_fits(&v, grp[s], tp[s], nin, j, i)) continue;
                    const int64_t w = max64(stage_time(&v, grp[s], tp[s], j, i), cc);
                    if (w < t_S || w > t_E) continue;
                    if (n == caps_room) {
                        caps_room *= 2;
                        caps = (int64_t *)realloc(caps, sizeof(int64_t) * caps_room);
                        if (!caps) return ORACLE_BAD_ARG;
                    }
                    caps[n++] = w;
                }
            }
        }
        qsort(caps, n, sizeof(int64_t), cmp_i64);
        int64_t best_T = ORACLE_INF, best_cap = ORACLE_INF;
        for (size_t q = 0; q < n; ++q) {
            if (q > 0 && caps[q] == caps[q - 1]) continue;
            n_caps[c] += 1;
            const int64_t F = capped_min_sum(&v, S, grp, tp, caps[q], D0, D1, arg, trial);
            if (F == ORACLE_INF) continue;
            const int64_t T = F + (int64_t)(p->M - 1) * caps[q];
            if (T < best_T) {
                best_T = T;
                best_cap = caps[q];
                for (int s = 0; s <= S; ++s) sp[s] = trial[s];
            }
        }
        if (best_T == ORACLE_INF) abort();          /* t_S itself is a cap and is feasible */
        int64_t b, t;
        if (score_partition(&v, S, grp, tp, sp, &b, &t) != CAND_OK || b != best_cap || t != best_T) abort();
        bottleneck[c] = best_cap;
        iter_time[c] = best_T;
    }
    free(D0); free(D1); free(arg); free(trial); free(caps);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------------------------
 * H-1F1B warm-up counts inside the capped recurrence (paper sections 4.1 and 5.2.3).
 *
 * Under H-1F1B the last stage launches one forward microbatch during warm-up and every earlier
 * stage launches delta more than the stage after it (eq. Ni), delta growing with the transfer
 * time of the cut between them relative to the cap t_max.  The recurrence is the paper's own
 * suffix form (eq. dp_general): a state is "the last s stages start at operator i"; its value is
 * the least sum of (t + 2c) under the cap, and it carries the warm-up count N of its first stage
 * as determined by the continuation that attained that least sum (eq. dp_ni), which the memory
 * constraint of the stage placed in front of it then uses (eq. mem_cons).  No search over N: a
 * continuation with a larger sum and a smaller N is not kept, as in the paper.
 *
 * Integer form of eq. dp_ni's increment, ceil(2c / t_max - eps) + 1 with eps = 1/64:
 *   delta(c; t_max) = 1                                    if 2c <= floor(t_max / 64)
 *                   = 1 + ceil((2c - floor(t_max/64)) / t_max)  otherwise   (2 or 3 when c <= t_max)
 * and counts never exceed the number of microbatches M.
 * ------------------------------------------------------------------------------------------- */
static int64_t h1f1b_delta(int64_t c, int64_t t_max)
{
    const int64_t x = 2 * c - t_max / 64;
    if (x <= 0) return 1;
    return 1 + ceil_div(x, t_max);                 /* x > 0 and c <= t_max imply t_max >= 1 */
}

/* One candidate under the cap t_max.  G and N are (S+1) x (L+1) tables: G[s][i] = least sum for
 * operators i..L-1 on the last s slots, N[s][i] = warm-up count of the first of those stages.
 * Ties keep the lowest end cut j of the first stage.  Returns the status; fills the outputs. */
/* Caps the capped entry points accept: below 2^47 us like every time of an accepted problem, and
 * small enough that a sum of at most 3 L terms plus (M - 1) caps stays inside int64 (magnitudes,
 * reading R13); a larger cap makes the candidate INVALID. */
static int cap_out_of_range(const oracle_problem *p, int64_t t_max)
{
    const int64_t by_sum = INT64_MAX / (3 * (int64_t)p->L + (int64_t)p->M);
    const int64_t limit = by_sum < ((int64_t)1 << 47) - 1 ? by_sum : ((int64_t)1 << 47) - 1;
    return t_max > limit;
}

static int plan_h1f1b_one(const tables_view *v, int S, int S_max, const int32_t *grp, const int32_t *tp,
                          int64_t t_max, int64_t *G, int64_t *N, int32_t *arg, int32_t *splits,
                          int32_t *dev_first, int32_t *warmup, int64_t *bott, int64_t *iter)
{
    const oracle_problem *p = v->p;
    const int L = p->L;
    fill_failed(S_max, splits, dev_first, bott, iter);
    for (int s = 0; s < S_max; ++s) warmup[s] = -1;
    if (!candidate_valid(p, S, S_max, grp, tp)) return CAND_INVALID;
    if (cap_out_of_range(p, t_max)) return CAND_INVALID;
    if (S > L || t_max < 0) return CAND_INFEASIBLE;
    const size_t W = (size_t)(L + 1);
    for (size_t x = 0; x < (size_t)(S + 1) * W; ++x) { G[x] = ORACLE_INF; N[x] = 0; arg[x] = -1; }
    G[(size_t)0 * W + L] = 0;                       /* no stages left, no operators left */
    for (int s = 1; s <= S; ++s) {
        const int slot = S - s;                     /* the stage this step places */
        for (int i = slot; i <= L - s; ++i) {
            int64_t best = ORACLE_INF, best_n = 0;
            int32_t best_j = -1;
            for (int j = i + 1; j <= L - (s - 1); ++j) {
                const int64_t rest = G[(size_t)(s - 1) * W + j];
                if (rest == ORACLE_INF) continue;
                const int64_t c = (s == 1) ? 0 : cut_time(p, grp[slot], grp[slot + 1], j);
                if (c > t_max) continue;                                   /* constraint (ii) */
                const int64_t t = stage_time(v, grp[slot], tp[slot], i, j);
                if (t > t_max) continue;                                   /* constraint (i) */
                int64_t n = h1f1b_delta(c, t_max) + N[(size_t)(s - 1) * W + j];   /* eq. dp_ni */
                if (n > p->M) n = p->M;
                if (!memory_fits(v, grp[slot], tp[slot], n, i, j)) continue;      /* constraint (iii) */
                const int64_t val = rest + t + 2 * c;
                if (val < best) { best = val; best_j = j; best_n = n; }
            }
            G[(size_t)s * W + i] = best;
            N[(size_t)s * W + i] = best_n;
            arg[(size_t)s * W + i] = best_j;
        }
    }
    if (G[(size_t)S * W + 0] == ORACLE_INF) return CAND_INFEASIBLE;
    int64_t worst = 0;
    int cutpos = 0;
    for (int slot = 0; slot < S; ++slot) {
        const int s = S - slot;
        const int next = arg[(size_t)s * W + cutpos];
        splits[slot] = cutpos;
        warmup[slot] = (int32_t)N[(size_t)s * W + cutpos];
        const int64_t c = (slot == S - 1) ? 0 : cut_time(p, grp[slot], grp[slot + 1], next);
        worst = max64(worst, max64(stage_time(v, grp[slot], tp[slot], cutpos, next), c));
        cutpos = next;
    }
    splits[S] = L;
    if (cutpos != L) abort();
    slot_devices(p, S, S_max, grp, tp, dev_first);
    *bott = worst;
    *iter = G[(size_t)S * W + 0] + (int64_t)(p->M - 1) * t_max;     /* T(t_max) of section 5.2.3 */
    return CAND_OK;
}

/* Capped H-1F1B recurrence for candidates c_begin..c_end-1, candidate c under the cap t_max[c].
 * splits, dev_first, status as oracle_plan_batch; warmup[c][s] = forward microbatches stage s
 * launches during warm-up (-1 beyond S or without a plan); bottleneck = the plan's own largest
 * stage or transfer time (<= the cap); iter_time = least sum + (M - 1) t_max[c]. */
int oracle_plan_h1f1b_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                            const int64_t *PR, int32_t C, int32_t S_max, const int32_t *cand_S,
                            const int32_t *cand_group, const int32_t *cand_tp, const int64_t *t_max,
                            int32_t c_begin, int32_t c_end, int32_t *splits, int32_t *dev_first,
                            int32_t *warmup, int64_t *bottleneck, int64_t *iter_time, int32_t *status)
{
    if (C < 0 || S_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end) return ORACLE_BAD_ARG;
    if (p->L > 65535) return ORACLE_BAD_ARG;
    const size_t cells = (size_t)(S_max + 1) * (size_t)(p->L + 1);
    int64_t *G = (int64_t *)malloc(sizeof(int64_t) * cells);
    int64_t *N = (int64_t *)malloc(sizeof(int64_t) * cells);
    int32_t *arg = (int32_t *)malloc(sizeof(int32_t) * cells);
    if (!G || !N || !arg) return ORACLE_BAD_ARG;
    for (int32_t c = c_begin; c < c_end; ++c)
        status[c] = plan_h1f1b_one(&(tables_view){ p, PF, PP, PS, PR }, cand_S[c], S_max,
                                   cand_group + (size_t)c * S_max, cand_tp + (size_t)c * S_max, t_max[c],
                                   G, N, arg, splits + (size_t)c * (S_max + 1),
                                   dev_first + (size_t)c * S_max, warmup + (size_t)c * S_max,
                                   bottleneck + c, iter_time + c);
    free(G); free(N); free(arg);
    return ORACLE_OK;
}

/* Warm-up counts and iteration time of given partitions under H-1F1B with the cap t_max[c]
 * (section 4.1: eq. Ni, eq. delta_i in the integer form above): INVALID for a malformed candidate
 * or cuts; INFEASIBLE when a stage or transfer time exceeds the cap or a stage does not fit in
 * memory with its warm-up count; otherwise warmup, bottleneck (own) and sum + (M - 1) t_max. */
int oracle_score_h1f1b(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                       const int64_t *PR, int32_t C, int32_t S_max, const int32_t *cand_S,
                       const int32_t *cand_group, const int32_t *cand_tp, const int32_t *splits,
                       const int64_t *t_max, int32_t *warmup, int64_t *bottleneck, int64_t *iter_time,
                       int32_t *status)
{
    if (C < 0 || S_max < 1) return ORACLE_BAD_ARG;
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    for (int32_t c = 0; c < C; ++c) {
        const int S = cand_S[c];
        const int32_t *grp = cand_group + (size_t)c * S_max, *tp = cand_tp + (size_t)c * S_max;
        const int32_t *sp = splits + (size_t)c * (S_max + 1);
        int32_t *wu = warmup + (size_t)c * S_max;
        for (int s = 0; s < S_max; ++s) wu[s] = -1;
        bottleneck[c] = ORACLE_INF;
        iter_time[c] = ORACLE_INF;
        status[c] = CAND_INVALID;
        if (!candidate_valid(p, S, S_max, grp, tp)) continue;
        int ok = sp[0] == 0 && sp[S] == L;
        for (int s = 0; s < S && ok; ++s) ok = sp[s + 1] > sp[s];
        if (!ok) continue;
        if (cap_out_of_range(p, t_max[c])) continue;
        status[c] = CAND_INFEASIBLE;
        if (t_max[c] < 0) continue;
        int64_t n = 0, sum = 0, worst = 0;
        int fits = 1;
        for (int s = S - 1; s >= 0; --s) {          /* counts accumulate from the last stage */
            const int64_t cc = (s == S - 1) ? 0 : cut_time(p, grp[s], grp[s + 1], sp[s + 1]);
            const int64_t t = stage_time(&v, grp[s], tp[s], sp[s], sp[s + 1]);
            if (cc > t_max[c] || t > t_max[c]) { fits = 0; break; }
            n += h1f1b_delta(cc, t_max[c]);
            if (n > p->M) n = p->M;
            if (!memory_fits(&v, grp[s], tp[s], n, sp[s], sp[s + 1])) { fits = 0; break; }
            wu[s] = (int32_t)n;
            sum += t + 2 * cc;
            worst = max64(worst, max64(t, cc));
        }
        if (!fits) {
            for (int s = 0; s < S_max; ++s) wu[s] = -1;
            continue;
        }
        status[c] = CAND_OK;
        bottleneck[c] = worst;
        iter_time[c] = sum + (int64_t)(p->M - 1) * t_max[c];
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Submesh choice inside the recurrence (paper section 5.2.3, eq. dp_general's third index).
 *
 * A candidate is an ORDER of device groups and a stage count S; how each group's devices are cut
 * into stages is decided by the recurrence itself.  With O_0 = 0, O_k = devices of the first k
 * groups of the order, the state (s, i, d) means: the first s stages hold the first i operators and
 * use exactly the first d devices of the ordered groups.  A stage placed at device offset d runs on
 * the group k with O_k <= d < O_{k+1} and takes tp of its devices, tp an allowed degree with
 * d + tp <= O_{k+1}; when that exhausts the group the next stage is on the next group and the cut
 * between them crosses the inter-group link, otherwise the intra-group link (the paper's rule for
 * C(j)).  Every device of every listed group is used: the answer is read at (S, L, O_K).
 * Min-max form, classic 1F1B counts, as on the hot path:
 *   D[s+1][i][d + tp] = min over (j, tp) of max(D[s][j][d], time, comm)
 * with ties resolved by the lowest previous cut j, then the smallest degree.
 * ------------------------------------------------------------------------------------------- */
/* Scratch of the three-index table for one call. */
typedef struct {
    int64_t *D;          /* (S_max + 1) x (L + 1) x (devices + 1) */
    int32_t *arg_j, *arg_k;
    int64_t *O;          /* offsets of the ordered groups */
    size_t W, Dn;
} mesh_tables;

#define MESH_AT(m, s, i, d) (((size_t)(s) * (m)->W + (size_t)(i)) * (m)->Dn + (size_t)(d))

/* Fills the table for one ordering (K groups og[], offsets m->O) and S stages.
 * capped = 0: min-max form.  capped = 1: least sum of (t + 2c) over transitions whose stage and
 * transfer times are at most cap (constraints (i), (ii)).  Ties: lowest previous cut, then
 * smallest degree.  If caps is not NULL, every fitting transition's max(time, comm) inside
 * [cap_lo, cap_hi] is appended to it (the candidate caps of section 5.2.4 (2)). */
static int mesh_fill(const tables_view *v, mesh_tables *m, int K, const int32_t *og, int S, int capped,
                     int64_t cap, int64_t **caps, size_t *n_caps, size_t *caps_room, int64_t cap_lo,
                     int64_t cap_hi)
{
    const oracle_problem *p = v->p;
    const int L = p->L;
    const int64_t Dtot = m->O[K];
    for (size_t x = 0; x < (size_t)(S + 1) * m->W * m->Dn; ++x) { m->D[x] = ORACLE_INF; m->arg_j[x] = -1; m->arg_k[x] = -1; }
    m->D[MESH_AT(m, 0, 0, 0)] = 0;
    for (int s = 0; s < S; ++s) {
        const int last = (s == S - 1);
        const int64_t n = (S - s) < p->M ? (S - s) : p->M;
        int k = 0;
        for (int64_t d = 0; d < Dtot; ++d) {
            while (m->O[k + 1] <= d) ++k;                      /* the group this stage runs on */
            const int g = og[k];
            for (int q = 0; q < p->n_tp; ++q) {
                const int tp = p->tp_degrees[q];
                const int64_t d2 = d + tp;
                if (d2 > m->O[k + 1]) continue;                /* a stage stays inside one group */
                if (last != (d2 == Dtot)) continue;            /* the last stage, and only it, uses up the devices */
                const int g_next = last ? g : (d2 == m->O[k + 1] ? og[k + 1] : g);
                for (int i = s + 1; i <= L - (S - 1 - s); ++i) {
                    if (last && i != L) continue;
                    const int64_t cc = last ? 0 : cut_time(p, g, g_next, i);
                    int64_t best = m->D[MESH_AT(m, s + 1, i, d2)];
                    int32_t bj = m->arg_j[MESH_AT(m, s + 1, i, d2)], bq = m->arg_k[MESH_AT(m, s + 1, i, d2)];
                    for (int j = s; j < i; ++j) {
                        if (!memory_fits(v, g, tp, n, j, i)) continue;
                        const int64_t t = stage_time(v, g, tp, j, i);
                        if (caps) {
                            const int64_t w = max64(t, cc);
                            if (w >= cap_lo && w <= cap_hi) {
                                if (*n_caps == *caps_room) {
                                    *caps_room *= 2;
                                    *caps = (int64_t *)realloc(*caps, sizeof(int64_t) * *caps_room);
                                    if (!*caps) return ORACLE_BAD_ARG;
                                }
                                (*caps)[(*n_caps)++] = w;
                            }
                        }
                        const int64_t prev = m->D[MESH_AT(m, s, j, d)];
                        if (prev == ORACLE_INF) continue;
                        int64_t val;
                        if (capped) {
                            if (t > cap || cc > cap) continue;
                            val = prev + t + 2 * cc;
                        } else {
                            val = max64(prev, max64(t, cc));
                        }
                        if (val < best || (val == best && (j < bj || (j == bj && q < bq)))) {
                            best = val; bj = j; bq = q;
                        }
                    }
                    m->D[MESH_AT(m, s + 1, i, d2)] = best;
                    m->arg_j[MESH_AT(m, s + 1, i, d2)] = bj;
                    m->arg_k[MESH_AT(m, s + 1, i, d2)] = bq;
                }
            }
        }
    }
    return ORACLE_OK;
}

/* Follows the back-pointers from (S, L, all devices): cuts, group and degree of every stage. */
static void mesh_backtrack(const tables_view *v, const mesh_tables *m, int K, const int32_t *og, int S,
                           int32_t *sp, int32_t *sg, int32_t *st)
{
    const oracle_problem *p = v->p;
    int i = p->L;
    int64_t d = m->O[K];
    sp[S] = p->L;
    for (int s = S; s >= 1; --s) {
        const int j = m->arg_j[MESH_AT(m, s, i, d)], q = m->arg_k[MESH_AT(m, s, i, d)];
        const int tp = p->tp_degrees[q];
        d -= tp;
        int k = 0;
        while (m->O[k + 1] <= d) ++k;
        sp[s - 1] = j;
        sg[s - 1] = og[k];
        st[s - 1] = tp;
        i = j;
    }
    if (i != 0 || d != 0) abort();
}

/* exact = 0: the min-max plan of every ordering.  exact = 1: the optimum of eq. gpipe_cost_model
 * over every slicing and partition, by the increasing sweep over the cap (section 5.2.4 (2)) with
 * the capped least-sum table at every cap; n_caps (may be NULL) receives the caps swept. */
static int mesh_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                      const int64_t *PR, int32_t C, int32_t G_max, int32_t S_max, const int32_t *ord_S,
                      const int32_t *ord_G, const int32_t *ord_group, int32_t c_begin, int32_t c_end,
                      int32_t *splits, int32_t *stage_group, int32_t *stage_tp, int32_t *dev_first,
                      int64_t *bottleneck, int64_t *iter_time, int32_t *status, int exact, int32_t *n_caps)
{
    if (C < 0 || S_max < 1 || G_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end) return ORACLE_BAD_ARG;
    if (p->L > 65535) return ORACLE_BAD_ARG;
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    int64_t total_dev = 0;
    for (int g = 0; g < p->G; ++g) total_dev += p->group_ndev[g];
    mesh_tables m;
    m.W = (size_t)(L + 1);
    m.Dn = (size_t)total_dev + 1;
    const size_t cells = (size_t)(S_max + 1) * m.W * m.Dn;
    m.D = (int64_t *)malloc(sizeof(int64_t) * cells);
    m.arg_j = (int32_t *)malloc(sizeof(int32_t) * cells);
    m.arg_k = (int32_t *)malloc(sizeof(int32_t) * cells);
    m.O = (int64_t *)malloc(sizeof(int64_t) * (size_t)(G_max + 1));
    char *seen = (char *)malloc((size_t)p->G);
    int32_t *trial = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)(S_max + 1));
    size_t caps_room = 1024;
    int64_t *caps = (int64_t *)malloc(sizeof(int64_t) * caps_room);
    if (!m.D || !m.arg_j || !m.arg_k || !m.O || !seen || !trial || !caps) return ORACLE_BAD_ARG;
    for (int32_t c = c_begin; c < c_end; ++c) {
        const int S = ord_S[c], K = ord_G[c];
        const int32_t *og = ord_group + (size_t)c * G_max;
        int32_t *sp = splits + (size_t)c * (S_max + 1), *sg = stage_group + (size_t)c * S_max;
        int32_t *st = stage_tp + (size_t)c * S_max, *df = dev_first + (size_t)c * S_max;
        fill_failed(S_max, sp, df, bottleneck + c, iter_time + c);
        for (int s = 0; s < S_max; ++s) { sg[s] = -1; st[s] = -1; }
        if (n_caps) n_caps[c] = 0;
        status[c] = CAND_INVALID;
        if (S < 1 || S > S_max || K < 1 || K > G_max) continue;
        int ok = 1;
        memset(seen, 0, (size_t)p->G);
        m.O[0] = 0;
        for (int k = 0; k < K && ok; ++k) {
            if (og[k] < 0 || og[k] >= p->G || seen[og[k]]) { ok = 0; break; }
            seen[og[k]] = 1;
            m.O[k + 1] = m.O[k] + p->group_ndev[og[k]];
        }
        if (!ok) continue;
        status[c] = CAND_INFEASIBLE;
        const int64_t Dtot = m.O[K];
        if (S > L || S < K || S > Dtot) continue;
        if (mesh_fill(&v, &m, K, og, S, 0, 0, NULL, NULL, NULL, 0, 0) != ORACLE_OK) return ORACLE_BAD_ARG;
        const int64_t t_S = m.D[MESH_AT(&m, S, L, Dtot)];
        if (t_S == ORACLE_INF) continue;
        mesh_backtrack(&v, &m, K, og, S, sp, sg, st);
        if (!candidate_valid(p, S, S_max, sg, st)) abort();      /* the slicing found is a well-formed candidate */
        if (score_partition(&v, S, sg, st, sp, bottleneck + c, iter_time + c) != CAND_OK || bottleneck[c] != t_S)
            abort();
        status[c] = CAND_OK;
        if (exact) {
            const int64_t t_E = ceil_div(iter_time[c], p->M);
            size_t n = 0;
            /* one more pass of the min-max table only to collect the candidate caps in [t_S, t_E] */
            if (mesh_fill(&v, &m, K, og, S, 0, 0, &caps, &n, &caps_room, t_S, t_E) != ORACLE_OK) return ORACLE_BAD_ARG;
            qsort(caps, n, sizeof(int64_t), cmp_i64);
            int64_t best_T = ORACLE_INF, best_cap = ORACLE_INF;
            int32_t *tsp = trial, *tsg = trial + (S_max + 1), *tst = trial + 2 * (S_max + 1);
            for (size_t q = 0; q < n; ++q) {
                if (q > 0 && caps[q] == caps[q - 1]) continue;
                if (n_caps) n_caps[c] += 1;
                if (mesh_fill(&v, &m, K, og, S, 1, caps[q], NULL, NULL, NULL, 0, 0) != ORACLE_OK) return ORACLE_BAD_ARG;
                const int64_t F = m.D[MESH_AT(&m, S, L, Dtot)];
                if (F == ORACLE_INF) continue;
                const int64_t T = F + (int64_t)(p->M - 1) * caps[q];
                if (T < best_T) {
                    best_T = T;
                    best_cap = caps[q];
                    mesh_backtrack(&v, &m, K, og, S, tsp, tsg, tst);
                    for (int s = 0; s <= S; ++s) sp[s] = tsp[s];
                    for (int s = 0; s < S; ++s) { sg[s] = tsg[s]; st[s] = tst[s]; }
                }
            }
            if (best_T == ORACLE_INF) abort();                   /* t_S itself is a cap and is feasible */
            int64_t b, t;
            if (score_partition(&v, S, sg, st, sp, &b, &t) != CAND_OK || b != best_cap || t != best_T) abort();
            bottleneck[c] = best_cap;
            iter_time[c] = best_T;
        }
        slot_devices(p, S, S_max, sg, st, df);
    }
    free(m.D); free(m.arg_j); free(m.arg_k); free(m.O); free(seen); free(trial); free(caps);
    return ORACLE_OK;
}

int oracle_plan_mesh_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP, const int64_t *PS,
                           const int64_t *PR, int32_t C, int32_t G_max, int32_t S_max, const int32_t *ord_S,
                           const int32_t *ord_G, const int32_t *ord_group, int32_t c_begin, int32_t c_end,
                           int32_t *splits, int32_t *stage_group, int32_t *stage_tp, int32_t *dev_first,
                           int64_t *bottleneck, int64_t *iter_time, int32_t *status)
{
    return mesh_batch(p, PF, PP, PS, PR, C, G_max, S_max, ord_S, ord_G, ord_group, c_begin, c_end, splits,
                      stage_group, stage_tp, dev_first, bottleneck, iter_time, status, 0, NULL);
}

/* The paper's full search for one ordering: eq. dp_general with its device index, swept over the
 * cap.  Outputs as oracle_plan_mesh_batch, with bottleneck = the winning cap (the plan's own largest
 * time) and iter_time = the optimum; n_caps[c] = caps swept. */
int oracle_plan_mesh_exact_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP,
                                 const int64_t *PS, const int64_t *PR, int32_t C, int32_t G_max, int32_t S_max,
                                 const int32_t *ord_S, const int32_t *ord_G, const int32_t *ord_group,
                                 int32_t c_begin, int32_t c_end, int32_t *splits, int32_t *stage_group,
                                 int32_t *stage_tp, int32_t *dev_first, int64_t *bottleneck, int64_t *iter_time,
                                 int32_t *status, int32_t *n_caps)
{
    return mesh_batch(p, PF, PP, PS, PR, C, G_max, S_max, ord_S, ord_G, ord_group, c_begin, c_end, splits,
                      stage_group, stage_tp, dev_first, bottleneck, iter_time, status, 1, n_caps);
}

/* ---------------------------------------------------------------------------------------------
 * The paper's recurrence in full for one cap (section 5.2.3): eq. dp_general with its device index
 * AND the H-1F1B warm-up count of eq. dp_ni in the state, in the suffix direction.
 *
 * State (s, i, e): the last s stages hold the operators i..L-1 and use exactly the last e devices
 * of the ordered groups; it keeps the least sum of (t + 2c) under the cap and the warm-up count N of
 * its first stage, as determined by the continuation that attained the least sum.  The first of
 * those stages starts at device offset D - e, runs on the group that offset falls in and takes tp
 * of its devices (not reaching beyond the group); the cut behind it crosses to the next group's
 * link when the stage exhausts its group.  Ties: lowest end cut j, then smallest degree.
 * ------------------------------------------------------------------------------------------- */
int oracle_plan_mesh_h1f1b_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP,
                                 const int64_t *PS, const int64_t *PR, int32_t C, int32_t G_max, int32_t S_max,
                                 const int32_t *ord_S, const int32_t *ord_G, const int32_t *ord_group,
                                 const int64_t *t_max, int32_t c_begin, int32_t c_end, int32_t *splits,
                                 int32_t *stage_group, int32_t *stage_tp, int32_t *dev_first, int32_t *warmup,
                                 int64_t *bottleneck, int64_t *iter_time, int32_t *status)
{
    if (C < 0 || S_max < 1 || G_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end) return ORACLE_BAD_ARG;
    if (p->L > 65535) return ORACLE_BAD_ARG;
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    int64_t total_dev = 0;
    for (int g = 0; g < p->G; ++g) total_dev += p->group_ndev[g];
    mesh_tables m;
    m.W = (size_t)(L + 1);
    m.Dn = (size_t)total_dev + 1;
    const size_t cells = (size_t)(S_max + 1) * m.W * m.Dn;
    m.D = (int64_t *)malloc(sizeof(int64_t) * cells);
    m.arg_j = (int32_t *)malloc(sizeof(int32_t) * cells);
    m.arg_k = (int32_t *)malloc(sizeof(int32_t) * cells);
    int32_t *N = (int32_t *)malloc(sizeof(int32_t) * cells);
    m.O = (int64_t *)malloc(sizeof(int64_t) * (size_t)(G_max + 1));
    char *seen = (char *)malloc((size_t)p->G);
    if (!m.D || !m.arg_j || !m.arg_k || !N || !m.O || !seen) return ORACLE_BAD_ARG;
    for (int32_t c = c_begin; c < c_end; ++c) {
        const int S = ord_S[c], K = ord_G[c];
        const int64_t cap = t_max[c];
        const int32_t *og = ord_group + (size_t)c * G_max;
        int32_t *sp = splits + (size_t)c * (S_max + 1), *sg = stage_group + (size_t)c * S_max;
        int32_t *st = stage_tp + (size_t)c * S_max, *df = dev_first + (size_t)c * S_max;
        int32_t *wu = warmup + (size_t)c * S_max;
        fill_failed(S_max, sp, df, bottleneck + c, iter_time + c);
        for (int s = 0; s < S_max; ++s) { sg[s] = -1; st[s] = -1; wu[s] = -1; }
        status[c] = CAND_INVALID;
        if (S < 1 || S > S_max || K < 1 || K > G_max) continue;
        int ok = 1;
        memset(seen, 0, (size_t)p->G);
        m.O[0] = 0;
        for (int k = 0; k < K && ok; ++k) {
            if (og[k] < 0 || og[k] >= p->G || seen[og[k]]) { ok = 0; break; }
            seen[og[k]] = 1;
            m.O[k + 1] = m.O[k] + p->group_ndev[og[k]];
        }
        if (!ok) continue;
        if (cap_out_of_range(p, cap)) continue;
        status[c] = CAND_INFEASIBLE;
        const int64_t Dtot = m.O[K];
        if (S > L || S < K || S > Dtot || cap < 0) continue;
        for (size_t x = 0; x < (size_t)(S + 1) * m.W * m.Dn; ++x) { m.D[x] = ORACLE_INF; N[x] = 0; m.arg_j[x] = -1; m.arg_k[x] = -1; }
        m.D[MESH_AT(&m, 0, L, 0)] = 0;                    /* no stages left, no operators, no devices */
        for (int s = 1; s <= S; ++s) {
            for (int64_t e = s; e <= Dtot - (S - s); ++e) {
                if ((s == S) != (e == Dtot)) continue;    /* the whole pipeline, and only it, uses every device */
                const int64_t d0 = Dtot - e;              /* first device of the stage this step places */
                int k = 0;
                while (m.O[k + 1] <= d0) ++k;
                const int g = og[k];
                for (int q = 0; q < p->n_tp; ++q) {
                    const int tp = p->tp_degrees[q];
                    if (d0 + tp > m.O[k + 1]) continue;   /* a stage stays inside one group */
                    const int64_t e0 = e - tp;            /* devices of the stages behind it */
                    if ((s == 1) != (e0 == 0)) continue;
                    const int g_next = (s == 1) ? g : (d0 + tp == m.O[k + 1] ? og[k + 1] : g);
                    for (int i = S - s; i <= L - s; ++i) {
                        if (s == S && i != 0) continue;
                        int64_t best = m.D[MESH_AT(&m, s, i, e)];
                        int32_t bj = m.arg_j[MESH_AT(&m, s, i, e)], bq = m.arg_k[MESH_AT(&m, s, i, e)];
                        int32_t bn = N[MESH_AT(&m, s, i, e)];
                        for (int j = i + 1; j <= L - (s - 1); ++j) {
                            const int64_t rest = m.D[MESH_AT(&m, s - 1, j, e0)];
                            if (rest == ORACLE_INF) continue;
                            const int64_t cc = (s == 1) ? 0 : cut_time(p, g, g_next, j);
                            if (cc > cap) continue;                                     /* constraint (ii) */
                            const int64_t t = stage_time(&v, g, tp, i, j);
                            if (t > cap) continue;                                      /* constraint (i) */
                            int64_t n = h1f1b_delta(cc, cap) + N[MESH_AT(&m, s - 1, j, e0)];   /* eq. dp_ni */
                            if (n > p->M) n = p->M;
                            if (!memory_fits(&v, g, tp, n, i, j)) continue;             /* constraint (iii) */
                            const int64_t val = rest + t + 2 * cc;
                            if (val < best || (val == best && (bj < 0 || j < bj || (j == bj && q < bq)))) {
                                best = val; bj = j; bq = q; bn = (int32_t)n;
                            }
                        }
                        m.D[MESH_AT(&m, s, i, e)] = best;
                        m.arg_j[MESH_AT(&m, s, i, e)] = bj;
                        m.arg_k[MESH_AT(&m, s, i, e)] = bq;
                        N[MESH_AT(&m, s, i, e)] = bn;
                    }
                }
            }
        }
        const int64_t sum = m.D[MESH_AT(&m, S, 0, Dtot)];
        if (sum == ORACLE_INF) continue;
        int i = 0;
        int64_t e = Dtot, worst = 0;
        for (int slot = 0; slot < S; ++slot) {
            const int s = S - slot;
            const int j = m.arg_j[MESH_AT(&m, s, i, e)], q = m.arg_k[MESH_AT(&m, s, i, e)];
            const int tp = p->tp_degrees[q];
            const int64_t d0 = Dtot - e;
            int k = 0;
            while (m.O[k + 1] <= d0) ++k;
            sp[slot] = i;
            sg[slot] = og[k];
            st[slot] = tp;
            wu[slot] = N[MESH_AT(&m, s, i, e)];
            i = j;
            e -= tp;
        }
        sp[S] = L;
        if (i != L || e != 0) abort();
        if (!candidate_valid(p, S, S_max, sg, st)) abort();
        for (int slot = 0; slot < S; ++slot) {
            const int64_t cc = (slot == S - 1) ? 0 : cut_time(p, sg[slot], sg[slot + 1], sp[slot + 1]);
            worst = max64(worst, max64(stage_time(&v, sg[slot], st[slot], sp[slot], sp[slot + 1]), cc));
        }
        slot_devices(p, S, S_max, sg, st, df);
        bottleneck[c] = worst;
        iter_time[c] = sum + (int64_t)(p->M - 1) * cap;
        status[c] = CAND_OK;
    }
    free(m.D); free(m.arg_j); free(m.arg_k); free(N); free(m.O); free(seen);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------------------------
 * The search of section 5.2.4 (2) around the full recurrence: the cap t_max swept over the sorted,
 * deduplicated candidate values, from the smallest feasible one up to t_E = ceil(T(t_S) / B).
 *
 * Candidate values of an ordering (what a profiler would hand over, independent of where in the
 * pipeline a stage sits): every stage time time(g, tp; j, i) for a group g of the ordering, an
 * allowed degree tp <= devices of g, and 0 <= j < i <= L; and every transfer time of a cut
 * 1 <= i <= L - 1 on the links the ordering can use (inside each listed group, and from each
 * listed group to the one after it).  These are the values at which the set of transitions that
 * constraints (i) and (ii) admit can change.
 *
 * Sweep, per ordering: the lower end is the classic min-max bottleneck (no cap below it admits a
 * plan, and H-1F1B's counts are never below the classic ones).  Caps are taken in increasing order
 * from there; each one is given to the full recurrence (oracle_plan_mesh_h1f1b_batch, one
 * ordering).  The first cap with a plan fixes t_E = ceil(T / B) from that plan's T; the sweep ends
 * past t_E, at the end of the list, or after max_caps caps.  The answer is the plan with the
 * smallest T = least sum + (B - 1) cap, the lower cap on equal T.  t_max_out receives the cap of
 * the answer (INF if none), n_caps the caps tried.
 * ------------------------------------------------------------------------------------------- */
int oracle_plan_mesh_h1f1b_sweep_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP,
                                       const int64_t *PS, const int64_t *PR, int32_t C, int32_t G_max,
                                       int32_t S_max, const int32_t *ord_S, const int32_t *ord_G,
                                       const int32_t *ord_group, int32_t max_caps, int32_t c_begin,
                                       int32_t c_end, int32_t *splits, int32_t *stage_group, int32_t *stage_tp,
                                       int32_t *dev_first, int32_t *warmup, int64_t *bottleneck,
                                       int64_t *iter_time, int32_t *status, int64_t *t_max_out, int32_t *n_caps)
{
    if (C < 0 || S_max < 1 || G_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end || max_caps < 1)
        return ORACLE_BAD_ARG;
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    /* one ordering's worth of outputs for the trial calls */
    int32_t *tsp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S_max + 1));
    int32_t *tsg = (int32_t *)malloc(sizeof(int32_t) * (size_t)S_max);
    int32_t *tst = (int32_t *)malloc(sizeof(int32_t) * (size_t)S_max);
    int32_t *tdf = (int32_t *)malloc(sizeof(int32_t) * (size_t)S_max);
    int32_t *twu = (int32_t *)malloc(sizeof(int32_t) * (size_t)S_max);
    size_t room = 1024, n = 0;
    int64_t *grid = (int64_t *)malloc(sizeof(int64_t) * room);
    if (!tsp || !tsg || !tst || !tdf || !twu || !grid) return ORACLE_BAD_ARG;
    for (int32_t c = c_begin; c < c_end; ++c) {
        const int32_t *og = ord_group + (size_t)c * G_max;
        int32_t *sp = splits + (size_t)c * (S_max + 1), *sg = stage_group + (size_t)c * S_max;
        int32_t *st = stage_tp + (size_t)c * S_max, *df = dev_first + (size_t)c * S_max;
        int32_t *wu = warmup + (size_t)c * S_max;
        for (int s = 0; s < S_max; ++s) wu[s] = -1;
        t_max_out[c] = ORACLE_INF;
        if (n_caps) n_caps[c] = 0;
        /* the classic min-max plan of this ordering: validity, and the lower end of the sweep */
        int64_t t_S, unused;
        int32_t st0;
        int rc = oracle_plan_mesh_batch(p, PF, PP, PS, PR, 1, G_max, S_max, ord_S + c, ord_G + c, og, 0, 1,
                                        sp, sg, st, df, &t_S, &unused, &st0);
        if (rc != ORACLE_OK) return rc;
        /* whatever happens next, the outputs start out as "no plan" */
        fill_failed(S_max, sp, df, bottleneck + c, iter_time + c);
        for (int s = 0; s < S_max; ++s) { sg[s] = -1; st[s] = -1; }
        status[c] = st0;
        if (st0 != CAND_OK) continue;
        status[c] = CAND_INFEASIBLE;
        const int K = ord_G[c];
        /* the candidate values at or above t_S */
        n = 0;
#define GRID_PUSH(x)                                                                          \
    do {                                                                                      \
        const int64_t val_ = (x);                                                             \
        if (val_ >= t_S) {                                                                    \
            if (n == room) {                                                                  \
                room *= 2;                                                                    \
                grid = (int64_t *)realloc(grid, sizeof(int64_t) * room);                      \
                if (!grid) return ORACLE_BAD_ARG;                                             \
            }                                                                                 \
            grid[n++] = val_;                                                                 \
        }                                                                                     \
    } while (0)
        for (int k = 0; k < K; ++k) {
            const int g = og[k];
            for (int q = 0; q < p->n_tp; ++q) {
                const int tp = p->tp_degrees[q];
                if (tp > p->group_ndev[g]) continue;
                for (int j = 0; j < L; ++j)
                    for (int i = j + 1; i <= L; ++i) GRID_PUSH(stage_time(&v, g, tp, j, i));
            }
            for (int i = 1; i <= L - 1; ++i) {
                GRID_PUSH(cut_time(p, g, g, i));
                if (k + 1 < K) GRID_PUSH(cut_time(p, g, og[k + 1], i));
            }
        }
#undef GRID_PUSH
        qsort(grid, n, sizeof(int64_t), cmp_i64);
        int64_t best_T = ORACLE_INF, t_E = ORACLE_INF;
        int tried = 0;
        for (size_t x = 0; x < n && tried < max_caps; ++x) {
            if (x > 0 && grid[x] == grid[x - 1]) continue;
            const int64_t cap = grid[x];
            if (cap > t_E) break;
            ++tried;
            int64_t b1, T1;
            int32_t s1;
            rc = oracle_plan_mesh_h1f1b_batch(p, PF, PP, PS, PR, 1, G_max, S_max, ord_S + c, ord_G + c, og, &cap,
                                              0, 1, tsp, tsg, tst, tdf, twu, &b1, &T1, &s1);
            if (rc != ORACLE_OK) return rc;
            if (s1 != CAND_OK) continue;
            if (t_E == ORACLE_INF) t_E = ceil_div(T1, p->M);
            if (T1 < best_T) {
                best_T = T1;
                for (int s = 0; s <= S_max; ++s) sp[s] = tsp[s];
                for (int s = 0; s < S_max; ++s) { sg[s] = tsg[s]; st[s] = tst[s]; df[s] = tdf[s]; wu[s] = twu[s]; }
                bottleneck[c] = b1;
                iter_time[c] = T1;
                t_max_out[c] = cap;
                status[c] = CAND_OK;
            }
        }
        if (n_caps) n_caps[c] = tried;
    }
    free(tsp); free(tsg); free(tst); free(tdf); free(twu); free(grid);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------------------------
 * The same search (section 5.2.4 (2)) for candidates, whose slicing is fixed: the cap swept over
 * the candidate values from the hot path's bottleneck up to t_E = ceil(T / B), the capped H-1F1B
 * recurrence (oracle_plan_h1f1b_batch, one candidate) at every cap.
 *
 * Candidate values of a candidate: every stage time time(g_s, tp_s; j, i) of one of its slots,
 * 0 <= j < i <= L, and every transfer time of a cut 1 <= i <= L - 1 on the link between two
 * consecutive slots (g_s, g_{s+1}).  Sweep, t_E, the answer, t_max_out and n_caps as for
 * oracle_plan_mesh_h1f1b_sweep_batch.
 * ------------------------------------------------------------------------------------------- */
int oracle_plan_h1f1b_sweep_batch(const oracle_problem *p, const int64_t *PF, const int64_t *PP,
                                  const int64_t *PS, const int64_t *PR, int32_t C, int32_t S_max,
                                  const int32_t *cand_S, const int32_t *cand_group, const int32_t *cand_tp,
                                  int32_t max_caps, int32_t c_begin, int32_t c_end, int32_t *splits,
                                  int32_t *dev_first, int32_t *warmup, int64_t *bottleneck, int64_t *iter_time,
                                  int32_t *status, int64_t *t_max_out, int32_t *n_caps)
{
    if (C < 0 || S_max < 1 || c_begin < 0 || c_end > C || c_begin > c_end || max_caps < 1) return ORACLE_BAD_ARG;
    const int L = p->L;
    tables_view v = { p, PF, PP, PS, PR };
    int32_t *tsp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S_max + 1));
    int32_t *tdf = (int32_t *)malloc(sizeof(int32_t) * (size_t)S_max);
    int32_t *twu = (int32_t *)malloc(sizeof(int32_t) * (size_t)S_max);
    size_t room = 1024, n = 0;
    int64_t *grid = (int64_t *)malloc(sizeof(int64_t) * room);
    if (!tsp || !tdf || !twu || !grid) return ORACLE_BAD_ARG;
    for (int32_t c = c_begin; c < c_end; ++c) {
        const int32_t *grp = cand_group + (size_t)c * S_max, *tp = cand_tp + (size_t)c * S_max;
        int32_t *sp = splits + (size_t)c * (S_max + 1), *df = dev_first + (size_t)c * S_max;
        int32_t *wu = warmup + (size_t)c * S_max;
        for (int s = 0; s < S_max; ++s) wu[s] = -1;
        t_max_out[c] = ORACLE_INF;
        if (n_caps) n_caps[c] = 0;
        /* the hot path's plan of this candidate: validity, and the lower end of the sweep */
        int64_t t_S, unused;
        int32_t st0;
        int rc = oracle_plan_batch(p, PF, PP, PS, PR, 1, S_max, cand_S + c, grp, tp, 0, 1, sp, df, &t_S, &unused, &st0);
        if (rc != ORACLE_OK) return rc;
        fill_failed(S_max, sp, df, bottleneck + c, iter_time + c);
        status[c] = st0;
        if (st0 != CAND_OK) continue;
        status[c] = CAND_INFEASIBLE;
        const int S = cand_S[c];
        n = 0;
        for (int s = 0; s < S; ++s) {
            for (int j = 0; j < L; ++j)
                for (int i = j + 1; i <= L; ++i) {
                    const int64_t val = stage_time(&v, grp[s], tp[s], j, i);
                    if (val < t_S) continue;
                    if (n == room) {
                        room *= 2;
                        grid = (int64_t *)realloc(grid, sizeof(int64_t) * room);
                        if (!grid) return ORACLE_BAD_ARG;
                    }
                    grid[n++] = val;
                }
            if (s + 1 < S)
                for (int i = 1; i <= L - 1; ++i) {
                    const int64_t val = cut_time(p, grp[s], grp[s + 1], i);
                    if (val < t_S) continue;
                    if (n == room) {
                        room *= 2;
                        grid = (int64_t *)realloc(grid, sizeof(int64_t) * room);
                        if (!grid) return ORACLE_BAD_ARG;
                    }
                    grid[n++] = val;
                }
        }
        qsort(grid, n, sizeof(int64_t), cmp_i64);
        int64_t best_T = ORACLE_INF, t_E = ORACLE_INF;
        int tried = 0;
        for (size_t x = 0; x < n && tried < max_caps; ++x) {
            if (x > 0 && grid[x] == grid[x - 1]) continue;
            const int64_t cap = grid[x];
            if (cap > t_E) break;
            ++tried;
            int64_t b1, T1;
            int32_t s1;
            rc = oracle_plan_h1f1b_batch(p, PF, PP, PS, PR, 1, S_max, cand_S + c, grp, tp, &cap, 0, 1, tsp, tdf, twu,
                                         &b1, &T1, &s1);
            if (rc != ORACLE_OK) return rc;
            if (s1 != CAND_OK) continue;
            if (t_E == ORACLE_INF) t_E = ceil_div(T1, p->M);
            if (T1 < best_T) {
                best_T = T1;
                for (int s = 0; s <= S_max; ++s) sp[s] = tsp[s];
                for (int s = 0; s < S_max; ++s) { df[s] = tdf[s]; wu[s] = twu[s]; }
                bottleneck[c] = b1;
                iter_time[c] = T1;
                t_max_out[c] = cap;
                status[c] = CAND_OK;
            }
        }
        if (n_caps) n_caps[c] = tried;
    }
    free(tsp); free(tdf); free(twu); free(grid);
    return ORACLE_OK;
}
