/*
 * harp.h - C ABI of the MI355X planner-search library.
 *
 * The library evaluates, on one GPU, a batch of candidate pipeline layouts for the inter-operator
 * planner of HARP (paper section 5.2).  A planning problem is an ordered sequence of L operators
 * with profiled per-GPU-type compute times and byte sizes, and a cluster of G homogeneous device
 * groups with intra- and inter-group link bandwidths (section 5.2.1, 5.2.3).  A candidate is an
 * ordered list of S stage slots; slot s is a submesh of tp_s devices of group g_s (the ordered
 * subclusters of section 5.2.1 together with the submesh choice of section 5.2.2, hoisted out of
 * the DP into the batch dimension).  For every candidate the library finds the partition of the
 * operators into S contiguous non-empty stages with the smallest feasible bottleneck t_max
 * (section 5.2.3, constraints (i)-(iii); the lower end t_S of the cap range of section 5.2.4 (2)) and
 * scores it with the iteration-time model of section 5.2.2 (eq. gpipe_cost_model).
 *
 * All quantities are integers: times in microseconds, sizes in bytes, bandwidths in bytes per
 * microsecond.  With segment [j, i) of operators on slot s = (g, tp), t = group_type[g]:
 *
 *   time(s; j, i) = ceil(sum_{j<=l<i} (fwd_us[t][l] + bwd_us[t][l]) / tp)
 *                   + sum_{j<=l<i} ceil(ar_count * 2 (tp-1) * act_bytes[l] / (tp * bw[g][g]))
 *                                                                   (second term 0 when tp == 1)
 *   comm(s; i)    = ceil(act_bytes[i-1] / bw[g_s][g_{s+1}])  for s < S-1,   0 for s == S-1
 *   fits(s; j, i) = sum param_bytes + N_s * sum stash_bytes <= tp * type_mem_bytes[t],
 *                   N_s = min(S - s, M)     (classic 1F1B in-flight microbatches, section 2.1;
 *                                            eq. mem_cons of section 5.2.3)
 *   bottleneck    = min over partitions with every stage fitting of
 *                   max_s max(time_s, comm_s)
 *   iter_time     = sum_s time_s + 2 sum_{s<S-1} comm_s + (M - 1) * bottleneck
 *
 * Among partitions of equal bottleneck the reported one is fixed by the recurrence
 *   D[s+1][i] = min_j max(D[s][j], time(s;j,i), comm(s;i))  over fitting j, lowest j on ties,
 * followed back from (S, L).
 *
 * Built on the same tables and cost model, further down in this header: the exact optimum of the
 * iteration-time model per candidate (harp_plan_exact_batch, section 5.2.4 (2)); the capped
 * recurrence with the warm-up counts of the H-1F1B scheduler in the memory constraint and as an
 * output (harp_plan_h1f1b_batch, harp_score_h1f1b; sections 4.1 and 5.2.3), and its search over
 * the cap (harp_plan_h1f1b_sweep_batch); the planner over ORDERINGS of device groups that chooses
 * every stage's devices inside the recurrence (harp_plan_mesh_batch, harp_plan_mesh_exact_batch,
 * harp_plan_mesh_h1f1b_batch; eq. dp_general's device index) and the paper's search in full around
 * it (harp_plan_mesh_h1f1b_sweep_batch); and the selection of the best plan of a batch
 * (harp_argmin_batch).
 *
 * Conventions.  Pointers marked DEVICE are device memory of the context's GPU, pointers marked
 * HOST are ordinary host memory.  The caller owns every buffer; the library allocates no device
 * memory.  Calls enqueue work on the given HIP stream (NULL = the default stream) and return
 * without waiting unless stated; outputs are valid once the stream has been synchronised.  Every
 * function returning int returns HARP_OK or a negative error code; harp_last_error gives the
 * message.  A context must not be used from two host threads at once.  No call falls back to the
 * CPU: without a usable GPU harp_create fails.
 */
#ifndef HARP_H
#define HARP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct harp_ctx harp_ctx;       /* opaque; host-side state of one GPU */
typedef struct harp_tables harp_tables; /* opaque host-side view of a caller-lent table buffer */

enum {
    HARP_OK = 0,
    HARP_ERR_INVALID_ARG = -1, /* null pointer, value out of range, malformed problem */
    HARP_ERR_SHAPE = -2,       /* sizes that do not fit together or exceed a stated limit */
    HARP_ERR_WORKSPACE = -3,   /* lent buffer too small or misaligned */
    HARP_ERR_HIP = -4,         /* a HIP runtime call failed */
    HARP_ERR_OVERFLOW = -5,    /* problem magnitudes outside the range the library guarantees */
    HARP_ERR_UNIMPLEMENTED = -6
};

/* per-candidate status written by harp_plan_batch and harp_score_1f1b */
enum { HARP_CAND_OK = 0, HARP_CAND_INFEASIBLE = 1, HARP_CAND_INVALID = 2 };

/* harp_plan_batch kernel selection (harp_set_plan_path).  Every path gives identical results. */
enum {
    HARP_PATH_AUTO = 0,    /* fastest path the tables allow */
    HARP_PATH_GENERIC = 1, /* int64 dense recurrence, one wave per DP cell; any degree, any size */
    HARP_PATH_FAST32 = 2   /* 32-bit times, bounded scan; needs harp_tables_fast32() != 0 */
};

#define HARP_INF INT64_MAX
#define HARP_MAX_TP_DEGREES 8
#define HARP_MAX_L_PLAN 65535

/* Creates the context for GPU `hip_device_ordinal`.  HARP_ERR_HIP when the device is missing. */
int harp_create(harp_ctx **out, int hip_device_ordinal);
void harp_destroy(harp_ctx *ctx);
/* Message of the last failed call on this context; owned by the context, never NULL. */
const char *harp_last_error(const harp_ctx *ctx);

/* The planning problem (paper section 5.2.2-5.2.3: layer sequence, profiled costs, subclusters).
 * All arrays row-major and contiguous. */
typedef struct {
    int32_t L;        /* operators, >= 1 */
    int32_t T;        /* GPU types, >= 1 */
    int32_t G;        /* device groups (homogeneous subclusters), >= 1 */
    int32_t M;        /* microbatches per iteration (the paper's B), >= 1 */
    int32_t ar_count; /* tensor-parallel all-reduces per operator per forward+backward, >= 0 */
    int32_t flags;    /* must be 0 */
    int32_t n_tp;     /* 1 .. HARP_MAX_TP_DEGREES */
    const int32_t *tp_degrees;     /* HOST   [n_tp] ascending, first == 1 */
    const int64_t *fwd_us;         /* DEVICE [T][L] forward time per operator and GPU type */
    const int64_t *bwd_us;         /* DEVICE [T][L] backward time */
    const int64_t *param_bytes;    /* DEVICE [L] parameters and buffers */
    const int64_t *stash_bytes;    /* DEVICE [L] activation kept per in-flight microbatch */
    const int64_t *act_bytes;      /* DEVICE [L] bytes crossing a cut placed right after l */
    const int32_t *group_type;     /* DEVICE [G] GPU type of each group */
    const int32_t *group_ndev;     /* DEVICE [G] devices in each group, >= 1 */
    const int64_t *type_mem_bytes; /* DEVICE [T] memory of one device */
    const int64_t *bw_bytes_per_us;/* DEVICE [G][G] symmetric, >= 1; diagonal = link inside a group */
} harp_problem;

/* Bytes of device memory the caller must lend to harp_build_segment_costs (0 on a malformed
 * problem).  Depends on L, T, G, n_tp only. */
size_t harp_tables_bytes(const harp_problem *problem);

/* Segment-cost tables (the stored stage costs that the search of section 5.2.3 looks up):
 * running sums over operators of compute time per GPU type, parameter bytes, stash bytes and
 * all-reduce time per (group, degree), so that any segment's time and memory is two lookups;
 * plus, when magnitudes allow, the 32-bit rows and per-link cut times of the fast path.
 * Also validates the device-resident problem (signs, ranges, magnitudes).
 *
 * table_buf: DEVICE, 256-byte aligned, at least harp_tables_bytes(problem) bytes; the returned
 * view aliases it and the problem's act_bytes, group_type, group_ndev, type_mem_bytes and
 * bw_bytes_per_us arrays, all of which must stay alive and unchanged until harp_tables_release.
 * Enqueues on `hip_stream` and returns; the verdict on the problem's values is collected by
 * harp_tables_finalize. */
int harp_build_segment_costs(harp_ctx *ctx, const harp_problem *problem, void *table_buf,
                             size_t table_bytes, harp_tables **out, void *hip_stream);

/* Waits for the build on its stream and returns its verdict: HARP_OK, HARP_ERR_INVALID_ARG
 * (negative input, bandwidth < 1, group type out of range, group without devices) or
 * HARP_ERR_OVERFLOW (sums that could leave int64, a stage or transfer time >= 2^47 us, or an
 * iteration time that could leave int64).  Idempotent.  harp_plan_batch and harp_score_1f1b call
 * it themselves on first use of a view. */
int harp_tables_finalize(harp_ctx *ctx, harp_tables *tables);

/* 1 when the finalized tables allow the 32-bit fast path (all degrees powers of two, every time
 * below 2^31 us, L <= 4096, per-link cut table within 256 MiB), else 0.  A batch runs on it when
 * its feasibility index (two tables of min(S_max, M, L) * T * n_tp rows of L + 1 16-bit entries)
 * stays within 256 MiB as well.  The min-max planner and the exact search use it for every such L;
 * the H-1F1B planner and the submesh planners, whose 32-bit kernels keep whole rows of several
 * arrays in LDS, use it up to L = 1024 and run on the int64 path beyond. */
int harp_tables_fast32(const harp_tables *tables);

/* DEVICE pointers into the table buffer, for inspection: running sums indexed [row][i],
 * i = 0..L, row pitch in elements returned through `pitch`.  PF [T], PP [1], PS [1],
 * PR [G * n_tp] (row g * n_tp + k for degree tp_degrees[k]). */
const int64_t *harp_tables_pf(const harp_tables *tables, size_t *pitch);
const int64_t *harp_tables_pp(const harp_tables *tables);
const int64_t *harp_tables_ps(const harp_tables *tables);
const int64_t *harp_tables_pr(const harp_tables *tables, size_t *pitch);

/* Frees the host-side view only. */
void harp_tables_release(harp_tables *tables);

/* A batch of candidates. */
typedef struct {
    int32_t C;     /* candidates, >= 0 */
    int32_t S_max; /* row length of the slot arrays, >= 1 */
    const int32_t *cand_S;     /* DEVICE [C]        stages of each candidate */
    const int32_t *cand_group; /* DEVICE [C][S_max] group of each slot (entries beyond S ignored) */
    const int32_t *cand_tp;    /* DEVICE [C][S_max] devices of each slot */
} harp_candidates;

/* Plans, all DEVICE, caller-allocated.  For a candidate whose status is not HARP_CAND_OK:
 * splits and dev_first all -1, bottleneck = iter_time = HARP_INF. */
typedef struct {
    int32_t *splits;     /* [C][S_max+1] cut positions b_0 = 0 < ... < b_S = L, rest -1 */
    int32_t *dev_first;  /* [C][S_max]   first global device id of each stage, rest -1; groups
                            number their devices consecutively in group order, a group's slots
                            take its devices in slot order */
    int64_t *bottleneck; /* [C] */
    int64_t *iter_time;  /* [C] */
    int32_t *status;     /* [C] HARP_CAND_* */
} harp_plans;

/* Chooses the kernel of harp_plan_batch for this context (HARP_PATH_*); for tests and
 * measurements.  HARP_ERR_INVALID_ARG on an unknown value. */
int harp_set_plan_path(harp_ctx *ctx, int path);

/* Bytes of DEVICE workspace harp_plan_batch needs for this batch (0 on malformed arguments). */
size_t harp_plan_workspace_bytes(harp_ctx *ctx, const harp_tables *tables,
                                 const harp_candidates *cands);

/* The search itself (section 5.2.3 recurrence per candidate, back-pointers, backtrack, and the
 * score of section 5.2.2), one wavefront or workgroup per candidate.  A candidate is HARP_CAND_INVALID when
 * S is outside 1..S_max, a group id or degree is not allowed, a group's slots are not adjacent
 * or use more devices than the group has; HARP_CAND_INFEASIBLE when S > L or no partition fits
 * in memory.  workspace: DEVICE, 256-byte aligned, >= harp_plan_workspace_bytes; contents are
 * scratch.  Needs L <= HARP_MAX_L_PLAN.  Asynchronous on `hip_stream`, except that the first use
 * of a view finalizes it. */
int harp_plan_batch(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                    const harp_plans *out, void *workspace, size_t workspace_bytes,
                    void *hip_stream);

/* harp_plan_batch for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs, statuses and kernel selection as harp_plan_batch; the planner workspace is a static
 * device array of HARP_STATIC_SCRATCH_BYTES inside the library (every GPU the library is used on
 * holds its own copy until the process ends; harp_create looks up its address).  The call
 * allocates and frees nothing, on the device or through any library.  It runs with as many
 * wavefronts (32-bit path, in fours) or workgroups (int64 path) as the array has room for, so large
 * batches are slower than with harp_plan_batch; a batch whose lists and reachability bands (about
 * 4 (S_max + 3) bytes per candidate), feasibility index (4 min(S_max, M, L) T n_tp (L + 1) bytes)
 * and the back-pointer slices of four wavefronts or one workgroup exceed the array is refused with
 * HARP_ERR_WORKSPACE and nothing is launched.  The tables must have been finalized (harp_tables_finalize) if the call is to stay
 * free of host waits.  Every call on one GPU uses the same array: calls that overlap on one GPU
 * (two streams, two contexts, two host threads) race; calls queued on one stream do not.  The
 * array keeps the previous call's contents; the kernels clear the counters they rely on. */
#define HARP_STATIC_SCRATCH_BYTES (32u << 20)
int harp_plan_batch_static(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                           const harp_plans *out, void *hip_stream);

/* Measurement support: harp_plan_batch with the work it does counted (an instrumented build of the
 * same kernel; slower, same outputs).  work: DEVICE [4], receives the number of transitions
 * (s, i, j) whose value max(D[s][j], time, comm) the kernel evaluated, the DP cells (s, i) it filled,
 * the groups of four previous cuts it read, and the candidates that reached the recurrence (the
 * others were rejected by the memory bounds of the pre-pass).  32-bit path only
 * (HARP_ERR_UNIMPLEMENTED otherwise).  Everything else as harp_plan_batch. */
int harp_plan_batch_count_work(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                               const harp_plans *out, void *workspace, size_t workspace_bytes,
                               uint64_t *work, void *hip_stream);

/* The exact optimum of eq. gpipe_cost_model per candidate: the sweep over the stage-time cap t_max
 * of section 5.2.4 (2), between t_S (the smallest feasible cap, found by the min-max search of
 * harp_plan_batch, which this call runs first) and t_E = ceil(T(t_S) / B), with the capped
 * least-sum recurrence of section 5.2.3 at each cap.  Outputs as for harp_plan_batch, except that
 * splits is the partition of least iteration time (ties: the smaller bottleneck, then the lowest
 * previous cut at every stage of the capped recurrence), bottleneck its largest stage or transfer
 * time and iter_time its iteration time; statuses are those of harp_plan_batch.
 * n_passes: DEVICE [C] or NULL; receives the number of capped recurrences run for the candidate
 * (0 when it has no plan or a single stage).
 * Kernel selection as for harp_plan_batch (harp_set_plan_path; identical results on every path);
 * workspace as for harp_plan_batch.  Asynchronous on `hip_stream`, except that the first use of a view
 * finalizes it. */
int harp_plan_exact_batch(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                          const harp_plans *out, int32_t *n_passes, void *workspace,
                          size_t workspace_bytes, void *hip_stream);

/* A batch of group orderings for harp_plan_mesh_batch: candidate c runs S = ord_S[c] stages on the
 * groups ord_group[c][0 .. ord_G[c]-1], in that order; the planner decides how each group's
 * devices are cut into stages. */
typedef struct {
    int32_t C;      /* orderings, >= 0 */
    int32_t G_max;  /* row length of ord_group, 1..1024 */
    int32_t S_max;  /* row length of the per-stage outputs, >= every ord_S */
    const int32_t *ord_S;     /* DEVICE [C] */
    const int32_t *ord_G;     /* DEVICE [C] groups listed, 1..G_max */
    const int32_t *ord_group; /* DEVICE [C][G_max] distinct group ids (entries beyond ord_G ignored) */
} harp_orderings;

/* Bytes of DEVICE workspace harp_plan_mesh_batch needs (0 on malformed arguments; finalizes the
 * view, because the size depends on the number of devices in the problem). */
size_t harp_plan_mesh_workspace_bytes(harp_ctx *ctx, harp_tables *tables, const harp_orderings *orders);

/* The search with the submesh of every stage chosen inside the recurrence (section 5.2.3, the third
 * index of eq. dp_general): state = (stages placed, operators placed, devices used across the
 * ordered groups).  A stage takes tp devices of the group its device offset falls in, tp an
 * allowed degree that does not reach beyond that group; the cut behind a stage that exhausts its
 * group crosses to the next group's link.  Every device of every listed group is used.  Min-max
 * form with the classic 1F1B counts, exactly the definitions of harp_plan_batch; ties: lowest
 * previous cut, then smallest degree.  The result for an ordering equals the best harp_plan_batch
 * result over all slicings of its groups into S stages.
 * out as for harp_plan_batch (rows of length S_max + 1 / S_max); stage_group, stage_tp: DEVICE
 * [C][S_max], the slicing found (-1 beyond S or without a plan).  HARP_CAND_INVALID: S outside
 * 1..S_max, ord_G outside 1..G_max, a group id out of range or listed twice; HARP_CAND_INFEASIBLE:
 * S > L, S < ord_G, S > devices, or no plan fits in memory.  At most 65535 devices, and
 * (devices + 1) x (L + 1) below 2^31 (HARP_ERR_SHAPE otherwise; also for the other entry points
 * with a device index).
 * Asynchronous on `hip_stream`, except that the first use of a view finalizes it. */
int harp_plan_mesh_batch(harp_ctx *ctx, harp_tables *tables, const harp_orderings *orders,
                         const harp_plans *out, int32_t *stage_group, int32_t *stage_tp,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* The paper's full search for every ordering (sections 5.2.3 and 5.2.4 (2)): the capped least-sum
 * table of eq. dp_general with its device index, swept over the cap t_max between t_S (what
 * harp_plan_mesh_batch finds) and t_E = ceil(T(t_S) / B).  Outputs as harp_plan_mesh_batch, except
 * that the plan is the one of least iteration time over every slicing and partition (ties: smaller
 * bottleneck, then lowest previous cut and smallest degree at every stage of the capped table),
 * bottleneck its largest stage or transfer time and iter_time its iteration time.  n_passes: DEVICE
 * [C] or NULL, capped tables filled per ordering.  Workspace as for harp_plan_mesh_batch. */
int harp_plan_mesh_exact_batch(harp_ctx *ctx, harp_tables *tables, const harp_orderings *orders,
                               const harp_plans *out, int32_t *stage_group, int32_t *stage_tp,
                               int32_t *n_passes, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* The paper's recurrence in full for one cap per ordering (section 5.2.3): eq. dp_general with its
 * device index and the H-1F1B warm-up count of eq. dp_ni in the state, suffix direction, the memory
 * constraint eq. mem_cons with that count; delta, the cap on counts and the tie rule as for
 * harp_plan_h1f1b_batch (ties: lowest end cut, then smallest degree); device model as for
 * harp_plan_mesh_batch.  t_max: DEVICE [C].  Outputs: out as for harp_plan_mesh_batch with
 * bottleneck = the plan's own largest time and iter_time = least sum + (M - 1) t_max[c];
 * stage_group, stage_tp, warmup: DEVICE [C][S_max].  With single-device groups this is
 * harp_plan_h1f1b_batch on the one slicing there is.  Workspace as for harp_plan_mesh_batch. */
int harp_plan_mesh_h1f1b_batch(harp_ctx *ctx, harp_tables *tables, const harp_orderings *orders,
                               const int64_t *t_max, const harp_plans *out, int32_t *stage_group,
                               int32_t *stage_tp, int32_t *warmup, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/* The search of section 5.2.4 (2) around that recurrence, per ordering: the cap t_max is swept over
 * the sorted, distinct candidate values, from the smallest feasible one up to t_E = ceil(T / B), and
 * harp_plan_mesh_h1f1b_batch's recurrence is evaluated at every one of them.  Candidate values of an
 * ordering: every stage time of a listed group, an allowed degree not above the group's device
 * count and an operator range [j, i), 0 <= j < i <= L; and every transfer time of a cut
 * 1 <= i <= L - 1 on the links the ordering can use (inside each listed group, and from each
 * listed group to the one after it).  The sweep starts at the bottleneck harp_plan_mesh_batch
 * finds (no smaller cap admits a plan, and H-1F1B's counts are never below the classic ones), takes
 * the values in increasing order, fixes t_E from the T of the first cap that has a plan, and ends
 * past t_E, when the values run out, or after max_caps (>= 1) caps.  The answer is the plan with
 * the smallest T = least sum + (M - 1) cap, the lower cap on equal T.  Outputs as
 * harp_plan_mesh_h1f1b_batch at that cap; t_max_out: DEVICE [C], the cap of the answer (INT64_MAX
 * when there is none); n_caps: DEVICE [C] or NULL, caps tried.  HARP_CAND_INFEASIBLE when no tried
 * cap has a plan.  The work per ordering is caps tried x one harp_plan_mesh_h1f1b_batch pass; when
 * the batch alone would leave compute units idle, several workgroups share the caps of one ordering
 * (same results).  Workspace: harp_plan_mesh_sweep_workspace_bytes (the slices of the resident
 * workgroups plus up to 33 kept plans per ordering), 256-byte aligned, contents irrelevant. */
size_t harp_plan_mesh_sweep_workspace_bytes(harp_ctx *ctx, harp_tables *tables, const harp_orderings *orders);
int harp_plan_mesh_h1f1b_sweep_batch(harp_ctx *ctx, harp_tables *tables, const harp_orderings *orders,
                                     int32_t max_caps, const harp_plans *out, int32_t *stage_group,
                                     int32_t *stage_tp, int32_t *warmup, int64_t *t_max_out,
                                     int32_t *n_caps, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/* The same search for candidates, whose slicing is fixed: the cap swept over the candidate values
 * from the bottleneck harp_plan_batch finds up to t_E = ceil(T / B), harp_plan_h1f1b_batch's
 * recurrence at every one of them.  Candidate values of a candidate: every stage time of one of
 * its slots (its group, its degree) over an operator range [j, i), 0 <= j < i <= L, and every
 * transfer time of a cut 1 <= i <= L - 1 on the link between two consecutive slots.  Order of the
 * sweep, t_E, the answer, max_caps, t_max_out and n_caps as for harp_plan_mesh_h1f1b_sweep_batch;
 * out and warmup as for harp_plan_h1f1b_batch at the cap of the answer; statuses as for
 * harp_plan_batch, and HARP_CAND_INFEASIBLE when no tried cap has a plan.  It runs on the submesh
 * kernels with every stage's group and degree given (one device offset per stage), not on the hot
 * path's: meant for batches of moderate size.  Workspace: harp_plan_h1f1b_sweep_workspace_bytes,
 * 256-byte aligned, contents irrelevant. */
size_t harp_plan_h1f1b_sweep_workspace_bytes(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands);
int harp_plan_h1f1b_sweep_batch(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                                int32_t max_caps, const harp_plans *out, int32_t *warmup,
                                int64_t *t_max_out, int32_t *n_caps, void *workspace,
                                size_t workspace_bytes, void *hip_stream);

/* The capped recurrence under the H-1F1B scheduler (sections 4.1 and 5.2.3): for candidate c and
 * the cap t_max[c] on every stage and transfer time (constraints (i), (ii)), the suffix recurrence
 * of eq. dp_general with the warm-up launch count carried in the state (eq. dp_ni) and used by the
 * memory constraint (eq. mem_cons):
 *   delta(c_cut; t_max) = 1 if 2 c_cut <= floor(t_max / 64), else 1 + ceil((2 c_cut - floor(t_max / 64)) / t_max)
 *   N(last stage) = 1,  N(stage s) = min(M, delta(cut behind s) + N(stage s + 1))        (eq. Ni)
 *   a state keeps the continuation of least sum (lowest end cut among equal sums) and its N.
 * t_max: DEVICE [C] (negative: no plan; above min(2^47 - 1, INT64_MAX / (3 L + M)), beyond which
 * sum + (M - 1) t_max could leave int64: the candidate is HARP_CAND_INVALID; the same bound holds
 * for every entry point that takes a cap).  warmup: DEVICE [C][S_max], receives N per stage, -1 beyond
 * S and for candidates without a plan.  out as for harp_plan_batch, with bottleneck = the plan's own
 * largest stage or transfer time (<= t_max[c]) and iter_time = least sum + (M - 1) t_max[c], the
 * T(t_max) of section 5.2.3; HARP_CAND_INFEASIBLE when no partition satisfies (i)-(iii) under the
 * cap.  Kernel selection, workspace and asynchrony as for harp_plan_batch. */
int harp_plan_h1f1b_batch(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                          const int64_t *t_max, const harp_plans *out, int32_t *warmup,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Warm-up counts and iteration time of caller-chosen partitions under H-1F1B with the cap
 * t_max[c] (section 4.1, eq. Ni; delta as above): splits DEVICE [C][S_max+1], t_max DEVICE [C];
 * outputs DEVICE: warmup [C][S_max], bottleneck (the partition's own), iter_time = sum of
 * (t + 2c) + (M - 1) t_max[c], status.  HARP_CAND_INVALID for a malformed candidate or cuts,
 * HARP_CAND_INFEASIBLE when a stage or transfer time exceeds the cap or a stage does not fit in
 * memory with its count (then warmup is -1 and the times HARP_INF). */
int harp_score_h1f1b(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                     const int32_t *splits, const int64_t *t_max, int32_t *warmup,
                     int64_t *bottleneck, int64_t *iter_time, int32_t *status, void *hip_stream);

/* Scores caller-chosen partitions with eq. gpipe_cost_model (section 5.2.2):
 * splits DEVICE [C][S_max+1].  Status HARP_CAND_INVALID when the candidate is malformed or its
 * cuts are not strictly increasing from 0 to L; HARP_CAND_INFEASIBLE when a stage does not fit
 * in memory; times are HARP_INF unless the status is HARP_CAND_OK.  Kernel selection as for
 * harp_plan_batch (harp_set_plan_path; the kernel for the 32-bit rows takes S_max <= 64, larger
 * batches run on the int64 one; identical results; HARP_ERR_UNIMPLEMENTED when HARP_PATH_FAST32 is
 * set and the tables have no 32-bit rows). */
int harp_score_1f1b(harp_ctx *ctx, harp_tables *tables, const harp_candidates *cands,
                    const int32_t *splits, int64_t *bottleneck, int64_t *iter_time,
                    int32_t *status, void *hip_stream);

/* Final selection over the batch (the min over evaluated candidates of section 5.2.3): smallest
 * iter_time among candidates with status HARP_CAND_OK, lowest index on ties.  best_time and
 * best_index are DEVICE scalars; -1 and HARP_INF when no candidate qualifies. */
int harp_argmin_batch(harp_ctx *ctx, int32_t C, const int64_t *iter_time, const int32_t *status,
                      int64_t *best_time, int32_t *best_index, void *hip_stream);

/* Measurement support for the roofline of the planner kernels (which are bound by integer vector
 * arithmetic, not by a contraction or by memory): launches `blocks` workgroups of 256 threads in
 * which every lane issues iters * 16 32-bit integer vector operations (8 independent chains of one
 * add and one max).  The caller times the launch; lane-operations = blocks * 256 * iters * 16.
 * sink: DEVICE [1], written only in a case that practically never occurs (it keeps the arithmetic
 * alive).  Asynchronous on `hip_stream`. */
int harp_measure_valu_int32(harp_ctx *ctx, int32_t blocks, int32_t iters, uint32_t *sink,
                            void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HARP_H */
