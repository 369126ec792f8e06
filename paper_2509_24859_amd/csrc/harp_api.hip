// Host layer of the C ABI declared in include/harp.h: argument checks, layout of the caller-lent
// buffers, kernel selection and launches.  Allocates no device memory (one small pinned host
// buffer per context receives the build verdict).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "harp_internal.h"

using namespace harp;

struct harp_ctx {
    int device;
    int n_cu;
    int plan_path;
    BuildHeader *pinned;   // host, pinned
    unsigned char *scratch;   // this device's copy of the library's static scratch array
    char err[512];
};

// Planner workspace of harp_plan_batch_static.  In host code this name is only a handle for
// hipGetSymbolAddress: harp_create asks for the device address once per context, with the
// context's device current, and every later use goes through harp_ctx::scratch.
static __device__ __align__(256) unsigned char scratch[HARP_STATIC_SCRATCH_BYTES];

struct harp_tables {
    TablesDev dev;
    BuildLimits lim;
    hipStream_t build_stream;
    int device;
    bool finalized;
    int verdict;
    bool fast32;
    long long total_devices;
    size_t bytes;
};

namespace {

int fail(harp_ctx *ctx, int code, const char *fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

int hip_fail(harp_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, HARP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t header, group_base, rows, chunk_sums, p32, cm, total;
    int64_t pitch, pitch32;
    int n_chunks;
    bool fast;
};

bool problem_shape_ok(const harp_problem *p) {
    if (!p) return false;
    if (p->L < 1 || p->L > (1 << 24) || p->T < 1 || p->T > 4096 || p->G < 1 || p->G > 4096) return false;
    if (p->M < 1 || p->ar_count < 0 || p->ar_count > (1 << 20) || p->flags != 0) return false;
    if (p->n_tp < 1 || p->n_tp > kMaxTp || !p->tp_degrees) return false;
    if (p->tp_degrees[0] != 1) return false;
    for (int k = 1; k < p->n_tp; ++k)
        if (p->tp_degrees[k] <= p->tp_degrees[k - 1] || p->tp_degrees[k] > 65536) return false;
    if (int64_t(p->T) + 2 + int64_t(p->G) * p->n_tp > 65535) return false;
    return true;
}

Layout make_layout(const harp_problem *p) {
    Layout y;
    const size_t L1 = size_t(p->L) + 1;
    y.pitch = (int64_t)align_up(L1, 16);
    y.pitch32 = (int64_t)align_up(L1, 16);
    y.n_chunks = (p->L + 255) / 256;     // scan scratch sized for the finest chunking (one wavefront)
    const size_t n_rows = size_t(p->T) + 2 + size_t(p->G) * p->n_tp;
    size_t off = 0;
    y.header = off; off += 256;
    y.group_base = off; off += align_up(size_t(p->G) * 4, 256);
    y.rows = off; off += align_up(n_rows * y.pitch * 8, 256);
    y.chunk_sums = off; off += align_up(n_rows * size_t(y.n_chunks) * 8, 256);
    bool pow2 = true;
    for (int k = 0; k < p->n_tp; ++k) pow2 = pow2 && (p->tp_degrees[k] & (p->tp_degrees[k] - 1)) == 0;
    const size_t cm_bytes = size_t(p->G) * p->G * y.pitch32 * 4;
    y.fast = pow2 && p->L <= kFastMaxL && cm_bytes <= kFastCutTableLimit &&
             size_t(p->G) * p->n_tp + size_t(p->G) * p->G <= 65535;
    y.p32 = off;
    if (y.fast) off += align_up(size_t(p->G) * p->n_tp * y.pitch32 * 4, 256);
    y.cm = off;
    if (y.fast) off += align_up(cm_bytes, 256);
    y.total = off;
    return y;
}

int finalize_tables(harp_ctx *ctx, harp_tables *t) {
    if (t->finalized) return t->verdict;
    hipError_t e = hipMemcpyAsync(ctx->pinned, t->dev.header, sizeof(BuildHeader), hipMemcpyDeviceToHost,
                                  t->build_stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "reading the build verdict");
    e = hipStreamSynchronize(t->build_stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "waiting for the table build");
    t->finalized = true;
    t->fast32 = ctx->pinned->fast32 != 0;
    t->total_devices = ctx->pinned->total_devices;
    if (ctx->pinned->bad_arg)
        t->verdict = fail(ctx, HARP_ERR_INVALID_ARG,
                          "problem arrays hold a negative value, a bandwidth below 1, a group type out of range or an empty group");
    else if (ctx->pinned->overflow)
        t->verdict = fail(ctx, HARP_ERR_OVERFLOW,
                          "problem magnitudes are outside the supported range (stage or transfer time >= 2^47 us, or sums that could leave int64)");
    else
        t->verdict = HARP_OK;
    return t->verdict;
}

int check_batch(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (!t || !cd) return fail(ctx, HARP_ERR_INVALID_ARG, "null tables or candidates");
    if (t->device != ctx->device) return fail(ctx, HARP_ERR_INVALID_ARG, "tables belong to another device");
    if (cd->C < 0) return fail(ctx, HARP_ERR_INVALID_ARG, "C must be >= 0");
    if (cd->C >= (1 << 30)) return fail(ctx, HARP_ERR_SHAPE, "at most 2^30 - 1 candidates per batch");
    if (cd->S_max < 1 || cd->S_max > kMaxStages)
        return fail(ctx, HARP_ERR_SHAPE, "S_max must be in 1..%d", kMaxStages);
    if (cd->C > 0 && (!cd->cand_S || !cd->cand_group || !cd->cand_tp))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null candidate array");
    if (t->dev.L > HARP_MAX_L_PLAN) return fail(ctx, HARP_ERR_SHAPE, "planning needs L <= %d", HARP_MAX_L_PLAN);
    return finalize_tables(ctx, t);
}

// Workgroups of the planner kernels that work one candidate per workgroup.
int n_plan_groups(const harp_ctx *ctx, int C, bool fast, int L, int S_max) {
    int resident = fast ? plan_fast_groups(L, S_max, ctx->n_cu) : ctx->n_cu * 8;
    if (resident < 1) resident = 1;
    return C < resident ? (C < 1 ? 1 : C) : resident;
}

// Back-pointer slices of the 32-bit path: one per resident wavefront of the min-max kernel (whole
// workgroups of kFastWaves) or per workgroup of the kernels built on it, whichever is more.
int n_fast_slices(const harp_ctx *ctx, int C, int L, int S_max) {
    int want = plan_fast_waves(L, S_max, ctx->n_cu);
    const int groups = plan_fast_groups(L, S_max, ctx->n_cu);
    if (want < groups) want = groups;
    if (want > C) want = C;
    want = (want + kFastWaves - 1) / kFastWaves * kFastWaves;
    return want < kFastWaves ? kFastWaves : want;
}

// Workspace of the min-max planner on the path that will run, with `units` slices (32-bit path) or
// workgroups (int64 path).
// The pre-pass keeps a feasibility index whose size grows with min(S_max, M) * T * n_tp * L; batches
// for which it would pass the limit run on the int64 path without bands.
bool fast_batch_ok(const harp_tables *t, const harp_candidates *cd) {
    return t->dev.L <= kIndexMaxL && plan_fast_index_bytes(t->dev, cd->S_max) <= kFastIndexLimit;
}

size_t plan_bytes_on_path(const harp_tables *t, const harp_candidates *cd, bool fast, int units) {
    if (fast) return plan_fast_ws_bytes(t->dev, cd->S_max, cd->C, units) + 256;
    // int64 path: the pre-pass area (lists, bands, index) when the index fits, then the workgroups' slices
    const size_t prepass = fast_batch_ok(t, cd) ? plan_fast_ws_bytes(t->dev, cd->S_max, cd->C, 0) : 0;
    return prepass + size_t(units) * plan_generic_ws_per_group(t->dev.L, cd->S_max) + 256;
}

// Workgroups of the submesh planner: resident ones, fewer when their slices would pass 16 GiB.
int n_mesh_groups(const harp_ctx *ctx, int C, size_t per_group, int threads) {
    long long n = (long long)ctx->n_cu * (2048 / threads);         // as many wavefronts as a CU holds
    const long long fit = (long long)((size_t(16) << 30) / (per_group ? per_group : 1));
    if (n > fit) n = fit;
    if (n > C) n = C;
    return n < 1 ? 1 : int(n);
}

// The search over the cap puts W workgroups on one ordering when the batch alone would leave
// compute units idle; its workspace holds the slices of the resident workgroups and W + 1 kept
// plans per ordering.
struct SweepLayout {
    int threads, groups, W, W_climb;
    size_t per_group, bytes;
};
SweepLayout sweep_layout(const harp_ctx *ctx, const harp_tables *t, const harp_orderings *od) {
    SweepLayout s;
    s.per_group = plan_mesh_ws_per_group(t->dev.L, od->S_max, t->total_devices);
    // up to 32 walkers share an ordering, so the batch fills the chip 32 times sooner than for one pass
    const long long walkers = (long long)(od->C > 0 ? od->C : 1) * 32;
    s.threads = plan_mesh_threads(t->dev.L, t->total_devices, int(walkers < (1 << 30) ? walkers : (1 << 30)), ctx->n_cu);
    long long resident = (long long)ctx->n_cu * (2048 / s.threads);
    const long long fit = (long long)((size_t(16) << 30) / (s.per_group ? s.per_group : 1));
    if (resident > fit) resident = fit;
    if (resident < 1) resident = 1;
    const long long C = od->C > 0 ? od->C : 1;
    long long W = resident / C;
    W = W < 1 ? 1 : (W > 32 ? 32 : W);
    s.W = int(W);
    // the climb to the first cap with a plan is deep for a few orderings only (those whose memory
    // fits once a larger cap has lowered the counts): it gets four times the walkers, drawn from
    // the same ticket, so that workgroups that are done with easy orderings join the deep ones
    long long Wc = 4 * resident / C;
    Wc = Wc < W ? W : (Wc > 32 ? 32 : Wc);
    s.W_climb = int(Wc);
    s.W = int(Wc);        // the rest of the sweep as well: more, shorter items even out orderings with many caps
    s.groups = int(resident < C * Wc ? resident : C * Wc);
    s.bytes = 256 + size_t(s.groups) * s.per_group + size_t(C) * size_t(Wc + 1) * plan_mesh_sweep_slot_bytes(od->S_max) +
              ((size_t(C) * (sizeof(int64_t) + sizeof(int)) + 255) & ~size_t(255));
    return s;
}

int check_orderings(harp_ctx *ctx, harp_tables *t, const harp_orderings *od) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (!t || !od) return fail(ctx, HARP_ERR_INVALID_ARG, "null tables or orderings");
    if (t->device != ctx->device) return fail(ctx, HARP_ERR_INVALID_ARG, "tables belong to another device");
    if (od->C < 0) return fail(ctx, HARP_ERR_INVALID_ARG, "C must be >= 0");
    if (od->S_max < 1 || od->S_max > kMaxStages) return fail(ctx, HARP_ERR_SHAPE, "S_max must be in 1..%d", kMaxStages);
    if (od->G_max < 1 || od->G_max > kMaxOrderGroups)
        return fail(ctx, HARP_ERR_SHAPE, "G_max must be in 1..%d", kMaxOrderGroups);
    if (od->C > 0 && (!od->ord_S || !od->ord_G || !od->ord_group))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null ordering array");
    if (t->dev.L > HARP_MAX_L_PLAN) return fail(ctx, HARP_ERR_SHAPE, "planning needs L <= %d", HARP_MAX_L_PLAN);
    return finalize_tables(ctx, t);
}

// The kernels with a device index address their state with 32-bit products of these two.
bool mesh_index_fits(const harp_tables *t) {
    return (t->total_devices + 1) * (int64_t(t->dev.L) + 1) < (int64_t(1) << 31);
}

// The 32-bit tables serve the min-max planner up to kFastMaxL operators; the kernels that keep
// whole rows of several arrays in LDS (H-1F1B, the submesh planners) stop at kFastRowsMaxL.
bool fast_allowed(const harp_tables *t, bool whole_rows) {
    return t->fast32 && (!whole_rows || t->dev.L <= kFastRowsMaxL);
}
bool use_fast_rows(const harp_ctx *ctx, const harp_tables *t) {
    return fast_allowed(t, true) && ctx->plan_path != HARP_PATH_GENERIC;
}
bool use_fast(const harp_ctx *ctx, const harp_tables *t, const harp_candidates *cd, bool whole_rows) {
    return fast_allowed(t, whole_rows) && ctx->plan_path != HARP_PATH_GENERIC && fast_batch_ok(t, cd);
}

}  // namespace

extern "C" {

int harp_create(harp_ctx **out, int hip_device_ordinal) {
    if (!out) return HARP_ERR_INVALID_ARG;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || hip_device_ordinal < 0 || hip_device_ordinal >= n)
        return HARP_ERR_HIP;
    if (hipSetDevice(hip_device_ordinal) != hipSuccess) return HARP_ERR_HIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, hip_device_ordinal) != hipSuccess) return HARP_ERR_HIP;
    harp_ctx *ctx = new (std::nothrow) harp_ctx;
    if (!ctx) return HARP_ERR_INVALID_ARG;
    ctx->device = hip_device_ordinal;
    ctx->n_cu = prop.multiProcessorCount;
    ctx->plan_path = HARP_PATH_AUTO;
    ctx->pinned = nullptr;
    ctx->scratch = nullptr;
    ctx->err[0] = 0;
    // each GPU holds its own copy of the static scratch array at its own address
    if (hipGetSymbolAddress(reinterpret_cast<void **>(&ctx->scratch), HIP_SYMBOL(scratch)) != hipSuccess ||
        !ctx->scratch) {
        delete ctx;
        return HARP_ERR_HIP;
    }
    if (hipHostMalloc(reinterpret_cast<void **>(&ctx->pinned), sizeof(BuildHeader), hipHostMallocDefault) != hipSuccess) {
        delete ctx;
        return HARP_ERR_HIP;
    }
    *out = ctx;
    return HARP_OK;
}

void harp_destroy(harp_ctx *ctx) {
    if (!ctx) return;
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    delete ctx;
}

const char *harp_last_error(const harp_ctx *ctx) { return ctx ? ctx->err : "null context"; }

size_t harp_tables_bytes(const harp_problem *problem) {
    if (!problem_shape_ok(problem)) return 0;
    return make_layout(problem).total;
}

int harp_build_segment_costs(harp_ctx *ctx, const harp_problem *p, void *table_buf, size_t table_bytes,
                             harp_tables **out, void *hip_stream) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (!out) return fail(ctx, HARP_ERR_INVALID_ARG, "null output pointer");
    *out = nullptr;
    if (!p) return fail(ctx, HARP_ERR_INVALID_ARG, "null problem");
    if (!problem_shape_ok(p))
        return fail(ctx, HARP_ERR_INVALID_ARG,
                    "malformed problem header (L, T, G, M, ar_count, flags or tp_degrees out of range)");
    if (!p->fwd_us || !p->bwd_us || !p->param_bytes || !p->stash_bytes || !p->act_bytes || !p->group_type ||
        !p->group_ndev || !p->type_mem_bytes || !p->bw_bytes_per_us)
        return fail(ctx, HARP_ERR_INVALID_ARG, "null problem array");
    const Layout y = make_layout(p);
    if (!table_buf || (reinterpret_cast<uintptr_t>(table_buf) & 255) != 0)
        return fail(ctx, HARP_ERR_WORKSPACE, "table buffer must be a 256-byte aligned device pointer");
    if (table_bytes < y.total)
        return fail(ctx, HARP_ERR_WORKSPACE, "table buffer holds %zu bytes, %zu needed", table_bytes, y.total);
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");

    harp_tables *t = new (std::nothrow) harp_tables;
    if (!t) return fail(ctx, HARP_ERR_INVALID_ARG, "out of host memory");
    unsigned char *base = static_cast<unsigned char *>(table_buf);
    TablesDev &d = t->dev;
    d.L = p->L; d.T = p->T; d.G = p->G; d.M = p->M; d.n_tp = p->n_tp; d.ar_count = p->ar_count;
    for (int k = 0; k < kMaxTp; ++k) { d.tp[k] = 0; d.tp_shift[k] = -1; }
    for (int k = 0; k < p->n_tp; ++k) {
        const int v = p->tp_degrees[k];
        d.tp[k] = v;
        if ((v & (v - 1)) == 0) { int s = 0; while ((1 << s) < v) ++s; d.tp_shift[k] = s; }
    }
    d.pitch = y.pitch; d.pitch32 = y.pitch32;
    d.header = reinterpret_cast<BuildHeader *>(base + y.header);
    d.group_base = reinterpret_cast<int32_t *>(base + y.group_base);
    d.rows = reinterpret_cast<int64_t *>(base + y.rows);
    d.chunk_sums = reinterpret_cast<int64_t *>(base + y.chunk_sums);
    d.P32 = y.fast ? reinterpret_cast<uint32_t *>(base + y.p32) : nullptr;
    d.CM = y.fast ? reinterpret_cast<uint32_t *>(base + y.cm) : nullptr;
    d.fwd_us = p->fwd_us; d.bwd_us = p->bwd_us; d.param_bytes = p->param_bytes;
    d.stash_bytes = p->stash_bytes; d.act_bytes = p->act_bytes; d.type_mem = p->type_mem_bytes;
    d.bw = p->bw_bytes_per_us; d.group_type = p->group_type; d.group_ndev = p->group_ndev;

    const int64_t tp_max = p->tp_degrees[p->n_tp - 1];
    const int64_t num_mul = int64_t(p->ar_count) * 2 * (tp_max - 1);
    t->lim.act_max = num_mul > 0 ? INT64_MAX / num_mul : INT64_MAX;
    t->lim.bw_max = INT64_MAX / tp_max;
    t->lim.mem_max = INT64_MAX / tp_max;
    t->lim.want_fast = y.fast ? 1 : 0;
    t->build_stream = static_cast<hipStream_t>(hip_stream);
    t->device = ctx->device;
    t->finalized = false;
    t->verdict = HARP_OK;
    t->fast32 = false;
    t->total_devices = 0;
    t->bytes = y.total;

    launch_build(d, t->lim, t->build_stream);
    e = hipGetLastError();
    if (e != hipSuccess) { delete t; return hip_fail(ctx, e, "launching the table build"); }
    *out = t;
    return HARP_OK;
}

int harp_tables_finalize(harp_ctx *ctx, harp_tables *tables) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (!tables) return fail(ctx, HARP_ERR_INVALID_ARG, "null tables");
    return finalize_tables(ctx, tables);
}

int harp_tables_fast32(const harp_tables *tables) { return tables && tables->finalized && tables->fast32; }

const int64_t *harp_tables_pf(const harp_tables *t, size_t *pitch) {
    if (!t) return nullptr;
    if (pitch) *pitch = (size_t)t->dev.pitch;
    return t->dev.PF(0);
}
const int64_t *harp_tables_pp(const harp_tables *t) { return t ? t->dev.PP() : nullptr; }
const int64_t *harp_tables_ps(const harp_tables *t) { return t ? t->dev.PS() : nullptr; }
const int64_t *harp_tables_pr(const harp_tables *t, size_t *pitch) {
    if (!t) return nullptr;
    if (pitch) *pitch = (size_t)t->dev.pitch;
    return t->dev.PR(0, 0);
}

void harp_tables_release(harp_tables *tables) { delete tables; }

int harp_set_plan_path(harp_ctx *ctx, int path) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (path != HARP_PATH_AUTO && path != HARP_PATH_GENERIC && path != HARP_PATH_FAST32)
        return fail(ctx, HARP_ERR_INVALID_ARG, "unknown plan path %d", path);
    ctx->plan_path = path;
    return HARP_OK;
}

size_t harp_plan_workspace_bytes(harp_ctx *ctx, const harp_tables *t, const harp_candidates *cd) {
    if (!ctx || !t || !cd || cd->C < 0 || cd->S_max < 1 || cd->S_max > kMaxStages) return 0;
    if (t->dev.L > HARP_MAX_L_PLAN) return 0;
    // sized for whichever path may run, so that the answer does not depend on the build verdict
    const int C = cd->C;
    const size_t per_group = plan_generic_ws_per_group(t->dev.L, cd->S_max) >
                                     plan_generic_h1f1b_ws_per_group(t->dev.L, cd->S_max)
                                 ? plan_generic_ws_per_group(t->dev.L, cd->S_max)
                                 : plan_generic_h1f1b_ws_per_group(t->dev.L, cd->S_max);
    size_t gen = size_t(n_plan_groups(ctx, C, false, t->dev.L, cd->S_max)) * per_group;
    if (fast_batch_ok(t, cd)) gen += plan_fast_ws_bytes(t->dev, cd->S_max, C, 0);
    size_t fast = 0;
    if (t->lim.want_fast && fast_batch_ok(t, cd))
        fast = plan_fast_ws_bytes(t->dev, cd->S_max, C, n_fast_slices(ctx, C, t->dev.L, cd->S_max));
    return (gen > fast ? gen : fast) + 256;
}

}  // extern "C"

namespace {

// What the candidate planners share: argument checks, the path that will run, and how many
// workgroups and back-pointer slices the lent memory allows.
struct PlanCall {
    CandDev c;
    PlansDev o;
    bool fast;
    bool banded;     // int64 path: the min-max planner runs behind the pre-pass (the index fits)
    int groups;      // workgroups of the one-candidate-per-workgroup kernels
    int slices;      // back-pointer slices of the 32-bit path (>= groups, a multiple of kFastWaves)
    hipStream_t st;
};

// limit_bytes: the memory at hand.  With shrink the unit count is cut down to what fits (the
// static-scratch entry point); without, the full resident count must fit.
int plan_prepare(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const harp_plans *out,
                 bool extra_null, bool whole_rows, const void *workspace, size_t limit_bytes, bool shrink,
                 void *hip_stream, PlanCall &pc) {
    int rc = check_batch(ctx, t, cd);
    if (rc != HARP_OK) return rc;
    if (!out || extra_null ||
        (cd->C > 0 && (!out->splits || !out->dev_first || !out->bottleneck || !out->iter_time || !out->status)))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    if (ctx->plan_path == HARP_PATH_FAST32 && !(fast_allowed(t, whole_rows) && fast_batch_ok(t, cd)))
        return fail(ctx, HARP_ERR_UNIMPLEMENTED,
                    "the 32-bit path was requested but these tables or this batch do not allow it");
    pc.c = CandDev{ cd->C, cd->S_max, cd->cand_S, cd->cand_group, cd->cand_tp };
    pc.o = PlansDev{ out->splits, out->dev_first, out->bottleneck, out->iter_time, out->status };
    pc.fast = use_fast(ctx, t, cd, whole_rows);
    pc.banded = !pc.fast && fast_batch_ok(t, cd);
    pc.groups = n_plan_groups(ctx, cd->C, pc.fast, t->dev.L, cd->S_max);
    pc.slices = pc.fast ? n_fast_slices(ctx, cd->C, t->dev.L, cd->S_max) : pc.groups;
    pc.st = static_cast<hipStream_t>(hip_stream);
    if (cd->C == 0) return HARP_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace must be a 256-byte aligned device pointer");
    if (!shrink) {
        const size_t need = harp_plan_workspace_bytes(ctx, t, cd);
        if (limit_bytes < need)
            return fail(ctx, HARP_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", limit_bytes, need);
    } else {
        const int unit = pc.fast ? kFastWaves : 1;
        const size_t least = plan_bytes_on_path(t, cd, pc.fast, unit);
        if (least > limit_bytes)
            return fail(ctx, HARP_ERR_WORKSPACE,
                        "this batch needs at least %zu bytes of planner workspace, the static scratch array holds %zu: "
                        "use harp_plan_batch with a caller-lent workspace, or split the batch", least, limit_bytes);
        const size_t per_unit = plan_bytes_on_path(t, cd, pc.fast, 2 * unit) - least;
        size_t room = ((limit_bytes - least) / (per_unit ? per_unit : 1) + 1) * size_t(unit);
        if (size_t(pc.slices) > room) pc.slices = int(room);
        if (pc.groups > pc.slices) pc.groups = pc.slices;
    }
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    return HARP_OK;
}

int plan_minmax(harp_ctx *ctx, harp_tables *t, const PlanCall &pc, void *ws, unsigned long long *work) {
    if (pc.fast) launch_plan_fast(t->dev, pc.c, pc.o, ws, pc.slices, ctx->n_cu, work, pc.st);
    else launch_plan_generic(t->dev, pc.c, pc.o, ws, pc.groups, pc.banded, pc.st);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the planner kernel");
    return HARP_OK;
}

}  // namespace

extern "C" {

int harp_plan_batch(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const harp_plans *out,
                    void *workspace, size_t workspace_bytes, void *hip_stream) {
    PlanCall pc;
    const int rc = plan_prepare(ctx, t, cd, out, false, false, workspace, workspace_bytes, false, hip_stream, pc);
    if (rc != HARP_OK || cd->C == 0) return rc;
    return plan_minmax(ctx, t, pc, workspace, nullptr);
}

int harp_plan_batch_static(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const harp_plans *out,
                           void *hip_stream) {
    PlanCall pc;
    const int rc = plan_prepare(ctx, t, cd, out, false, false, ctx ? ctx->scratch : nullptr,
                                size_t(HARP_STATIC_SCRATCH_BYTES), true, hip_stream, pc);
    if (rc != HARP_OK || cd->C == 0) return rc;
    return plan_minmax(ctx, t, pc, ctx->scratch, nullptr);
}

int harp_plan_batch_count_work(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const harp_plans *out,
                               void *workspace, size_t workspace_bytes, uint64_t *work, void *hip_stream) {
    PlanCall pc;
    const int rc = plan_prepare(ctx, t, cd, out, work == nullptr, false, workspace, workspace_bytes, false, hip_stream,
                                pc);
    if (rc != HARP_OK) return rc;
    if (!pc.fast)
        return fail(ctx, HARP_ERR_UNIMPLEMENTED, "work is counted on the 32-bit path only");
    launch_clear_work(reinterpret_cast<unsigned long long *>(work), pc.st);
    if (cd->C == 0) return HARP_OK;
    return plan_minmax(ctx, t, pc, workspace, reinterpret_cast<unsigned long long *>(work));
}

int harp_plan_exact_batch(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const harp_plans *out,
                          int32_t *n_passes, void *workspace, size_t workspace_bytes, void *hip_stream) {
    PlanCall pc;
    // (the exact search's two rows of 8- or 16-byte entries fit LDS for every L of the 32-bit tables)
    int rc = plan_prepare(ctx, t, cd, out, false, false, workspace, workspace_bytes, false, hip_stream, pc);
    if (rc != HARP_OK || cd->C == 0) return rc;
    if (pc.fast) {
        rc = plan_minmax(ctx, t, pc, workspace, nullptr);
        if (rc != HARP_OK) return rc;
        launch_plan_exact(t->dev, pc.c, pc.o, n_passes, workspace, pc.groups, pc.slices, ctx->n_cu, pc.st);
    } else {
        launch_plan_generic_exact(t->dev, pc.c, pc.o, n_passes, workspace, pc.groups, pc.banded, pc.st);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the exact-search kernels");
    return HARP_OK;
}

int harp_plan_h1f1b_batch(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const int64_t *t_max,
                          const harp_plans *out, int32_t *warmup, void *workspace, size_t workspace_bytes,
                          void *hip_stream) {
    PlanCall pc;
    const int rc = plan_prepare(ctx, t, cd, out, cd && cd->C > 0 && (!warmup || !t_max), true, workspace,
                                workspace_bytes, false, hip_stream, pc);
    if (rc != HARP_OK || cd->C == 0) return rc;
    if (pc.fast) launch_plan_h1f1b(t->dev, pc.c, t_max, pc.o, warmup, workspace, pc.groups, pc.slices, ctx->n_cu, pc.st);
    else launch_plan_generic_h1f1b(t->dev, pc.c, t_max, pc.o, warmup, workspace, pc.groups, pc.banded, pc.st);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the H-1F1B planner kernels");
    return HARP_OK;
}

size_t harp_plan_mesh_workspace_bytes(harp_ctx *ctx, harp_tables *t, const harp_orderings *od) {
    if (check_orderings(ctx, t, od) != HARP_OK) return 0;
    const size_t per_group = plan_mesh_ws_per_group(t->dev.L, od->S_max, t->total_devices);
    return 256 + size_t(n_mesh_groups(ctx, od->C, per_group,
                                      plan_mesh_threads(t->dev.L, t->total_devices, od->C, ctx->n_cu))) * per_group;
}

size_t harp_plan_mesh_sweep_workspace_bytes(harp_ctx *ctx, harp_tables *t, const harp_orderings *od) {
    if (check_orderings(ctx, t, od) != HARP_OK) return 0;
    return sweep_layout(ctx, t, od).bytes;
}

}  // extern "C"

namespace {

int plan_mesh_common(harp_ctx *ctx, harp_tables *t, const harp_orderings *od, const harp_plans *out,
                     int32_t *stage_group, int32_t *stage_tp, int32_t *n_passes, bool exact, void *workspace,
                     size_t workspace_bytes, void *hip_stream) {
    int rc = check_orderings(ctx, t, od);
    if (rc != HARP_OK) return rc;
    if (!out || (od->C > 0 && (!out->splits || !out->dev_first || !out->bottleneck || !out->iter_time ||
                               !out->status || !stage_group || !stage_tp)))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null output array");
    if (ctx->plan_path == HARP_PATH_FAST32 && !t->fast32)
        return fail(ctx, HARP_ERR_UNIMPLEMENTED, "the 32-bit path was requested but these tables do not allow it");
    if (od->C == 0) return HARP_OK;
    if (t->total_devices > 65535) return fail(ctx, HARP_ERR_SHAPE, "the submesh planner handles at most 65535 devices");
    if (!mesh_index_fits(t)) return fail(ctx, HARP_ERR_SHAPE, "(devices + 1) x (L + 1) must stay below 2^31 for the kernels with a device index");
    const size_t per_group = plan_mesh_ws_per_group(t->dev.L, od->S_max, t->total_devices);
    const int threads = plan_mesh_threads(t->dev.L, t->total_devices, od->C, ctx->n_cu);
    const int groups = n_mesh_groups(ctx, od->C, per_group, threads);
    const size_t need = 256 + size_t(groups) * per_group;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const OrdDev o = { od->C, od->G_max, od->S_max, od->ord_S, od->ord_G, od->ord_group };
    const PlansDev pl = { out->splits, out->dev_first, out->bottleneck, out->iter_time, out->status };
    launch_plan_mesh(t->dev, o, pl, stage_group, stage_tp, n_passes, exact, use_fast_rows(ctx, t), workspace, groups,
                     threads, t->total_devices,
                     static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the submesh planner kernel");
    return HARP_OK;
}

}  // namespace

extern "C" {

int harp_plan_mesh_batch(harp_ctx *ctx, harp_tables *t, const harp_orderings *od, const harp_plans *out,
                         int32_t *stage_group, int32_t *stage_tp, void *workspace, size_t workspace_bytes,
                         void *hip_stream) {
    return plan_mesh_common(ctx, t, od, out, stage_group, stage_tp, nullptr, false, workspace, workspace_bytes,
                            hip_stream);
}

int harp_plan_mesh_h1f1b_batch(harp_ctx *ctx, harp_tables *t, const harp_orderings *od, const int64_t *t_max,
                               const harp_plans *out, int32_t *stage_group, int32_t *stage_tp, int32_t *warmup,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    int rc = check_orderings(ctx, t, od);
    if (rc != HARP_OK) return rc;
    if (!out || (od->C > 0 && (!out->splits || !out->dev_first || !out->bottleneck || !out->iter_time ||
                               !out->status || !stage_group || !stage_tp || !warmup || !t_max)))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    if (ctx->plan_path == HARP_PATH_FAST32 && !t->fast32)
        return fail(ctx, HARP_ERR_UNIMPLEMENTED, "the 32-bit path was requested but these tables do not allow it");
    if (od->C == 0) return HARP_OK;
    if (t->total_devices > 65535) return fail(ctx, HARP_ERR_SHAPE, "the submesh planner handles at most 65535 devices");
    if (!mesh_index_fits(t)) return fail(ctx, HARP_ERR_SHAPE, "(devices + 1) x (L + 1) must stay below 2^31 for the kernels with a device index");
    const size_t per_group = plan_mesh_ws_per_group(t->dev.L, od->S_max, t->total_devices);
    const int threads = plan_mesh_threads(t->dev.L, t->total_devices, od->C, ctx->n_cu);
    const int groups = n_mesh_groups(ctx, od->C, per_group, threads);
    const size_t need = 256 + size_t(groups) * per_group;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const OrdDev o = { od->C, od->G_max, od->S_max, od->ord_S, od->ord_G, od->ord_group };
    const PlansDev pl = { out->splits, out->dev_first, out->bottleneck, out->iter_time, out->status };
    launch_plan_mesh_h1f1b(t->dev, o, t_max, pl, stage_group, stage_tp, warmup, use_fast_rows(ctx, t), workspace, groups,
                           threads, t->total_devices, static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the submesh H-1F1B kernel");
    return HARP_OK;
}

int harp_plan_mesh_h1f1b_sweep_batch(harp_ctx *ctx, harp_tables *t, const harp_orderings *od, int32_t max_caps,
                                     const harp_plans *out, int32_t *stage_group, int32_t *stage_tp,
                                     int32_t *warmup, int64_t *t_max_out, int32_t *n_caps, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
    int rc = check_orderings(ctx, t, od);
    if (rc != HARP_OK) return rc;
    if (max_caps < 1) return fail(ctx, HARP_ERR_INVALID_ARG, "max_caps must be >= 1");
    if (!out || (od->C > 0 && (!out->splits || !out->dev_first || !out->bottleneck || !out->iter_time ||
                               !out->status || !stage_group || !stage_tp || !warmup || !t_max_out)))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    if (ctx->plan_path == HARP_PATH_FAST32 && !t->fast32)
        return fail(ctx, HARP_ERR_UNIMPLEMENTED, "the 32-bit path was requested but these tables do not allow it");
    if (od->C == 0) return HARP_OK;
    if (t->total_devices > 65535) return fail(ctx, HARP_ERR_SHAPE, "the submesh planner handles at most 65535 devices");
    if (!mesh_index_fits(t)) return fail(ctx, HARP_ERR_SHAPE, "(devices + 1) x (L + 1) must stay below 2^31 for the kernels with a device index");
    const SweepLayout lay = sweep_layout(ctx, t, od);
    const size_t need = lay.bytes;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < need)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const OrdDev o = { od->C, od->G_max, od->S_max, od->ord_S, od->ord_G, od->ord_group };
    const PlansDev pl = { out->splits, out->dev_first, out->bottleneck, out->iter_time, out->status };
    launch_plan_mesh_h1f1b_sweep(t->dev, o, nullptr, nullptr, max_caps, pl, stage_group, stage_tp, warmup, t_max_out, n_caps,
                                 use_fast_rows(ctx, t), workspace, lay.groups, lay.threads, lay.W_climb, lay.W, t->total_devices,
                                 static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the submesh H-1F1B sweep kernel");
    return HARP_OK;
}

size_t harp_plan_h1f1b_sweep_workspace_bytes(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd) {
    if (check_batch(ctx, t, cd) != HARP_OK) return 0;
    const harp_orderings shape = { cd->C, 1, cd->S_max, nullptr, nullptr, nullptr };
    return sweep_layout(ctx, t, &shape).bytes;
}

int harp_plan_h1f1b_sweep_batch(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, int32_t max_caps,
                                const harp_plans *out, int32_t *warmup, int64_t *t_max_out, int32_t *n_caps,
                                void *workspace, size_t workspace_bytes, void *hip_stream) {
    int rc = check_batch(ctx, t, cd);
    if (rc != HARP_OK) return rc;
    if (max_caps < 1) return fail(ctx, HARP_ERR_INVALID_ARG, "max_caps must be >= 1");
    if (!out || (cd->C > 0 && (!out->splits || !out->dev_first || !out->bottleneck || !out->iter_time ||
                               !out->status || !warmup || !t_max_out)))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    if (ctx->plan_path == HARP_PATH_FAST32 && !t->fast32)
        return fail(ctx, HARP_ERR_UNIMPLEMENTED, "the 32-bit path was requested but these tables do not allow it");
    if (cd->C == 0) return HARP_OK;
    if (t->total_devices > 65535) return fail(ctx, HARP_ERR_SHAPE, "the search over the cap handles at most 65535 devices");
    if (!mesh_index_fits(t)) return fail(ctx, HARP_ERR_SHAPE, "(devices + 1) x (L + 1) must stay below 2^31 for the kernels with a device index");
    const harp_orderings shape = { cd->C, 1, cd->S_max, nullptr, nullptr, nullptr };
    const SweepLayout lay = sweep_layout(ctx, t, &shape);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < lay.bytes)
        return fail(ctx, HARP_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, lay.bytes);
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const OrdDev o = { cd->C, 1, cd->S_max, cd->cand_S, nullptr, nullptr };
    const PlansDev pl = { out->splits, out->dev_first, out->bottleneck, out->iter_time, out->status };
    launch_plan_mesh_h1f1b_sweep(t->dev, o, cd->cand_group, cd->cand_tp, max_caps, pl, nullptr, nullptr, warmup,
                                 t_max_out, n_caps, use_fast_rows(ctx, t), workspace, lay.groups, lay.threads, lay.W_climb, lay.W,
                                 t->total_devices, static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the search over the cap");
    return HARP_OK;
}

int harp_plan_mesh_exact_batch(harp_ctx *ctx, harp_tables *t, const harp_orderings *od, const harp_plans *out,
                               int32_t *stage_group, int32_t *stage_tp, int32_t *n_passes, void *workspace,
                               size_t workspace_bytes, void *hip_stream) {
    return plan_mesh_common(ctx, t, od, out, stage_group, stage_tp, n_passes, true, workspace, workspace_bytes,
                            hip_stream);
}

int harp_score_h1f1b(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const int32_t *splits,
                     const int64_t *t_max, int32_t *warmup, int64_t *bottleneck, int64_t *iter_time,
                     int32_t *status, void *hip_stream) {
    int rc = check_batch(ctx, t, cd);
    if (rc != HARP_OK) return rc;
    if (cd->C == 0) return HARP_OK;
    if (!splits || !t_max || !warmup || !bottleneck || !iter_time || !status)
        return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const CandDev c = { cd->C, cd->S_max, cd->cand_S, cd->cand_group, cd->cand_tp };
    launch_score_h1f1b(t->dev, c, splits, t_max, warmup, bottleneck, iter_time, status,
                       static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the H-1F1B scorer kernel");
    return HARP_OK;
}

int harp_score_1f1b(harp_ctx *ctx, harp_tables *t, const harp_candidates *cd, const int32_t *splits,
                    int64_t *bottleneck, int64_t *iter_time, int32_t *status, void *hip_stream) {
    int rc = check_batch(ctx, t, cd);
    if (rc != HARP_OK) return rc;
    if (cd->C == 0) return HARP_OK;
    if (!splits || !bottleneck || !iter_time || !status) return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const CandDev c = { cd->C, cd->S_max, cd->cand_S, cd->cand_group, cd->cand_tp };
    if (ctx->plan_path == HARP_PATH_FAST32 && !t->fast32)
        return fail(ctx, HARP_ERR_UNIMPLEMENTED, "these tables have no 32-bit rows");
    launch_score(t->dev, c, splits, bottleneck, iter_time, status, t->fast32 && ctx->plan_path != HARP_PATH_GENERIC,
                 ctx->n_cu, static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the scorer kernel");
    return HARP_OK;
}

int harp_argmin_batch(harp_ctx *ctx, int32_t C, const int64_t *iter_time, const int32_t *status,
                      int64_t *best_time, int32_t *best_index, void *hip_stream) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (C < 0) return fail(ctx, HARP_ERR_INVALID_ARG, "C must be >= 0");
    if (!best_time || !best_index || (C > 0 && (!iter_time || !status)))
        return fail(ctx, HARP_ERR_INVALID_ARG, "null array");
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    launch_argmin(C, iter_time, status, best_time, best_index, static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the selection kernel");
    return HARP_OK;
}

int harp_measure_valu_int32(harp_ctx *ctx, int32_t blocks, int32_t iters, uint32_t *sink, void *hip_stream) {
    if (!ctx) return HARP_ERR_INVALID_ARG;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || !sink)
        return fail(ctx, HARP_ERR_INVALID_ARG, "blocks must be in 1..2^20, iters >= 1, sink non-null");
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    launch_valu_int32(blocks, iters, sink, static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e, "launching the VALU measurement kernel");
    return HARP_OK;
}

}  // extern "C"
