"""ctypes binding of the C ABI in include/harp.h.

Argument marshalling only: every step of the planner search runs in the HIP kernels behind the
ABI.  PyTorch is used to own device memory and to name the stream; nothing is computed with it.
There is no CPU fallback: if the library is not built, or no GPU is visible, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libharp_hip.so")

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_WORKSPACE, ERR_HIP, ERR_OVERFLOW, ERR_UNIMPLEMENTED = \
    0, -1, -2, -3, -4, -5, -6
CAND_OK, CAND_INFEASIBLE, CAND_INVALID = 0, 1, 2
PATH_AUTO, PATH_GENERIC, PATH_FAST32 = 0, 1, 2
INF = (1 << 63) - 1

EXPORTS = (
    "harp_create", "harp_destroy", "harp_last_error", "harp_tables_bytes",
    "harp_build_segment_costs", "harp_tables_finalize", "harp_tables_fast32", "harp_tables_pf",
    "harp_tables_pp", "harp_tables_ps", "harp_tables_pr", "harp_tables_release",
    "harp_set_plan_path", "harp_plan_workspace_bytes", "harp_plan_batch", "harp_plan_batch_static",
    "harp_plan_batch_count_work",
    "harp_plan_exact_batch",
    "harp_plan_h1f1b_batch", "harp_score_h1f1b",
    "harp_plan_mesh_workspace_bytes", "harp_plan_mesh_batch", "harp_plan_mesh_exact_batch", "harp_plan_mesh_h1f1b_batch",
    "harp_plan_mesh_h1f1b_sweep_batch", "harp_plan_mesh_sweep_workspace_bytes",
    "harp_plan_h1f1b_sweep_batch", "harp_plan_h1f1b_sweep_workspace_bytes",
    "harp_score_1f1b", "harp_argmin_batch", "harp_measure_valu_int32",
)


class HarpError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("harp error %d: %s" % (code, message))
        self.code = code


class harp_problem(C.Structure):
    _fields_ = [("L", C.c_int32), ("T", C.c_int32), ("G", C.c_int32), ("M", C.c_int32),
                ("ar_count", C.c_int32), ("flags", C.c_int32), ("n_tp", C.c_int32),
                ("tp_degrees", C.c_void_p), ("fwd_us", C.c_void_p), ("bwd_us", C.c_void_p),
                ("param_bytes", C.c_void_p), ("stash_bytes", C.c_void_p), ("act_bytes", C.c_void_p),
                ("group_type", C.c_void_p), ("group_ndev", C.c_void_p),
                ("type_mem_bytes", C.c_void_p), ("bw_bytes_per_us", C.c_void_p)]


class harp_orderings(C.Structure):
    _fields_ = [("C", C.c_int32), ("G_max", C.c_int32), ("S_max", C.c_int32), ("ord_S", C.c_void_p),
                ("ord_G", C.c_void_p), ("ord_group", C.c_void_p)]


class harp_candidates(C.Structure):
    _fields_ = [("C", C.c_int32), ("S_max", C.c_int32), ("cand_S", C.c_void_p),
                ("cand_group", C.c_void_p), ("cand_tp", C.c_void_p)]


class harp_plans(C.Structure):
    _fields_ = [("splits", C.c_void_p), ("dev_first", C.c_void_p), ("bottleneck", C.c_void_p),
                ("iter_time", C.c_void_p), ("status", C.c_void_p)]


_lib = None


def load_library() -> C.CDLL:
    """Loads libharp_hip.so; raises when it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(or paper_2509_24859_amd.build.build_library()) first" % LIB_PATH)
    # torch first: it brings its own HIP runtime, and the library must bind to that same runtime
    # (device pointers and streams are torch's), not load a second one beside it
    _torch()
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.harp_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.harp_destroy.argtypes = [vp]
    lib.harp_destroy.restype = None
    lib.harp_last_error.argtypes = [vp]
    lib.harp_last_error.restype = C.c_char_p
    lib.harp_tables_bytes.argtypes = [C.POINTER(harp_problem)]
    lib.harp_tables_bytes.restype = sz
    lib.harp_build_segment_costs.argtypes = [vp, C.POINTER(harp_problem), vp, sz, C.POINTER(vp), vp]
    lib.harp_tables_finalize.argtypes = [vp, vp]
    lib.harp_tables_fast32.argtypes = [vp]
    for name in ("harp_tables_pf", "harp_tables_pr"):
        getattr(lib, name).argtypes = [vp, C.POINTER(sz)]
        getattr(lib, name).restype = vp
    for name in ("harp_tables_pp", "harp_tables_ps"):
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = vp
    lib.harp_tables_release.argtypes = [vp]
    lib.harp_tables_release.restype = None
    lib.harp_set_plan_path.argtypes = [vp, C.c_int]
    lib.harp_plan_workspace_bytes.argtypes = [vp, vp, C.POINTER(harp_candidates)]
    lib.harp_plan_workspace_bytes.restype = sz
    lib.harp_plan_batch.argtypes = [vp, vp, C.POINTER(harp_candidates), C.POINTER(harp_plans), vp, sz, vp]
    lib.harp_plan_batch_count_work.argtypes = [vp, vp, C.POINTER(harp_candidates), C.POINTER(harp_plans), vp, sz, vp, vp]
    lib.harp_plan_batch_static.argtypes = [vp, vp, C.POINTER(harp_candidates), C.POINTER(harp_plans), vp]
    lib.harp_plan_exact_batch.argtypes = [vp, vp, C.POINTER(harp_candidates), C.POINTER(harp_plans), vp, vp, sz, vp]
    lib.harp_plan_h1f1b_batch.argtypes = [vp, vp, C.POINTER(harp_candidates), vp, C.POINTER(harp_plans), vp, vp, sz, vp]
    lib.harp_score_h1f1b.argtypes = [vp, vp, C.POINTER(harp_candidates), vp, vp, vp, vp, vp, vp, vp]
    lib.harp_plan_mesh_workspace_bytes.argtypes = [vp, vp, C.POINTER(harp_orderings)]
    lib.harp_plan_mesh_workspace_bytes.restype = sz
    lib.harp_plan_h1f1b_sweep_workspace_bytes.argtypes = [vp, vp, C.POINTER(harp_candidates)]
    lib.harp_plan_h1f1b_sweep_workspace_bytes.restype = sz
    lib.harp_plan_h1f1b_sweep_batch.argtypes = [vp, vp, C.POINTER(harp_candidates), i32, C.POINTER(harp_plans),
                                                vp, vp, vp, vp, sz, vp]
    lib.harp_plan_mesh_sweep_workspace_bytes.argtypes = [vp, vp, C.POINTER(harp_orderings)]
    lib.harp_plan_mesh_sweep_workspace_bytes.restype = sz
    lib.harp_plan_mesh_batch.argtypes = [vp, vp, C.POINTER(harp_orderings), C.POINTER(harp_plans), vp, vp, vp, sz, vp]
    lib.harp_plan_mesh_exact_batch.argtypes = [vp, vp, C.POINTER(harp_orderings), C.POINTER(harp_plans), vp, vp, vp,
                                               vp, sz, vp]
    lib.harp_plan_mesh_h1f1b_batch.argtypes = [vp, vp, C.POINTER(harp_orderings), vp, C.POINTER(harp_plans), vp, vp,
                                               vp, vp, sz, vp]
    lib.harp_plan_mesh_h1f1b_sweep_batch.argtypes = [vp, vp, C.POINTER(harp_orderings), i32, C.POINTER(harp_plans),
                                                     vp, vp, vp, vp, vp, vp, sz, vp]
    lib.harp_score_1f1b.argtypes = [vp, vp, C.POINTER(harp_candidates), vp, vp, vp, vp, vp]
    lib.harp_argmin_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.harp_measure_valu_int32.argtypes = [vp, i32, i32, vp, vp]
    _lib = lib
    return lib


def _torch():
    import torch
    return torch


def _stream_handle(stream=None) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dev(a, dtype, device):
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=dtype))
    return t.to(device)


class Context:
    """harp_create / harp_destroy."""

    def __init__(self, device_ordinal: int = 0):
        self.lib = load_library()
        torch = _torch()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the planner has no CPU path")
        self.device = torch.device("cuda", device_ordinal)
        h = C.c_void_p()
        rc = self.lib.harp_create(C.byref(h), device_ordinal)
        if rc != OK:
            raise HarpError(rc, "harp_create failed")
        self.handle = h

    def check(self, rc: int):
        if rc != OK:
            raise HarpError(rc, self.lib.harp_last_error(self.handle).decode())

    def set_plan_path(self, path: int):
        self.check(self.lib.harp_set_plan_path(self.handle, path))

    def close(self):
        if getattr(self, "handle", None):
            self.lib.harp_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DeviceProblem:
    """A problem's arrays resident on the GPU plus the harp_problem struct naming them."""

    def __init__(self, ctx: Context, p):
        d = ctx.device
        self.host = p
        self.tp_host = np.ascontiguousarray(p.tp_degrees, dtype=np.int32)
        self.fwd = _dev(p.fwd_us, np.int64, d)
        self.bwd = _dev(p.bwd_us, np.int64, d)
        self.par = _dev(p.param_bytes, np.int64, d)
        self.sta = _dev(p.stash_bytes, np.int64, d)
        self.act = _dev(p.act_bytes, np.int64, d)
        self.gt = _dev(p.group_type, np.int32, d)
        self.gn = _dev(p.group_ndev, np.int32, d)
        self.mem = _dev(p.type_mem_bytes, np.int64, d)
        self.bw = _dev(p.bw, np.int64, d)
        self.c = harp_problem(p.L, p.T, p.G, p.M, p.ar_count, 0, len(self.tp_host),
                              self.tp_host.ctypes.data, self.fwd.data_ptr(), self.bwd.data_ptr(),
                              self.par.data_ptr(), self.sta.data_ptr(), self.act.data_ptr(),
                              self.gt.data_ptr(), self.gn.data_ptr(), self.mem.data_ptr(),
                              self.bw.data_ptr())


class Tables:
    """harp_build_segment_costs / harp_tables_finalize / harp_tables_release."""

    def __init__(self, ctx: Context, problem, stream=None, finalize: bool = True):
        torch = _torch()
        self.ctx = ctx
        self.dp = problem if isinstance(problem, DeviceProblem) else DeviceProblem(ctx, problem)
        n = ctx.lib.harp_tables_bytes(C.byref(self.dp.c))
        if n == 0:
            raise HarpError(ERR_INVALID_ARG, "harp_tables_bytes rejected the problem header")
        self.buf = torch.empty(n, dtype=torch.uint8, device=ctx.device)
        self.nbytes = n
        h = C.c_void_p()
        ctx.check(ctx.lib.harp_build_segment_costs(ctx.handle, C.byref(self.dp.c), self.buf.data_ptr(),
                                                   n, C.byref(h), _stream_handle(stream)))
        self.handle = h
        if finalize:
            self.finalize()

    def rebuild(self, stream=None):
        """Enqueue the build again into the same buffer (for timing); returns without waiting."""
        self.release()
        h = C.c_void_p()
        self.ctx.check(self.ctx.lib.harp_build_segment_costs(
            self.ctx.handle, C.byref(self.dp.c), self.buf.data_ptr(), self.nbytes, C.byref(h),
            _stream_handle(stream)))
        self.handle = h

    def finalize(self):
        self.ctx.check(self.ctx.lib.harp_tables_finalize(self.ctx.handle, self.handle))

    @property
    def fast32(self) -> bool:
        return bool(self.ctx.lib.harp_tables_fast32(self.handle))

    def _rows(self, ptr: int, n_rows: int, pitch: int) -> np.ndarray:
        """Copy n_rows table rows (L+1 entries each) back to the host for inspection."""
        torch = _torch()
        base = self.buf.data_ptr()
        off = ptr - base
        L1 = self.dp.host.L + 1
        flat = self.buf[off: off + n_rows * pitch * 8].view(torch.int64).reshape(n_rows, pitch)
        return flat[:, :L1].cpu().numpy()

    def host_copies(self):
        """(PF [T][L+1], PP [L+1], PS [L+1], PR [G][n_tp][L+1]) as numpy arrays."""
        lib, p = self.ctx.lib, self.dp.host
        pitch = C.c_size_t()
        pf = lib.harp_tables_pf(self.handle, C.byref(pitch))
        PF = self._rows(pf, p.T, pitch.value)
        PP = self._rows(lib.harp_tables_pp(self.handle), 1, pitch.value)[0]
        PS = self._rows(lib.harp_tables_ps(self.handle), 1, pitch.value)[0]
        pr = lib.harp_tables_pr(self.handle, C.byref(pitch))
        PR = self._rows(pr, p.G * len(self.dp.tp_host), pitch.value).reshape(p.G, len(self.dp.tp_host), -1)
        return PF, PP, PS, PR

    def release(self):
        if getattr(self, "handle", None):
            self.ctx.lib.harp_tables_release(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass


class DeviceCandidates:
    def __init__(self, ctx: Context, cands):
        d = ctx.device
        self.C, self.S_max = int(cands.C), int(cands.S_max)
        self.cs = _dev(cands.cand_S, np.int32, d)
        self.cg = _dev(cands.cand_group, np.int32, d)
        self.ct = _dev(cands.cand_tp, np.int32, d)
        self.c = harp_candidates(self.C, self.S_max, self.cs.data_ptr(), self.cg.data_ptr(),
                                 self.ct.data_ptr())


class DevicePlans:
    def __init__(self, ctx: Context, C_: int, S_max: int):
        torch = _torch()
        d = ctx.device
        self.splits = torch.empty((C_, S_max + 1), dtype=torch.int32, device=d)
        self.dev_first = torch.empty((C_, S_max), dtype=torch.int32, device=d)
        self.bottleneck = torch.empty(C_, dtype=torch.int64, device=d)
        self.iter_time = torch.empty(C_, dtype=torch.int64, device=d)
        self.status = torch.empty(C_, dtype=torch.int32, device=d)
        self.c = harp_plans(self.splits.data_ptr(), self.dev_first.data_ptr(),
                            self.bottleneck.data_ptr(), self.iter_time.data_ptr(),
                            self.status.data_ptr())

    def poison(self):
        """Fill every output with a value no correct run leaves behind."""
        for t in (self.splits, self.dev_first, self.status):
            t.fill_(-7)
        self.bottleneck.fill_(-7)
        self.iter_time.fill_(-7)

    def to_host(self):
        class _P:
            pass
        o = _P()
        o.splits = self.splits.cpu().numpy()
        o.dev_first = self.dev_first.cpu().numpy()
        o.bottleneck = self.bottleneck.cpu().numpy()
        o.iter_time = self.iter_time.cpu().numpy()
        o.status = self.status.cpu().numpy()
        return o


def plan_workspace(ctx: Context, tables: Tables, dc: DeviceCandidates):
    torch = _torch()
    n = ctx.lib.harp_plan_workspace_bytes(ctx.handle, tables.handle, C.byref(dc.c))
    if n == 0 and dc.C > 0:
        raise HarpError(ERR_SHAPE, "harp_plan_workspace_bytes rejected the batch")
    return torch.empty(max(n, 256), dtype=torch.uint8, device=ctx.device)


def harp_plan_batch(ctx: Context, tables: Tables, dc: DeviceCandidates, out: DevicePlans,
                    workspace, stream=None):
    ctx.check(ctx.lib.harp_plan_batch(ctx.handle, tables.handle, C.byref(dc.c), C.byref(out.c),
                                      workspace.data_ptr(), workspace.numel(), _stream_handle(stream)))


def harp_plan_batch_count_work(ctx: Context, tables: Tables, dc: DeviceCandidates, out: DevicePlans, workspace, work,
                               stream=None):
    """work: int64 device tensor of 4 entries (transitions, cells, groups of four, candidates planned)."""
    ctx.check(ctx.lib.harp_plan_batch_count_work(ctx.handle, tables.handle, C.byref(dc.c), C.byref(out.c),
                                                 workspace.data_ptr(), workspace.numel(), work.data_ptr(),
                                                 _stream_handle(stream)))


def harp_plan_batch_static(ctx: Context, tables: Tables, dc: DeviceCandidates, out: DevicePlans, stream=None):
    ctx.check(ctx.lib.harp_plan_batch_static(ctx.handle, tables.handle, C.byref(dc.c), C.byref(out.c),
                                             _stream_handle(stream)))


def harp_plan_exact_batch(ctx: Context, tables: Tables, dc: DeviceCandidates, out: DevicePlans,
                          workspace, n_passes=None, stream=None):
    ctx.check(ctx.lib.harp_plan_exact_batch(ctx.handle, tables.handle, C.byref(dc.c), C.byref(out.c),
                                            n_passes.data_ptr() if n_passes is not None else None,
                                            workspace.data_ptr(), workspace.numel(), _stream_handle(stream)))


def harp_plan_h1f1b_batch(ctx: Context, tables: Tables, dc: DeviceCandidates, t_max, out: DevicePlans,
                          warmup, workspace, stream=None):
    ctx.check(ctx.lib.harp_plan_h1f1b_batch(ctx.handle, tables.handle, C.byref(dc.c), t_max.data_ptr(),
                                            C.byref(out.c), warmup.data_ptr(), workspace.data_ptr(),
                                            workspace.numel(), _stream_handle(stream)))


def harp_score_h1f1b(ctx: Context, tables: Tables, dc: DeviceCandidates, splits, t_max, warmup, bottleneck,
                     iter_time, status, stream=None):
    ctx.check(ctx.lib.harp_score_h1f1b(ctx.handle, tables.handle, C.byref(dc.c), splits.data_ptr(),
                                       t_max.data_ptr(), warmup.data_ptr(), bottleneck.data_ptr(),
                                       iter_time.data_ptr(), status.data_ptr(), _stream_handle(stream)))


def harp_score_1f1b(ctx: Context, tables: Tables, dc: DeviceCandidates, splits, bottleneck,
                    iter_time, status, stream=None):
    ctx.check(ctx.lib.harp_score_1f1b(ctx.handle, tables.handle, C.byref(dc.c), splits.data_ptr(),
                                      bottleneck.data_ptr(), iter_time.data_ptr(), status.data_ptr(),
                                      _stream_handle(stream)))


def harp_argmin_batch(ctx: Context, C_: int, iter_time, status, best_time, best_index, stream=None):
    ctx.check(ctx.lib.harp_argmin_batch(ctx.handle, C_, iter_time.data_ptr(), status.data_ptr(),
                                        best_time.data_ptr(), best_index.data_ptr(),
                                        _stream_handle(stream)))


def harp_measure_valu_int32(ctx: Context, blocks: int, iters: int, sink, stream=None):
    ctx.check(ctx.lib.harp_measure_valu_int32(ctx.handle, blocks, iters, sink.data_ptr(), _stream_handle(stream)))


def harp_build_segment_costs(ctx: Context, problem, stream=None, finalize: bool = True) -> Tables:
    return Tables(ctx, problem, stream, finalize)


def plan(ctx: Context, problem, cands, path: int = PATH_AUTO):
    """Convenience for tests: build tables, plan a batch, return host copies of the plans."""
    torch = _torch()
    tables = Tables(ctx, problem)
    dc = DeviceCandidates(ctx, cands)
    out = DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    ws = plan_workspace(ctx, tables, dc)
    ctx.set_plan_path(path)
    try:
        harp_plan_batch(ctx, tables, dc, out, ws)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    return out.to_host(), tables


class DeviceOrderings:
    def __init__(self, ctx: Context, orders):
        self.C, self.G_max, self.S_max = int(orders.C), int(orders.G_max), int(orders.S_max)
        self.ord_S = _dev(orders.ord_S, np.int32, ctx.device)
        self.ord_G = _dev(orders.ord_G, np.int32, ctx.device)
        self.ord_group = _dev(orders.ord_group, np.int32, ctx.device)
        self.c = harp_orderings(self.C, self.G_max, self.S_max, self.ord_S.data_ptr(), self.ord_G.data_ptr(),
                                self.ord_group.data_ptr())


def harp_plan_mesh_batch(ctx: Context, tables: Tables, do: DeviceOrderings, out: DevicePlans, stage_group,
                         stage_tp, workspace, stream=None):
    ctx.check(ctx.lib.harp_plan_mesh_batch(ctx.handle, tables.handle, C.byref(do.c), C.byref(out.c),
                                           stage_group.data_ptr(), stage_tp.data_ptr(), workspace.data_ptr(),
                                           workspace.numel(), _stream_handle(stream)))


def harp_plan_mesh_exact_batch(ctx: Context, tables: Tables, do: DeviceOrderings, out: DevicePlans, stage_group,
                               stage_tp, workspace, n_passes=None, stream=None):
    ctx.check(ctx.lib.harp_plan_mesh_exact_batch(ctx.handle, tables.handle, C.byref(do.c), C.byref(out.c),
                                                 stage_group.data_ptr(), stage_tp.data_ptr(),
                                                 n_passes.data_ptr() if n_passes is not None else None,
                                                 workspace.data_ptr(), workspace.numel(), _stream_handle(stream)))


def harp_plan_mesh_h1f1b_batch(ctx: Context, tables: Tables, do: DeviceOrderings, t_max, out: DevicePlans,
                               stage_group, stage_tp, warmup, workspace, stream=None):
    ctx.check(ctx.lib.harp_plan_mesh_h1f1b_batch(ctx.handle, tables.handle, C.byref(do.c), t_max.data_ptr(),
                                                 C.byref(out.c), stage_group.data_ptr(), stage_tp.data_ptr(),
                                                 warmup.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                                 _stream_handle(stream)))


def plan_mesh_h1f1b(ctx: Context, problem, orders, t_max, path: int = PATH_AUTO):
    """Convenience for tests: the full recurrence for one cap per ordering; host copies of the plans
    with `.stage_group`, `.stage_tp`, `.warmup`."""
    torch = _torch()
    tables = Tables(ctx, problem)
    do = DeviceOrderings(ctx, orders)
    out = DevicePlans(ctx, do.C, do.S_max)
    out.poison()
    sg = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    st = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    wu = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    caps = _dev(np.asarray(t_max, dtype=np.int64).reshape(-1), np.int64, ctx.device)
    ws = mesh_workspace(ctx, tables, do)
    ctx.set_plan_path(path)
    try:
        harp_plan_mesh_h1f1b_batch(ctx, tables, do, caps, out, sg, st, wu, ws)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    got = out.to_host()
    got.stage_group = sg[:do.C].cpu().numpy()
    got.stage_tp = st[:do.C].cpu().numpy()
    got.warmup = wu[:do.C].cpu().numpy()
    return got, tables


def harp_plan_mesh_h1f1b_sweep_batch(ctx: Context, tables: Tables, do: DeviceOrderings, max_caps: int,
                                     out: DevicePlans, stage_group, stage_tp, warmup, t_max_out, workspace,
                                     n_caps=None, stream=None):
    ctx.check(ctx.lib.harp_plan_mesh_h1f1b_sweep_batch(
        ctx.handle, tables.handle, C.byref(do.c), int(max_caps), C.byref(out.c), stage_group.data_ptr(),
        stage_tp.data_ptr(), warmup.data_ptr(), t_max_out.data_ptr(),
        n_caps.data_ptr() if n_caps is not None else None, workspace.data_ptr(), workspace.numel(),
        _stream_handle(stream)))


def plan_mesh_h1f1b_sweep(ctx: Context, problem, orders, max_caps: int = 1 << 20, path: int = PATH_AUTO):
    """Convenience for tests: the search around the full recurrence; host copies of the plans with
    `.stage_group`, `.stage_tp`, `.warmup`, `.t_max`, `.n_caps`."""
    torch = _torch()
    tables = Tables(ctx, problem)
    do = DeviceOrderings(ctx, orders)
    out = DevicePlans(ctx, do.C, do.S_max)
    out.poison()
    sg = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    st = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    wu = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    tm = torch.full((max(do.C, 1),), -7, dtype=torch.int64, device=ctx.device)
    nc = torch.full((max(do.C, 1),), -7, dtype=torch.int32, device=ctx.device)
    ws = mesh_sweep_workspace(ctx, tables, do)
    ctx.set_plan_path(path)
    try:
        harp_plan_mesh_h1f1b_sweep_batch(ctx, tables, do, max_caps, out, sg, st, wu, tm, ws, nc)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    got = out.to_host()
    got.stage_group = sg[:do.C].cpu().numpy()
    got.stage_tp = st[:do.C].cpu().numpy()
    got.warmup = wu[:do.C].cpu().numpy()
    got.t_max = tm[:do.C].cpu().numpy()
    got.n_caps = nc[:do.C].cpu().numpy()
    return got, tables


def mesh_workspace(ctx: Context, tables: Tables, do: DeviceOrderings):
    torch = _torch()
    n = ctx.lib.harp_plan_mesh_workspace_bytes(ctx.handle, tables.handle, C.byref(do.c))
    if n == 0:
        raise HarpError(ERR_INVALID_ARG, ctx.lib.harp_last_error(ctx.handle).decode() or "malformed orderings")
    return torch.empty(n, dtype=torch.uint8, device=ctx.device)


def harp_plan_h1f1b_sweep_batch(ctx: Context, tables: Tables, dc: DeviceCandidates, max_caps: int,
                                out: DevicePlans, warmup, t_max_out, workspace, n_caps=None, stream=None):
    ctx.check(ctx.lib.harp_plan_h1f1b_sweep_batch(
        ctx.handle, tables.handle, C.byref(dc.c), int(max_caps), C.byref(out.c), warmup.data_ptr(),
        t_max_out.data_ptr(), n_caps.data_ptr() if n_caps is not None else None, workspace.data_ptr(),
        workspace.numel(), _stream_handle(stream)))


def h1f1b_sweep_workspace(ctx: Context, tables: Tables, dc: DeviceCandidates):
    torch = _torch()
    n = ctx.lib.harp_plan_h1f1b_sweep_workspace_bytes(ctx.handle, tables.handle, C.byref(dc.c))
    if n == 0:
        raise HarpError(ERR_INVALID_ARG, ctx.lib.harp_last_error(ctx.handle).decode() or "malformed candidates")
    return torch.empty(n, dtype=torch.uint8, device=ctx.device)


def plan_h1f1b_sweep(ctx: Context, problem, cands, max_caps: int = 1 << 20, path: int = PATH_AUTO):
    """Convenience for tests: the search over the cap for candidates; host copies of the plans with
    `.warmup`, `.t_max`, `.n_caps`."""
    torch = _torch()
    tables = Tables(ctx, problem)
    dc = DeviceCandidates(ctx, cands)
    out = DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    wu = torch.full((max(dc.C, 1), dc.S_max), -7, dtype=torch.int32, device=ctx.device)
    tm = torch.full((max(dc.C, 1),), -7, dtype=torch.int64, device=ctx.device)
    nc = torch.full((max(dc.C, 1),), -7, dtype=torch.int32, device=ctx.device)
    ws = h1f1b_sweep_workspace(ctx, tables, dc)
    ctx.set_plan_path(path)
    try:
        harp_plan_h1f1b_sweep_batch(ctx, tables, dc, max_caps, out, wu, tm, ws, nc)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    got = out.to_host()
    got.warmup = wu[:dc.C].cpu().numpy()
    got.t_max = tm[:dc.C].cpu().numpy()
    got.n_caps = nc[:dc.C].cpu().numpy()
    return got, tables


def mesh_sweep_workspace(ctx: Context, tables: Tables, do: DeviceOrderings):
    torch = _torch()
    n = ctx.lib.harp_plan_mesh_sweep_workspace_bytes(ctx.handle, tables.handle, C.byref(do.c))
    if n == 0:
        raise HarpError(ERR_INVALID_ARG, ctx.lib.harp_last_error(ctx.handle).decode() or "malformed orderings")
    return torch.empty(n, dtype=torch.uint8, device=ctx.device)


def plan_mesh(ctx: Context, problem, orders, exact: bool = False, path: int = PATH_AUTO):
    """Convenience for tests: tables, submesh planner over a batch of orderings (min-max, or the
    exact search); host copies of the plans with `.stage_group`, `.stage_tp` (and `.n_passes`)."""
    torch = _torch()
    tables = Tables(ctx, problem)
    do = DeviceOrderings(ctx, orders)
    out = DevicePlans(ctx, do.C, do.S_max)
    out.poison()
    sg = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    st = torch.full((max(do.C, 1), do.S_max), -7, dtype=torch.int32, device=ctx.device)
    n_passes = torch.full((max(do.C, 1),), -7, dtype=torch.int32, device=ctx.device)
    ws = mesh_workspace(ctx, tables, do)
    ctx.set_plan_path(path)
    try:
        if exact:
            harp_plan_mesh_exact_batch(ctx, tables, do, out, sg, st, ws, n_passes)
        else:
            harp_plan_mesh_batch(ctx, tables, do, out, sg, st, ws)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    got = out.to_host()
    got.stage_group = sg[:do.C].cpu().numpy()
    got.stage_tp = st[:do.C].cpu().numpy()
    got.n_passes = n_passes[:do.C].cpu().numpy()
    return got, tables


def plan_h1f1b(ctx: Context, problem, cands, t_max, path: int = PATH_AUTO):
    """Convenience for tests: tables, capped H-1F1B recurrence over a batch; host copies of the
    plans (with `.warmup`) and the tables."""
    torch = _torch()
    tables = Tables(ctx, problem)
    dc = DeviceCandidates(ctx, cands)
    out = DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    ws = plan_workspace(ctx, tables, dc)
    caps = _dev(np.asarray(t_max, dtype=np.int64).reshape(-1), np.int64, ctx.device)
    warmup = torch.full((max(dc.C, 1), dc.S_max), -7, dtype=torch.int32, device=ctx.device)
    ctx.set_plan_path(path)
    try:
        harp_plan_h1f1b_batch(ctx, tables, dc, caps, out, warmup, ws)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    got = out.to_host()
    got.warmup = warmup[:dc.C].cpu().numpy()
    return got, tables


def plan_exact(ctx: Context, problem, cands, path: int = PATH_AUTO):
    """Convenience for tests: tables, exact search over a batch; host copies of the plans and of
    the number of capped passes per candidate."""
    torch = _torch()
    tables = Tables(ctx, problem)
    dc = DeviceCandidates(ctx, cands)
    out = DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    ws = plan_workspace(ctx, tables, dc)
    n_passes = torch.full((max(dc.C, 1),), -7, dtype=torch.int32, device=ctx.device)
    ctx.set_plan_path(path)
    try:
        harp_plan_exact_batch(ctx, tables, dc, out, ws, n_passes)
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_path(PATH_AUTO)
    return out.to_host(), n_passes[:dc.C].cpu().numpy(), tables
