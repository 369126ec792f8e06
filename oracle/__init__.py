"""CPU oracle for the HARP planner search (paper section 5.2).  TEST INFRASTRUCTURE ONLY.

Python front end of `harp_oracle.c` (compiled with gcc on first use) plus a brute-force twin in
`brute.py`.  Nothing here is imported by the product package; only tests, the smoke check and the
benchmark's cpu_baseline leg use it.  It shares no code with the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "harp_oracle.c")
_LIB = os.path.join(_HERE, "libharp_oracle.so")

INF = np.iinfo(np.int64).max
OK, INFEASIBLE, INVALID = 0, 1, 2
ERR_BAD_ARG, ERR_OVERFLOW = -1, -5


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared library next to its source."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _CProblem(C.Structure):
    _fields_ = [("L", C.c_int32), ("T", C.c_int32), ("G", C.c_int32), ("M", C.c_int32),
                ("ar_count", C.c_int32), ("n_tp", C.c_int32),
                ("tp_degrees", C.c_void_p), ("fwd_us", C.c_void_p), ("bwd_us", C.c_void_p),
                ("param_bytes", C.c_void_p), ("stash_bytes", C.c_void_p), ("act_bytes", C.c_void_p),
                ("group_type", C.c_void_p), ("group_ndev", C.c_void_p),
                ("type_mem_bytes", C.c_void_p), ("bw", C.c_void_p)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("oracle_build_tables", "oracle_plan_batch", "oracle_score_1f1b",
                     "oracle_argmin_batch", "oracle_plan_exact_batch", "oracle_plan_h1f1b_batch",
                     "oracle_score_h1f1b", "oracle_plan_mesh_batch",
                     "oracle_plan_mesh_exact_batch", "oracle_plan_mesh_h1f1b_batch",
                     "oracle_plan_mesh_h1f1b_sweep_batch", "oracle_plan_h1f1b_sweep_batch"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _ptr(a: np.ndarray):
    return C.c_void_p(a.ctypes.data)


def _c64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _c32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Tables:
    """Running-sum tables of one problem, built by the C oracle; keeps every array alive."""

    def __init__(self, problem):
        p = problem
        self.problem = p
        self._keep = dict(
            tp=_c32(p.tp_degrees), fwd=_c64(p.fwd_us), bwd=_c64(p.bwd_us), par=_c64(p.param_bytes),
            sta=_c64(p.stash_bytes), act=_c64(p.act_bytes), gt=_c32(p.group_type),
            gn=_c32(p.group_ndev), mem=_c64(p.type_mem_bytes), bw=_c64(p.bw))
        k = self._keep
        self.c = _CProblem(p.L, p.T, p.G, p.M, p.ar_count, len(k["tp"]), k["tp"].ctypes.data,
                           k["fwd"].ctypes.data, k["bwd"].ctypes.data, k["par"].ctypes.data,
                           k["sta"].ctypes.data, k["act"].ctypes.data, k["gt"].ctypes.data,
                           k["gn"].ctypes.data, k["mem"].ctypes.data, k["bw"].ctypes.data)
        L1 = p.L + 1
        self.PF = np.zeros((p.T, L1), dtype=np.int64)
        self.PP = np.zeros(L1, dtype=np.int64)
        self.PS = np.zeros(L1, dtype=np.int64)
        self.PR = np.zeros((p.G, len(k["tp"]), L1), dtype=np.int64)
        self.rc = _load().oracle_build_tables(C.byref(self.c), _ptr(self.PF), _ptr(self.PP),
                                               _ptr(self.PS), _ptr(self.PR))


class Plans:
    def __init__(self, n, S_max):
        self.splits = np.full((n, S_max + 1), -1, dtype=np.int32)
        self.dev_first = np.full((n, S_max), -1, dtype=np.int32)
        self.bottleneck = np.full(n, INF, dtype=np.int64)
        self.iter_time = np.full(n, INF, dtype=np.int64)
        self.status = np.full(n, -1, dtype=np.int32)


def build_tables(problem) -> Tables:
    t = Tables(problem)
    if t.rc != 0:
        raise ValueError("oracle_build_tables failed with code %d" % t.rc)
    return t


def plan_batch(tables: Tables, cands, c_begin: int = 0, c_end: int | None = None,
               out: Plans | None = None) -> Plans:
    """Plan candidates c_begin..c_end-1; outputs are indexed by absolute candidate number."""
    c_end = cands.C if c_end is None else c_end
    out = Plans(cands.C, cands.S_max) if out is None else out
    cs, cg, ct = _c32(cands.cand_S), _c32(cands.cand_group), _c32(cands.cand_tp)
    rc = _load().oracle_plan_batch(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(cands.C), C.c_int32(cands.S_max), _ptr(cs), _ptr(cg), _ptr(ct),
        C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.dev_first),
        _ptr(out.bottleneck), _ptr(out.iter_time), _ptr(out.status))
    if rc != 0:
        raise ValueError("oracle_plan_batch failed with code %d" % rc)
    return out


def plan_exact_batch(tables: Tables, cands, c_begin: int = 0, c_end: int | None = None,
                     out: Plans | None = None) -> Plans:
    """Exact optimum of the iteration-time model per candidate (cap sweep); `out.n_caps` counts the
    caps swept."""
    c_end = cands.C if c_end is None else c_end
    out = Plans(cands.C, cands.S_max) if out is None else out
    if not hasattr(out, "n_caps"):
        out.n_caps = np.zeros(cands.C, dtype=np.int32)
    cs, cg, ct = _c32(cands.cand_S), _c32(cands.cand_group), _c32(cands.cand_tp)
    rc = _load().oracle_plan_exact_batch(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(cands.C), C.c_int32(cands.S_max), _ptr(cs), _ptr(cg), _ptr(ct),
        C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.dev_first),
        _ptr(out.bottleneck), _ptr(out.iter_time), _ptr(out.status), _ptr(out.n_caps))
    if rc != 0:
        raise ValueError("oracle_plan_exact_batch failed with code %d" % rc)
    return out


def plan_h1f1b_batch(tables: Tables, cands, t_max, c_begin: int = 0, c_end: int | None = None,
                     out: Plans | None = None) -> Plans:
    """Capped suffix recurrence with H-1F1B warm-up counts, candidate c under the cap t_max[c];
    `out.warmup[c][s]` = forward microbatches stage s launches during warm-up."""
    c_end = cands.C if c_end is None else c_end
    out = Plans(cands.C, cands.S_max) if out is None else out
    if not hasattr(out, "warmup"):
        out.warmup = np.full((cands.C, cands.S_max), -1, dtype=np.int32)
    caps = np.ascontiguousarray(t_max, dtype=np.int64)
    assert caps.shape == (cands.C,)
    cs, cg, ct = _c32(cands.cand_S), _c32(cands.cand_group), _c32(cands.cand_tp)
    rc = _load().oracle_plan_h1f1b_batch(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(cands.C), C.c_int32(cands.S_max), _ptr(cs), _ptr(cg), _ptr(ct), _ptr(caps),
        C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.dev_first), _ptr(out.warmup),
        _ptr(out.bottleneck), _ptr(out.iter_time), _ptr(out.status))
    if rc != 0:
        raise ValueError("oracle_plan_h1f1b_batch failed with code %d" % rc)
    return out


def score_h1f1b(tables: Tables, cands, splits, t_max):
    """Warm-up counts, bottleneck, iteration time and status of given partitions under H-1F1B."""
    sp = _c32(splits)
    assert sp.shape == (cands.C, cands.S_max + 1)
    caps = np.ascontiguousarray(t_max, dtype=np.int64)
    cs, cg, ct = _c32(cands.cand_S), _c32(cands.cand_group), _c32(cands.cand_tp)
    warmup = np.full((cands.C, cands.S_max), -1, dtype=np.int32)
    bott = np.full(cands.C, INF, dtype=np.int64)
    it = np.full(cands.C, INF, dtype=np.int64)
    st = np.full(cands.C, -1, dtype=np.int32)
    rc = _load().oracle_score_h1f1b(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(cands.C), C.c_int32(cands.S_max), _ptr(cs), _ptr(cg), _ptr(ct), _ptr(sp), _ptr(caps),
        _ptr(warmup), _ptr(bott), _ptr(it), _ptr(st))
    if rc != 0:
        raise ValueError("oracle_score_h1f1b failed with code %d" % rc)
    return warmup, bott, it, st


def plan_mesh_batch(tables: Tables, orders, c_begin: int = 0, c_end: int | None = None,
                    out: Plans | None = None, exact: bool = False) -> Plans:
    """Recurrence with the submesh of every stage chosen inside it; `orders` is a batch of group
    orderings.  exact=False: the min-max plan; exact=True: the optimum of the iteration-time model by
    the sweep over the cap (`out.n_caps` counts the caps).  `out.stage_group`, `out.stage_tp` give
    the slicing found."""
    c_end = orders.C if c_end is None else c_end
    out = Plans(orders.C, orders.S_max) if out is None else out
    if not hasattr(out, "stage_group"):
        out.stage_group = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
        out.stage_tp = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    if exact and not hasattr(out, "n_caps"):
        out.n_caps = np.zeros(orders.C, dtype=np.int32)
    os_, og_, ogr = _c32(orders.ord_S), _c32(orders.ord_G), _c32(orders.ord_group)
    args = [C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
            C.c_int32(orders.C), C.c_int32(orders.G_max), C.c_int32(orders.S_max), _ptr(os_), _ptr(og_), _ptr(ogr),
            C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.stage_group), _ptr(out.stage_tp),
            _ptr(out.dev_first), _ptr(out.bottleneck), _ptr(out.iter_time), _ptr(out.status)]
    if exact:
        rc = _load().oracle_plan_mesh_exact_batch(*args, _ptr(out.n_caps))
    else:
        rc = _load().oracle_plan_mesh_batch(*args)
    if rc != 0:
        raise ValueError("oracle mesh planner failed with code %d" % rc)
    return out


def plan_mesh_h1f1b_batch(tables: Tables, orders, t_max, c_begin: int = 0, c_end: int | None = None,
                          out: Plans | None = None) -> Plans:
    """The full recurrence for one cap per ordering: device index and H-1F1B warm-up count in the
    state.  `out.stage_group`, `out.stage_tp`, `out.warmup` describe the plan found."""
    c_end = orders.C if c_end is None else c_end
    out = Plans(orders.C, orders.S_max) if out is None else out
    if not hasattr(out, "stage_group"):
        out.stage_group = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
        out.stage_tp = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    if not hasattr(out, "warmup"):
        out.warmup = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    caps = np.ascontiguousarray(t_max, dtype=np.int64)
    assert caps.shape == (orders.C,)
    os_, og_, ogr = _c32(orders.ord_S), _c32(orders.ord_G), _c32(orders.ord_group)
    rc = _load().oracle_plan_mesh_h1f1b_batch(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(orders.C), C.c_int32(orders.G_max), C.c_int32(orders.S_max), _ptr(os_), _ptr(og_), _ptr(ogr),
        _ptr(caps), C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.stage_group),
        _ptr(out.stage_tp), _ptr(out.dev_first), _ptr(out.warmup), _ptr(out.bottleneck), _ptr(out.iter_time),
        _ptr(out.status))
    if rc != 0:
        raise ValueError("oracle_plan_mesh_h1f1b_batch failed with code %d" % rc)
    return out


def plan_mesh_h1f1b_sweep_batch(tables: Tables, orders, max_caps: int = 1 << 20, c_begin: int = 0,
                                c_end: int | None = None, out: Plans | None = None) -> Plans:
    """The search in full: the cap swept over the candidate values from the smallest feasible one
    to ceil(T / B), the full recurrence at every cap.  `out.t_max` is the cap of the answer,
    `out.n_caps` the caps tried."""
    c_end = orders.C if c_end is None else c_end
    out = Plans(orders.C, orders.S_max) if out is None else out
    if not hasattr(out, "stage_group"):
        out.stage_group = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
        out.stage_tp = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    if not hasattr(out, "warmup"):
        out.warmup = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    if not hasattr(out, "t_max"):
        out.t_max = np.full(orders.C, INF, dtype=np.int64)
        out.n_caps = np.zeros(orders.C, dtype=np.int32)
    os_, og_, ogr = _c32(orders.ord_S), _c32(orders.ord_G), _c32(orders.ord_group)
    rc = _load().oracle_plan_mesh_h1f1b_sweep_batch(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(orders.C), C.c_int32(orders.G_max), C.c_int32(orders.S_max), _ptr(os_), _ptr(og_), _ptr(ogr),
        C.c_int32(max_caps), C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.stage_group),
        _ptr(out.stage_tp), _ptr(out.dev_first), _ptr(out.warmup), _ptr(out.bottleneck), _ptr(out.iter_time),
        _ptr(out.status), _ptr(out.t_max), _ptr(out.n_caps))
    if rc != 0:
        raise ValueError("oracle_plan_mesh_h1f1b_sweep_batch failed with code %d" % rc)
    return out


def plan_h1f1b_sweep_batch(tables: Tables, cands, max_caps: int = 1 << 20, c_begin: int = 0,
                           c_end: int | None = None, out: Plans | None = None) -> Plans:
    """The same search for candidates (fixed slicing): the cap swept from the hot path's bottleneck
    to ceil(T / B), the capped H-1F1B recurrence at every cap.  `out.warmup`, `out.t_max`,
    `out.n_caps` as for the submesh form."""
    c_end = cands.C if c_end is None else c_end
    out = Plans(cands.C, cands.S_max) if out is None else out
    if not hasattr(out, "warmup"):
        out.warmup = np.full((cands.C, cands.S_max), -1, dtype=np.int32)
    if not hasattr(out, "t_max"):
        out.t_max = np.full(cands.C, INF, dtype=np.int64)
        out.n_caps = np.zeros(cands.C, dtype=np.int32)
    cs, cg, ct = _c32(cands.cand_S), _c32(cands.cand_group), _c32(cands.cand_tp)
    rc = _load().oracle_plan_h1f1b_sweep_batch(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(cands.C), C.c_int32(cands.S_max), _ptr(cs), _ptr(cg), _ptr(ct), C.c_int32(max_caps),
        C.c_int32(c_begin), C.c_int32(c_end), _ptr(out.splits), _ptr(out.dev_first), _ptr(out.warmup),
        _ptr(out.bottleneck), _ptr(out.iter_time), _ptr(out.status), _ptr(out.t_max), _ptr(out.n_caps))
    if rc != 0:
        raise ValueError("oracle_plan_h1f1b_sweep_batch failed with code %d" % rc)
    return out


def score_1f1b(tables: Tables, cands, splits):
    sp = _c32(splits)
    assert sp.shape == (cands.C, cands.S_max + 1)
    cs, cg, ct = _c32(cands.cand_S), _c32(cands.cand_group), _c32(cands.cand_tp)
    bott = np.full(cands.C, INF, dtype=np.int64)
    it = np.full(cands.C, INF, dtype=np.int64)
    st = np.full(cands.C, -1, dtype=np.int32)
    rc = _load().oracle_score_1f1b(
        C.byref(tables.c), _ptr(tables.PF), _ptr(tables.PP), _ptr(tables.PS), _ptr(tables.PR),
        C.c_int32(cands.C), C.c_int32(cands.S_max), _ptr(cs), _ptr(cg), _ptr(ct), _ptr(sp),
        _ptr(bott), _ptr(it), _ptr(st))
    if rc != 0:
        raise ValueError("oracle_score_1f1b failed with code %d" % rc)
    return bott, it, st


def argmin_batch(iter_time, status):
    it, st = _c64(iter_time), _c32(status)
    bt = C.c_int64(0)
    bi = C.c_int32(0)
    _load().oracle_argmin_batch(C.c_int32(it.shape[0]), _ptr(it), _ptr(st), C.byref(bt), C.byref(bi))
    return int(bt.value), int(bi.value)
