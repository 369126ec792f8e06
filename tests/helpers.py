"""Small constructors shared by the tests (inputs only, no planner arithmetic)."""
import numpy as np

from paper_2509_24859_amd.workloads import Candidates, Problem

BIG = 1 << 40


def simple_problem(costs, M=1, T=1, G=1, ndev=(1,), tp=(1,), act=None, params=None, stash=None,
                   mem=None, bw=None, gtype=None, fwd=None, bwd=None, ar_count=4):
    """Problem whose operator l costs costs[l] (forward+backward, all in the forward entry)."""
    costs = np.asarray(costs, dtype=np.int64)
    L = costs.shape[-1]
    if fwd is None:
        fwd = np.tile(costs, (T, 1)) if costs.ndim == 1 else costs
        bwd = np.zeros_like(fwd)
    z = np.zeros(L, dtype=np.int64)
    return Problem(
        L=L, T=T, G=G, M=M, ar_count=ar_count, tp_degrees=np.asarray(tp, dtype=np.int32),
        fwd_us=np.ascontiguousarray(fwd, dtype=np.int64),
        bwd_us=np.ascontiguousarray(bwd, dtype=np.int64),
        param_bytes=z.copy() if params is None else np.asarray(params, dtype=np.int64),
        stash_bytes=z.copy() if stash is None else np.asarray(stash, dtype=np.int64),
        act_bytes=z.copy() if act is None else np.asarray(act, dtype=np.int64),
        group_type=np.zeros(G, dtype=np.int32) if gtype is None else np.asarray(gtype, np.int32),
        group_ndev=np.asarray(ndev, dtype=np.int32),
        type_mem_bytes=np.full(T, BIG, dtype=np.int64) if mem is None else np.asarray(mem, np.int64),
        bw=np.full((G, G), 1, dtype=np.int64) if bw is None else np.asarray(bw, dtype=np.int64))


def cands_from_lists(slot_lists, S_max=None):
    """slot_lists: per candidate a list of (group, tp)."""
    S_max = max(len(s) for s in slot_lists) if S_max is None else S_max
    C = len(slot_lists)
    cg = np.full((C, S_max), -1, dtype=np.int32)
    ct = np.zeros((C, S_max), dtype=np.int32)
    cs = np.zeros(C, dtype=np.int32)
    for c, sl in enumerate(slot_lists):
        cs[c] = len(sl)
        for s, (g, t) in enumerate(sl[:S_max]):
            cg[c, s], ct[c, s] = g, t
    return Candidates(C, S_max, cs, cg, ct)


def same_slot(S, g=0, tp=1):
    return [(g, tp)] * S


def read_golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line)
    return rows


def oracle_plan_threaded(tables, cands, threads=None, step=16):
    """Oracle plans for a whole batch, candidates spread over host threads (ctypes drops the GIL)."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(cands.C, cands.S_max)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda lo: oracle.plan_batch(tables, cands, lo, min(lo + step, cands.C), out),
                    range(0, cands.C, step)))
    return out


def oracle_plan_exact_threaded(tables, cands, threads=None):
    """Oracle exact-optimum plans for a whole batch, one candidate per task over host threads."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(cands.C, cands.S_max)
    out.n_caps = np.zeros(cands.C, dtype=np.int32)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda c: oracle.plan_exact_batch(tables, cands, c, c + 1, out), range(cands.C)))
    return out


def oracle_plan_h1f1b_threaded(tables, cands, t_max, threads=None, step=8):
    """Oracle H-1F1B plans for a whole batch, candidates spread over host threads."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(cands.C, cands.S_max)
    out.warmup = np.full((cands.C, cands.S_max), -1, dtype=np.int32)
    caps = np.ascontiguousarray(t_max, dtype=np.int64)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda lo: oracle.plan_h1f1b_batch(tables, cands, caps, lo, min(lo + step, cands.C), out),
                    range(0, cands.C, step)))
    return out


def oracle_plan_mesh_threaded(tables, orders, threads=None, exact=False):
    """Oracle submesh plans for a whole batch of orderings, one ordering per task over host threads."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(orders.C, orders.S_max)
    out.stage_group = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.stage_tp = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.n_caps = np.zeros(orders.C, dtype=np.int32)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda c: oracle.plan_mesh_batch(tables, orders, c, c + 1, out, exact), range(orders.C)))
    return out


def oracle_plan_mesh_h1f1b_threaded(tables, orders, t_max, threads=None):
    """Oracle plans of the full recurrence (device index and H-1F1B count) for a batch of orderings."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(orders.C, orders.S_max)
    out.stage_group = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.stage_tp = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.warmup = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    caps = np.ascontiguousarray(t_max, dtype=np.int64)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda c: oracle.plan_mesh_h1f1b_batch(tables, orders, caps, c, c + 1, out), range(orders.C)))
    return out


def oracle_plan_mesh_h1f1b_sweep_threaded(tables, orders, max_caps=1 << 20, threads=None):
    """Oracle answers of the search around the full recurrence for a batch of orderings."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(orders.C, orders.S_max)
    out.stage_group = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.stage_tp = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.warmup = np.full((orders.C, orders.S_max), -1, dtype=np.int32)
    out.t_max = np.full(orders.C, oracle.INF, dtype=np.int64)
    out.n_caps = np.zeros(orders.C, dtype=np.int32)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda c: oracle.plan_mesh_h1f1b_sweep_batch(tables, orders, max_caps, c, c + 1, out),
                    range(orders.C)))
    return out


def oracle_plan_h1f1b_sweep_threaded(tables, cands, max_caps=1 << 20, threads=None):
    """Oracle answers of the search over the cap for a batch of candidates (fixed slicing)."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    out = oracle.Plans(cands.C, cands.S_max)
    out.warmup = np.full((cands.C, cands.S_max), -1, dtype=np.int32)
    out.t_max = np.full(cands.C, oracle.INF, dtype=np.int64)
    out.n_caps = np.zeros(cands.C, dtype=np.int32)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda c: oracle.plan_h1f1b_sweep_batch(tables, cands, max_caps, c, c + 1, out), range(cands.C)))
    return out


def assert_plans_equal(got, want, label=""):
    """Bit-exact comparison of every output array of a batch."""
    for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
        a, b = getattr(got, name), getattr(want, name)
        if not (a == b).all():
            bad = np.nonzero((a != b).reshape(a.shape[0], -1).any(axis=1))[0]
            raise AssertionError("%s: %s differs at %d candidates, first %d: got %s want %s"
                                 % (label, name, bad.size, bad[0], a[bad[0]], b[bad[0]]))
