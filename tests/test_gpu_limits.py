"""GPU parity at the stated limits of the entry points: the largest stage count, the longest
sequence the 32-bit path takes, sequences beyond it (int64 path), and S = L."""
import numpy as np
import pytest

import oracle
from paper_2509_24859_amd import workloads as W

from helpers import (assert_plans_equal, cands_from_lists, oracle_plan_exact_threaded, oracle_plan_h1f1b_threaded,
                     oracle_plan_threaded, same_slot, simple_problem)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(harp):
    c = harp.Context(0)
    yield c
    c.close()


ROWS_MAX_L = 1024      # the 32-bit H-1F1B and submesh kernels keep whole rows of several arrays in LDS


def _all_entry_points(harp, ctx, p, cands, label, exact=True):
    tables = oracle.build_tables(p)
    want = oracle_plan_threaded(tables, cands)
    fast32 = harp.Tables(ctx, p).fast32
    paths = [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if fast32 else [])
    row_paths = [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if fast32 and p.L <= ROWS_MAX_L else [])
    for path in paths:
        got, _ = harp.plan(ctx, p, cands, path)
        assert_plans_equal(got, want, "%s min-max path %d" % (label, path))
    caps = np.where(want.status == oracle.OK, want.bottleneck // 8 * 9, 3).astype(np.int64)
    want_h = oracle_plan_h1f1b_threaded(tables, cands, caps)
    for path in row_paths:
        got, _ = harp.plan_h1f1b(ctx, p, cands, caps, path)
        assert_plans_equal(got, want_h, "%s H-1F1B path %d" % (label, path))
        assert (got.warmup == want_h.warmup).all()
    if fast32 and p.L > ROWS_MAX_L:          # asked for by name where it does not exist: an error, no fallback
        with pytest.raises(harp.HarpError) as e:
            harp.plan_h1f1b(ctx, p, cands, caps, harp.PATH_FAST32)
        assert e.value.code == harp.ERR_UNIMPLEMENTED
    if exact:
        want_e = oracle_plan_exact_threaded(tables, cands)
        for path in paths:
            got, _, _ = harp.plan_exact(ctx, p, cands, path)
            assert_plans_equal(got, want_e, "%s exact path %d" % (label, path))
    elif fast32:
        # too long for the oracle's sweep to stay in seconds: the two arithmetic paths against each other
        a, _, _ = harp.plan_exact(ctx, p, cands, harp.PATH_GENERIC)
        b, _, _ = harp.plan_exact(ctx, p, cands, harp.PATH_FAST32)
        assert_plans_equal(b, a, "%s exact, 32-bit against int64" % label)
        assert ((a.iter_time <= want.iter_time) | (want.status != oracle.OK)).all()
    return want, fast32


def test_largest_stage_count(harp, ctx):
    """S = S_max = 256 stages on one group of 256 devices."""
    rng = np.random.default_rng(41)
    L = 300
    p = simple_problem(np.zeros(L), M=300, G=1, ndev=(256,), tp=(1, 2),
                       fwd=rng.integers(1, 500, size=(1, L)), bwd=rng.integers(1, 900, size=(1, L)),
                       act=rng.integers(0, 10**4, size=L), params=rng.integers(0, 1000, size=L),
                       stash=rng.integers(0, 50, size=L), mem=[40000], bw=[[50]])
    cands = cands_from_lists([same_slot(256), same_slot(255), same_slot(200), [(0, 2)] * 128, [(0, 2)] * 129],
                             S_max=256)
    want, fast32 = _all_entry_points(harp, ctx, p, cands, "256 stages", exact=False)
    assert fast32 and list(want.status[:4]) == [0, 0, 0, 0] and want.status[4] == oracle.INVALID
    # one beyond the limit is an argument error, not a silent truncation
    import torch
    tables = harp.Tables(ctx, p)
    over = cands_from_lists([same_slot(256)], S_max=257)
    with pytest.raises(harp.HarpError) as e:
        dc = harp.DeviceCandidates(ctx, over)
        out = harp.DevicePlans(ctx, 1, 257)
        harp.harp_plan_batch(ctx, tables, dc, out, torch.empty(1 << 20, dtype=torch.uint8, device=ctx.device))
    assert e.value.code == harp.ERR_SHAPE


def test_every_operator_its_own_stage(harp, ctx):
    """S = L: the only partition has one operator per stage; S = L + 1 has none."""
    rng = np.random.default_rng(42)
    L = 64
    p = simple_problem(rng.integers(1, 100, size=L), M=7, G=2, ndev=(40, 40), tp=(1, 2),
                       act=rng.integers(0, 2000, size=L), bw=[[100, 7], [7, 90]])
    slots = [(0, 1)] * 30 + [(1, 1)] * 34
    cands = cands_from_lists([slots, slots + [(1, 1)], slots[:-1]], S_max=65)
    want, _ = _all_entry_points(harp, ctx, p, cands, "S = L")
    assert list(want.status) == [oracle.OK, oracle.INFEASIBLE, oracle.OK]
    assert list(want.splits[0, :L + 1]) == list(range(L + 1))


def test_longest_sequence_of_the_32_bit_path_and_beyond(harp, ctx):
    """L = 1024 is the last length with 32-bit kernels behind every entry point, 4096 the last for
    the min-max planner and the exact search; past each limit the int64 path takes over with the same
    results."""
    rng = np.random.default_rng(43)
    for L, expect_fast in ((1024, True), (1025, True), (2048, True), (4096, True), (4097, False)):
        G = 3
        bw = rng.integers(20, 4000, size=(G, G))
        # many microbatches keep [t_S, t_E] narrow, so that the oracle's sweep stays in seconds
        p = simple_problem(np.zeros(L), M=5000, T=2, G=G, ndev=(8, 8, 8), tp=(1, 2, 4),
                           fwd=rng.integers(1, 2000, size=(2, L)), bwd=rng.integers(1, 3000, size=(2, L)),
                           act=rng.integers(0, 10**6, size=L), params=rng.integers(1, 10**5, size=L),
                           stash=rng.integers(0, 10**3, size=L), gtype=[0, 1, 0],
                           mem=[int(4e7), int(3e7)], bw=np.minimum(bw, bw.T))
        cands = W.make_candidates(p, L, 91, G, 6, 0, 6 if L > 2000 else 16)
        print("L = %d" % L, flush=True)
        want, fast32 = _all_entry_points(harp, ctx, p, cands, "L = %d" % L, exact=(L <= 2048))
        assert fast32 == expect_fast and (want.status == oracle.OK).any()


def test_many_device_groups(harp, ctx):
    """More than 64 groups (the pre-pass checks re-entered groups against the slot list instead of a
    bit mask) and more than 2,048 (group types and sizes are read from memory, not LDS; the per-link
    table of the 32-bit path is out of reach, so only the int64 path runs)."""
    rng = np.random.default_rng(48)
    for G, L in ((100, 150), (2100, 60)):
        T = 3
        bw = rng.integers(5, 3000, size=(G, G))
        p = simple_problem(np.zeros(L), M=6, T=T, G=G, ndev=rng.integers(1, 3, size=G) * 2, tp=(1, 2),
                           fwd=rng.integers(1, 900, size=(T, L)), bwd=rng.integers(1, 900, size=(T, L)),
                           act=rng.integers(0, 10**5, size=L), params=rng.integers(1, 10**4, size=L),
                           stash=rng.integers(0, 10**3, size=L), gtype=rng.integers(0, T, size=G),
                           mem=[int(6e4 * L / 150), int(4e4 * L / 150), int(3e4 * L / 150)], bw=np.minimum(bw, bw.T))
        lists = []
        for n in range(40):
            S = int(rng.integers(2, 101 if G == 100 else 50))      # up to 100 stages: the pre-pass's 128-thread shape
            order = rng.permutation(G)[:S]
            lists.append([(int(g), int(rng.integers(1, 3))) for g in order])
        a, b = int(rng.integers(0, G)), int(rng.integers(0, G - 1))
        b += b >= a
        lists.append([(a, 1), (b, 1), (a, 1)])                      # a group left and entered again
        lists.append([(a, 1)] * (int(p.group_ndev[a]) + 1))         # more devices than the group has
        lists.append([(G - 1, 2), (0, 1), (G - 2, 1), (G - 2, 1)])
        cands = cands_from_lists(lists)
        want = oracle_plan_threaded(oracle.build_tables(p), cands)
        assert list(want.status[40:42]) == [oracle.INVALID, oracle.INVALID]
        assert (want.status == oracle.OK).sum() >= 10 and (want.status == oracle.INFEASIBLE).sum() >= 5
        fast32 = harp.Tables(ctx, p).fast32
        assert fast32 == (G == 100)
        for path in [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if fast32 else []):
            got, _ = harp.plan(ctx, p, cands, path)
            assert_plans_equal(got, want, "%d groups path %d" % (G, path))


def test_sequences_beyond_the_feasibility_index(harp, ctx):
    """The pre-pass builds its index of fitting ranges for sequences of up to 16,383 operators and up to
    256 MiB; beyond either limit the int64 planner runs without bands (the dense kernel), with the
    same results."""
    rng = np.random.default_rng(47)
    # (L, T, degrees, M, S_max): the first is too long for the index, the second makes it too large
    for L, T, tp, M, S_max in ((17000, 2, (1, 2), 40, 4), (12000, 8, (1, 2, 4, 8, 16, 32, 64, 128), 100, 100)):
        G = 3
        bw = rng.integers(20, 4000, size=(G, G))
        p = simple_problem(np.zeros(L), M=M, T=T, G=G, ndev=(128, 128, 128), tp=tp,
                           fwd=rng.integers(1, 200, size=(T, L)), bwd=rng.integers(1, 300, size=(T, L)),
                           act=rng.integers(0, 10**6, size=L), params=rng.integers(1, 10**5, size=L),
                           stash=rng.integers(0, 10**3, size=L), gtype=rng.integers(0, T, size=G),
                           mem=[int(6e8)] * T, bw=np.minimum(bw, bw.T))
        slots = [[(0, 1), (1, 2), (2, 1)], [(2, 2), (0, 1), (0, 1), (1, 1)], [(1, 1), (1, 1)], [(0, 2)] * 3 + [(1, 1)]]
        cands = cands_from_lists(slots[:3] if L > 16383 else slots, S_max=S_max)
        print("L = %d, S_max = %d" % (L, S_max), flush=True)
        want = oracle_plan_threaded(oracle.build_tables(p), cands)
        assert not harp.Tables(ctx, p).fast32 and (want.status == oracle.OK).any()
        got, _ = harp.plan(ctx, p, cands, harp.PATH_GENERIC)
        assert_plans_equal(got, want, "L = %d without the index" % L)


def test_argument_errors_of_the_newer_entry_points(harp, ctx):
    """Every planner entry point refuses a short or misaligned workspace, null arrays and shapes
    beyond its limits with an error code, and launches nothing."""
    import torch
    w = W.make("tiny")
    tables = harp.Tables(ctx, w.problem)
    dc = harp.DeviceCandidates(ctx, w.candidates())
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    ws = harp.plan_workspace(ctx, tables, dc)
    small = torch.empty(256, dtype=torch.uint8, device=ctx.device)
    caps = torch.zeros(dc.C, dtype=torch.int64, device=ctx.device)
    warm = torch.zeros((dc.C, dc.S_max), dtype=torch.int32, device=ctx.device)

    class Null:
        @staticmethod
        def data_ptr():
            return None

    calls = {
        "exact": lambda work: harp.harp_plan_exact_batch(ctx, tables, dc, out, work),
        "h1f1b": lambda work: harp.harp_plan_h1f1b_batch(ctx, tables, dc, caps, out, warm, work),
    }
    for name, call in calls.items():
        for work, code in ((small, harp.ERR_WORKSPACE), (ws[1:], harp.ERR_WORKSPACE)):
            with pytest.raises(harp.HarpError) as e:
                call(work)
            assert e.value.code == code, name
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_h1f1b_batch(ctx, tables, dc, Null, out, warm, ws)
    assert e.value.code == harp.ERR_INVALID_ARG
    with pytest.raises(harp.HarpError) as e:
        harp.harp_score_h1f1b(ctx, tables, dc, out.splits, caps, Null, out.bottleneck, out.iter_time, out.status)
    assert e.value.code == harp.ERR_INVALID_ARG

    orders = W.make_orderings(w.problem, 0, 1, 2, 4, 0, 8)
    do = harp.DeviceOrderings(ctx, orders)
    mout = harp.DevicePlans(ctx, do.C, do.S_max)
    sg = torch.zeros((do.C, do.S_max), dtype=torch.int32, device=ctx.device)
    mws = harp.mesh_workspace(ctx, tables, do)
    for work in (small, mws[1:]):
        with pytest.raises(harp.HarpError) as e:
            harp.harp_plan_mesh_batch(ctx, tables, do, mout, sg, sg.clone(), work)
        assert e.value.code == harp.ERR_WORKSPACE
        with pytest.raises(harp.HarpError) as e:
            harp.harp_plan_mesh_exact_batch(ctx, tables, do, mout, sg, sg.clone(), work)
        assert e.value.code == harp.ERR_WORKSPACE
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_mesh_batch(ctx, tables, do, mout, Null, sg, mws)
    assert e.value.code == harp.ERR_INVALID_ARG
    do.c.G_max = 5000
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_mesh_batch(ctx, tables, do, mout, sg, sg.clone(), mws)
    assert e.value.code == harp.ERR_SHAPE
    with pytest.raises(harp.HarpError) as e:
        harp.harp_measure_valu_int32(ctx, 0, 10, small)
    assert e.value.code == harp.ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert (out.to_host().status == -7).all()          # nothing ran


def test_device_index_larger_than_32_bits_is_refused(harp, ctx):
    """The kernels with a device index address (devices + 1) x (L + 1) states per stage with 32-bit
    products: a problem beyond that is refused on the host with a shape error (it would need tens of
    GB of workspace anyway), never run with a wrapped index."""
    import torch
    L = 60000
    p = simple_problem(np.ones(L, dtype=np.int64), M=2, G=1, ndev=(40000,), tp=(1,))
    tables = harp.Tables(ctx, p)
    orders = W.Orderings(1, 1, 2, np.array([2], dtype=np.int32), np.array([1], dtype=np.int32),
                         np.zeros((1, 1), dtype=np.int32))
    do = harp.DeviceOrderings(ctx, orders)
    out = harp.DevicePlans(ctx, 1, 2)
    out.poison()
    sg = torch.zeros((1, 2), dtype=torch.int32, device=ctx.device)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=ctx.device)
    for call in (lambda: harp.harp_plan_mesh_batch(ctx, tables, do, out, sg, sg.clone(), ws),
                 lambda: harp.harp_plan_mesh_exact_batch(ctx, tables, do, out, sg, sg.clone(), ws)):
        with pytest.raises(harp.HarpError) as e:
            call()
        assert e.value.code == harp.ERR_SHAPE and "2^31" in str(e.value)
    torch.cuda.synchronize()
    assert (out.to_host().status == -7).all()


def test_calls_on_a_caller_stream_and_back_to_back(harp, ctx):
    """Every entry point enqueues on the stream it is given; calls queued back to back on one stream
    with one workspace (each after the other, no host synchronisation in between) give the same
    results as calls made one at a time."""
    import torch
    w = W.make("llama70b")
    cands = w.candidates(0, 2048)
    ref, _ = harp.plan(ctx, w.problem, cands)
    ref_exact, _, _ = harp.plan_exact(ctx, w.problem, cands)
    side = torch.cuda.Stream()                      # default priority
    with torch.cuda.stream(side):
        tables = harp.Tables(ctx, w.problem, side)
        dc = harp.DeviceCandidates(ctx, cands)
        out1 = harp.DevicePlans(ctx, dc.C, dc.S_max)
        out2 = harp.DevicePlans(ctx, dc.C, dc.S_max)
        out3 = harp.DevicePlans(ctx, dc.C, dc.S_max)
        ws = harp.plan_workspace(ctx, tables, dc)
        best_t = torch.empty(1, dtype=torch.int64, device=ctx.device)
        best_i = torch.empty(1, dtype=torch.int32, device=ctx.device)
        harp.harp_plan_batch(ctx, tables, dc, out1, ws, side)
        harp.harp_plan_exact_batch(ctx, tables, dc, out2, ws, None, side)
        harp.harp_plan_batch(ctx, tables, dc, out3, ws, side)
        harp.harp_argmin_batch(ctx, dc.C, out2.iter_time, out2.status, best_t, best_i, side)
    side.synchronize()
    a, b, c = out1.to_host(), out2.to_host(), out3.to_host()
    for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
        assert (getattr(a, name) == getattr(ref, name)).all(), name
        assert (getattr(c, name) == getattr(ref, name)).all(), name
        assert (getattr(b, name) == getattr(ref_exact, name)).all(), name
    assert (int(best_t.item()), int(best_i.item())) == oracle.argmin_batch(ref_exact.iter_time, ref_exact.status)


def test_planner_calls_inside_a_hip_graph(harp, ctx):
    """The planner launches are plain kernel launches on the caller's stream (counters are cleared by
    a kernel, never by a memset), so a caller may capture them: a graph of plan + exact + argmin is
    replayed several times, with the candidates changed in place and eager work in between, and
    every replay is compared with eager calls on the same inputs."""
    import torch
    w = W.make("llama7b")
    all_cands = w.candidates()
    tables = harp.Tables(ctx, w.problem)                 # built and finalized outside the graph
    first = all_cands.slice(0, 256)
    dc = harp.DeviceCandidates(ctx, first)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    out_e = harp.DevicePlans(ctx, dc.C, dc.S_max)
    ws = harp.plan_workspace(ctx, tables, dc)
    best_t = torch.empty(1, dtype=torch.int64, device=ctx.device)
    best_i = torch.empty(1, dtype=torch.int32, device=ctx.device)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                        # warm-up on the capture stream
        harp.harp_plan_batch(ctx, tables, dc, out, ws, side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        s = torch.cuda.current_stream()
        harp.harp_plan_batch(ctx, tables, dc, out, ws, s)
        harp.harp_plan_exact_batch(ctx, tables, dc, out_e, ws, None, s)
        harp.harp_argmin_batch(ctx, dc.C, out_e.iter_time, out_e.status, best_t, best_i, s)
    for k in range(4):
        batch = all_cands.slice(256 * k, 256 * (k + 1))
        dc.cs.copy_(torch.from_numpy(batch.cand_S))
        dc.cg.copy_(torch.from_numpy(batch.cand_group))
        dc.ct.copy_(torch.from_numpy(batch.cand_tp))
        out.poison()
        out_e.poison()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, got_e = out.to_host(), out_e.to_host()
        want, _ = harp.plan(ctx, w.problem, batch)       # eager work between the replays
        want_e, _, _ = harp.plan_exact(ctx, w.problem, batch)
        for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
            assert (getattr(got, name) == getattr(want, name)).all(), (k, name)
            assert (getattr(got_e, name) == getattr(want_e, name)).all(), (k, name)
        assert (int(best_t.item()), int(best_i.item())) == oracle.argmin_batch(want_e.iter_time, want_e.status)
