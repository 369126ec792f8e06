"""GPU parity: the HIP library behind the C ABI against the CPU oracle, bit for bit."""
import os

import numpy as np
import pytest

import oracle
from paper_2509_24859_amd import workloads as W

from helpers import (BIG, assert_plans_equal, cands_from_lists, oracle_plan_threaded, same_slot,
                     simple_problem)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(harp):
    c = harp.Context(0)
    yield c
    c.close()


def _paths(harp, tables):
    return [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if tables.fast32 else [])


def _plan_all_paths(harp, ctx, problem, cands, want, label):
    import torch
    tables = harp.Tables(ctx, problem)
    dc = harp.DeviceCandidates(ctx, cands)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    ws = harp.plan_workspace(ctx, tables, dc)
    ran = []
    for path in _paths(harp, tables):
        out.poison()
        ctx.set_plan_path(path)
        try:
            harp.harp_plan_batch(ctx, tables, dc, out, ws)
            torch.cuda.synchronize()
        finally:
            ctx.set_plan_path(harp.PATH_AUTO)
        assert_plans_equal(out.to_host(), want, "%s path %d" % (label, path))
        ran.append(path)
    return tables, ran


# ------------------------------------------------------------------ tables (a1)

@pytest.mark.parametrize("name", W.ORDER)
def test_tables_match_oracle(harp, ctx, name):
    w = W.make(name)
    want = oracle.build_tables(w.problem)
    tables = harp.Tables(ctx, w.problem)
    PF, PP, PS, PR = tables.host_copies()
    assert (PF == want.PF).all() and (PP == want.PP).all() and (PS == want.PS).all()
    assert (PR == want.PR).all()
    assert tables.fast32


def test_tables_match_oracle_long_rows(harp, ctx):
    """Rows spanning several scan chunks with a ragged tail (L = 5000: 4 full chunks + 904)."""
    rng = np.random.default_rng(1)
    L, T, G = 5000, 3, 5
    fwd = rng.integers(0, 5000, size=(T, L))
    bwd = rng.integers(0, 9000, size=(T, L))
    bw = rng.integers(1, 500, size=(G, G))
    bw = np.minimum(bw, bw.T)
    p = simple_problem(np.zeros(L), M=7, T=T, G=G, ndev=[8] * G, tp=(1, 2, 3, 8),
                       fwd=fwd, bwd=bwd, params=rng.integers(0, 10**9, size=L),
                       stash=rng.integers(0, 10**8, size=L), act=rng.integers(0, 10**7, size=L),
                       gtype=rng.integers(0, T, size=G), bw=bw)
    want = oracle.build_tables(p)
    tables = harp.Tables(ctx, p)
    PF, PP, PS, PR = tables.host_copies()
    assert (PF == want.PF).all() and (PP == want.PP).all() and (PS == want.PS).all()
    assert (PR == want.PR).all()
    assert not tables.fast32          # degree 3 and L > 1024


def test_tables_match_oracle_operator_level(harp, ctx):
    """The long-sequence problem of the streaming measurement at a length the oracle finishes in
    seconds: 300,001 operators = 1,171 full wavefront runs and a ragged tail, 138 rows, built by
    the chunk-major kernels; 262,144, their shortest sequence, which ends with a full run (the last
    table entry then lies one past the last run's window of stores); and 100,003 operators, built by
    the row-parallel ones."""
    for L in (300001, 262144, 100003):
        _check_operator_level(harp, ctx, L)
    # groups whose own links differ (every third one alike): the chunk-major kernels reuse a row only
    # when the one walked just before it has the same link speed and degree
    _check_operator_level(harp, ctx, 270001, own_links=lambda g: 400_000 - 1000 * (g % 3) - (17 * g if g > 20 else 0))


def test_tables_beyond_a_million_operators(harp, ctx):
    """1,100,003 operators, 7 table rows: more than 4,096 runs of 256 operators per row, so a thread of
    the scan over the run sums takes more sums than it keeps in registers; and few enough rows that a
    launch has a single row part."""
    rng = np.random.default_rng(77)
    L = 1_100_003
    fwd = rng.integers(1, 3000, size=(1, L))
    p = simple_problem(np.zeros(L), M=4, T=1, G=2, ndev=(4, 4), tp=(1, 2), fwd=fwd, bwd=2 * fwd,
                       params=rng.integers(0, 1 << 22, size=L), stash=rng.integers(0, 1 << 18, size=L),
                       act=rng.integers(0, 1 << 26, size=L), bw=[[40000, 125], [125, 35000]])
    want = oracle.build_tables(p)
    tables = harp.Tables(ctx, p)
    PF, PP, PS, PR = tables.host_copies()
    assert (PF == want.PF).all() and (PP == want.PP).all() and (PS == want.PS).all()
    assert (PR == want.PR).all()


def _check_operator_level(harp, ctx, L, own_links=None):
    p = W.long_sequence(L)
    if own_links is not None:
        for g in range(p.G):
            p.bw[g, g] = own_links(g)
    want = oracle.build_tables(p)
    tables = harp.Tables(ctx, p)
    PF, PP, PS, PR = tables.host_copies()
    assert (PF == want.PF).all() and (PP == want.PP).all() and (PS == want.PS).all()
    assert (PR == want.PR).all()


def test_tables_large_quotients(harp, ctx):
    """All-reduce and cut times whose operands leave the range of the fast division."""
    rng = np.random.default_rng(6)
    L = 300
    act = rng.integers(0, 1 << 58, size=L)
    act[::7] = rng.integers(0, 1 << 20, size=act[::7].shape)
    p = simple_problem([1] * L, M=2, G=2, ndev=(4, 4), tp=(1, 2, 4), act=act, ar_count=1,
                       bw=[[3, 1 << 55], [1 << 55, (1 << 53) + 5]])
    want = oracle.Tables(p)
    assert want.rc == oracle.ERR_OVERFLOW          # times beyond 2^47: both sides must refuse
    with pytest.raises(harp.HarpError):
        harp.Tables(ctx, p)
    act = rng.integers(0, 1 << 40, size=L)
    p = simple_problem([1] * L, M=2, G=2, ndev=(4, 4), tp=(1, 2, 4), act=act, ar_count=3,
                       bw=[[7, 1 << 30], [1 << 30, (1 << 33) + 5]])
    want = oracle.build_tables(p)
    PF, PP, PS, PR = harp.Tables(ctx, p).host_copies()
    assert (PR == want.PR).all() and (PF == want.PF).all()


def test_tables_random_small(harp, ctx):
    for seed in range(60):
        w = W.random_small(seed)
        want = oracle.build_tables(w.problem)
        PF, PP, PS, PR = harp.Tables(ctx, w.problem).host_copies()
        assert (PF == want.PF).all() and (PP == want.PP).all() and (PS == want.PS).all()
        assert (PR == want.PR).all(), seed


def test_build_verdicts(harp, ctx):
    cases = [
        (simple_problem([1, -1], ndev=(2,)), harp.ERR_INVALID_ARG),
        (simple_problem([1, 1], ndev=(2,), bw=[[0]]), harp.ERR_INVALID_ARG),
        (simple_problem([1, 1], ndev=(0,)), harp.ERR_INVALID_ARG),
        (simple_problem([1, 1], ndev=(2,), gtype=[3]), harp.ERR_INVALID_ARG),
        (simple_problem([1, 1], ndev=(2,), mem=[-5]), harp.ERR_INVALID_ARG),
        (simple_problem([1 << 46, 1 << 46], ndev=(2,)), harp.ERR_OVERFLOW),
        (simple_problem([1 << 45, 1 << 45], M=1 << 17, ndev=(2,)), harp.ERR_OVERFLOW),
        (simple_problem([1 << 61, 1 << 61], ndev=(2,)), harp.ERR_OVERFLOW),
        (simple_problem([1, 1], ndev=(2,), params=[(1 << 61) - 1] * 2, stash=[(1 << 61) - 1] * 2, M=64),
         harp.ERR_OVERFLOW),
    ]
    for p, code in cases:
        assert oracle.Tables(p).rc == (oracle.ERR_BAD_ARG if code == harp.ERR_INVALID_ARG
                                       else oracle.ERR_OVERFLOW)
        with pytest.raises(harp.HarpError) as e:
            harp.Tables(ctx, p)
        assert e.value.code == code
    ok = simple_problem([1 << 40, 1 << 40], ndev=(2,))
    assert oracle.Tables(ok).rc == 0
    t = harp.Tables(ctx, ok)
    assert not t.fast32                      # times beyond 32 bits: only the int64 path


def _verdict_cases():
    """Problems on both sides of every magnitude limit (all sums, products and times that must stay
    inside int64 or below 2^47 us): (label, problem)."""
    top = (1 << 63) - 1
    cases = []

    def add(label, p):
        cases.append((label, p))
    # largest stage time any plan can see: below 2^47
    add("time 2^47 - 1", simple_problem([1 << 46, (1 << 46) - 1], ndev=(2,)))
    add("time 2^47", simple_problem([1 << 46, 1 << 46], ndev=(2,)))
    # a long sequence (chunk-major build): the iteration-time bound worst x (3 L + M) decides
    long_costs = np.zeros(300001, dtype=np.int64)
    long_costs[123456] = ((1 << 63) - 1) // (3 * 300001 + 1)
    add("one huge operator among 300,001, at the limit", simple_problem(long_costs, ndev=(2,)))
    long_costs = long_costs.copy()
    long_costs[299999] = 1
    add("one huge operator among 300,001, beyond", simple_problem(long_costs, ndev=(2,)))
    # iteration time: worst x (3 L + M) inside int64
    w = 1 << 40
    m_ok = top // w - 3 * 2
    add("iteration time at the limit", simple_problem([w - 1, 1], M=int(m_ok), ndev=(2,)))
    add("iteration time beyond", simple_problem([w - 1, 1], M=int(m_ok) + 1, ndev=(2,)))
    # parameter bytes: the running sum may pass 2^62 but not 2^63
    add("parameters 1.5 x 2^62", simple_problem([1, 1], ndev=(2,), params=[3 << 60, 3 << 60]))
    add("parameters 2^63", simple_problem([1, 1], ndev=(2,), params=[1 << 62, 1 << 62]))
    add("parameters 2^63 over chunks", simple_problem(np.ones(3000, dtype=np.int64), ndev=(2,),
                                                      params=[1 << 62] + [0] * 2998 + [1 << 62]))
    add("parameters 2^63 - 1 over chunks", simple_problem(np.ones(3000, dtype=np.int64), ndev=(2,),
                                                          params=[1 << 62] + [0] * 2998 + [(1 << 62) - 1]))
    # memory need with the in-flight count: PP + min(M, L) PS
    ps = 1 << 40
    add("need at the limit", simple_problem([1, 1], M=8, ndev=(2,), params=[top - 2 * 2 * ps, 0], stash=[ps, ps]))
    add("need beyond", simple_problem([1, 1], M=8, ndev=(2,), params=[top - 2 * 2 * ps + 1, 0], stash=[ps, ps]))
    # degree x device memory
    add("tp x memory at the limit", simple_problem([1, 1], ndev=(8,), tp=(1, 8), mem=[top // 8]))
    add("tp x memory beyond", simple_problem([1, 1], ndev=(8,), tp=(1, 8), mem=[top // 8 + 1]))
    # all-reduce numerator ar_count 2 (tp - 1) act, with links fast enough that every time stays small
    fast = [[1 << 50]]
    lim = top // (4 * 2 * 7)
    add("all-reduce numerator at the limit", simple_problem([1, 1], ndev=(8,), tp=(1, 8), act=[lim, 5], bw=fast))
    add("all-reduce numerator beyond", simple_problem([1, 1], ndev=(8,), tp=(1, 8), act=[lim + 1, 5], bw=fast))
    add("large act without tensor parallelism", simple_problem([1, 1], ndev=(8,), tp=(1,), act=[lim + 1, 5], bw=fast))
    # degree x bandwidth of a group's own link; other links may be as fast as they like
    two = lambda own, other: [[own, other], [other, own]]
    add("tp x own link at the limit", simple_problem([1, 1], G=2, ndev=(8, 8), tp=(1, 8), act=[9, 9], bw=two(top // 8, 7)))
    add("tp x own link beyond", simple_problem([1, 1], G=2, ndev=(8, 8), tp=(1, 8), act=[9, 9], bw=two(top // 8 + 1, 7)))
    add("other links beyond int64 / tp", simple_problem([1, 1], G=2, ndev=(8, 8), tp=(1, 8), act=[9, 9], bw=two(7, top)))
    add("own link beyond int64 / tp without tensor parallelism",
        simple_problem([1, 1], G=2, ndev=(8, 8), tp=(1,), act=[9, 9], bw=two(top, 7)))
    # the slowest of 400 links (20 groups) decides the largest transfer time
    slow = np.full((20, 20), 1 << 20, dtype=np.int64)
    slow[19, 18] = slow[18, 19] = 1
    add("transfer over the slowest of 400 links at the limit",
        simple_problem([1, 1], G=20, ndev=(1,) * 20, act=[(1 << 47) - 1, 5], bw=slow))
    add("transfer over the slowest of 400 links beyond",
        simple_problem([1, 1], G=20, ndev=(1,) * 20, act=[1 << 47, 5], bw=slow))
    return cases


def test_build_verdicts_are_the_oracles_at_every_limit(harp, ctx):
    """The library's verdict on magnitudes equals the oracle's 128-bit check on both sides of every
    limit, and accepted problems give the oracle's tables."""
    seen = set()
    for label, p in _verdict_cases():
        rc = oracle.Tables(p).rc
        seen.add(rc)
        if rc == 0:
            tables = harp.Tables(ctx, p)
            want = oracle.build_tables(p)
            PF, PP, PS, PR = tables.host_copies()
            assert (PF == want.PF).all() and (PP == want.PP).all() and (PS == want.PS).all() and (PR == want.PR).all(), label
        else:
            assert rc == oracle.ERR_OVERFLOW, label
            with pytest.raises(harp.HarpError) as e:
                harp.Tables(ctx, p)
            assert e.value.code == harp.ERR_OVERFLOW, label
    assert seen == {0, oracle.ERR_OVERFLOW}


# ------------------------------------------------------------------ planner (a2-a4)

def test_plan_tiny_all_paths(harp, ctx):
    w = W.make("tiny")
    cands = w.candidates()
    want = oracle.plan_batch(oracle.build_tables(w.problem), cands)
    _, ran = _plan_all_paths(harp, ctx, w.problem, cands, want, "tiny")
    assert harp.PATH_FAST32 in ran


@pytest.mark.parametrize("name,n", [("llama7b", 1024), ("llama70b", 16384), ("finegrained", 65536),
                                    ("stress", 16384)])
def test_plan_workloads_all_paths(harp, ctx, name, n):
    w = W.make(name)
    cands = w.candidates(0, n)
    want = oracle_plan_threaded(oracle.build_tables(w.problem), cands)
    assert (want.status == oracle.OK).any()
    _, ran = _plan_all_paths(harp, ctx, w.problem, cands, want, name)
    assert harp.PATH_FAST32 in ran


def test_plan_random_small_all_paths(harp, ctx):
    fast_runs = 0
    for seed in range(400):
        w = W.random_small(seed)
        cands = w.candidates()
        want = oracle.plan_batch(oracle.build_tables(w.problem), cands)
        _, ran = _plan_all_paths(harp, ctx, w.problem, cands, want, "seed %d" % seed)
        fast_runs += harp.PATH_FAST32 in ran
    assert fast_runs > 200


def test_plan_medium_random_problems(harp, ctx):
    """Sizes that span several tiles with ragged tails: L not a multiple of 64, tight memory."""
    rng = np.random.default_rng(21)
    for case in range(12):
        L = int(rng.integers(65, 700))
        T, G = int(rng.integers(1, 4)), int(rng.integers(1, 6))
        ndev = rng.choice([2, 4, 8], size=G)
        fwd = rng.integers(1, 4000, size=(T, L))
        bw = rng.integers(50, 4000, size=(G, G))
        bw = np.minimum(bw, bw.T)
        params = rng.integers(0, 10**6, size=L)
        stash = rng.integers(0, 10**5, size=L)
        S_max = int(rng.integers(G, G + 8))
        tp = (1, 2, 4, 8)[:int(rng.integers(1, 5))]
        per_stage = int(params.sum() + 0.5 * S_max * stash.sum()) // S_max
        mem = (rng.uniform(0.5, 1.6, size=T) * per_stage / np.sqrt(tp[-1])).astype(np.int64)
        p = simple_problem(np.zeros(L), M=int(rng.integers(1, 40)), T=T, G=G, ndev=ndev, tp=tp,
                           fwd=fwd, bwd=2 * fwd, params=params, stash=stash,
                           act=rng.integers(0, 10**6, size=L), gtype=rng.integers(0, T, size=G),
                           mem=mem, bw=bw)
        p.group_ndev = np.maximum(p.group_ndev, p.tp_degrees[-1]).astype(np.int32)
        cands = W.make_candidates(p, case, 77, G, S_max, 0, 48)
        want = oracle_plan_threaded(oracle.build_tables(p), cands)
        _plan_all_paths(harp, ctx, p, cands, want, "medium %d (L=%d)" % (case, L))


def test_plan_wide_bands(harp, ctx):
    """Loose memory: every DP row is reachable over its whole width, wider than a workgroup, so
    cells and staged rows take several trips; and memory so tight that bands are a few cells."""
    rng = np.random.default_rng(31)
    for L, G, S_max, scale in ((600, 3, 9, 1000.0), (1024, 2, 5, 1000.0), (700, 4, 24, 1.02), (333, 2, 40, 1.3)):
        T = 2
        fwd = rng.integers(1, 3000, size=(T, L))
        params = rng.integers(1, 10**6, size=L)
        stash = rng.integers(0, 10**4, size=L)
        bw = rng.integers(20, 4000, size=(G, G))
        bw = np.minimum(bw, bw.T)
        mem = np.full(T, int(scale * (params.sum() + S_max * stash.sum()) / S_max))
        p = simple_problem(np.zeros(L), M=12, T=T, G=G, ndev=[16] * G, tp=(1, 2), fwd=fwd, bwd=fwd,
                           params=params, stash=stash, act=rng.integers(0, 10**6, size=L),
                           gtype=rng.integers(0, T, size=G), mem=mem, bw=bw)
        cands = W.make_candidates(p, L, 81, G, S_max, 0, 40)
        want = oracle_plan_threaded(oracle.build_tables(p), cands)
        _, ran = _plan_all_paths(harp, ctx, p, cands, want, "wide bands L=%d" % L)
        assert harp.PATH_FAST32 in ran


def test_plan_sequence_of_4096_operators(harp, ctx):
    """The longest sequence the 32-bit min-max path takes (the stress workload's cluster with 4,096
    operators): with tight memory the bands are narrow and every candidate is planned in the first
    pass of the kernel; with loose memory the widest stage spans hundreds of cuts more than a
    wavefront's first-pass share of LDS holds, so candidates go through the second pass."""
    for scale, n in ((2.4, 24), (8.0, 6)):
        p = W.long_sequence(4096, seed=3)
        p.type_mem_bytes = (p.type_mem_bytes * scale).astype(np.int64)
        cands = W.make_candidates(p, 3, 77, p.G, 48, 0, n)
        print("L = 4096, memory x %.1f" % scale, flush=True)
        want = oracle_plan_threaded(oracle.build_tables(p), cands)
        assert (want.status == oracle.OK).any()
        _, ran = _plan_all_paths(harp, ctx, p, cands, want, "L=4096 memory x%.1f" % scale)
        assert harp.PATH_FAST32 in ran
        if scale < 3:
            assert (want.status == oracle.INFEASIBLE).any()


def test_plan_adversarial_rows(harp, ctx):
    """Inputs built to break shortcuts: huge transfers on some cuts (non-monotone DP rows), zero
    cost operators (long runs of ties), memory that only fits one-operator stages."""
    rng = np.random.default_rng(4)
    L = 200
    fwd = rng.integers(0, 3, size=(1, L)) * rng.integers(0, 50, size=(1, L))
    act = np.where(rng.random(L) < 0.3, 10**9, rng.integers(0, 1000, size=L))
    p = simple_problem(np.zeros(L), M=9, G=3, ndev=(8, 8, 8), tp=(1, 2, 4), fwd=fwd, bwd=fwd,
                       act=act, bw=[[1000, 3, 1], [3, 1000, 7], [1, 7, 1000]])
    cands = W.make_candidates(p, 0, 78, 3, 12, 0, 64)
    want = oracle_plan_threaded(oracle.build_tables(p), cands)
    _plan_all_paths(harp, ctx, p, cands, want, "adversarial transfers")

    L = 90
    p = simple_problem([0] * L, M=5, ndev=(8,), tp=(1, 2))
    cands = cands_from_lists([same_slot(S) for S in (1, 2, 7, 8)], S_max=8)
    want = oracle.plan_batch(oracle.build_tables(p), cands)
    _plan_all_paths(harp, ctx, p, cands, want, "all-zero costs")

    L = 12
    p = simple_problem(list(range(1, L + 1)), M=3, ndev=(16,), tp=(1,), params=[10] * L, mem=[10])
    cands = cands_from_lists([same_slot(S) for S in (11, 12, 13)], S_max=16)
    want = oracle.plan_batch(oracle.build_tables(p), cands)
    assert list(want.status) == [oracle.INFEASIBLE, oracle.OK, oracle.INFEASIBLE]
    _plan_all_paths(harp, ctx, p, cands, want, "one operator per stage")


def test_plan_odd_degrees_use_generic_path(harp, ctx):
    rng = np.random.default_rng(8)
    L = 70
    p = simple_problem(np.zeros(L), M=6, G=2, ndev=(6, 6), tp=(1, 2, 3, 6),
                       fwd=rng.integers(1, 1000, size=(1, L)), bwd=rng.integers(1, 1000, size=(1, L)),
                       act=rng.integers(0, 10**5, size=L), bw=[[900, 10], [10, 700]])
    cands = W.make_candidates(p, 0, 79, 2, 6, 0, 40)
    want = oracle.plan_batch(oracle.build_tables(p), cands)
    tables, ran = _plan_all_paths(harp, ctx, p, cands, want, "odd degrees")
    assert ran == [harp.PATH_GENERIC]
    # asking for the 32-bit path on such tables is an error, not a silent switch
    dc = harp.DeviceCandidates(ctx, cands)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    ws = harp.plan_workspace(ctx, tables, dc)
    ctx.set_plan_path(harp.PATH_FAST32)
    try:
        with pytest.raises(harp.HarpError) as e:
            harp.harp_plan_batch(ctx, tables, dc, out, ws)
        assert e.value.code == harp.ERR_UNIMPLEMENTED
    finally:
        ctx.set_plan_path(harp.PATH_AUTO)


def test_plan_wide_times_use_generic_path(harp, ctx):
    """Times beyond 32 bits: the int64 path must carry them exactly."""
    rng = np.random.default_rng(9)
    L = 40
    fwd = rng.integers(1, 1 << 36, size=(2, L))
    p = simple_problem(np.zeros(L), M=50, T=2, G=2, ndev=(4, 4), tp=(1, 2, 4), fwd=fwd, bwd=fwd // 3,
                       act=rng.integers(0, 1 << 40, size=L), gtype=[0, 1], bw=[[1 << 20, 5], [5, 1 << 18]])
    cands = W.make_candidates(p, 0, 80, 2, 8, 0, 64)
    want = oracle.plan_batch(oracle.build_tables(p), cands)
    assert (want.status == oracle.OK).all() and want.iter_time.max() > (1 << 40)
    _, ran = _plan_all_paths(harp, ctx, p, cands, want, "wide times")
    assert ran == [harp.PATH_GENERIC]


def test_invalid_and_degenerate_candidates(harp, ctx):
    p = simple_problem([3, 1, 4, 1, 5, 9], G=2, ndev=(2, 2), tp=(1, 2), bw=np.full((2, 2), 2),
                       act=[5] * 6)
    lists = [
        [(0, 1), (1, 1), (0, 1)],       # group revisited
        [(0, 2), (0, 1)],               # over-subscribed
        [(0, 3)],                       # degree not allowed
        [(2, 1)],                       # no such group
        [(-1, 1)],                      # negative group
        [(0, 0)],                       # degree below 1
        [],                             # no stage
        [(0, 1), (1, 2)],               # fine
        [(1, 1)] * 2 + [(0, 1)] * 2,    # fine, S = 4
    ]
    cands = cands_from_lists(lists, S_max=8)
    extra = cands_from_lists([[(0, 1)] * 2 + [(1, 1)] * 2], S_max=8)
    extra.cand_S[0] = 9                 # S beyond S_max
    cands = W.Candidates(cands.C + 1, 8, np.concatenate([cands.cand_S, extra.cand_S]),
                         np.concatenate([cands.cand_group, extra.cand_group]),
                         np.concatenate([cands.cand_tp, extra.cand_tp]))
    want = oracle.plan_batch(oracle.build_tables(p), cands)
    assert list(want.status) == [2, 2, 2, 2, 2, 2, 2, 0, 0, 2]
    _plan_all_paths(harp, ctx, p, cands, want, "invalid candidates")
    # more stages than operators
    p = simple_problem([1, 1], ndev=(4,))
    cands = cands_from_lists([same_slot(3), same_slot(2), same_slot(1)])
    want = oracle.plan_batch(oracle.build_tables(p), cands)
    assert list(want.status) == [1, 0, 0]
    _plan_all_paths(harp, ctx, p, cands, want, "S > L")


def test_empty_batch_and_argument_errors(harp, ctx):
    import torch
    w = W.make("tiny")
    tables = harp.Tables(ctx, w.problem)
    empty = w.candidates(0, 0)
    dc = harp.DeviceCandidates(ctx, empty)
    out = harp.DevicePlans(ctx, 0, dc.S_max)
    ws = harp.plan_workspace(ctx, tables, dc)
    harp.harp_plan_batch(ctx, tables, dc, out, ws)          # C = 0: nothing to do, no error
    torch.cuda.synchronize()
    dc = harp.DeviceCandidates(ctx, w.candidates())
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    small = torch.empty(256, dtype=torch.uint8, device=ctx.device)
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_batch(ctx, tables, dc, out, small)
    assert e.value.code == harp.ERR_WORKSPACE
    ws = harp.plan_workspace(ctx, tables, dc)
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_batch(ctx, tables, dc, out, ws[1:])  # misaligned
    assert e.value.code == harp.ERR_WORKSPACE
    dc.c.S_max = 0
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_batch(ctx, tables, dc, out, ws)
    assert e.value.code == harp.ERR_SHAPE
    with pytest.raises(harp.HarpError) as e:
        ctx.set_plan_path(9)
    assert e.value.code == harp.ERR_INVALID_ARG


def _bands_from_the_memory_constraint(p, S, groups, degrees):
    """Per DP row s the lowest cut from which stages s .. S-1 can still hold the rest and the highest
    cut that s stages can reach, by exhaustive set propagation over eq. mem_cons (non-empty stages,
    classic in-flight counts min(S - s, M)); None when some row has no cut left."""
    L = p.L
    PP = np.concatenate([[0], np.cumsum(p.param_bytes)]).astype(object)
    PS = np.concatenate([[0], np.cumsum(p.stash_bytes)]).astype(object)

    def fits(s, j, i):
        n = min(S - s, p.M)
        cap = int(degrees[s]) * int(p.type_mem_bytes[p.group_type[groups[s]]])
        return (PP[i] - PP[j]) + n * (PS[i] - PS[j]) <= cap

    reach = [{0}]
    for s in range(S):
        last = L - (S - 1 - s)                      # leaves an operator to every later stage
        reach.append({i for j in reach[s] for i in range(j + 1, last + 1) if fits(s, j, i)})
    done = [set() for _ in range(S + 1)]
    done[S] = {L}
    for s in range(S - 1, -1, -1):
        done[s] = {j for j in range(s, L) for i in done[s + 1] if j < i and fits(s, j, i)}
    if any(not r for r in reach) or any(not d for d in done) or L not in reach[S] or 0 not in done[0]:
        return None
    rows = [(min(done[s]), max(reach[s])) for s in range(S + 1)]
    return None if any(lo > hi for lo, hi in rows) else rows


def test_counted_work_matches_the_bands_of_the_memory_constraint(harp, ctx):
    """harp_plan_batch_count_work: same plans as harp_plan_batch; the cells it reports are exactly the
    cells of the reachability bands (worked out here by exhaustive propagation of eq. mem_cons), the
    candidates it reports are those with a band in every row, and the transitions lie between one
    per cell with a fitting predecessor and all fitting predecessors inside the bands."""
    import torch
    cases = [W.make("tiny"), W.make("llama7b")] + [W.random_small(seed, odd_degrees=False) for seed in range(40)]
    checked = 0
    for w in cases:
        p = w.problem
        cands = w.candidates(0, min(w.C, 96))
        tables = harp.Tables(ctx, p)
        if not tables.fast32:
            continue
        dc = harp.DeviceCandidates(ctx, cands)
        out, out2 = harp.DevicePlans(ctx, dc.C, dc.S_max), harp.DevicePlans(ctx, dc.C, dc.S_max)
        ws = harp.plan_workspace(ctx, tables, dc)
        work = torch.full((4,), -7, dtype=torch.int64, device=ctx.device)
        out.poison(); out2.poison()
        harp.harp_plan_batch(ctx, tables, dc, out, ws)
        harp.harp_plan_batch_count_work(ctx, tables, dc, out2, ws, work)
        torch.cuda.synchronize()
        assert_plans_equal(out2.to_host(), out.to_host(), "%s counted launch" % w.name)
        transitions, cells, groups_of_four, planned = (int(x) for x in work.cpu().numpy())
        want_cells = want_planned = most = least = 0
        PP = np.concatenate([[0], np.cumsum(p.param_bytes)]).astype(object)
        PS = np.concatenate([[0], np.cumsum(p.stash_bytes)]).astype(object)
        statuses = oracle.plan_batch(oracle.build_tables(p), cands).status
        for c in range(cands.C):
            S = int(cands.cand_S[c])
            if statuses[c] == oracle.INVALID:
                continue
            rows = _bands_from_the_memory_constraint(p, S, cands.cand_group[c], cands.cand_tp[c])
            if rows is None:
                continue
            want_planned += 1
            if S == 1:                              # one stage holds everything: no recurrence, no cells
                continue
            for s in range(S):                      # stage s fills row s + 1 from row s
                (jl, jh), (il, ih) = rows[s], rows[s + 1]
                n = min(S - s, p.M)
                cap = int(cands.cand_tp[c][s]) * int(p.type_mem_bytes[p.group_type[cands.cand_group[c][s]]])
                for i in range(il, ih + 1):
                    fitting = sum(1 for j in range(jl, min(i - 1, jh) + 1)
                                  if (PP[i] - PP[j]) + n * (PS[i] - PS[j]) <= cap)
                    want_cells += 1
                    most += fitting
                    least += 1 if fitting else 0
        assert (cells, planned) == (want_cells, want_planned), w.name
        assert least <= transitions <= most and 4 * groups_of_four >= transitions, w.name
        checked += want_planned
    assert checked > 200
    # the int64 path has no counting build
    ctx.set_plan_path(harp.PATH_GENERIC)
    try:
        with pytest.raises(harp.HarpError) as e:
            harp.harp_plan_batch_count_work(ctx, tables, dc, out2, ws, work)
        assert e.value.code == harp.ERR_UNIMPLEMENTED
    finally:
        ctx.set_plan_path(harp.PATH_AUTO)


# ------------------------------------------------------------------ scorer and selection

def test_score_parity_on_arbitrary_partitions(harp, ctx):
    import torch
    rng = np.random.default_rng(2)
    seen = set()
    for name, n in (("tiny", 16), ("llama7b", 1024), ("llama70b", 2048), ("stress", 2048)):
        w = W.make(name)
        cands = w.candidates(0, n)
        L = w.problem.L
        splits = np.full((n, cands.S_max + 1), -1, dtype=np.int32)
        for c in range(n):
            S = int(cands.cand_S[c])
            cut = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False))
            splits[c, :S + 1] = [0, *cut, L]
        splits[3, 1] = splits[3, 2]                 # not strictly increasing
        splits[5, 0] = 1                            # does not start at 0
        splits[7, int(cands.cand_S[7])] = L - 1     # does not end at L
        want = oracle.score_1f1b(oracle.build_tables(w.problem), cands, splits)
        tables = harp.Tables(ctx, w.problem)
        dc = harp.DeviceCandidates(ctx, cands)
        sp = torch.from_numpy(splits).to(ctx.device)
        b = torch.full((n,), -7, dtype=torch.int64, device=ctx.device)
        t = torch.full((n,), -7, dtype=torch.int64, device=ctx.device)
        st = torch.full((n,), -7, dtype=torch.int32, device=ctx.device)
        for path in (harp.PATH_AUTO, harp.PATH_GENERIC):        # the kernel for the 32-bit tables, the int64 one
            b.fill_(-7); t.fill_(-7); st.fill_(-7)
            ctx.set_plan_path(path)
            try:
                harp.harp_score_1f1b(ctx, tables, dc, sp, b, t, st)
                torch.cuda.synchronize()
            finally:
                ctx.set_plan_path(harp.PATH_AUTO)
            assert (st.cpu().numpy() == want[2]).all()
            assert (b.cpu().numpy() == want[0]).all() and (t.cpu().numpy() == want[1]).all()
        seen |= set(int(x) for x in np.unique(want[2]))
    assert seen == {0, 1, 2}


def test_score_checks_the_slot_lists_on_both_paths(harp, ctx):
    """The scorer's own checks of a candidate (stage count, group ids, degrees, a group entered twice,
    more devices than a group has) and of a partition, on the kernel for the 32-bit tables and on the
    int64 one, against the oracle; S_max = 64 and 65 (the first kernel takes at most 64 stages)."""
    import torch
    rng = np.random.default_rng(12)
    L = 90
    p = simple_problem(np.zeros(L), M=5, T=2, G=4, ndev=(4, 2, 8, 4), tp=(1, 2, 4),
                       fwd=rng.integers(1, 500, size=(2, L)), bwd=rng.integers(1, 900, size=(2, L)),
                       act=rng.integers(0, 10**5, size=L), params=rng.integers(0, 1000, size=L),
                       stash=rng.integers(0, 100, size=L), gtype=[0, 1, 1, 0], mem=[30000, 20000],
                       bw=[[900, 7, 9, 5], [7, 800, 6, 4], [9, 6, 700, 3], [5, 4, 3, 950]])
    lists = [
        [(0, 2), (0, 2), (1, 1), (2, 4)],           # fine
        [(0, 2), (1, 1), (0, 2)],                   # group 0 entered twice
        [(1, 1), (1, 1), (1, 1)],                   # three devices of a group of two
        [(2, 4), (2, 4), (3, 1)],                   # exactly the devices of group 2
        [(2, 4), (2, 4), (2, 1)],                   # one too many
        [(0, 3), (1, 1)],                           # a degree that is not allowed
        [(4, 1), (1, 1)],                           # a group that does not exist
        [(-1, 1), (1, 1)],
        [(3, 4)],                                   # a single stage
        [(3, 1), (3, 1), (3, 1), (3, 1), (0, 1), (0, 1), (0, 1), (0, 1), (2, 2), (2, 2), (2, 2), (2, 2), (1, 2)],
    ]
    for S_max in (64, 65):
        cands = cands_from_lists(lists * 3, S_max=S_max)
        cands.cand_S[len(lists)] = 0                # no stage
        cands.cand_S[len(lists) + 3] = S_max + 1    # more stages than the arrays hold
        n = cands.C
        splits = np.full((n, S_max + 1), -1, dtype=np.int32)
        for c in range(n):
            S = int(cands.cand_S[c])
            if 1 <= S <= S_max:
                cut = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False))
                splits[c, :S + 1] = [0, *cut, L]
        splits[2 * len(lists), 1] = 0               # a fine slot list with cuts that do not rise
        want = oracle.score_1f1b(oracle.build_tables(p), cands, splits)
        assert set(int(x) for x in np.unique(want[2])) == {0, 1, 2} or set(int(x) for x in np.unique(want[2])) == {0, 2}
        tables = harp.Tables(ctx, p)
        assert tables.fast32
        dc = harp.DeviceCandidates(ctx, cands)
        sp = torch.from_numpy(splits).to(ctx.device)
        for path in (harp.PATH_AUTO, harp.PATH_GENERIC):
            b = torch.full((n,), -7, dtype=torch.int64, device=ctx.device)
            t = torch.full((n,), -7, dtype=torch.int64, device=ctx.device)
            st = torch.full((n,), -7, dtype=torch.int32, device=ctx.device)
            ctx.set_plan_path(path)
            try:
                harp.harp_score_1f1b(ctx, tables, dc, sp, b, t, st)
                torch.cuda.synchronize()
            finally:
                ctx.set_plan_path(harp.PATH_AUTO)
            assert (st.cpu().numpy() == want[2]).all(), (S_max, path, st.cpu().numpy(), want[2])
            assert (b.cpu().numpy() == want[0]).all() and (t.cpu().numpy() == want[1]).all(), (S_max, path)


def test_argmin_parity(harp, ctx):
    import torch
    rng = np.random.default_rng(3)
    for n in (0, 1, 63, 64, 1000, 32767, 32768, 70001, 600011):   # one workgroup below 2^15, many from there on
        it = rng.integers(10, 50, size=n).astype(np.int64)
        st = rng.integers(0, 3, size=n).astype(np.int32)
        for status in (st, np.ones(n, dtype=np.int32)):
            want = oracle.argmin_batch(it, status)
            bt = torch.full((1,), -7, dtype=torch.int64, device=ctx.device)
            bi = torch.full((1,), -7, dtype=torch.int32, device=ctx.device)
            harp.harp_argmin_batch(ctx, n, torch.from_numpy(it).to(ctx.device),
                                   torch.from_numpy(status).to(ctx.device), bt, bi)
            torch.cuda.synchronize()
            assert (int(bt.item()), int(bi.item())) == want


# ------------------------------------------------------------------ full size, bench configuration

def test_stress_full_batch_properties_and_samples(harp, ctx):
    """The whole stress batch in the configuration bench.py times (auto path): sampled candidates
    against the oracle one by one, and properties that hold at any size for all of them."""
    import torch
    w = W.make("stress")
    cands = w.candidates()
    tables = harp.Tables(ctx, w.problem)
    assert tables.fast32
    dc = harp.DeviceCandidates(ctx, cands)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    ws = harp.plan_workspace(ctx, tables, dc)
    out.poison()
    harp.harp_plan_batch(ctx, tables, dc, out, ws)
    torch.cuda.synchronize()
    got = out.to_host()
    # determinism: a second launch is byte-identical (integer min/max has no order dependence)
    out2 = harp.DevicePlans(ctx, dc.C, dc.S_max)
    harp.harp_plan_batch(ctx, tables, dc, out2, ws)
    torch.cuda.synchronize()
    assert_plans_equal(out2.to_host(), got, "second launch")
    # sampled candidates against the oracle
    idx = np.random.default_rng(0).choice(w.C, size=320, replace=False)
    sample = cands.take(idx)
    want = oracle_plan_threaded(oracle.build_tables(w.problem), sample)
    class _Sub:
        pass
    sub = _Sub()
    for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
        setattr(sub, name, getattr(got, name)[idx])
    assert_plans_equal(sub, want, "stress sample")
    # properties over the whole batch
    ok = got.status == 0
    frac_bad = float((got.status == 1).mean())
    assert 0.25 < frac_bad < 0.35 and (got.status != 2).all()
    S = cands.cand_S.astype(np.int64)
    rows = np.arange(w.C)
    assert (got.splits[ok, 0] == 0).all() and (got.splits[rows[ok], S[ok]] == w.problem.L).all()
    width = np.arange(cands.S_max + 1)[None, :]
    inside = width <= S[:, None]
    d = np.diff(got.splits.astype(np.int64), axis=1)
    assert (d[ok][inside[ok][:, 1:]] > 0).all()
    assert (got.splits[ok][~inside[ok]] == -1).all()
    assert (got.splits[~ok] == -1).all() and (got.bottleneck[~ok] == oracle.INF).all()
    # the stand-alone scorer reproduces the planner's own numbers from its cuts
    b = torch.empty_like(out.bottleneck)
    t = torch.empty_like(out.iter_time)
    st = torch.empty_like(out.status)
    harp.harp_score_1f1b(ctx, tables, dc, out.splits, b, t, st)
    torch.cuda.synchronize()
    assert (b.cpu().numpy()[ok] == got.bottleneck[ok]).all()
    assert (t.cpu().numpy()[ok] == got.iter_time[ok]).all()
    assert (st.cpu().numpy()[ok] == 0).all() and (st.cpu().numpy()[~ok] == 2).all()
    # selection
    bt = torch.empty(1, dtype=torch.int64, device=ctx.device)
    bi = torch.empty(1, dtype=torch.int32, device=ctx.device)
    harp.harp_argmin_batch(ctx, w.C, out.iter_time, out.status, bt, bi)
    torch.cuda.synchronize()
    assert (int(bt.item()), int(bi.item())) == oracle.argmin_batch(got.iter_time, got.status)


@pytest.fixture(scope="module")
def stress_full(harp, ctx):
    """The whole stress batch planned once on each path, in the launch configuration bench.py times."""
    import torch
    w = W.make("stress")
    cands = w.candidates()
    tables = harp.Tables(ctx, w.problem)
    dc = harp.DeviceCandidates(ctx, cands)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    ws = harp.plan_workspace(ctx, tables, dc)
    plans = {}
    for path in (harp.PATH_FAST32, harp.PATH_GENERIC):
        out.poison()
        ctx.set_plan_path(path)
        try:
            harp.harp_plan_batch(ctx, tables, dc, out, ws)
            torch.cuda.synchronize()
        finally:
            ctx.set_plan_path(harp.PATH_AUTO)
        plans[path] = out.to_host()
    return w, cands, plans


def test_stress_full_batch_both_paths_agree(harp, stress_full):
    """All 262,144 candidates: the int64 kernel (dense scans, no bands, no index) and the 32-bit
    kernel share no device code beyond the scorer and must give the same plans."""
    _, _, plans = stress_full
    assert_plans_equal(plans[harp.PATH_FAST32], plans[harp.PATH_GENERIC], "stress, 32-bit against int64 path")


@pytest.mark.parametrize("quarter", range(4))
def test_stress_full_batch_against_oracle(harp, stress_full, quarter):
    """All 262,144 candidates of the stress batch against the oracle, a quarter of the batch per case
    (about 25 s of oracle time on 16 host threads each).  Includes the candidates that pass the
    memory bounds of the pre-pass and are found infeasible by the recurrence."""
    w, cands, plans = stress_full
    n = w.C // 4
    lo, hi = quarter * n, (quarter + 1) * n if quarter < 3 else w.C
    want = oracle_plan_threaded(oracle.build_tables(w.problem), cands.slice(lo, hi))
    got = plans[harp.PATH_FAST32]

    class _Sub:
        pass
    sub = _Sub()
    for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
        setattr(sub, name, getattr(got, name)[lo:hi])
    assert_plans_equal(sub, want, "stress candidates %d..%d" % (lo, hi))
    assert (want.status == oracle.INFEASIBLE).any() and (want.status == oracle.OK).any()


def test_case_study_of_the_paper_on_the_gpu(harp, ctx):
    """Section 2.2, Table 1 (tests/golden/case_study_shares.txt): the kernels give the oracle's plans
    for the table's two pipelines, whose 128-layer stage sizes follow the submeshes' FLOP shares."""
    from helpers import read_golden
    rows = read_golden(os.path.join(os.path.dirname(__file__), "golden", "case_study_shares.txt"))
    for row in rows:
        L, flops, layers = (part.split() for part in row.split("|"))
        L, flops, layers = int(L[0]), [int(x) for x in flops], [int(x) for x in layers]
        scale = flops[0] * flops[1]
        fwd = np.array([[scale // f] * L for f in flops], dtype=np.int64)
        p = simple_problem(np.zeros(L), M=8, T=3, G=3, ndev=(1, 1, 1), gtype=[0, 1, 2], fwd=fwd,
                           bwd=np.zeros_like(fwd))
        cands = cands_from_lists([[(0, 1), (1, 1), (2, 1)]])
        want = oracle.plan_batch(oracle.build_tables(p), cands)
        _plan_all_paths(harp, ctx, p, cands, want, "case study, %d layers" % L)
        if L == 128:
            sizes = np.diff(want.splits[0, :4])
            assert max(abs(1000 * n / L - s) for n, s in zip(sizes, layers)) <= 12
