"""GPU parity of the exact search (cap sweep of section 5.2.4 (2)): harp_plan_exact_batch against the
oracle's increasing sweep over every distinct stage cost, bit for bit."""
import os

import numpy as np
import pytest

import oracle
from paper_2509_24859_amd import workloads as W

from helpers import (assert_plans_equal, cands_from_lists, oracle_plan_exact_threaded, oracle_plan_threaded,
                     read_golden, same_slot, simple_problem)

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def ctx(harp):
    c = harp.Context(0)
    yield c
    c.close()


def _check(harp, ctx, problem, cands, label, need_fast=True):
    """Both kernel paths (int64 always, 32-bit when the tables allow it) against the oracle's sweep."""
    tables = oracle.build_tables(problem)
    want = oracle_plan_exact_threaded(tables, cands)
    ok = (want.status == oracle.OK) & (cands.cand_S >= 2)
    fast32 = harp.Tables(ctx, problem).fast32
    assert fast32 or not need_fast, label
    for path in [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if fast32 else []):
        tag = "%s (path %d)" % (label, path)
        got, n_passes, _ = harp.plan_exact(ctx, problem, cands, path)
        assert_plans_equal(got, want, tag)
        assert (n_passes[ok] >= 1).all() and (n_passes[~ok] == 0).all(), tag
        # never more capped recurrences than the increasing sweep would run, the opening pass at t_S aside
        assert (n_passes[ok] <= want.n_caps[ok] + 1).all(), tag
    return got, want, n_passes


def test_exact_hand_examples(harp, ctx):
    for row in read_golden(os.path.join(GOLD, "hand_examples_exact.txt")):
        M, splits, cap, T = [f.strip() for f in row.split("|")]
        p = simple_problem([6, 2, 2, 6], M=int(M), G=2, ndev=(1, 1), act=[0, 5, 0, 0],
                           bw=[[1000, 1], [1, 1000]])
        cands = cands_from_lists([[(0, 1), (1, 1)]])
        got, _, _ = harp.plan_exact(ctx, p, cands)
        assert list(got.splits[0]) == [int(x) for x in splits.split()]
        assert got.bottleneck[0] == int(cap) and got.iter_time[0] == int(T)


def test_exact_tiny(harp, ctx):
    w = W.make("tiny")
    _check(harp, ctx, w.problem, w.candidates(), "tiny")


def test_exact_random_small(harp, ctx):
    fast_runs = 0
    for seed in range(400):
        w = W.random_small(seed)
        fast_runs += harp.Tables(ctx, w.problem).fast32
        _check(harp, ctx, w.problem, w.candidates(), "seed %d" % seed, need_fast=False)
    assert fast_runs > 200


@pytest.mark.parametrize("name,n,stride", [("llama7b", 1024, 1), ("llama70b", 384, 171), ("finegrained", 32, 1021),
                                           ("stress", 16, 16553)])
def test_exact_workloads(harp, ctx, name, n, stride):
    """Candidates spread over the whole batch (every stride-th), as many as the oracle's sweep can
    do in seconds."""
    w = W.make(name)
    idx = (np.arange(n, dtype=np.int64) * stride) % w.C
    cands = w.candidates().take(idx) if stride > 1 else w.candidates(0, n)
    got, want, n_passes = _check(harp, ctx, w.problem, cands, name)
    assert (want.status == oracle.OK).any()
    print("%s: passes per candidate mean %.1f max %d; oracle caps mean %.0f"
          % (name, n_passes.mean(), n_passes.max(), want.n_caps.mean()))


def test_exact_medium_random_problems(harp, ctx):
    """Sizes that span several wavefronts with ragged tails, tight memory, transfers that matter."""
    rng = np.random.default_rng(121)
    for case in range(8):
        L = int(rng.integers(65, 300))
        T, G = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        ndev = rng.choice([2, 4, 8], size=G)
        fwd = rng.integers(1, 4000, size=(T, L))
        bw = rng.integers(50, 4000, size=(G, G))
        bw = np.minimum(bw, bw.T)
        params = rng.integers(0, 10**6, size=L)
        stash = rng.integers(0, 10**5, size=L)
        S_max = int(rng.integers(G, G + 6))
        tp = (1, 2, 4, 8)[:int(rng.integers(1, 5))]
        per_stage = int(params.sum() + 0.5 * S_max * stash.sum()) // S_max
        mem = (rng.uniform(0.7, 2.0, size=T) * per_stage / np.sqrt(tp[-1])).astype(np.int64)
        p = simple_problem(np.zeros(L), M=int(rng.integers(1, 40)), T=T, G=G, ndev=ndev, tp=tp,
                           fwd=fwd, bwd=2 * fwd, params=params, stash=stash,
                           act=rng.integers(0, 4 * 10**6, size=L), gtype=rng.integers(0, T, size=G),
                           mem=mem, bw=bw)
        p.group_ndev = np.maximum(p.group_ndev, p.tp_degrees[-1]).astype(np.int32)
        cands = W.make_candidates(p, case, 177, G, S_max, 0, 24)
        _check(harp, ctx, p, cands, "medium %d (L=%d)" % (case, L))


def test_exact_wide_bands_and_ties(harp, ctx):
    """Loose memory with bands wider than a workgroup; long runs of equal sums (zero-cost operators,
    uniform operators); transfers that exceed the cap on most cuts."""
    rng = np.random.default_rng(131)
    L, G, T = 600, 2, 2
    fwd = rng.integers(1, 3000, size=(T, L))
    bw = np.array([[4000, 30], [30, 3000]])
    p = simple_problem(np.zeros(L), M=12, T=T, G=G, ndev=[16] * G, tp=(1, 2), fwd=fwd, bwd=fwd,
                       params=rng.integers(1, 10**6, size=L), stash=rng.integers(0, 10**4, size=L),
                       act=rng.integers(0, 10**6, size=L), gtype=[0, 1], mem=[1 << 50, 1 << 50], bw=bw)
    _check(harp, ctx, p, W.make_candidates(p, 0, 181, G, 5, 0, 12), "wide bands")

    L = 200
    fwd = rng.integers(0, 3, size=(1, L)) * rng.integers(0, 50, size=(1, L))
    act = np.where(rng.random(L) < 0.3, 10**6, rng.integers(0, 1000, size=L))
    p = simple_problem(np.zeros(L), M=9, G=3, ndev=(8, 8, 8), tp=(1, 2, 4), fwd=fwd, bwd=fwd,
                       act=act, bw=[[1000, 3, 1], [3, 1000, 7], [1, 7, 1000]])
    _check(harp, ctx, p, W.make_candidates(p, 0, 178, 3, 12, 0, 48), "expensive transfers, zero-cost operators")

    p = simple_problem([7] * 90, M=5, ndev=(8,), tp=(1, 2))
    _check(harp, ctx, p, cands_from_lists([same_slot(S) for S in (1, 2, 7, 8)], S_max=8), "uniform operators")
    p = simple_problem([0] * 90, M=5, ndev=(8,), tp=(1, 2))
    _check(harp, ctx, p, cands_from_lists([same_slot(S) for S in (1, 2, 7, 8)], S_max=8), "all-zero costs")


def test_exact_invalid_infeasible_and_single_stage(harp, ctx):
    L = 12
    p = simple_problem(list(range(1, L + 1)), M=3, ndev=(16,), tp=(1,), params=[10] * L, mem=[25])
    lists = [same_slot(S) for S in (1, 5, 6, 12, 13)] + [[(0, 3)], [(1, 1)]]
    cands = cands_from_lists(lists, S_max=16)
    got, want, _ = _check(harp, ctx, p, cands, "mixed statuses")
    assert set(want.status) == {oracle.OK, oracle.INFEASIBLE, oracle.INVALID}


def test_exact_sums_beyond_32_bits(harp, ctx):
    """Transfers so long that a plan's sum leaves 31 bits while every single time stays below 2^31:
    those candidates take the 64-bit instantiation; the rest of the batch stays on 32-bit sums."""
    rng = np.random.default_rng(19)
    L, G = 60, 5
    act = rng.integers(11, 20, size=L) * 10**8
    act[rng.choice(L - 1, size=3, replace=False)] = 1000    # three cheap cuts, four links to cross
    bw = np.ones((G, G), dtype=np.int64) + np.eye(G, dtype=np.int64) * 10**6   # slow links between groups only
    p = simple_problem(np.zeros(L), M=3, G=G, ndev=(4,) * G, tp=(1, 2),
                       fwd=rng.integers(1, 10**6, size=(1, L)), bwd=rng.integers(1, 10**6, size=(1, L)),
                       act=act, bw=bw)
    full = W.make_candidates(p, 0, 83, G, 9, 0, 48)
    lists = []
    for c in range(full.C):
        slots = [(int(g), int(t)) for g, t in zip(full.cand_group[c, :full.cand_S[c]], full.cand_tp[c, :full.cand_S[c]])]
        if c % 2:                                           # leave the last group out: three links
            slots = [x for x in slots if x[0] != G - 1]
        lists.append(slots)
    cands = cands_from_lists(lists, S_max=9)
    got, want, _ = _check(harp, ctx, p, cands, "wide sums")
    ok = want.status == oracle.OK
    sums = want.iter_time[ok] - (p.M - 1) * want.bottleneck[ok]
    assert (sums >= 1 << 31).any() and (sums < 1 << 31).any()


def test_exact_odd_degrees_and_wide_times_use_int64_path(harp, ctx):
    rng = np.random.default_rng(9)
    L = 50
    p = simple_problem(np.zeros(L), M=6, G=2, ndev=(6, 6), tp=(1, 2, 3, 6),
                       fwd=rng.integers(1, 1000, size=(1, L)), bwd=rng.integers(1, 1000, size=(1, L)),
                       act=rng.integers(0, 10**5, size=L), bw=[[900, 10], [10, 700]])
    cands = W.make_candidates(p, 0, 79, 2, 6, 0, 32)
    _check(harp, ctx, p, cands, "odd degrees", need_fast=False)
    assert not harp.Tables(ctx, p).fast32
    # asking for the 32-bit path on such tables is an error, not a silent switch
    with pytest.raises(harp.HarpError) as e:
        harp.plan_exact(ctx, p, cands, harp.PATH_FAST32)
    assert e.value.code == harp.ERR_UNIMPLEMENTED

    L = 40
    fwd = rng.integers(1, 1 << 36, size=(2, L))
    p = simple_problem(np.zeros(L), M=50, T=2, G=2, ndev=(4, 4), tp=(1, 2, 4), fwd=fwd, bwd=fwd // 3,
                       act=rng.integers(0, 1 << 40, size=L), gtype=[0, 1], bw=[[1 << 20, 5], [5, 1 << 18]])
    cands = W.make_candidates(p, 0, 80, 2, 8, 0, 32)
    got, want, _ = _check(harp, ctx, p, cands, "times beyond 32 bits", need_fast=False)
    assert not harp.Tables(ctx, p).fast32 and want.iter_time.max() > (1 << 40)


def test_exact_empty_batch(harp, ctx):
    w = W.make("tiny")
    got, n_passes, _ = harp.plan_exact(ctx, w.problem, w.candidates(0, 0))
    assert got.status.shape == (0,) and n_passes.shape == (0,)


def test_exact_full_finegrained_batch_both_paths_and_sample(harp, ctx):
    """The whole fine-grained batch (65,536 candidates) through the exact search on both kernel paths,
    which share no search code: identical plans and pass counts; and a sample spread over the batch
    against the oracle's full increasing sweep (which does about 6 candidates a second on 16 host
    threads, so the oracle itself cannot cover the batch)."""
    w = W.make("finegrained")
    cands = w.candidates()
    fast, n_fast, _ = harp.plan_exact(ctx, w.problem, cands, harp.PATH_FAST32)
    gen, n_gen, _ = harp.plan_exact(ctx, w.problem, cands, harp.PATH_GENERIC)
    assert_plans_equal(fast, gen, "finegrained exact, 32-bit against int64 path")
    assert (n_fast == n_gen).all()
    idx = (np.arange(48, dtype=np.int64) * 1361) % w.C
    want = oracle_plan_exact_threaded(oracle.build_tables(w.problem), cands.take(idx))

    class _Sub:
        pass
    sub = _Sub()
    for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
        setattr(sub, name, getattr(fast, name)[idx])
    assert_plans_equal(sub, want, "finegrained exact sample")


def test_exact_stress_sample_both_paths(harp, ctx):
    """Every 16th candidate of the stress batch through the exact search on both kernel paths, which
    share no search code: identical plans and pass counts.  About one candidate in sixteen there has
    a stage too wide for a wavefront's share of LDS and takes the 32-bit path's second launch, and
    candidates of every width meet the int64 kernels."""
    w = W.make("stress")
    idx = np.arange(0, w.C, 16, dtype=np.int64)
    cands = w.candidates().take(idx)
    fast, n_fast, _ = harp.plan_exact(ctx, w.problem, cands, harp.PATH_FAST32)
    gen, n_gen, _ = harp.plan_exact(ctx, w.problem, cands, harp.PATH_GENERIC)
    assert_plans_equal(fast, gen, "stress exact, 32-bit against int64 path")
    assert (n_fast == n_gen).all()
    assert (fast.status == oracle.OK).sum() > 8000


def test_exact_full_stress_batch_properties(harp, ctx):
    """The whole stress batch in the launch configuration the benchmark times: what must hold for
    every candidate whatever its size."""
    import torch
    w = W.make("stress")
    cands = w.candidates()
    minmax, tables = harp.plan(ctx, w.problem, cands)
    got, n_passes, tables = harp.plan_exact(ctx, w.problem, cands)
    ok = minmax.status == oracle.OK
    assert (got.status == minmax.status).all()
    assert (got.dev_first == minmax.dev_first).all()
    assert (got.iter_time[ok] <= minmax.iter_time[ok]).all()
    assert (got.bottleneck[ok] >= minmax.bottleneck[ok]).all()
    assert (got.iter_time[~ok] == oracle.INF).all() and (got.splits[~ok] == -1).all()
    # the reported times are the cost model's for the reported cuts (scorer kernel and, on a sample, oracle)
    dc = harp.DeviceCandidates(ctx, cands)
    sp = torch.from_numpy(got.splits).to(ctx.device)
    b = torch.empty(cands.C, dtype=torch.int64, device=ctx.device)
    t = torch.empty_like(b)
    st = torch.empty(cands.C, dtype=torch.int32, device=ctx.device)
    harp.harp_score_1f1b(ctx, tables, dc, sp, b, t, st)
    torch.cuda.synchronize()
    assert (b.cpu().numpy() == got.bottleneck).all() and (t.cpu().numpy() == got.iter_time).all()
    assert (st.cpu().numpy()[ok] == oracle.OK).all()
    idx = np.nonzero(ok)[0][::997]
    sub = cands.take(idx)
    ob, ot, ost = oracle.score_1f1b(oracle.build_tables(w.problem), sub, got.splits[idx])
    assert (ob == got.bottleneck[idx]).all() and (ot == got.iter_time[idx]).all() and (ost == 0).all()
    # the min-max plan is one of the partitions the sweep considers: strictly better somewhere
    assert (got.iter_time[ok] < minmax.iter_time[ok]).any()
