"""GPU parity of the capped recurrence with H-1F1B warm-up counts (sections 4.1, 5.2.3) and of its
scorer: harp_plan_h1f1b_batch and harp_score_h1f1b against the oracle, bit for bit, on both
kernel paths."""
import os

import numpy as np
import pytest

import oracle
from paper_2509_24859_amd import workloads as W

from helpers import (BIG, assert_plans_equal, cands_from_lists, oracle_plan_h1f1b_threaded,
                     oracle_plan_threaded, read_golden, same_slot, simple_problem)

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def ctx(harp):
    c = harp.Context(0)
    yield c
    c.close()


def _check(harp, ctx, problem, cands, caps, label, need_fast=True):
    caps = np.ascontiguousarray(caps, dtype=np.int64)
    tables = oracle.build_tables(problem)
    want = oracle_plan_h1f1b_threaded(tables, cands, caps)
    fast32 = harp.Tables(ctx, problem).fast32
    assert fast32 or not need_fast, label
    for path in [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if fast32 else []):
        tag = "%s (path %d)" % (label, path)
        got, dev_tables = harp.plan_h1f1b(ctx, problem, cands, caps, path)
        assert_plans_equal(got, want, tag)
        if not (got.warmup == want.warmup).all():
            bad = np.nonzero((got.warmup != want.warmup).any(axis=1))[0]
            raise AssertionError("%s: warmup differs at %d candidates, first %d: got %s want %s"
                                 % (tag, bad.size, bad[0], got.warmup[bad[0]], want.warmup[bad[0]]))
    return got, want, dev_tables


def _score(harp, ctx, dev_tables, cands, splits, caps):
    import torch
    dc = harp.DeviceCandidates(ctx, cands)
    sp = torch.from_numpy(np.ascontiguousarray(splits, dtype=np.int32)).to(ctx.device)
    tm = torch.from_numpy(np.ascontiguousarray(caps, dtype=np.int64)).to(ctx.device)
    wu = torch.full((max(cands.C, 1), cands.S_max), -7, dtype=torch.int32, device=ctx.device)
    b = torch.full((max(cands.C, 1),), -7, dtype=torch.int64, device=ctx.device)
    t = torch.full_like(b, -7)
    st = torch.full((max(cands.C, 1),), -7, dtype=torch.int32, device=ctx.device)
    harp.harp_score_h1f1b(ctx, dev_tables, dc, sp, tm, wu, b, t, st)
    torch.cuda.synchronize()
    n = cands.C
    return wu[:n].cpu().numpy(), b[:n].cpu().numpy(), t[:n].cpu().numpy(), st[:n].cpu().numpy()


def _caps_from_min_max(problem, cands, num, den, fallback=7):
    mm = oracle_plan_threaded(oracle.build_tables(problem), cands)
    return np.where(mm.status == oracle.OK, mm.bottleneck // den * num, fallback).astype(np.int64), mm


def test_h1f1b_paper_examples(harp, ctx):
    for row in read_golden(os.path.join(GOLD, "h1f1b_warmup_examples.txt")):
        t_max, cuts, counts = [f.strip() for f in row.split("|")]
        cuts = [int(x) for x in cuts.split()]
        S = len(cuts) + 1
        p = simple_problem([int(t_max)] * S, M=16, G=S, ndev=(1,) * S, act=cuts + [0],
                           bw=np.ones((S, S), dtype=np.int64))
        cands = cands_from_lists([[(g, 1) for g in range(S)]])
        got, _, _ = _check(harp, ctx, p, cands, [int(t_max)], row)
        assert list(got.warmup[0]) == [int(x) for x in counts.split()]


def test_h1f1b_tiny_and_random_small(harp, ctx):
    w = W.make("tiny")
    for num, den in ((1, 1), (9, 8), (2, 1)):
        caps, _ = _caps_from_min_max(w.problem, w.candidates(), num, den)
        _check(harp, ctx, w.problem, w.candidates(), caps, "tiny x%d/%d" % (num, den))
    fast_runs = 0
    for seed in range(300):
        w = W.random_small(seed)
        cands = w.candidates()
        fast_runs += harp.Tables(ctx, w.problem).fast32
        for num, den in ((1, 1), (5, 4), (4, 1)):
            caps, _ = _caps_from_min_max(w.problem, cands, num, den)
            _check(harp, ctx, w.problem, cands, caps, "seed %d x%d/%d" % (seed, num, den), need_fast=False)
    assert fast_runs > 150
    # caps at the edges of the 32-bit arithmetic: zero, one, around 2^31 and 2^32, far above every time
    edge = np.array([0, 1, 2 ** 31 - 1, 2 ** 31, 2 ** 32 + 5, 2 ** 40], dtype=np.int64)
    for seed in range(40):
        w = W.random_small(seed)
        cands = w.candidates()
        _check(harp, ctx, w.problem, cands, edge[np.arange(cands.C) % edge.size], "edge caps, seed %d" % seed,
               need_fast=False)


@pytest.mark.parametrize("name,n,stride", [("llama7b", 1024, 1), ("llama70b", 2048, 8), ("finegrained", 512, 127),
                                           ("stress", 384, 681)])
def test_h1f1b_workloads(harp, ctx, name, n, stride):
    w = W.make(name)
    idx = (np.arange(n, dtype=np.int64) * stride) % w.C
    cands = w.candidates().take(idx)
    feasible = 0
    for num, den in ((1, 1), (33, 32), (3, 2)):
        caps, mm = _caps_from_min_max(w.problem, cands, num, den)
        got, want, dev_tables = _check(harp, ctx, w.problem, cands, caps, "%s x%d/%d" % (name, num, den))
        ok = want.status == oracle.OK
        feasible += int(ok.sum())
        # the scorer (a second code path) reproduces counts and times of the reported plans
        wu, b, t, st = _score(harp, ctx, dev_tables, cands, got.splits, caps)
        assert (st[ok] == oracle.OK).all() and (wu[ok] == got.warmup[ok]).all()
        assert (b[ok] == got.bottleneck[ok]).all() and (t[ok] == got.iter_time[ok]).all()
        assert (got.bottleneck[ok] <= caps[ok]).all()
        # H-1F1B keeps at least the classic number of microbatches in flight
        S = cands.cand_S[:, None]
        s = np.arange(cands.S_max)[None, :]
        classic = np.minimum(S - s, w.problem.M)
        assert ((got.warmup >= classic) | (s >= S) | ~ok[:, None]).all()
    assert feasible > 0


def test_h1f1b_medium_random_problems(harp, ctx):
    rng = np.random.default_rng(221)
    for case in range(8):
        L = int(rng.integers(65, 400))
        T, G = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        ndev = rng.choice([2, 4, 8], size=G)
        fwd = rng.integers(1, 4000, size=(T, L))
        bw = rng.integers(50, 4000, size=(G, G))
        bw = np.minimum(bw, bw.T)
        params = rng.integers(0, 10**6, size=L)
        stash = rng.integers(0, 10**5, size=L)
        S_max = int(rng.integers(G, G + 8))
        tp = (1, 2, 4, 8)[:int(rng.integers(1, 5))]
        per_stage = int(params.sum() + 1.5 * S_max * stash.sum()) // S_max
        mem = (rng.uniform(0.7, 2.0, size=T) * per_stage / np.sqrt(tp[-1])).astype(np.int64)
        p = simple_problem(np.zeros(L), M=int(rng.integers(1, 40)), T=T, G=G, ndev=ndev, tp=tp,
                           fwd=fwd, bwd=2 * fwd, params=params, stash=stash,
                           act=rng.integers(0, 4 * 10**6, size=L), gtype=rng.integers(0, T, size=G),
                           mem=mem, bw=bw)
        p.group_ndev = np.maximum(p.group_ndev, p.tp_degrees[-1]).astype(np.int32)
        cands = W.make_candidates(p, case, 277, G, S_max, 0, 48)
        for num, den in ((1, 1), (5, 4), (3, 1)):
            caps, _ = _caps_from_min_max(p, cands, num, den)
            _check(harp, ctx, p, cands, caps, "medium %d (L=%d) x%d/%d" % (case, L, num, den))


def test_h1f1b_wide_bands_ties_and_degenerate(harp, ctx):
    rng = np.random.default_rng(231)
    L, G, T = 600, 2, 2
    fwd = rng.integers(1, 3000, size=(T, L))
    p = simple_problem(np.zeros(L), M=12, T=T, G=G, ndev=[16] * G, tp=(1, 2), fwd=fwd, bwd=fwd,
                       params=rng.integers(1, 10**6, size=L), stash=rng.integers(0, 10**4, size=L),
                       act=rng.integers(0, 10**6, size=L), gtype=[0, 1], mem=[1 << 50, 1 << 50],
                       bw=np.array([[4000, 30], [30, 3000]]))
    cands = W.make_candidates(p, 0, 281, G, 5, 0, 12)
    caps, _ = _caps_from_min_max(p, cands, 9, 8)
    _check(harp, ctx, p, cands, caps, "wide bands")

    p = simple_problem([7] * 90, M=5, ndev=(8,), tp=(1, 2))
    cands = cands_from_lists([same_slot(S) for S in (1, 2, 7, 8)], S_max=8)
    _check(harp, ctx, p, cands, [7 * 90, 7 * 45, 7 * 13, 7 * 12], "uniform operators, exact caps")
    _check(harp, ctx, p, cands, [7 * 90 - 1, 7 * 45 - 1, 7 * 13 - 1, 7 * 12 - 1], "caps one below the optimum")
    p = simple_problem([0] * 90, M=5, ndev=(8,), tp=(1, 2))
    _check(harp, ctx, p, cands, [0, 0, 0, 0], "all-zero costs under a zero cap")

    L = 12
    p = simple_problem(list(range(1, L + 1)), M=3, ndev=(16,), tp=(1,), params=[10] * L, mem=[25])
    lists = [same_slot(S) for S in (1, 5, 6, 12, 13)] + [[(0, 3)], [(1, 1)]]
    cands = cands_from_lists(lists, S_max=16)
    got, want, _ = _check(harp, ctx, p, cands, [100, 100, 100, -1, 100, 100, 100], "mixed statuses")
    assert set(want.status) == {oracle.OK, oracle.INFEASIBLE, oracle.INVALID}
    w = W.make("tiny")
    got, _ = harp.plan_h1f1b(ctx, w.problem, w.candidates(0, 0), np.zeros(0, dtype=np.int64))
    assert got.status.shape == (0,)


def test_h1f1b_counts_decide_feasibility(harp, ctx):
    # three one-operator stages, stash 10 each, slow link then fast link: counts 5, 2, 1
    for mem, st in ((50, oracle.OK), (49, oracle.INFEASIBLE)):
        p = simple_problem([1000] * 3, M=16, G=3, ndev=(1, 1, 1), act=[750, 0, 0], stash=[10] * 3,
                           bw=np.ones((3, 3), dtype=np.int64), mem=[mem])
        cands = cands_from_lists([[(0, 1), (1, 1), (2, 1)]])
        got, want, _ = _check(harp, ctx, p, cands, [1000], "memory %d" % mem)
        assert want.status[0] == st


def test_h1f1b_sums_beyond_32_bits_and_int64_tables(harp, ctx):
    rng = np.random.default_rng(19)
    L, G = 60, 5
    act = rng.integers(11, 20, size=L) * 10**8
    act[rng.choice(L - 1, size=3, replace=False)] = 1000
    bw = np.ones((G, G), dtype=np.int64) + np.eye(G, dtype=np.int64) * 10**6
    p = simple_problem(np.zeros(L), M=3, G=G, ndev=(4,) * G, tp=(1, 2),
                       fwd=rng.integers(1, 10**6, size=(1, L)), bwd=rng.integers(1, 10**6, size=(1, L)),
                       act=act, bw=bw)
    full = W.make_candidates(p, 0, 83, G, 9, 0, 48)
    lists = []
    for c in range(full.C):
        slots = [(int(g), int(t)) for g, t in zip(full.cand_group[c, :full.cand_S[c]], full.cand_tp[c, :full.cand_S[c]])]
        lists.append([x for x in slots if x[0] != G - 1] if c % 2 else slots)
    cands = cands_from_lists(lists, S_max=9)
    caps, _ = _caps_from_min_max(p, cands, 1, 1)
    got, want, _ = _check(harp, ctx, p, cands, caps, "wide sums")
    ok = want.status == oracle.OK
    sums = want.iter_time[ok] - (p.M - 1) * caps[ok]
    assert (sums >= 1 << 31).any() and (sums < 1 << 30).any()

    L = 50
    p = simple_problem(np.zeros(L), M=6, G=2, ndev=(6, 6), tp=(1, 2, 3, 6),
                       fwd=rng.integers(1, 1000, size=(1, L)), bwd=rng.integers(1, 1000, size=(1, L)),
                       act=rng.integers(0, 10**5, size=L), stash=rng.integers(0, 100, size=L),
                       mem=[4000], bw=[[900, 10], [10, 700]])
    cands = W.make_candidates(p, 0, 79, 2, 6, 0, 32)
    caps, _ = _caps_from_min_max(p, cands, 5, 4)
    _check(harp, ctx, p, cands, caps, "odd degrees", need_fast=False)
    assert not harp.Tables(ctx, p).fast32


def test_h1f1b_scorer_on_arbitrary_partitions(harp, ctx):
    rng = np.random.default_rng(5)
    w = W.make("llama70b")
    cands = w.candidates(0, 1024)
    L, S_max = w.problem.L, cands.S_max
    splits = np.full((cands.C, S_max + 1), -1, dtype=np.int32)
    for c in range(cands.C):
        S = int(cands.cand_S[c])
        inner = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False)) if S > 1 else []
        splits[c, :S + 1] = [0, *inner, L]
    splits[5, 2] = splits[5, 1]                 # not strictly increasing
    splits[9, 0] = 1                            # does not start at 0
    w.problem.type_mem_bytes[:] *= 4             # random cuts rarely fit the real devices
    caps = 4 * rng.integers(10**5, 3 * 10**6, size=cands.C)     # some above, some below the stage times
    caps[11] = -5
    tables = oracle.build_tables(w.problem)
    wu, b, t, st = oracle.score_h1f1b(tables, cands, splits, caps)
    dev_tables = harp.Tables(ctx, w.problem)
    gwu, gb, gt, gst = _score(harp, ctx, dev_tables, cands, splits, caps)
    assert (gst == st).all() and (gwu == wu).all() and (gb == b).all() and (gt == t).all()
    assert set(st) == {oracle.OK, oracle.INFEASIBLE, oracle.INVALID}


def test_caps_beyond_the_accepted_range_are_invalid(harp, ctx):
    """The largest accepted cap gives a plan with an exact iteration time; one more, or INT64_MAX passed
    as "no cap", makes the candidate INVALID on every entry point that takes a cap, on both paths and
    in the oracle (sum + (M - 1) t_max would otherwise leave int64)."""
    w = W.make("llama7b")
    p = w.problem
    top = min(2 ** 47 - 1, (2 ** 63 - 1) // (3 * p.L + p.M))
    cands = w.candidates(0, 8)
    cands.cand_group[7, 0] = p.G + 3                      # malformed whatever the cap
    caps = np.array([top, top + 1, 2 ** 63 - 1, 2 ** 62, top, -1, top - 1, top + 1], dtype=np.int64)
    got, want, dev_tables = _check(harp, ctx, p, cands, caps, "caps at the limit")
    assert list(want.status) == [0, 2, 2, 2, 0, 1, 0, 2]
    splits = oracle.plan_batch(oracle.build_tables(p), cands).splits       # each candidate's own min-max cuts
    wu, b, t, st = oracle.score_h1f1b(oracle.build_tables(p), cands, splits, caps)
    gwu, gb, gt, gst = _score(harp, ctx, dev_tables, cands, splits, caps)
    assert (gst == st).all() and (gwu == wu).all() and (gb == b).all() and (gt == t).all()
    assert list(st) == [0, 2, 2, 2, 0, 1, 0, 2]
    # a candidate the memory bounds reject keeps INVALID under such a cap (32-bit path: rejected by the pre-pass)
    tight = simple_problem([5] * 6, M=2, ndev=(4,), tp=(1,), params=[10] * 6, mem=[15])
    tc = cands_from_lists([same_slot(2), same_slot(2)])
    _, tw, _ = _check(harp, ctx, tight, tc, np.array([100, 2 ** 63 - 1], dtype=np.int64), "rejected by memory")
    assert list(tw.status) == [1, 2]


def test_h1f1b_stress_sample_both_paths(harp, ctx):
    """Every 16th candidate of the stress batch, at the caps the exact search finds, through the
    H-1F1B recurrence on both kernel paths, which share no code: identical plans and warm-up counts.
    A third of these candidates have a slot too wide for a wavefront's share of LDS and take the
    32-bit path's second launch."""
    w = W.make("stress")
    idx = np.arange(0, w.C, 16, dtype=np.int64)
    cands = w.candidates().take(idx)
    exact, _, _ = harp.plan_exact(ctx, w.problem, cands)
    caps = np.where(exact.status == oracle.OK, exact.bottleneck, 0).astype(np.int64)
    fast, _ = harp.plan_h1f1b(ctx, w.problem, cands, caps, harp.PATH_FAST32)
    gen, _ = harp.plan_h1f1b(ctx, w.problem, cands, caps, harp.PATH_GENERIC)
    assert_plans_equal(fast, gen, "stress H-1F1B, 32-bit against int64 path")
    assert (fast.warmup == gen.warmup).all()
    assert (fast.status == oracle.OK).any() and (fast.status != oracle.OK).any()


def test_h1f1b_full_stress_batch_properties(harp, ctx):
    """The whole stress batch at the caps the exact search found, in the launch configuration the
    benchmark times: what must hold for every candidate whatever its size."""
    w = W.make("stress")
    cands = w.candidates()
    exact, _, _ = harp.plan_exact(ctx, w.problem, cands)
    caps = np.where(exact.status == oracle.OK, exact.bottleneck, 0).astype(np.int64)
    got, dev_tables = harp.plan_h1f1b(ctx, w.problem, cands, caps)
    ok = got.status == oracle.OK
    assert ok.any() and ((exact.status == oracle.OK) | ~ok).all()     # H-1F1B needs at least as much memory
    assert (got.bottleneck[ok] <= caps[ok]).all()
    # under the same cap the least sum cannot beat the one found without the larger counts
    assert (got.iter_time[ok] >= exact.iter_time[ok]).all()
    wu, b, t, st = _score(harp, ctx, dev_tables, cands, got.splits, caps)
    assert (st[ok] == oracle.OK).all() and (wu[ok] == got.warmup[ok]).all()
    assert (b[ok] == got.bottleneck[ok]).all() and (t[ok] == got.iter_time[ok]).all()
    assert (got.warmup[~ok] == -1).all() and (got.splits[~ok] == -1).all()
    idx = np.nonzero(ok)[0][::1499]
    sub = cands.take(idx)
    owu, ob, ot, ost = oracle.score_h1f1b(oracle.build_tables(w.problem), sub, got.splits[idx], caps[idx])
    assert (ost == 0).all() and (owu == got.warmup[idx]).all() and (ot == got.iter_time[idx]).all()
    print("stress: %d of %d feasible under H-1F1B counts at the exact search's caps (classic counts: %d)"
          % (ok.sum(), cands.C, (exact.status == oracle.OK).sum()))


def _check_sweep(harp, ctx, problem, cands, label, max_caps=1 << 20):
    from helpers import oracle_plan_h1f1b_sweep_threaded
    want = oracle_plan_h1f1b_sweep_threaded(oracle.build_tables(problem), cands, max_caps)
    fast32 = harp.Tables(ctx, problem).fast32
    for path in [harp.PATH_GENERIC] + ([harp.PATH_FAST32] if fast32 else []):
        tag = "%s (path %d)" % (label, path)
        got, _ = harp.plan_h1f1b_sweep(ctx, problem, cands, max_caps, path)
        assert_plans_equal(got, want, tag)
        for name in ("warmup", "t_max", "n_caps"):
            a, b = getattr(got, name), getattr(want, name)
            if not (a == b).all():
                bad = np.nonzero((a != b).reshape(a.shape[0], -1).any(axis=1))[0]
                raise AssertionError("%s: %s differs at %d candidates, first %d: got %s want %s"
                                     % (tag, name, bad.size, bad[0], a[bad[0]], b[bad[0]]))
    return got, want


def test_h1f1b_sweep_of_candidates(harp, ctx):
    """The search over the cap for candidates with a fixed slicing (section 5.2.4 (2) around the
    capped H-1F1B recurrence) against the oracle: plans, counts, chosen cap and caps tried."""
    feasible = moved = 0
    for seed in range(150):
        w = W.random_small(seed)
        cands = w.candidates()
        got, want = _check_sweep(harp, ctx, w.problem, cands, "seed %d" % seed)
        ok = want.status == oracle.OK
        feasible += int(ok.sum())
        mm, _ = harp.plan(ctx, w.problem, cands)
        moved += int((want.t_max[ok] != mm.bottleneck[ok]).sum())
        if seed % 10 == 0:
            _check_sweep(harp, ctx, w.problem, cands, "seed %d, 2 caps" % seed, max_caps=2)
    assert feasible > 500 and moved > 20
    # malformed and infeasible candidates; an empty batch
    p = simple_problem([5, 3, 8, 2, 7, 4], M=3, G=3, ndev=(2, 2, 1), tp=(1, 2), bw=np.full((3, 3), 2),
                       act=[4, 9, 2, 7, 5, 3], params=[1] * 6, stash=[1] * 6, mem=[40])
    lists = [[(0, 1), (0, 1), (1, 2)], [(0, 2), (1, 1), (2, 1)], [(0, 1), (1, 1), (0, 1)], [(0, 2), (0, 1)],
             [(0, 3)], [(5, 1)], [(2, 1)] * 1 + [(1, 1)] * 2 + [(0, 1)] * 2 + [(0, 2)], [(1, 2)]]
    cands = cands_from_lists(lists, S_max=7)
    _, want = _check_sweep(harp, ctx, p, cands, "statuses")
    assert {oracle.OK, oracle.INVALID} <= set(want.status)
    got, _ = harp.plan_h1f1b_sweep(ctx, p, cands.slice(0, 0))
    assert got.status.shape == (0,)
    for name, n in (("tiny", 16), ("llama7b", 64), ("llama70b", 24)):
        w = W.make(name)
        cands = w.candidates(0, n)
        got, want = _check_sweep(harp, ctx, w.problem, cands, name)
        ok = want.status == oracle.OK
        assert ok.any() and (name != "llama70b" or (want.status == oracle.INFEASIBLE).any())
        at, _ = harp.plan_h1f1b(ctx, w.problem, cands, np.where(ok, want.t_max, -1))
        for field in ("splits", "warmup", "iter_time"):
            assert (getattr(at, field)[ok] == getattr(got, field)[ok]).all(), (name, field)
