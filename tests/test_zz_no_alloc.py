"""The allocation-free entry point against the entry point it is a variant of.

harp_plan_batch_static plans with the library's static scratch array in place of a caller-lent
workspace.  Its outputs must equal harp_plan_batch's bit for bit, on two calls in a row that share
the array (the second with a smaller batch of another shape, so that whatever the first call left
behind is still there), on both kernel paths; it must not allocate device memory; and it must refuse
a batch whose workspace cannot fit.
"""
import gc

import numpy as np
import pytest

from paper_2509_24859_amd import workloads as W

from helpers import assert_plans_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(harp):
    c = harp.Context(0)
    yield c
    c.close()


def _reference(harp, ctx, tables, dc):
    import torch
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    ws = harp.plan_workspace(ctx, tables, dc)
    harp.harp_plan_batch(ctx, tables, dc, out, ws)
    torch.cuda.synchronize()
    return out.to_host()


@pytest.mark.parametrize("path_name", ["auto", "generic"])
def test_static_scratch_matches_workspace_entry_point(harp, ctx, path_name):
    import torch
    path = {"auto": harp.PATH_AUTO, "generic": harp.PATH_GENERIC}[path_name]
    first = ("finegrained", 0, 6000 if path_name == "auto" else 600)      # more candidates than resident workgroups
    second = ("llama70b", 300, 1500 if path_name == "auto" else 300)      # smaller, other shape, other slice
    ctx.set_plan_path(path)
    try:
        for name, lo, n in (first, second):
            w = W.make(name)
            cands = w.candidates(lo, lo + n)
            tables = harp.Tables(ctx, w.problem)
            dc = harp.DeviceCandidates(ctx, cands)
            want = _reference(harp, ctx, tables, dc)
            assert (want.status == 0).any()
            out = harp.DevicePlans(ctx, dc.C, dc.S_max)
            out.poison()
            torch.cuda.synchronize()
            # no collection of earlier tests' garbage (which would free tensors) between the two readings
            gc.collect()
            gc.disable()
            try:
                before = torch.cuda.memory_allocated(ctx.device)
                harp.harp_plan_batch_static(ctx, tables, dc, out)
                assert torch.cuda.memory_allocated(ctx.device) == before     # nothing came from torch's allocator
            finally:
                gc.enable()
            torch.cuda.synchronize()
            assert_plans_equal(out.to_host(), want, "%s static, path %s" % (name, path_name))
    finally:
        ctx.set_plan_path(harp.PATH_AUTO)


def test_static_scratch_runs_with_few_workgroups(harp, ctx):
    """A stress-shaped batch whose lists and bands take most of the array: the call runs with the
    workgroups that still fit and gives the same plans."""
    import torch
    w = W.make("stress")
    cands = w.candidates(1000, 1000 + 100_000)
    tables = harp.Tables(ctx, w.problem)
    dc = harp.DeviceCandidates(ctx, cands)
    want = _reference(harp, ctx, tables, dc)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    harp.harp_plan_batch_static(ctx, tables, dc, out)
    torch.cuda.synchronize()
    assert_plans_equal(out.to_host(), want, "stress static")


def test_static_scratch_refuses_what_cannot_fit(harp, ctx):
    w = W.make("stress")
    cands = w.candidates(0, 200_000)          # lists and bands alone pass 32 MiB
    tables = harp.Tables(ctx, w.problem)
    dc = harp.DeviceCandidates(ctx, cands)
    out = harp.DevicePlans(ctx, dc.C, dc.S_max)
    out.poison()
    with pytest.raises(harp.HarpError) as e:
        harp.harp_plan_batch_static(ctx, tables, dc, out)
    assert e.value.code == harp.ERR_WORKSPACE
    assert "static scratch" in str(e.value)
    assert (out.status.cpu().numpy() == -7).all()          # nothing was launched


def test_static_scratch_empty_batch(harp, ctx):
    w = W.make("tiny")
    tables = harp.Tables(ctx, w.problem)
    dc = harp.DeviceCandidates(ctx, w.candidates(0, 0))
    out = harp.DevicePlans(ctx, 0, dc.S_max)
    harp.harp_plan_batch_static(ctx, tables, dc, out)
