"""Finds the device-memory scale of the stress workload.  TEST INFRASTRUCTURE ONLY.

Bisects the scalar that multiplies the stress workload's per-type device memories until the C
oracle marks about 30% (accepted: 28-32%) of the first 4096 seed-0 candidates infeasible, then
prints the value rounded to 6 significant digits.  The printed value is frozen by hand as
`STRESS_MEMORY_SCALE` in the workload generator.  Calls only the oracle and the generator.

Run from the repository root:  python -m oracle.calibrate_stress_memory
"""
from __future__ import annotations

import os
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import oracle  # noqa: E402
from paper_2509_24859_amd import workloads  # noqa: E402

N = 4096


def infeasible_fraction(scale: float, threads: int) -> float:
    w = workloads.stress(0, memory_scale=scale)
    cands = w.candidates(0, N)
    tables = oracle.build_tables(w.problem)
    out = oracle.Plans(N, cands.S_max)
    step = 32
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda lo: oracle.plan_batch(tables, cands, lo, min(lo + step, N), out),
                    range(0, N, step)))
    return float((out.status == oracle.INFEASIBLE).mean())


def main():
    threads = len(os.sched_getaffinity(0))
    lo, hi = 0.05, 4.0           # fraction infeasible falls as the scale grows
    best = None
    for it in range(24):
        mid = float("%.6g" % ((lo * hi) ** 0.5))
        f = infeasible_fraction(mid, threads)
        print("scale %.6g -> infeasible %.4f" % (mid, f), flush=True)
        if 0.295 <= f <= 0.305:
            best = mid
            break
        if 0.28 <= f <= 0.32:
            best = mid
        if f > 0.30:
            lo = mid
        else:
            hi = mid
    print("STRESS_MEMORY_SCALE =", best)


if __name__ == "__main__":
    main()
