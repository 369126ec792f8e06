"""Host-side choice of candidate group orderings (paper section 5.2.1): part of the product, not of
the input generators, and never used by the oracle."""
from __future__ import annotations

import numpy as np


def memory_to_compute_order(p) -> np.ndarray:
    """Group ids in the order the paper's heuristic would run them (section 5.2.1): groups whose
    devices have the most memory per unit of compute throughput first, because earlier stages of a
    1F1B-style schedule keep more microbatches in flight.  Throughput of a GPU type is taken as the
    reciprocal of its total forward+backward time over the model; ties go to the lower group id.
    A host-side pre-filter for candidate orderings; the planner kernels take whatever orderings
    the caller lists."""
    work = (p.fwd_us + p.bwd_us).sum(axis=1).astype(np.float64)          # per type, us for the whole model
    ratio = p.type_mem_bytes.astype(np.float64) * work                   # memory / (1 / time)
    per_group = ratio[p.group_type]
    return np.lexsort((np.arange(p.G), -per_group)).astype(np.int32)
