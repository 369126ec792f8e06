"""Host-side choice of candidate group orderings (paper section 5.2.1): part of the product, not of
the input generators, and never used by the oracle (which has a twin of its own to check it)."""
from __future__ import annotations

import numpy as np


def memory_to_compute_order(p) -> np.ndarray:
    """Group ids in the order the paper's heuristic would run them (section 5.2.1): groups whose
    devices have the most memory per unit of compute throughput first, because earlier stages of a
    1F1B-style schedule keep more microbatches in flight.  Throughput of a GPU type is taken as the
    reciprocal of its total forward+backward time over the model, so the key of a group is the
    product memory x time of its type: an exact integer (Python integers: the product of two
    int64 values does not fit a double, and rounding it could reorder near-ties); ties go to the
    lower group id.  A host-side pre-filter for candidate orderings; the planner kernels take
    whatever orderings the caller lists."""
    work = [sum(int(f) + int(b) for f, b in zip(p.fwd_us[t], p.bwd_us[t])) for t in range(p.T)]
    key = [int(p.type_mem_bytes[t]) * work[t] for t in range(p.T)]       # memory / (1 / time), exact
    order = sorted(range(p.G), key=lambda g: (-key[int(p.group_type[g])], g))
    return np.asarray(order, dtype=np.int32)
