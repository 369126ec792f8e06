"""DAG model of a 1F1B-style pipeline (paper section 4.2.1), as a checker of the cost model.

Test infrastructure, like everything under oracle/: the product never imports it.

For microbatch k at stage s the DAG has the nodes F[k,s], B[k,s] (forward and backward compute),
CF[k,s] and CB[k,s] (the transfers between stages s and s+1, forward and backward).  Edges:
  E_comp  the computations of one stage run one after the other, in the order of a 1F1B-style
          schedule: N_s forwards during warm-up, then backward and forward alternate, then the
          remaining backwards;
  E_comm  transfers in the same direction over one link run one after the other (full duplex);
  E_dep   F[k,s] -> CF[k,s] -> F[k,s+1];  F[k,S] -> B[k,S];  B[k,s+1] -> CB[k,s] -> B[k,s].
Every edge u -> v carries d(u) and means s(v) - s(u) >= d(u) (eq. precedence); every node starts as
soon as all its predecessors have finished, s(F[1,1]) = 0.  The end-to-end latency is the largest
finish time.  Plain Python, exact integers.
"""
from __future__ import annotations


def stage_order(B: int, n_warmup: int):
    """Computation order of one stage: ('F', k) / ('B', k) for microbatches k = 0..B-1."""
    n = min(n_warmup, B)
    order = [("F", k) for k in range(n)]
    for k in range(B):
        order.append(("B", k))
        if k + n < B:
            order.append(("F", k + n))
    return order


def simulate(f, b, c, B: int, warmup):
    """f[s], b[s]: forward and backward time of stage s; c[s]: transfer time between s and s+1
    (len S-1); B microbatches; warmup[s] = forwards stage s launches before its first backward.
    Returns (latency, start) with start[(kind, k, s)] for kind in F, B, CF, CB."""
    S = len(f)
    assert len(b) == S and len(c) == S - 1 and len(warmup) == S
    queue = [stage_order(B, warmup[s]) for s in range(S)]
    pos = [0] * S
    stage_free = [0] * S
    link_free = {("CF", s): 0 for s in range(S - 1)}
    link_free.update({("CB", s): 0 for s in range(S - 1)})
    start, finish = {}, {}

    def transfer(kind, k, s, ready):
        # transfers of one direction leave in the order their data is produced, which on every link
        # is the microbatch order
        t0 = max(link_free[(kind, s)], ready)
        start[(kind, k, s)] = t0
        finish[(kind, k, s)] = t0 + c[s]
        link_free[(kind, s)] = t0 + c[s]

    progress = True
    while progress:
        progress = False
        for s in range(S):
            while pos[s] < len(queue[s]):
                kind, k = queue[s][pos[s]]
                if kind == "F":
                    ready = 0 if s == 0 else finish.get(("CF", k, s - 1))
                    dur = f[s]
                else:
                    ready = finish.get(("F", k, s)) if s == S - 1 else finish.get(("CB", k, s))
                    dur = b[s]
                if ready is None:
                    break
                t0 = max(stage_free[s], ready)
                start[(kind, k, s)] = t0
                finish[(kind, k, s)] = stage_free[s] = t0 + dur
                pos[s] += 1
                progress = True
                if kind == "F" and s < S - 1:
                    transfer("CF", k, s, t0 + dur)
                if kind == "B" and s > 0:
                    transfer("CB", k, s - 1, t0 + dur)
    if any(pos[s] < len(queue[s]) for s in range(S)):
        raise ValueError("the schedule deadlocks: a stage waits for a backward its warm-up count never lets arrive")
    return max(stage_free), start


def cost_model(f, b, c, B: int) -> int:
    """eq. gpipe_cost_model for given stage and transfer times."""
    t = [x + y for x, y in zip(f, b)]
    return sum(t) + 2 * sum(c) + (B - 1) * max(t)
