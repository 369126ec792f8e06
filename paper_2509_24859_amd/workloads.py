"""Seeded synthetic planning problems and candidate batches.

This module only draws numbers and lays them out as flat integer arrays.  It holds none of the
planner's arithmetic (no prefix sums, no cost model, no feasibility logic): the CPU oracle and the
HIP library both receive exactly these arrays and do all the computing themselves.

The five workloads stand in for the profiled GPT/MoE operator graphs and clusters of the paper's
evaluation (section 6 and appendix B: L around 10^2 layers, 3-15 stages, tensor-parallel degrees
1-8, 5-10 Gb/s links across subclusters against 200 Gb/s-300 GB/s inside one, 16-40 GB devices).

Random numbers: splitmix64 (Steele, Lea, Flood 2014) used as a counter-based generator, one
independent stream per array and one per candidate, so any slice of a batch can be generated on
its own and is identical on every machine.  Real-valued draws (log-uniform bandwidths, log-normal
costs) go through numpy's libm once, here, and are rounded to integers before anyone computes
with them.

Units: times in microseconds, sizes in bytes, bandwidths in bytes per microsecond
(1 MB = 10^6 B, 1 GB = 10^9 B, 1 Gb/s = 125 B/us, 1 GB/s = 1000 B/us).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

MB = 10**6
GB = 10**9
GBIT = 125          # bytes per microsecond in one Gb/s
GBYTE = 1000        # bytes per microsecond in one GB/s


def _mix(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


class Streams:
    """A batch of independent splitmix64 streams advanced in lock step.

    `state` has one entry per stream; `u64()` returns the next output of every stream.
    """

    def __init__(self, state: np.ndarray):
        self.state = np.array(state, dtype=np.uint64, copy=True).reshape(-1)

    def u64(self) -> np.ndarray:
        with np.errstate(over="ignore"):
            self.state = self.state + _GAMMA
        return _mix(self.state)

    def below(self, n) -> np.ndarray:
        """Integer in [0, n) per stream (n may be an array); plain modulo of the 64-bit draw."""
        return (self.u64() % np.asarray(n, dtype=np.uint64)).astype(np.int64)


def _stream_state(seed: int, config_id: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * _GAMMA + np.uint64(config_id)
        return _mix(np.uint64(base) + np.uint64(stream) * np.uint64(0xD1342543DE82EF95))


def _draw_u64(seed: int, config_id: int, stream: int, n: int) -> np.ndarray:
    """n successive outputs of one named stream."""
    s0 = _stream_state(seed, config_id, stream)
    with np.errstate(over="ignore"):
        ctr = s0 + (np.arange(1, n + 1, dtype=np.uint64) * _GAMMA)
    return _mix(ctr)


def _uniform_int(x: np.ndarray, lo: int, hi: int) -> np.ndarray:
    return (np.int64(lo) + (x % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int64)


def _unit_real(x: np.ndarray) -> np.ndarray:
    return (x >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def _log_uniform(x: np.ndarray, lo: float, hi: float) -> np.ndarray:
    return np.exp(np.log(lo) + _unit_real(x) * np.log(hi / lo))


def _normal(x1: np.ndarray, x2: np.ndarray) -> np.ndarray:
    u1 = np.maximum(_unit_real(x1), 2.0 ** -53)
    u2 = _unit_real(x2)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


@dataclass
class Problem:
    """One planning problem: operator profiles per GPU type and the cluster description."""
    L: int
    T: int
    G: int
    M: int
    ar_count: int
    tp_degrees: np.ndarray          # [n_tp] int32, ascending, first == 1
    fwd_us: np.ndarray              # [T][L] int64
    bwd_us: np.ndarray              # [T][L] int64
    param_bytes: np.ndarray         # [L] int64
    stash_bytes: np.ndarray         # [L] int64
    act_bytes: np.ndarray           # [L] int64
    group_type: np.ndarray          # [G] int32
    group_ndev: np.ndarray          # [G] int32
    type_mem_bytes: np.ndarray      # [T] int64
    bw: np.ndarray                  # [G][G] int64 bytes/us, symmetric

    @property
    def n_tp(self) -> int:
        return int(self.tp_degrees.shape[0])


@dataclass
class Candidates:
    """A batch of candidate slot lists (ordered device-group slicings)."""
    C: int
    S_max: int
    cand_S: np.ndarray              # [C] int32
    cand_group: np.ndarray          # [C][S_max] int32, unused slots -1
    cand_tp: np.ndarray             # [C][S_max] int32, unused slots 0

    def slice(self, lo: int, hi: int) -> "Candidates":
        return Candidates(hi - lo, self.S_max, self.cand_S[lo:hi].copy(),
                          self.cand_group[lo:hi].copy(), self.cand_tp[lo:hi].copy())

    def take(self, idx) -> "Candidates":
        idx = np.asarray(idx)
        return Candidates(int(idx.size), self.S_max, self.cand_S[idx].copy(),
                          self.cand_group[idx].copy(), self.cand_tp[idx].copy())


@dataclass
class Workload:
    name: str
    config_id: int
    seed: int
    problem: Problem
    C: int
    S_max: int
    S_min: int
    notes: dict = field(default_factory=dict)

    def candidates(self, lo: int = 0, hi: int | None = None) -> Candidates:
        hi = self.C if hi is None else hi
        return make_candidates(self.problem, self.seed, self.config_id, self.S_min, self.S_max,
                               lo, hi)


def _problem(L, T, G, M, tp, fwd, params, stash, act, gtype, gndev, mem, bw, ar_count=4):
    fwd = np.ascontiguousarray(fwd, dtype=np.int64)
    return Problem(
        L=L, T=T, G=G, M=M, ar_count=ar_count,
        tp_degrees=np.asarray(tp, dtype=np.int32),
        fwd_us=fwd, bwd_us=np.ascontiguousarray(2 * fwd, dtype=np.int64),
        param_bytes=np.ascontiguousarray(params, dtype=np.int64),
        stash_bytes=np.ascontiguousarray(stash, dtype=np.int64),
        act_bytes=np.ascontiguousarray(act, dtype=np.int64),
        group_type=np.asarray(gtype, dtype=np.int32),
        group_ndev=np.asarray(gndev, dtype=np.int32),
        type_mem_bytes=np.asarray(mem, dtype=np.int64),
        bw=np.ascontiguousarray(bw, dtype=np.int64))


def _scaled(base: np.ndarray, factors, divide: bool) -> np.ndarray:
    rows = []
    for f in factors:
        v = base.astype(np.float64) / f if divide else base.astype(np.float64) * f
        rows.append(np.maximum(1, np.rint(v)).astype(np.int64))
    return np.stack(rows)


def _bw_matrix(G: int, intra: int, inter_pairs: np.ndarray) -> np.ndarray:
    bw = np.zeros((G, G), dtype=np.int64)
    k = 0
    for a in range(G):
        bw[a, a] = intra
        for b in range(a + 1, G):
            bw[a, b] = bw[b, a] = max(1, int(inter_pairs[k]))
            k += 1
    return bw


# Frozen by oracle/calibrate_stress_memory.py: scale on the stress workload's device memories at
# which the oracle finds about 30% of the first 4096 seed-0 candidates infeasible.
STRESS_MEMORY_SCALE = 0.249897


def tiny(seed: int = 0) -> Workload:
    cid, L, T, G = 1, 8, 2, 2
    base = _uniform_int(_draw_u64(seed, cid, 0, L), 200, 2000)
    fwd = _scaled(base, (1.0, 0.55), divide=False)
    params = _uniform_int(_draw_u64(seed, cid, 1, L), 50, 400) * MB
    act = _uniform_int(_draw_u64(seed, cid, 2, L), 8, 64) * MB
    bw = _bw_matrix(G, 300 * GBYTE, np.full(1, 25 * GBIT))
    p = _problem(L, T, G, 4, (1, 2), fwd, params, act, act, [0, 1], [2, 2],
                 [40 * GB, 40 * GB], bw)
    return Workload("tiny", cid, seed, p, C=16, S_max=4, S_min=2)


def llama7b(seed: int = 0) -> Workload:
    cid, L, T, G = 2, 32, 3, 4
    base = _uniform_int(_draw_u64(seed, cid, 0, L), 9500, 10500)
    fwd = _scaled(base, (1.0, 0.6, 0.35), divide=True)
    act = np.full(L, 33554432, dtype=np.int64)
    inter = _uniform_int(_draw_u64(seed, cid, 3, G * (G - 1) // 2), 10, 100) * GBIT
    bw = _bw_matrix(G, 400 * GBYTE, inter)
    p = _problem(L, T, G, 32, (1, 2, 4), fwd, np.full(L, 3200 * MB), 16 * act, act,
                 [g % T for g in range(G)], [4] * G, [80 * GB, 40 * GB, 24 * GB], bw)
    return Workload("llama7b", cid, seed, p, C=1024, S_max=8, S_min=G)


def llama70b(seed: int = 0) -> Workload:
    cid, L, T, G = 3, 82, 4, 8
    layer = _uniform_int(_draw_u64(seed, cid, 0, L), 42750, 47250)
    layer[0] *= 4
    layer[L - 1] *= 4
    fwd = _scaled(layer, (1.0, 0.7, 0.45, 0.3), divide=True)
    act = np.full(L, 67108864, dtype=np.int64)
    x = _draw_u64(seed, cid, 3, G * (G - 1) // 2)
    inter = np.rint(_log_uniform(x, 5.0, 200.0) * GBIT).astype(np.int64)
    bw = _bw_matrix(G, 400 * GBYTE, inter)
    p = _problem(L, T, G, 64, (1, 2, 4, 8), fwd, np.full(L, 13700 * MB), 16 * act, act,
                 [g % T for g in range(G)], [8] * G,
                 [192 * GB, 80 * GB, 40 * GB, 24 * GB], bw)
    return Workload("llama70b", cid, seed, p, C=16384, S_max=16, S_min=G)


def finegrained(seed: int = 0) -> Workload:
    cid, L, T, G = 4, 160, 4, 16
    attn = _uniform_int(_draw_u64(seed, cid, 0, L // 2), 14250, 15750)
    base = np.empty(L, dtype=np.int64)
    base[0::2] = attn
    base[1::2] = 2 * attn
    fwd = _scaled(base, (1.0, 0.7, 0.45, 0.3), divide=True)
    params = np.empty(L, dtype=np.int64)
    params[0::2] = 4600 * MB
    params[1::2] = 9100 * MB
    act = np.empty(L, dtype=np.int64)
    act[0::2] = 134217728
    act[1::2] = 67108864
    stash = np.empty(L, dtype=np.int64)
    stash[0::2] = 6 * 67108864
    stash[1::2] = 10 * 67108864
    x = _draw_u64(seed, cid, 3, G * (G - 1) // 2)
    inter = np.rint(_log_uniform(x, 1.0, 100.0) * GBIT).astype(np.int64)
    bw = _bw_matrix(G, 400 * GBYTE, inter)
    p = _problem(L, T, G, 128, (1, 2, 4, 8), fwd, params, stash, act,
                 [g % T for g in range(G)], [16] * G,
                 [192 * GB, 80 * GB, 40 * GB, 24 * GB], bw)
    return Workload("finegrained", cid, seed, p, C=65536, S_max=32, S_min=G)


def stress(seed: int = 0, memory_scale: float | None = None) -> Workload:
    cid, L, T, G = 5, 512, 8, 32
    kappa = STRESS_MEMORY_SCALE if memory_scale is None else memory_scale
    z = _normal(_draw_u64(seed, cid, 0, L), _draw_u64(seed, cid, 4, L))
    base = np.maximum(1, np.rint(np.exp(np.log(800.0) + 0.6 * z))).astype(np.int64)
    fwd = _scaled(base, (1.0, 0.85, 0.7, 0.6, 0.5, 0.4, 0.3, 0.25), divide=True)
    params = base * 2 * MB
    act = _uniform_int(_draw_u64(seed, cid, 2, L), 8, 64) * MB
    x = _draw_u64(seed, cid, 3, G * (G - 1) // 2)
    inter = np.rint(_log_uniform(x, 1.0, 100.0) * GBIT).astype(np.int64)
    bw = _bw_matrix(G, 400 * GBYTE, inter)
    mem_gb = np.array([192, 141, 96, 80, 64, 48, 40, 24], dtype=np.float64)
    mem = np.rint(mem_gb * GB * kappa).astype(np.int64)
    p = _problem(L, T, G, 256, (1, 2, 4, 8), fwd, params, 4 * act, act,
                 [g % T for g in range(G)], [8] * G, mem, bw)
    return Workload("stress", cid, seed, p, C=262144, S_max=64, S_min=G,
                    notes={"memory_scale": kappa})


def random_small(seed: int, L_max: int = 10, S_cap: int = 5, odd_degrees: bool = True) -> Workload:
    """A small random problem for property tests: mixed GPU types, degrees and tight memory.

    Sizes: L in [2, L_max], up to 3 types, up to 3 groups of 1-4 devices, S_max in [G, S_cap].
    Roughly a third of the draws have memory tight enough to make some candidates infeasible, a
    sixth have one very slow link, and (with odd_degrees) a fifth allow a degree of 3.
    """
    cid = 99
    x = _draw_u64(seed, cid, 0, 16)
    L = 2 + int(x[0] % np.uint64(L_max - 1))
    T = 1 + int(x[1] % np.uint64(3))
    G = 1 + int(x[2] % np.uint64(3))
    M = 1 + int(x[3] % np.uint64(8))
    S_max = G + int(x[4] % np.uint64(max(1, S_cap - G + 1)))
    degree_sets = [(1,), (1, 2), (1, 2, 4), (1, 2, 4, 8)] + ([(1, 2, 3, 4)] if odd_degrees else [])
    tp = degree_sets[int(x[5] % np.uint64(len(degree_sets)))]
    ndev = _uniform_int(_draw_u64(seed, cid, 1, G), 1, 4)
    if tp[-1] == 8:
        ndev = ndev * 2
    gtype = _uniform_int(_draw_u64(seed, cid, 2, G), 0, T - 1)
    base = _uniform_int(_draw_u64(seed, cid, 3, L), 1, 60)
    speed = 1.0 + _unit_real(_draw_u64(seed, cid, 4, T)) * 2.0
    fwd = _scaled(base, speed, divide=False)
    fwd = fwd + _uniform_int(_draw_u64(seed, cid, 5, T * L), 0, 3).reshape(T, L)
    params = _uniform_int(_draw_u64(seed, cid, 6, L), 0, 40)
    stash = _uniform_int(_draw_u64(seed, cid, 7, L), 0, 12)
    act = _uniform_int(_draw_u64(seed, cid, 8, L), 0, 400)
    tight = int(x[6] % np.uint64(3))
    per_dev = int(params.sum() + min(M, S_max) * stash.sum())
    hi = max(2, per_dev if tight else 4 * per_dev)
    lo = max(1, hi // (6 if tight == 2 else 2))
    mem = _uniform_int(_draw_u64(seed, cid, 9, T), lo, hi)
    inter = _uniform_int(_draw_u64(seed, cid, 10, max(1, G * (G - 1) // 2)), 1, 40)
    if int(x[7] % np.uint64(6)) == 0:
        inter[0] = 1
    bw = _bw_matrix(G, int(20 + x[8] % np.uint64(200)), inter)
    p = _problem(L, T, G, M, tp, fwd, params, stash, act, gtype, ndev, mem, bw,
                 ar_count=int(x[9] % np.uint64(5)))
    p.bwd_us = np.ascontiguousarray(
        p.fwd_us + _uniform_int(_draw_u64(seed, cid, 11, T * L), 0, 50).reshape(T, L))
    return Workload("random_small", cid, seed, p, C=8, S_max=S_max, S_min=G)


def long_sequence(L: int = 1 << 20, seed: int = 0) -> Problem:
    """Operator-level problem for the table build alone: the stress workload's cluster (8 GPU
    types, 32 groups, degrees 1-8) with L operators, standing in for the 10^4-10^5 operator graphs
    that the paper's layer construction (section 5.1) starts from.  Too long to plan; it exists to
    show the table build streaming at HBM rate."""
    cid, T, G = 6, 8, 32
    base = _uniform_int(_draw_u64(seed, cid, 0, L), 200, 3000)
    fwd = _scaled(base, (1.0, 0.85, 0.7, 0.6, 0.5, 0.4, 0.3, 0.25), divide=True)
    params = base * 2 * MB
    act = _uniform_int(_draw_u64(seed, cid, 2, L), 8, 64) * MB
    x = _draw_u64(seed, cid, 3, G * (G - 1) // 2)
    inter = np.rint(_log_uniform(x, 1.0, 100.0) * GBIT).astype(np.int64)
    bw = _bw_matrix(G, 400 * GBYTE, inter)
    mem = np.array([192, 141, 96, 80, 64, 48, 40, 24], dtype=np.int64) * GB
    return _problem(L, T, G, 256, (1, 2, 4, 8), fwd, params, 4 * act, act,
                    [g % T for g in range(G)], [8] * G, mem, bw)


WORKLOADS = {"tiny": tiny, "llama7b": llama7b, "llama70b": llama70b,
             "finegrained": finegrained, "stress": stress}
ORDER = ("tiny", "llama7b", "llama70b", "finegrained", "stress")


def make(name: str, seed: int = 0) -> Workload:
    return WORKLOADS[name](seed)


@dataclass
class Orderings:
    """A batch of group orderings: candidate c runs its S stages on the groups ord_group[c, :ord_G[c]]
    in that order; how each group's devices are cut into stages is left to the planner."""
    C: int
    G_max: int
    S_max: int
    ord_S: np.ndarray        # [C] int32
    ord_G: np.ndarray        # [C] int32
    ord_group: np.ndarray    # [C][G_max] int32, -1 beyond ord_G

    def slice(self, lo: int, hi: int) -> "Orderings":
        return Orderings(hi - lo, self.G_max, self.S_max, self.ord_S[lo:hi].copy(), self.ord_G[lo:hi].copy(),
                         self.ord_group[lo:hi].copy())

    def take(self, idx) -> "Orderings":
        idx = np.asarray(idx, dtype=np.int64)
        return Orderings(int(idx.size), self.G_max, self.S_max, self.ord_S[idx].copy(), self.ord_G[idx].copy(),
                         self.ord_group[idx].copy())


def orderings_from_lists(lists, S_max=None, G_max=None) -> Orderings:
    """lists: per candidate (S, [group ids in order])."""
    G_max = max(len(g) for _, g in lists) if G_max is None else G_max
    S_max = max(S for S, _ in lists) if S_max is None else S_max
    C = len(lists)
    og = np.full((C, G_max), -1, dtype=np.int32)
    for c, (_, groups) in enumerate(lists):
        og[c, :len(groups)] = groups[:G_max]
    return Orderings(C, G_max, max(S_max, 1), np.array([S for S, _ in lists], dtype=np.int32),
                     np.array([len(g) for _, g in lists], dtype=np.int32), og)


def make_orderings(p: Problem, seed: int, config_id: int, S_min: int, S_max: int, lo: int, hi: int) -> Orderings:
    """Orderings lo..hi-1 of a batch; ordering c depends only on (seed, config_id, c): a uniformly
    random order of all G groups (Fisher-Yates) and a stage count drawn from [max(S_min, G),
    min(S_max, devices)]."""
    n = hi - lo
    G = p.G
    cs = np.arange(lo, hi, dtype=np.uint64)
    with np.errstate(over="ignore"):
        st = _mix(_stream_state(seed, config_id, 2000) + cs * np.uint64(0xA0761D6478BD642F))
    rng = Streams(st)
    order = np.tile(np.arange(G, dtype=np.int64), (n, 1))
    rows = np.arange(n)
    for k in range(G - 1, 0, -1):
        r = rng.below(k + 1)
        a = order[rows, k].copy()
        order[rows, k] = order[rows, r]
        order[rows, r] = a
    top = min(S_max, int(p.group_ndev.sum()))
    low = max(S_min, G)
    if top < low:
        raise ValueError("no stage count between the number of groups and the number of devices")
    S = low + rng.below(top - low + 1)
    return Orderings(n, G, S_max, S.astype(np.int32), np.full(n, G, dtype=np.int32), order.astype(np.int32))


def make_candidates(p: Problem, seed: int, config_id: int, S_min: int, S_max: int,
                    lo: int, hi: int) -> Candidates:
    """Candidates lo..hi-1 of the batch; candidate c depends only on (seed, config_id, c).

    Per candidate: a uniformly random order of the G groups (Fisher-Yates); a stage count S drawn
    from [S_min, S_max]; every group gets one slot and the S - G extra slots go one at a time to a
    uniformly drawn group that still has fewer slots than devices; within a group holding k slots,
    each slot's degree is drawn uniformly from the allowed degrees not above floor(ndev / k), so a
    group is never over-subscribed.  Slots of one group are adjacent, in the drawn group order.
    """
    n = hi - lo
    G = p.G
    cs = np.arange(lo, hi, dtype=np.uint64)
    with np.errstate(over="ignore"):
        st = _mix(_stream_state(seed, config_id, 1000) + cs * np.uint64(0xA0761D6478BD642F))
    rng = Streams(st)

    order = np.tile(np.arange(G, dtype=np.int64), (n, 1))
    rows = np.arange(n)
    for k in range(G - 1, 0, -1):
        r = rng.below(k + 1)
        a = order[rows, k].copy()
        order[rows, k] = order[rows, r]
        order[rows, r] = a

    if S_max < G:
        raise ValueError("every group needs a slot: S_max must be at least G")
    S_min = max(S_min, G)
    S = S_min + rng.below(S_max - S_min + 1)
    cap = np.minimum(p.group_ndev.astype(np.int64), S_max)
    S = np.minimum(S, int(cap.sum()))
    slots = np.ones((n, G), dtype=np.int64)          # indexed by group id
    for _ in range(S_max - G):
        need = slots.sum(axis=1) < S
        elig = slots < cap[None, :]
        cnt = np.maximum(elig.sum(axis=1), 1)
        r = rng.below(cnt)
        pick = (np.cumsum(elig, axis=1) > r[:, None]).argmax(axis=1)
        slots[rows, pick] += need.astype(np.int64) * elig[rows, pick]

    cand_group = np.full((n, S_max), -1, dtype=np.int32)
    cand_tp = np.zeros((n, S_max), dtype=np.int32)
    tp = p.tp_degrees.astype(np.int64)
    ndev = p.group_ndev.astype(np.int64)
    ends = np.cumsum(slots[rows[:, None], order], axis=1)     # slots used up to each ordered group
    for s in range(S_max):
        live = s < S
        k = np.minimum((ends <= s).sum(axis=1), G - 1)
        g = order[rows, k]
        lim = ndev[g] // slots[rows, g]
        n_ok = np.maximum((tp[None, :] <= lim[:, None]).sum(axis=1), 1)
        d = tp[rng.below(n_ok)]
        cand_group[:, s] = np.where(live, g, -1)
        cand_tp[:, s] = np.where(live, d, 0)
    return Candidates(n, S_max, S.astype(np.int32), cand_group, cand_tp)


def dense_counts(L: int, S: np.ndarray):
    """(cells, transitions) per candidate of the dense stage-by-stage recurrence.

    Fixed formulas, independent of how an implementation prunes: cells = S (L - S + 1);
    transitions = (S - 2) R (R + 1) / 2 + 2 R with R = L - S + 1 for S >= 2, and 1 for S == 1.
    Candidates with S > L count as zero.
    """
    S = np.asarray(S, dtype=np.int64)
    R = L - S + 1
    cells = np.where(R > 0, S * R, 0)
    trans = np.where(S >= 2, (S - 2) * R * (R + 1) // 2 + 2 * R, 1)
    trans = np.where(R > 0, trans, 0)
    return cells, trans
