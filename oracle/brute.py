"""Brute-force twin of the oracle for tiny inputs.  TEST INFRASTRUCTURE ONLY.

Everything is recomputed from the raw problem arrays by literal summation over operators and
literal enumeration of all ways to cut the operator sequence (no tables, no recurrence, nothing
shared with `harp_oracle.c`), in Python's unbounded integers.  It exists to pin the C oracle.

Stage cost, transfer cost and memory rule follow the paper's section 5.2.2 / 5.2.3 constraints
(i)-(iii) under the integer readings stated at the top of `harp_oracle.c`.
"""
from __future__ import annotations

from itertools import combinations

INF = (1 << 63) - 1


def _cdiv(a: int, b: int) -> int:
    return -((-a) // b)


def stage_time(p, g: int, tp: int, j: int, i: int) -> int:
    t = int(p.group_type[g])
    work = sum(int(p.fwd_us[t][l]) + int(p.bwd_us[t][l]) for l in range(j, i))
    ar = 0
    if tp > 1:
        for l in range(j, i):
            ar += _cdiv(int(p.ar_count) * 2 * (tp - 1) * int(p.act_bytes[l]), tp * int(p.bw[g][g]))
    return _cdiv(work, tp) + ar


def cut_time(p, g: int, h: int, i: int) -> int:
    return _cdiv(int(p.act_bytes[i - 1]), int(p.bw[g][h]))


def memory_fits(p, g: int, tp: int, n: int, j: int, i: int) -> bool:
    par = sum(int(p.param_bytes[l]) for l in range(j, i))
    sta = sum(int(p.stash_bytes[l]) for l in range(j, i))
    return par + n * sta <= tp * int(p.type_mem_bytes[int(p.group_type[g])])


def stage_cost(p, S: int, grp, tp, s: int, j: int, i: int) -> int:
    """w(s; j, i): INF if the stage does not fit, else max(stage time, transfer after it)."""
    n = min(S - s, int(p.M))
    if not memory_fits(p, int(grp[s]), int(tp[s]), n, j, i):
        return INF
    c = 0 if s == S - 1 else cut_time(p, int(grp[s]), int(grp[s + 1]), i)
    return max(stage_time(p, int(grp[s]), int(tp[s]), j, i), c)


def valid(p, S: int, S_max: int, grp, tp) -> bool:
    if not 1 <= S <= S_max:
        return False
    allowed = set(int(x) for x in p.tp_degrees)
    used, order = {}, []
    for s in range(S):
        g, d = int(grp[s]), int(tp[s])
        if not (0 <= g < p.G) or d not in allowed:
            return False
        if order and order[-1] != g and g in order:
            return False
        order.append(g)
        used[g] = used.get(g, 0) + d
        if used[g] > int(p.group_ndev[g]):
            return False
    return True


def partitions(n_items: int, n_parts: int):
    """All cut vectors (0, b_1, ..., n_items) with n_parts non-empty parts."""
    for mids in combinations(range(1, n_items), n_parts - 1):
        yield (0,) + mids + (n_items,)


def opt(p, S: int, grp, tp, s: int, i: int) -> int:
    """Smallest bottleneck of the first i operators on slots 0..s-1, by enumeration."""
    if s == 0:
        return 0 if i == 0 else INF
    if i < s:
        return INF
    best = INF
    for b in partitions(i, s):
        worst = 0
        for q in range(s):
            w = stage_cost(p, S, grp, tp, q, b[q], b[q + 1])
            worst = max(worst, w)
            if worst == INF:
                break
        best = min(best, worst)
    return best


def score(p, S: int, grp, tp, b):
    """(bottleneck, iteration time) of a feasible partition: sum(t + 2c) + (M - 1) bottleneck."""
    worst, single = 0, 0
    for s in range(S):
        t = stage_time(p, int(grp[s]), int(tp[s]), b[s], b[s + 1])
        c = 0 if s == S - 1 else cut_time(p, int(grp[s]), int(grp[s + 1]), b[s + 1])
        worst = max(worst, t, c)
        single += t + 2 * c
    return worst, single + (int(p.M) - 1) * worst


def plan(p, S: int, S_max: int, grp, tp):
    """Status, cut vector, bottleneck, iteration time of the reported plan.

    Reported plan: b_S = L; going down, b_s is the smallest j for which the best bottleneck of
    the first j operators on s slots, combined with stage s over [j, b_{s+1}), attains the best
    bottleneck of the first b_{s+1} operators on s+1 slots.
    """
    L = int(p.L)
    if not valid(p, S, S_max, grp, tp):
        return 2, None, INF, INF
    if S > L or opt(p, S, grp, tp, S, L) == INF:
        return 1, None, INF, INF
    b = [0] * (S + 1)
    b[S] = L
    for s in range(S - 1, -1, -1):
        target = opt(p, S, grp, tp, s + 1, b[s + 1])
        for j in range(s, b[s + 1]):
            left = opt(p, S, grp, tp, s, j)
            if left == INF:
                continue
            if max(left, stage_cost(p, S, grp, tp, s, j, b[s + 1])) == target:
                b[s] = j
                break
        else:
            raise AssertionError("no predecessor attains the optimum")
    bott, it = score(p, S, grp, tp, b)
    assert bott == opt(p, S, grp, tp, S, L)
    return 0, b, bott, it


def best_iteration_time(p, S: int, S_max: int, grp, tp):
    """Exhaustive optimum of eq. gpipe_cost_model over every feasible partition (T* of the
    candidate), with t_max taken as the partition's own max over stage and transfer times."""
    if not valid(p, S, S_max, grp, tp) or S > int(p.L):
        return INF
    best = INF
    for b in partitions(int(p.L), S):
        if any(stage_cost(p, S, grp, tp, s, b[s], b[s + 1]) == INF for s in range(S)):
            continue
        best = min(best, score(p, S, grp, tp, b)[1])
    return best


def _stage_terms(p, S, grp, tp, s, j, i):
    """(fits, stage time, transfer time) of stage s over [j, i)."""
    n = min(S - s, int(p.M))
    fits = memory_fits(p, int(grp[s]), int(tp[s]), n, j, i)
    t = stage_time(p, int(grp[s]), int(tp[s]), j, i)
    c = 0 if s == S - 1 else cut_time(p, int(grp[s]), int(grp[s + 1]), i)
    return fits, t, c


def opt_sum(p, S, grp, tp, s, i, cap):
    """Smallest sum of (t + 2c) over the first i operators on slots 0..s-1 with every stage
    fitting and every stage and transfer time at most cap, by enumeration."""
    if s == 0:
        return 0 if i == 0 else INF
    if i < s:
        return INF
    best = INF
    for b in partitions(i, s):
        total = 0
        for q in range(s):
            fits, t, c = _stage_terms(p, S, grp, tp, q, b[q], b[q + 1])
            if not fits or t > cap or c > cap:
                total = INF
                break
            total += t + 2 * c
        best = min(best, total)
    return best


def plan_exact(p, S: int, S_max: int, grp, tp):
    """Status, cuts, winning cap, optimum of the iteration-time model (section 5.2.2-5.2.4).

    The optimum is taken over every feasible partition; among the partitions attaining it the
    reported one has the smallest bottleneck b*, and under the cap b* the cuts are fixed from the
    back: b_s is the smallest j for which the best capped sum of the first j operators on s slots
    plus stage s over [j, b_{s+1}) attains the best capped sum of the first b_{s+1} operators."""
    L = int(p.L)
    if not valid(p, S, S_max, grp, tp):
        return 2, None, INF, INF
    best_T, best_b = INF, INF
    if S <= L:
        for b in partitions(L, S):
            if any(stage_cost(p, S, grp, tp, s, b[s], b[s + 1]) == INF for s in range(S)):
                continue
            bott, T = score(p, S, grp, tp, b)
            if T < best_T or (T == best_T and bott < best_b):
                best_T, best_b = T, bott
    if best_T == INF:
        return 1, None, INF, INF
    cap = best_b
    cuts = [0] * (S + 1)
    cuts[S] = L
    for s in range(S - 1, -1, -1):
        target = opt_sum(p, S, grp, tp, s + 1, cuts[s + 1], cap)
        for j in range(s, cuts[s + 1]):
            left = opt_sum(p, S, grp, tp, s, j, cap)
            fits, t, c = _stage_terms(p, S, grp, tp, s, j, cuts[s + 1])
            if left == INF or not fits or t > cap or c > cap:
                continue
            if left + t + 2 * c == target:
                cuts[s] = j
                break
        else:
            raise AssertionError("no predecessor attains the capped optimum")
    bott, T = score(p, S, grp, tp, cuts)
    assert T == best_T and bott == cap
    return 0, cuts, cap, best_T


# ---------------------------------------------------------------- H-1F1B warm-up counts

def h1f1b_delta(c: int, t_max: int) -> int:
    """Extra forward microbatches a stage launches over the next one (sections 4.1, 5.2.3):
    ceil(2c / t_max - 1/64) + 1 in integers, the 1/64 of t_max rounded down."""
    slack = t_max // 64
    if 2 * c <= slack:
        return 1
    return 1 + _cdiv(2 * c - slack, t_max)


def h1f1b_evaluate(p, S: int, grp, tp, b, t_max: int):
    """Warm-up counts of the partition b under the cap t_max by eq. Ni (1 + the deltas of all later
    cuts, never more than M), and the sum of (t + 2c); None when a stage or transfer time exceeds
    the cap or a stage does not fit with its count."""
    M = int(p.M)
    deltas = [h1f1b_delta(cut_time(p, int(grp[s]), int(grp[s + 1]), b[s + 1]), t_max) for s in range(S - 1)]
    total, counts = 0, []
    for s in range(S):
        n = min(M, 1 + sum(deltas[s:]))
        t = stage_time(p, int(grp[s]), int(tp[s]), b[s], b[s + 1])
        c = 0 if s == S - 1 else cut_time(p, int(grp[s]), int(grp[s + 1]), b[s + 1])
        if t > t_max or c > t_max or not memory_fits(p, int(grp[s]), int(tp[s]), n, b[s], b[s + 1]):
            return None
        counts.append(n)
        total += t + 2 * c
    return counts, total


def h1f1b_best_sum(p, S: int, grp, tp, t_max: int) -> int:
    """Least sum of (t + 2c) over ALL partitions that are feasible under H-1F1B with the cap t_max,
    by enumeration: a lower bound for the recurrence, which keeps only the least-sum continuation
    of every state and may therefore miss a plan whose tail is costlier but needs fewer warm-up
    launches."""
    best = INF
    if S <= int(p.L):
        for b in partitions(int(p.L), S):
            r = h1f1b_evaluate(p, S, grp, tp, b, t_max)
            if r is not None:
                best = min(best, r[1])
    return best


def plan_h1f1b(p, S: int, S_max: int, grp, tp, t_max: int):
    """The capped suffix recurrence with the warm-up count carried by the least-sum continuation
    (eq. dp_general, eq. dp_ni), written as a memoised recursion over (first operator, first slot):
    returns (status, cuts, counts, least sum)."""
    L, M = int(p.L), int(p.M)
    if not valid(p, S, S_max, grp, tp):
        return 2, None, None, INF
    if S > L or t_max < 0:
        return 1, None, None, INF
    memo = {}

    def state(i: int, slot: int):
        """(least sum, count of the first stage, its end cut) for operators i.. on slots slot.."""
        if slot == S:
            return (0, 0, -1) if i == L else (INF, 0, -1)
        key = (i, slot)
        if key in memo:
            return memo[key]
        g, d = int(grp[slot]), int(tp[slot])
        best = (INF, 0, -1)
        for j in range(i + 1, L - (S - slot - 1) + 1):
            rest, n_next, _ = state(j, slot + 1)
            if rest == INF:
                continue
            c = 0 if slot == S - 1 else cut_time(p, g, int(grp[slot + 1]), j)
            t = stage_time(p, g, d, i, j)
            if c > t_max or t > t_max:
                continue
            n = min(M, h1f1b_delta(c, t_max) + n_next)
            if not memory_fits(p, g, d, n, i, j):
                continue
            if rest + t + 2 * c < best[0]:
                best = (rest + t + 2 * c, n, j)
        memo[key] = best
        return best

    total = state(0, 0)[0]
    if total == INF:
        return 1, None, None, INF
    cuts, counts, i = [0], [], 0
    for slot in range(S):
        _, n, j = state(i, slot)
        counts.append(n)
        cuts.append(j)
        i = j
    return 0, cuts, counts, total


# ---------------------------------------------------------------- submesh choice inside the recurrence

def slicings(p, groups, S: int):
    """Every way to cut the devices of the ordered groups into S stages: each group's devices are
    split into an ordered sequence of allowed degrees that uses all of them.  Yields slot lists
    [(group, degree), ...] of length S."""
    degrees = [int(x) for x in p.tp_degrees]

    def compositions(n):
        if n == 0:
            yield ()
            return
        for d in degrees:
            if d <= n:
                for rest in compositions(n - d):
                    yield (d,) + rest

    def rec(k, left):
        if k == len(groups):
            if left == 0:
                yield []
            return
        g = int(groups[k])
        for comp in compositions(int(p.group_ndev[g])):
            if len(comp) <= left - (len(groups) - k - 1):
                for tail in rec(k + 1, left - len(comp)):
                    yield [(g, d) for d in comp] + tail

    yield from rec(0, S)


def mesh_valid(p, S: int, S_max: int, groups) -> bool:
    groups = [int(g) for g in groups]
    return 1 <= S <= S_max and len(groups) >= 1 and len(set(groups)) == len(groups) and \
        all(0 <= g < int(p.G) for g in groups)


def mesh_best_bottleneck(p, S: int, groups) -> int:
    """Smallest bottleneck over EVERY slicing of the ordered groups into S stages and every
    partition of the operators, by enumeration (INF when none is feasible)."""
    L = int(p.L)
    best = INF
    if S <= L:
        for slots in slicings(p, groups, S):
            grp = [g for g, _ in slots]
            tp = [d for _, d in slots]
            for b in partitions(L, S):
                w = 0
                for s in range(S):
                    w = max(w, stage_cost(p, S, grp, tp, s, b[s], b[s + 1]))
                    if w >= best:
                        break
                best = min(best, w)
    return best


def plan_mesh(p, S: int, S_max: int, groups):
    """The recurrence over (stages, operators, devices used) as a memoised recursion: returns
    (status, bottleneck, cuts, slot list).  state(s, i, d) = best value with the first s stages on the
    first i operators and the first d devices; ties: lowest previous cut, then smallest degree."""
    L, M = int(p.L), int(p.M)
    if not mesh_valid(p, S, S_max, groups):
        return 2, INF, None, None
    groups = [int(g) for g in groups]
    bounds = [0]
    for g in groups:
        bounds.append(bounds[-1] + int(p.group_ndev[g]))
    total = bounds[-1]
    degrees = [int(x) for x in p.tp_degrees]
    if S > L or S < len(groups) or S > total:
        return 1, INF, None, None
    memo = {}

    def group_at(d):
        return max(k for k in range(len(groups)) if bounds[k] <= d)

    def state(s, i, d):
        if s == 0:
            return (0, -1, -1) if (i == 0 and d == 0) else (INF, -1, -1)
        key = (s, i, d)
        if key in memo:
            return memo[key]
        best = (INF, -1, -1)
        last = s == S
        n = min(S - (s - 1), M)
        for q, deg in enumerate(degrees):
            d0 = d - deg
            if d0 < 0:
                continue
            k = group_at(d0)
            if d > bounds[k + 1] or (d == total) != last:
                continue
            g = groups[k]
            g_next = g if (last or d < bounds[k + 1]) else groups[k + 1]
            c = 0 if last else cut_time(p, g, g_next, i)
            for j in range(s - 1, i):
                prev = state(s - 1, j, d0)[0]
                if prev == INF or not memory_fits(p, g, deg, n, j, i):
                    continue
                val = max(prev, stage_time(p, g, deg, j, i), c)
                if (val, j, q) < best:
                    best = (val, j, q)
        memo[key] = best
        return best

    value = state(S, L, total)[0]
    if value == INF:
        return 1, INF, None, None
    cuts, slots = [L], []
    i, d = L, total
    for s in range(S, 0, -1):
        _, j, q = state(s, i, d)
        d -= degrees[q]
        slots.append((groups[group_at(d)], degrees[q]))
        cuts.append(j)
        i = j
    return 0, value, cuts[::-1], slots[::-1]


def mesh_best_iteration_time(p, S: int, groups):
    """(T*, bottleneck) of the best plan over EVERY slicing of the ordered groups into S stages and
    every partition, by enumeration; among equal iteration times the smaller bottleneck."""
    L = int(p.L)
    best = (INF, INF)
    if S <= L:
        for slots in slicings(p, groups, S):
            grp = [g for g, _ in slots]
            tp = [d for _, d in slots]
            for b in partitions(L, S):
                if any(stage_cost(p, S, grp, tp, s, b[s], b[s + 1]) == INF for s in range(S)):
                    continue
                bott, T = score(p, S, grp, tp, b)
                best = min(best, (T, bott))
    return best


def plan_mesh_capped(p, S: int, groups, cap: int):
    """Least sum of (t + 2c) with every stage and transfer time at most cap, over slicings and
    partitions, as a memoised recursion over (stages, operators, devices); ties: lowest previous
    cut, then smallest degree.  Returns (sum, cuts, slot list) or (INF, None, None)."""
    L, M = int(p.L), int(p.M)
    groups = [int(g) for g in groups]
    bounds = [0]
    for g in groups:
        bounds.append(bounds[-1] + int(p.group_ndev[g]))
    total = bounds[-1]
    degrees = [int(x) for x in p.tp_degrees]
    memo = {}

    def group_at(d):
        return max(k for k in range(len(groups)) if bounds[k] <= d)

    def state(s, i, d):
        if s == 0:
            return (0, -1, -1) if (i == 0 and d == 0) else (INF, -1, -1)
        key = (s, i, d)
        if key in memo:
            return memo[key]
        best = (INF, -1, -1)
        last = s == S
        n = min(S - (s - 1), M)
        for q, deg in enumerate(degrees):
            d0 = d - deg
            if d0 < 0:
                continue
            k = group_at(d0)
            if d > bounds[k + 1] or (d == total) != last:
                continue
            g = groups[k]
            g_next = g if (last or d < bounds[k + 1]) else groups[k + 1]
            c = 0 if last else cut_time(p, g, g_next, i)
            if c > cap:
                continue
            for j in range(s - 1, i):
                prev = state(s - 1, j, d0)[0]
                t = stage_time(p, g, deg, j, i)
                if prev == INF or t > cap or not memory_fits(p, g, deg, n, j, i):
                    continue
                if (prev + t + 2 * c, j, q) < best:
                    best = (prev + t + 2 * c, j, q)
        memo[key] = best
        return best

    if S > L or S < len(groups) or S > total:
        return INF, None, None
    value = state(S, L, total)[0]
    if value == INF:
        return INF, None, None
    cuts, slots = [L], []
    i, d = L, total
    for s in range(S, 0, -1):
        _, j, q = state(s, i, d)
        d -= degrees[q]
        slots.append((groups[group_at(d)], degrees[q]))
        cuts.append(j)
        i = j
    return value, cuts[::-1], slots[::-1]


def plan_mesh_h1f1b(p, S: int, S_max: int, groups, t_max: int):
    """The full recurrence of section 5.2.3 for one cap (device index and H-1F1B count in the
    state, suffix direction) as a memoised recursion: (status, cuts, slot list, counts, least sum).
    state(i, slot, d) = the stages from `slot` on start at operator i and at device offset d."""
    L, M = int(p.L), int(p.M)
    if not mesh_valid(p, S, S_max, groups):
        return 2, None, None, None, INF
    groups = [int(g) for g in groups]
    bounds = [0]
    for g in groups:
        bounds.append(bounds[-1] + int(p.group_ndev[g]))
    total = bounds[-1]
    degrees = [int(x) for x in p.tp_degrees]
    if S > L or S < len(groups) or S > total or t_max < 0:
        return 1, None, None, None, INF
    memo = {}

    def group_at(d):
        return max(k for k in range(len(groups)) if bounds[k] <= d)

    def state(i, slot, d):
        if slot == S:
            return (0, 0, -1, -1) if (i == L and d == total) else (INF, 0, -1, -1)
        key = (i, slot, d)
        if key in memo:
            return memo[key]
        best = (INF, 0, -1, -1)
        if d < total:
            k = group_at(d)
            g = groups[k]
            last = slot == S - 1
            for j in range(i + 1, L - (S - slot - 1) + 1):
                for q, deg in enumerate(degrees):
                    d2 = d + deg
                    if d2 > bounds[k + 1] or (d2 == total) != last:
                        continue
                    rest, n_next, _, _ = state(j, slot + 1, d2)
                    if rest == INF:
                        continue
                    g_next = g if (last or d2 < bounds[k + 1]) else groups[k + 1]
                    c = 0 if last else cut_time(p, g, g_next, j)
                    t = stage_time(p, g, deg, i, j)
                    if c > t_max or t > t_max:
                        continue
                    n = min(M, h1f1b_delta(c, t_max) + n_next)
                    if not memory_fits(p, g, deg, n, i, j):
                        continue
                    if (rest + t + 2 * c, j, q) < (best[0], best[2] if best[2] >= 0 else INF, best[3]):
                        best = (rest + t + 2 * c, n, j, q)
        memo[key] = best
        return best

    total_sum = state(0, 0, 0)[0]
    if total_sum == INF:
        return 1, None, None, None, INF
    cuts, slots, counts, i, d = [0], [], [], 0, 0
    for slot in range(S):
        _, n, j, q = state(i, slot, d)
        slots.append((groups[group_at(d)], degrees[q]))
        counts.append(n)
        cuts.append(j)
        i, d = j, d + degrees[q]
    return 0, cuts, slots, counts, total_sum


def mesh_cap_values(p, groups):
    """Candidate caps of an ordering (section 5.2.4 (2)): every stage time of every listed group,
    usable degree and operator range, and every transfer time of an inner cut on the links the
    ordering can use (inside a group, and to the group after it).  Sorted, distinct."""
    L = int(p.L)
    groups = [int(g) for g in groups]
    values = set()
    for k, g in enumerate(groups):
        for deg in (int(x) for x in p.tp_degrees):
            if deg <= int(p.group_ndev[g]):
                values.update(stage_time(p, g, deg, j, i) for j in range(L) for i in range(j + 1, L + 1))
        links = [g] + ([groups[k + 1]] if k + 1 < len(groups) else [])
        values.update(cut_time(p, g, h, i) for h in links for i in range(1, L))
    return sorted(values)


def sweep_mesh_h1f1b(p, S: int, S_max: int, groups, max_caps: int = 1 << 20):
    """The search around the full recurrence, twin of the oracle's: caps in increasing order from
    the classic min-max bottleneck; the first cap with a plan fixes t_E = ceil(T / M); smallest
    T = least sum + (M - 1) cap wins, the lower cap on ties.
    Returns (status, cap, cuts, slot list, counts, T, caps tried)."""
    status, t_S, _, _ = plan_mesh(p, S, S_max, groups)
    if status != 0:
        return status, INF, None, None, None, INF, 0
    M = int(p.M)
    best = (1, INF, None, None, None, INF)
    t_E, tried = INF, 0
    for cap in mesh_cap_values(p, groups):
        if cap < t_S:
            continue
        if cap > t_E or tried >= max_caps:
            break
        tried += 1
        st, cuts, slots, counts, total = plan_mesh_h1f1b(p, S, S_max, groups, cap)
        if st != 0:
            continue
        T = total + (M - 1) * cap
        if t_E == INF:
            t_E = _cdiv(T, M)
        if T < best[5]:
            best = (0, cap, cuts, slots, counts, T)
    return best + (tried,)


def cap_values(p, S: int, grp, tp):
    """Candidate caps of a candidate (fixed slicing): the stage times of its slots over every
    operator range, and the transfer times of the inner cuts on the links between consecutive slots."""
    L = int(p.L)
    values = set()
    for s in range(S):
        g, d = int(grp[s]), int(tp[s])
        values.update(stage_time(p, g, d, j, i) for j in range(L) for i in range(j + 1, L + 1))
        if s + 1 < S:
            values.update(cut_time(p, g, int(grp[s + 1]), i) for i in range(1, L))
    return sorted(values)


def sweep_h1f1b(p, S: int, S_max: int, grp, tp, max_caps: int = 1 << 20):
    """The search around the capped H-1F1B recurrence for one candidate, twin of the oracle's.
    Returns (status, cap, cuts, counts, T, caps tried)."""
    status, _, t_S, _ = plan(p, S, S_max, grp, tp)
    if status != 0:
        return status, INF, None, None, INF, 0
    M = int(p.M)
    best = (1, INF, None, None, INF)
    t_E, tried = INF, 0
    for cap in cap_values(p, S, grp, tp):
        if cap < t_S:
            continue
        if cap > t_E or tried >= max_caps:
            break
        tried += 1
        st, cuts, counts, total = plan_h1f1b(p, S, S_max, grp, tp, cap)
        if st != 0:
            continue
        T = total + (M - 1) * cap
        if t_E == INF:
            t_E = _cdiv(T, M)
        if T < best[4]:
            best = (0, cap, cuts, counts, T)
    return best + (tried,)


def subcluster_order(p):
    """Order of the subclusters by the heuristic of section 5.2.1, as a check of the product's
    pre-filter: a group goes before another when its devices have more memory per unit of compute
    throughput, throughput of a GPU type = 1 / (its forward+backward time over the whole model);
    equal ratios keep the lower group id first.  Written as the definition: exact fractions, and a
    selection that asks, for every position, which remaining group no other remaining group beats."""
    from fractions import Fraction

    def ratio(g):
        t = int(p.group_type[g])
        time = sum(int(x) for x in p.fwd_us[t]) + sum(int(x) for x in p.bwd_us[t])
        if time == 0:
            return Fraction(0)                       # infinite throughput: no memory per unit of it
        return Fraction(int(p.type_mem_bytes[t])) / Fraction(1, time)

    left = list(range(p.G))
    out = []
    while left:
        pick = next(g for g in left
                    if all(ratio(g) > ratio(h) or (ratio(g) == ratio(h) and g <= h) for h in left))
        out.append(pick)
        left.remove(pick)
    return out
