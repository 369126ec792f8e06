"""Pins of the cost model itself: the DAG pipeline simulator (section 4.2.1) against the closed
forms the paper proves (Lemma 1, Lemma 2, eq. result2h), the case study of section 2.3, and the
warm-up counts the H-1F1B oracle emits."""
import math

import numpy as np

import oracle
from oracle import dag_sim

from helpers import cands_from_lists, simple_problem


def test_lemma_1_and_2_two_balanced_stages():
    f, b, B = 30, 70, 40
    for c in (0, 1, 10, 49, 50, 51, 99, 100):
        for K in (2, 3, 4, 5):
            T, start = dag_sim.simulate([f, f], [b, b], [c], B, [K, 1])
            for i in (12, 20, 27):                      # microbatches well inside the steady phase
                # Lemma 1: backward of a microbatch after its forward, local path vs round trip
                assert start[("B", i, 0)] - start[("F", i, 0)] == max(K * f + (K - 1) * b, 2 * f + b + 2 * c)
                # Lemma 2: one K-block
                assert start[("F", i + K, 0)] - start[("F", i, 0)] == max(K * (f + b), 2 * (f + b + c))


def test_smallest_bubble_free_warmup_is_eq_result2h():
    f, b, B = 40, 60, 64
    for c in (0, 3, 25, 50, 51, 75, 100):
        delta = math.ceil(1 + 2 * c / (f + b))          # eq. result2h
        model = dag_sim.cost_model([f, f], [b, b], [c], B)
        assert model == (B + 1) * (f + b) + 2 * c
        # with that many extra launches the pipeline reaches the cost model exactly ...
        assert dag_sim.simulate([f, f], [b, b], [c], B, [1 + delta, 1])[0] == model
        # ... and with one fewer it does not, unless no transfer has to be hidden at all
        if delta > 1:
            T_less = dag_sim.simulate([f, f], [b, b], [c], B, [delta, 1])[0]
            assert T_less > model or c == 0


def test_case_study_counts():
    # three balanced stages, slow first link (between half a stage time and a full one), fast
    # second link: the tailored {5, 2, 1} hides everything; Eager-1F1B's {5, 3, 1} and the classic
    # {3, 2, 1} leave bubbles (section 2.3)
    f, b, c, B = [100] * 3, [200] * 3, [250, 0], 24
    model = dag_sim.cost_model(f, b, c, B)
    assert dag_sim.simulate(f, b, c, B, [5, 2, 1])[0] == model
    assert dag_sim.simulate(f, b, c, B, [5, 3, 1])[0] > model
    assert dag_sim.simulate(f, b, c, B, [3, 2, 1])[0] > dag_sim.simulate(f, b, c, B, [5, 3, 1])[0]


def test_counts_of_the_h1f1b_oracle_reach_the_cost_model():
    """The warm-up counts the oracle derives (eq. Ni with the integer delta) fed to the simulator:
    on balanced chains the simulated latency is the iteration time the oracle reports, while the
    classic counts are slower whenever a transfer has to be hidden."""
    rng = np.random.default_rng(3)
    hidden = 0
    for case in range(60):
        S = int(rng.integers(2, 5))
        fwd = int(rng.integers(20, 200))
        t = 3 * fwd                                       # forward + backward = fwd + 2 fwd
        # transfers outside the 1/64 slack bands, where the integer delta equals ceil(1 + 2c/t)
        cuts = [int(rng.choice([0, rng.integers(t // 60 + 1, t // 2 + 1), rng.integers(t // 2 + t // 60 + 1, t + 1)]))
                for _ in range(S - 1)]
        M = int(rng.integers(4 * S + 8, 48))
        p = simple_problem(np.zeros(S), M=M, G=S, ndev=(1,) * S, fwd=np.full((1, S), fwd),
                           bwd=np.full((1, S), 2 * fwd), act=cuts + [0], bw=np.ones((S, S), dtype=np.int64))
        cands = cands_from_lists([[(g, 1) for g in range(S)]])
        out = oracle.plan_h1f1b_batch(oracle.build_tables(p), cands, [t])
        assert out.status[0] == oracle.OK
        counts = [int(x) for x in out.warmup[0, :S]]
        assert counts == [1 + sum(math.ceil(1 + 2 * c / t) for c in cuts[s:]) for s in range(S)]
        f, b = [fwd] * S, [2 * fwd] * S
        T_h = dag_sim.simulate(f, b, cuts, M, counts)[0]
        T_classic = dag_sim.simulate(f, b, cuts, M, list(range(S, 0, -1)))[0]
        assert T_h <= T_classic
        if S == 2:
            assert T_h == out.iter_time[0] == dag_sim.cost_model(f, b, cuts, M)
        if any(c > 0 for c in cuts):
            hidden += T_classic > T_h
    assert hidden > 20


def test_order_and_deadlock():
    assert dag_sim.stage_order(4, 2) == [("F", 0), ("F", 1), ("B", 0), ("F", 2), ("B", 1), ("F", 3), ("B", 2), ("B", 3)]
    # a first stage that waits for a backward before the second stage could have seen any forward
    try:
        dag_sim.simulate([1, 1], [1, 1], [0], 4, [0, 1])
    except ValueError:
        pass
    else:
        raise AssertionError("a schedule that starts with a backward cannot run")


def _counts_without_slack(c, t_max):
    """eq. Ni with eq. result2h's delta = ceil(1 + 2c / t_max) per link (no eps band)."""
    n = [1] * (len(c) + 1)
    for s in range(len(c) - 1, -1, -1):
        n[s] = n[s + 1] + (1 if c[s] == 0 else 1 + -(-2 * c[s] // t_max))
    return n


def test_cost_model_against_the_simulated_pipeline():
    """How far eq. gpipe_cost_model is from the simulated schedule, recorded as assertions.

    Equality holds for balanced stages without transfers (any number of stages, classic counts) and,
    with transfers, for two balanced stages with eq. result2h's warm-up (tested above).  Otherwise the
    model is neither an upper nor a lower bound.  On 3,000 seeded random unbalanced pipelines with
    H-1F1B counts the simulation is slower than the model in 7% of the cases, by at most 14.2% and
    never by more than (S - 1) t_max (one bottleneck time of bubble per link); faster in 64%, by at
    most 15.5% (stages shorter than the bottleneck overlap their neighbours' work, which the sum of
    all stage times in the model does not credit); and never below max(B t_max, one microbatch end
    to end).  Without transfers and with the classic counts the simulation never exceeds the model."""
    import random
    rnd = random.Random(7)
    for _ in range(300):
        S, B, f0 = rnd.randint(2, 8), rnd.randint(1, 50), rnd.randint(1, 100)
        f, b, c = [f0] * S, [2 * f0] * S, [0] * (S - 1)
        assert dag_sim.simulate(f, b, c, B, list(range(S, 0, -1)))[0] == dag_sim.cost_model(f, b, c, B)
    for _ in range(600):
        S = rnd.randint(2, 6)
        B = rnd.randint(S + 8, 40)
        f = [rnd.randint(5, 100) for _ in range(S)]
        b = [2 * x for x in f]
        c = [0] * (S - 1)
        assert dag_sim.simulate(f, b, c, B, list(range(S, 0, -1)))[0] <= dag_sim.cost_model(f, b, c, B)
    rnd = random.Random(1)
    above = below = 0
    worst_above = worst_below = 0.0
    for _ in range(3000):
        S = rnd.randint(2, 6)
        B = rnd.randint(S + 8, 40)
        f = [rnd.randint(5, 100) for _ in range(S)]
        b = [2 * x for x in f]
        t_max = max(x + y for x, y in zip(f, b))
        c = [rnd.choice([0, rnd.randint(0, t_max // 60), rnd.randint(0, t_max // 2), rnd.randint(0, t_max)])
             for _ in range(S - 1)]
        model = dag_sim.cost_model(f, b, c, B)
        T = dag_sim.simulate(f, b, c, B, _counts_without_slack(c, t_max))[0]
        assert T - model <= (S - 1) * t_max
        assert T >= max(B * t_max, sum(f) + sum(b) + 2 * sum(c))
        above += T > model
        below += T < model
        worst_above = max(worst_above, (T - model) / model)
        worst_below = max(worst_below, (model - T) / model)
    assert (above, below) == (221, 1922)
    assert 0.141 < worst_above < 0.142 and 0.154 < worst_below < 0.155


def test_subcluster_order_heuristic():
    """Section 5.2.1: subclusters with more memory per unit of compute go first.  The product's
    pre-filter against the twin in oracle/brute.py, which states the rule with exact fractions."""
    from oracle import brute
    from paper_2509_24859_amd import ordering, workloads as W
    # three types: (memory, relative time per operator); ratio memory x time: 80, 96, 72
    p = simple_problem(np.zeros(4), T=3, G=5, ndev=(2,) * 5, gtype=[0, 1, 2, 1, 0],
                       fwd=np.array([[10] * 4, [24] * 4, [30] * 4]), bwd=np.zeros((3, 4), dtype=np.int64),
                       mem=[80, 40, 24])
    assert list(ordering.memory_to_compute_order(p)) == [1, 3, 0, 4, 2] == brute.subcluster_order(p)
    # keys that differ by one part in 2^60: equal once rounded to a double, ordered as integers
    a = 1 << 30
    p = simple_problem(np.zeros(1), T=3, G=3, ndev=(1,) * 3, gtype=[0, 1, 2],
                       fwd=np.array([[a], [a - 1], [a]]), bwd=np.zeros((3, 1), dtype=np.int64),
                       mem=[a, a + 1, a])
    assert float(a) * float(a) == float(a + 1) * float(a - 1)
    assert list(ordering.memory_to_compute_order(p)) == [0, 2, 1] == brute.subcluster_order(p)
    for name in W.ORDER:
        w = W.make(name)
        assert list(ordering.memory_to_compute_order(w.problem)) == brute.subcluster_order(w.problem)
    for seed in range(200):
        w = W.random_small(seed)
        assert list(ordering.memory_to_compute_order(w.problem)) == brute.subcluster_order(w.problem), seed
