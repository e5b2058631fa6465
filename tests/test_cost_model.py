"""Cost-model arithmetic (Eq. 1, Eq. 4, Eq. 5): pins of the Python oracle, then the library's
C entry points against it.  CPU only."""
import os
import random
from fractions import Fraction

import pytest

import paper_2512_20953_amd as P
from oracle import cost_ref as CR

GOLD = os.path.join(os.path.dirname(__file__), "golden", "toy_pipeline_idle.txt")


def _gold():
    vals = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = v
    return vals


# ---------------------------------------------------------------- oracle pins
def test_oracle_reproduces_the_papers_toy_idle_shares():
    g = _gold()
    t = [float(x) for x in g["stage_times"]]
    idle, mean = CR.idle_fractions(t, int(g["K"][0]))
    assert abs(idle[0] - float(Fraction(g["idle_a100"][0]))) < 1e-15 and abs(idle[1] - idle[0]) < 1e-15
    assert abs(idle[2] - float(Fraction(g["idle_h800"][0]))) < 1e-15 and abs(idle[3] - idle[2]) < 1e-15
    assert abs(mean - float(Fraction(g["idle_overall"][0]))) < 1e-15


def test_oracle_equal_stages_give_the_textbook_pipeline_time():
    # P equal stages, K micro-batches: (P + K - 1) * t; one stage: K * t; one micro-batch: sum
    assert CR.pipeline_time([3.0] * 4, 8) == (4 + 8 - 1) * 3.0
    assert CR.pipeline_time([5.0], 7) == 35.0
    assert CR.pipeline_time([1.0, 2.0, 4.0], 1) == 7.0
    # the slowest stage paces the steady state, wherever it sits
    assert CR.pipeline_time([1.0, 4.0, 2.0], 5) == 7.0 + 4 * 4.0
    assert CR.iteration_time([[1.0, 1.0], [3.0]], 4, 0.5) == max(2 + 3 * 1, 3 + 3 * 3) + 0.5


def test_oracle_binary_decomposition():
    t = [1.0, 1.9, 3.7, 7.2]
    assert CR.layers_time(8, t) == 7.2 and CR.layers_time(1, t) == 1.0
    assert CR.layers_time(10, t) == 7.2 + 1.9
    assert CR.layers_time(7, t) == 1.0 + 1.9 + 3.7
    # exactly additive layers reproduce n * t(1)
    assert CR.layers_time(13, [2.0, 4.0, 8.0, 16.0]) == 26.0


def test_oracle_partition_small_cases():
    # two GPUs, the second twice as fast, no memory limit: 12 layers split 4 / 8
    best, sols = CR.partition_layers(12, [2.0, 1.0], [1e9, 1e9], 1.0, 0.0, [1, 1])
    assert best == 8.0 and sols == {(4, 8)}
    # a memory cap on the fast GPU pushes layers back to the slow one
    best, sols = CR.partition_layers(12, [2.0, 1.0], [1e9, 6.0], 1.0, 0.0, [1, 1])
    assert best == 12.0 and sols == {(6, 6)}
    # activations of earlier stages count once per in-flight micro-batch
    best, sols = CR.partition_layers(6, [1.0, 1.0], [8.0, 8.0], 1.0, 1.0, [3, 1])
    assert sols == {(2, 4)} and best == 4.0
    assert CR.partition_layers(6, [1.0, 1.0], [2.0, 2.0], 1.0, 0.0, [1, 1]) == (None, set())


# ---------------------------------------------------------------- library vs oracle
def test_library_matches_oracle_on_the_toy_example():
    g = _gold()
    t = [float(x) for x in g["stage_times"]]
    idle, mean = P.cost_idle_fractions(t, 1)
    ref_idle, ref_mean = CR.idle_fractions(t, 1)
    assert idle == ref_idle and mean == ref_mean
    assert P.cost_pipeline_time(t, 1) == 6.0


def test_library_matches_oracle_on_random_pipelines():
    rng = random.Random(20953)
    for _ in range(200):
        groups = [[rng.uniform(0.1, 9.0) for _ in range(rng.randint(1, 6))] for _ in range(rng.randint(1, 4))]
        K, ts = rng.randint(1, 32), rng.uniform(0, 3)
        assert P.cost_iteration_time(groups, K, ts) == pytest.approx(CR.iteration_time(groups, K, ts), rel=1e-14)
        for g in groups:
            assert P.cost_pipeline_time(g, K) == pytest.approx(CR.pipeline_time(g, K), rel=1e-14)
            idle, mean = P.cost_idle_fractions(g, K)
            ridle, rmean = CR.idle_fractions(g, K)
            assert idle == pytest.approx(ridle, abs=1e-14) and mean == pytest.approx(rmean, abs=1e-14)
        t = [rng.uniform(0.5, 2.0) * (1 << i) for i in range(6)]
        n = rng.randint(1, 63)
        assert P.cost_layers_time(n, t) == pytest.approx(CR.layers_time(n, t), rel=1e-14)


def test_library_partition_is_optimal_and_valid():
    rng = random.Random(7)
    for case in range(300):
        Pn = rng.randint(1, 4)
        N = rng.randint(Pn, 12)
        t = [rng.choice([0.5, 1.0, 1.5, 2.0, 3.0]) for _ in range(Pn)]
        fixed, act = rng.choice([0.0, 1.0, 2.0]), rng.choice([0.0, 0.5, 1.0])
        infl = [Pn - i for i in range(Pn)]
        mem = [rng.choice([4.0, 8.0, 16.0, 1e9]) for _ in range(Pn)]
        best, sols = CR.partition_layers(N, t, mem, fixed, act, infl)
        if best is None:
            with pytest.raises(P.AhError) as e:
                P.cost_partition_layers(N, t, mem, fixed, act, infl)
            assert e.value.status == 5
            continue
        l, worst = P.cost_partition_layers(N, t, mem, fixed, act, infl)
        assert worst == best, (case, l, worst, best)
        assert tuple(l) in sols
        assert sum(l) == N and min(l) >= 1


def test_library_refuses_bad_arguments():
    with pytest.raises(P.AhError):
        P.cost_layers_time(9, [1.0, 2.0, 4.0])        # 9 needs the 8-layer profile
    with pytest.raises(P.AhError):
        P.cost_pipeline_time([1.0, -1.0], 2)
    with pytest.raises(P.AhError):
        P.cost_partition_layers(2, [1.0, 1.0, 1.0], [1e9] * 3, 0, 0, [1, 1, 1])   # fewer layers than stages
