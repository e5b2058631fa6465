"""Plain Python definition of the paper's cost-model arithmetic (test infrastructure only).

Eq. 1 (Section III-A): iteration time under 1F1B = max over DP groups of
(sum of stage times + (K - 1) * slowest stage) + T_sync.
Eq. 5 (Section III-D): time of n layers = sum of the profiled power-of-two blocks of n.
Eq. 4 (Section III-C): layer partition; its printed objective g_i / l_i is read as balancing
time, max_i l_i * t_i with t_i the per-layer time of stage i's GPU (1 / computing power), under
the memory constraint (4c).  The partition is found by exhaustive enumeration.

Pins (tests/test_cost_model.py): the idle shares of the paper's toy pipeline (Section II-D:
75 %, 2/3, 5/6), the textbook (P + K - 1) * t for equal stages, powers of two in Eq. 5.
"""
import itertools

__all__ = ["layers_time", "pipeline_time", "iteration_time", "idle_fractions", "partition_layers"]


def layers_time(n, t_pow2):
    total, i = 0.0, 0
    while n:
        if n & 1:
            total += t_pow2[i]
        n >>= 1
        i += 1
    return total


def pipeline_time(t_stage, K):
    return sum(t_stage) + (K - 1) * max(t_stage)


def iteration_time(groups, K, t_sync):
    return max(pipeline_time(g, K) for g in groups) + t_sync


def idle_fractions(t_stage, K):
    total = pipeline_time(t_stage, K)
    idle = [1.0 - K * t / total for t in t_stage]
    return idle, sum(idle) / len(idle)


def partition_layers(n_layers, t_layer, mem_bytes, fixed_per_layer, act_per_layer, in_flight):
    """Exhaustive search.  Returns (best bottleneck, set of all optimal assignments) or (None, set())."""
    P = len(t_layer)
    best, argbest = None, set()
    for cuts in itertools.combinations(range(1, n_layers), P - 1):
        l = [b - a for a, b in zip((0,) + cuts, cuts + (n_layers,))]
        if any(li * (fixed_per_layer + act_per_layer * f) > m for li, f, m in zip(l, in_flight, mem_bytes)):
            continue
        worst = max(li * ti for li, ti in zip(l, t_layer))
        if best is None or worst < best:
            best, argbest = worst, {tuple(l)}
        elif worst == best:
            argbest.add(tuple(l))
    return best, argbest
