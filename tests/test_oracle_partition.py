"""Pins for the partitioner oracle (Section 3.2): exhaustive enumeration on small problems, special cases with a
closed form, a hand-worked example, and NOAM for the configurations of Table 1."""
import itertools
import math

import numpy as np
import pytest

from oracle.partition import StageAssign, noam_of, partition, pipeline_time, stage_time, sync_time


def _compositions(total, parts):
    """All ways to write ``total`` as an ordered sum of ``parts`` positive integers."""
    for cuts in itertools.combinations(range(1, total), parts - 1):
        yield [b - a for a, b in zip((0,) + cuts, cuts + (total,))]


def _cost_by_definition(T, a, w, layer_counts, machine_counts, bw):
    """Slowest element of one concrete pipeline, written out from the problem statement (not via the oracle)."""
    worst, first = 0.0, 0
    for k, (nl, m) in enumerate(zip(layer_counts, machine_counts)):
        layers = range(first, first + nl)
        compute = sum(T[l] for l in layers)
        sync = sum(4.0 * (m - 1) * w[l] / m / bw for l in layers)
        worst = max(worst, max(compute, sync) / m)
        first += nl
        if k + 1 < len(layer_counts):
            worst = max(worst, 2.0 * a[first - 1] / bw)
    return worst


def _brute_force(T, a, w, M, bw):
    N = len(T)
    best = math.inf
    for k in range(1, min(N, M) + 1):
        for lc in _compositions(N, k):
            for mc in _compositions(M, k):
                best = min(best, _cost_by_definition(T, a, w, lc, mc, bw))
    return best


def _check_feasible(stages, N, M):
    assert stages[0].first == 0 and stages[-1].last == N - 1
    for p, q in zip(stages, stages[1:]):
        assert q.first == p.last + 1
    assert all(s.first <= s.last and s.replicas >= 1 for s in stages)
    assert sum(s.replicas for s in stages) == M


@pytest.mark.parametrize("seed", range(12))
def test_dp_equals_exhaustive_enumeration(seed):
    rng = np.random.default_rng(100 + seed)
    for N in range(1, 7):
        for M in range(1, 7):
            T = rng.uniform(0.5, 4.0, N).tolist()
            # mix the regimes: cheap / expensive boundaries, cheap / expensive synchronisation
            a = (rng.uniform(0.0, 1.0, N) * rng.choice([0.1, 1.0, 10.0])).tolist()
            w = (rng.uniform(0.0, 1.0, N) * rng.choice([0.0, 1.0, 20.0])).tolist()
            bw = float(rng.choice([0.5, 1.0, 8.0]))
            best, stages, noam = partition(T, a, w, M, bw)
            ref = _brute_force(T, a, w, M, bw)
            assert best == pytest.approx(ref, rel=1e-12, abs=0), (N, M)
            _check_feasible(stages, N, M)
            assert pipeline_time(T, a, w, stages, bw) == pytest.approx(best, rel=1e-12)
            lc = [s.last - s.first + 1 for s in stages]
            mc = [s.replicas for s in stages]
            assert _cost_by_definition(T, a, w, lc, mc, bw) == pytest.approx(ref, rel=1e-12)
            assert noam == math.ceil(M / stages[0].replicas)


def test_one_machine_is_one_stage():
    T, a, w = [1.0, 2.5, 0.5, 3.0], [9.0] * 4, [7.0] * 4
    best, stages, noam = partition(T, a, w, 1, 1.0)
    assert best == pytest.approx(7.0) and stages == [StageAssign(0, 3, 1)] and noam == 1


def test_free_communication_balances_equal_layers():
    # no parameters, (almost) free boundaries: N equal layers on N machines cost one layer time,
    # whether as a straight pipeline or as one replicated stage
    N, t = 5, 2.0
    best, stages, _ = partition([t] * N, [1e-9] * N, [0.0] * N, N, 1.0)
    assert best == pytest.approx(t)
    _check_feasible(stages, N, N)


def test_huge_activations_force_data_parallelism():
    # boundaries cost far more than compute, parameters are tiny: one stage replicated M times
    T = [1.0, 2.0, 3.0, 2.0]
    best, stages, noam = partition(T, [1e6] * 4, [1e-9] * 4, 4, 1.0)
    assert stages == [StageAssign(0, 3, 4)] and best == pytest.approx(8.0 / 4) and noam == 1


def test_huge_parameters_force_a_straight_pipeline():
    # synchronisation of any replicated stage dwarfs compute, boundaries are free: no stage is replicated
    T = [1.0, 1.0, 1.0]
    best, stages, noam = partition(T, [1e-9] * 3, [1e6] * 3, 3, 1.0)
    assert [s.replicas for s in stages] == [1, 1, 1] and best == pytest.approx(1.0) and noam == 3


def test_hand_worked_example():
    # T = [4, 2, 2], parameters 10 bytes in total, bandwidth 1, two machines.
    #   one stage on 2 machines: compute 8, synchronisation 4*(1)*10/2 = 20 -> max/2 = 10
    #   split after layer 1: max(T(1->1,1) = 4, 2*C_1 = 2*1, T(2->3,1) = 4) = 4
    #   split after layer 2: max(6, 2*0.5, 2) = 6
    T, a, w = [4.0, 2.0, 2.0], [1.0, 0.5, 0.25], [5.0, 3.0, 2.0]
    assert sync_time(10.0, 2, 1.0) == pytest.approx(20.0)
    assert stage_time(T, w, 1, 3, 2, 1.0) == pytest.approx(10.0)
    best, stages, noam = partition(T, a, w, 2, 1.0)
    assert best == pytest.approx(4.0)
    assert stages == [StageAssign(0, 0, 1), StageAssign(1, 2, 1)] and noam == 2
    # a boundary that costs more than the alternative moves the optimum: C_1 = 3.5 -> 2*C_1 = 7 > 6
    best, stages, _ = partition(T, [3.5, 0.5, 0.25], w, 2, 1.0)
    assert best == pytest.approx(6.0) and stages == [StageAssign(0, 1, 1), StageAssign(2, 2, 1)]


def test_stage_time_has_the_one_over_m_factor_on_both_terms():
    T, w = [6.0], [3.0]
    # m = 3: compute 6, synchronisation 4*2*3/3 = 8 -> max 8, / 3
    assert stage_time(T, w, 1, 1, 3, 1.0) == pytest.approx(8.0 / 3.0)
    assert stage_time(T, [0.0], 1, 1, 3, 1.0) == pytest.approx(2.0)
    assert sync_time(3.0, 1, 1.0) == 0.0


def test_noam_of_table1_configurations():
    # VGG16 rows of Table 1: "2-1-1" on 4 machines, "7-1" on 8, "9-5-1-1" on 16; Inception-v3 "8" (data parallel)
    def cfg(*replicas):
        return [StageAssign(i, i, r) for i, r in enumerate(replicas)]
    assert noam_of(cfg(2, 1, 1)) == 2
    assert noam_of(cfg(7, 1)) == 2
    assert noam_of(cfg(9, 5, 1, 1)) == 2
    assert noam_of(cfg(8)) == 1
    assert noam_of(cfg(1, 1, 1, 1)) == 4


def test_more_machines_never_hurt_when_synchronisation_is_free():
    rng = np.random.default_rng(7)
    T = rng.uniform(1, 3, 6).tolist()
    a = rng.uniform(0, 0.2, 6).tolist()
    prev = math.inf
    for M in range(1, 8):
        best, _, _ = partition(T, a, [0.0] * 6, M, 1.0)
        assert best <= prev + 1e-12
        prev = best


def test_argument_errors():
    with pytest.raises(ValueError):
        partition([], [], [], 2, 1.0)
    with pytest.raises(ValueError):
        partition([1.0], [1.0], [1.0], 0, 1.0)
    with pytest.raises(ValueError):
        partition([1.0], [1.0, 2.0], [1.0], 1, 1.0)
    with pytest.raises(ValueError):
        partition([1.0], [1.0], [1.0], 1, 0.0)
