"""Oracle for the layer partitioner (Section 3.2: profiling quantities, the dynamic program, NOAM).

Test infrastructure only (see package docstring).  Plain Python floats (fp64), loops in the paper's
order and notation: layers l = 1..N, machines m = 1..M, ``A(j, m)`` the time of the slowest stage of
the best pipeline over layers 1..j on exactly m machines, ``T(i -> j, m)`` the time of one stage
holding layers i..j replicated over m machines.

Inputs are the three per-layer profile quantities of Section 3.2 -- ``T[l]`` (forward + backward
compute time), ``a[l]`` (bytes of the layer's output activations, also of the gradient that comes
back) and ``w[l]`` (bytes of its parameters) -- and one link bandwidth in bytes per time unit.

Readings where the text leaves room:
  * ``C_l = a_l / bandwidth`` (one direction); a boundary after layer i costs ``2 C_i``.
  * ``W_l^m = 4 (m - 1) |w_l| / m / bandwidth``: the per-worker traffic the text gives for a
    data-parallel stage of m replicas, divided by the bandwidth; zero for m = 1.
  * ``T(i -> j, m)`` carries the printed factor 1/m over both terms of the max.
  * Ties between partitions of equal cost are broken towards the earlier split point and the smaller
    replica count of the last stage (first minimum found in the printed order of the two ``min``);
    only the optimum value is unique, callers compare that and check the partition is feasible.
"""
from __future__ import annotations

import math
from typing import List, NamedTuple, Sequence, Tuple


class StageAssign(NamedTuple):
    first: int      # first layer of the stage, 0-based
    last: int       # last layer of the stage, 0-based, inclusive
    replicas: int   # machines the stage is replicated over


def comm_time(a_bytes: float, bandwidth: float) -> float:
    """C_l: time to move layer l's output activations (or the gradient of the same size) one way."""
    return a_bytes / bandwidth


def sync_time(w_bytes: float, m: int, bandwidth: float) -> float:
    """W_l^m: weight synchronisation time of layer l in a stage replicated over m machines."""
    return 4.0 * (m - 1) * w_bytes / m / bandwidth


def stage_time(T: Sequence[float], w: Sequence[float], i: int, j: int, m: int, bandwidth: float) -> float:
    """T(i -> j, m) for 1-based inclusive layers i..j: (1/m) max(sum of T_l, sum of W_l^m)."""
    compute = 0.0
    sync = 0.0
    for l in range(i, j + 1):
        compute += T[l - 1]
        sync += sync_time(w[l - 1], m, bandwidth)
    return max(compute, sync) / m


def partition(T: Sequence[float], a: Sequence[float], w: Sequence[float], M: int,
              bandwidth: float) -> Tuple[float, List[StageAssign], int]:
    """The dynamic program of Section 3.2.  Returns (A(N, M), stages, NOAM)."""
    N = len(T)
    if N < 1 or M < 1 or len(a) != N or len(w) != N or not bandwidth > 0:
        raise ValueError("bad partition problem")
    INF = math.inf
    A = [[INF] * (M + 1) for _ in range(N + 1)]          # A[j][m], 1-based
    choice = [[None] * (M + 1) for _ in range(N + 1)]    # None = one stage; else (i, m')
    for j in range(1, N + 1):
        for m in range(1, M + 1):
            # Case 1: one stage replicated m times (this is also the printed initialisation of
            # A(1, m) and A(j, 1), for which Case 2 has no admissible (i, m'))
            best = stage_time(T, w, 1, j, m, bandwidth)
            pick = None
            # Case 2: best pipeline over layers 1..i on m - m' machines, then one stage i+1..j on m'
            for i in range(1, j):
                for mp in range(1, m):
                    cand = max(A[i][m - mp], 2.0 * comm_time(a[i - 1], bandwidth),
                               stage_time(T, w, i + 1, j, mp, bandwidth))
                    if cand < best:
                        best, pick = cand, (i, mp)
            A[j][m] = best
            choice[j][m] = pick
    stages: List[StageAssign] = []
    j, m = N, M
    while True:
        pick = choice[j][m]
        if pick is None:
            stages.append(StageAssign(0, j - 1, m))
            break
        i, mp = pick
        stages.append(StageAssign(i, j - 1, mp))
        j, m = i, m - mp
    stages.reverse()
    return A[N][M], stages, noam_of(stages)


def noam_of(stages: Sequence[StageAssign]) -> int:
    """NUM_OPT_ACTIVE_MINIBATCHES: ceil(machines / machines of the input stage) (end of Section 3.2)."""
    total = sum(s.replicas for s in stages)
    return math.ceil(total / stages[0].replicas)


def pipeline_time(T: Sequence[float], a: Sequence[float], w: Sequence[float],
                  stages: Sequence[StageAssign], bandwidth: float) -> float:
    """Time of the slowest element of a given pipeline: each stage's T(i -> j, m) and each boundary's 2 C_i."""
    worst = 0.0
    for k, s in enumerate(stages):
        worst = max(worst, stage_time(T, w, s.first + 1, s.last + 1, s.replicas, bandwidth))
        if k + 1 < len(stages):
            worst = max(worst, 2.0 * comm_time(a[s.last], bandwidth))
    return worst
