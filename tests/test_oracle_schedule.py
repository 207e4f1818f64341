"""Pins for the integer side of the oracle: NOAM, depth, 1F1B order, versions, simulator."""
import itertools
import os

import pytest

from oracle.schedule import (OP_B, OP_F, OP_U, in_flight_depth, noam, schedule_1f1b, simulate,
                             stashed_version_closed_form)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example_4stage.txt")


def _facts():
    out = []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, s, mb, v = line.split()
            out.append((k, int(s), int(mb), int(v)))
    return out


def test_noam_formula():
    # Section 3.2 (end): ceil(#machines / #machines of the input stage); the three VGG16
    # configurations of Table 1 (2-1-1 on 4, 7-1 on 8, 9-5-1-1 on 16) and a straight pipeline.
    assert noam(4, 1) == 4
    assert noam(4, 2) == 2
    assert noam(8, 7) == 2
    assert noam(16, 9) == 2
    assert noam(8, 8) == 1


def test_worked_example_golden():
    S, NOAM, M = 4, 4, 16
    ev = {s: schedule_1f1b(S, NOAM, M, s) for s in range(S)}
    for fact, stage1, mb1, value in _facts():
        ops = ev[stage1 - 1]
        mb = mb1 - 1
        if fact == "startup_forwards":
            first_b = next(i for i, o in enumerate(ops) if o.kind == OP_B)
            assert first_b == value and all(o.kind == OP_F for o in ops[:first_b])
            continue
        idx_f = next(i for i, o in enumerate(ops) if o.kind == OP_F and o.mb == mb)
        idx_b = next(i for i, o in enumerate(ops) if o.kind == OP_B and o.mb == mb)
        u_before_f = sum(1 for o in ops[:idx_f] if o.kind == OP_U)
        u_before_b = sum(1 for o in ops[:idx_b] if o.kind == OP_U)
        if fact == "updates_before_forward":
            assert u_before_f == value == ops[idx_f].version
        elif fact == "updates_before_backward":
            assert u_before_b == value
        elif fact == "interleaved_updates":
            assert u_before_b - u_before_f == value
        else:
            raise AssertionError(fact)


def test_stage0_order_prefix():
    # Section 3.3/3.4: four forwards, then B of the first minibatch comes before F of the fifth.
    ops = [(o.kind, o.mb) for o in schedule_1f1b(4, 4, 8, 0) if o.kind != OP_U]
    assert ops[:8] == [(OP_F, 0), (OP_F, 1), (OP_F, 2), (OP_F, 3), (OP_B, 0), (OP_F, 4), (OP_B, 1), (OP_F, 5)]
    last = [(o.kind, o.mb) for o in schedule_1f1b(4, 4, 8, 3) if o.kind != OP_U]
    assert last[:4] == [(OP_F, 0), (OP_B, 0), (OP_F, 1), (OP_B, 1)]


@pytest.mark.parametrize("S,NOAM,M", [(s, n, m) for s in range(1, 7) for n in range(1, s + 1)
                                       for m in (1, 2, 3, 5, 3 * s)])
def test_invariants(S, NOAM, M):
    for s in range(S):
        ops = schedule_1f1b(S, NOAM, M, s)
        depth = in_flight_depth(S, NOAM, s)
        f = {o.mb: o for o in ops if o.kind == OP_F}
        b = {o.mb: o for o in ops if o.kind == OP_B}
        u = [o for o in ops if o.kind == OP_U]
        # drain: every minibatch gets exactly one F, B and U; final version = M
        assert sorted(f) == sorted(b) == list(range(M)) and len(u) == M and u[-1].version == M
        live, in_flight, latest = {}, 0, 0
        for o in ops:
            if o.kind == OP_F:
                in_flight += 1
                assert in_flight <= depth                        # Section 3.5: bounded state
                assert o.version == latest                       # F reads the latest version
                live[o.mb] = o.version
            elif o.kind == OP_B:
                in_flight -= 1
                assert o.version == f[o.mb].version              # Section 3.4: same version for F and B
                assert o.mb == min(live)                          # FIFO
                del live[o.mb]
            else:
                latest += 1
                assert o.version == latest
                # ring rule: the slot being overwritten holds no version an in-flight minibatch needs
                assert all(v % depth != o.slot for v in live.values())
            assert o.slot == o.version % depth
            assert len(set(live.values()) | {latest}) <= depth + 1
        # closed form read off the staleness equation (Section 3.4)
        for i in range(M):
            assert f[i].version == stashed_version_closed_form(i, depth)
        if True:
            assert min(depth, M) == max(sum(1 for o in ops[:k] if o.kind == OP_F) - sum(1 for o in ops[:k] if o.kind == OP_B)
                       for k in range(len(ops) + 1))


def test_depth_rule():
    assert [in_flight_depth(4, 4, s) for s in range(4)] == [4, 3, 2, 1]
    # one active minibatch = plain model parallelism (Section 3.1, first timeline)
    assert [in_flight_depth(4, 1, s) for s in range(4)] == [1, 1, 1, 1]
    assert [in_flight_depth(2, 2, s) for s in range(2)] == [2, 1]      # the 7-1 configuration of Table 1


def test_sequential_when_one_in_flight():
    # S = 1, or NOAM = 1: version seen by minibatch i is i (ordinary minibatch SGD, Section 3.4 first equation)
    for S, NOAM in [(1, 1), (4, 1), (3, 1)]:
        for s in range(S):
            ops = schedule_1f1b(S, NOAM, 9, s)
            assert [o.version for o in ops if o.kind == OP_F] == list(range(9))
            kinds = [o.kind for o in ops]
            assert kinds == [OP_F, OP_B, OP_U] * 9


def test_simulator_terminates_everywhere():
    for S in range(1, 9):
        for NOAM in range(1, S + 1):
            for M in (1, 2, S, 3 * S):
                ev = simulate(S, NOAM, M)
                assert len(ev) == 3 * M * S


def test_steady_state_has_no_idle_slot():
    # Section 3.3: balanced pipeline (unit F and B), NOAM = S: in steady state every stage is busy.
    for S in (2, 3, 4, 6):
        M = 10 * S
        ev = [e for e in simulate(S, S, M) if e.op.kind != OP_U]
        for s in range(S):
            mine = sorted((e for e in ev if e.stage == s), key=lambda e: e.start)
            # steady state: after the first backward of this stage, before the last forward
            first_b = next(i for i, e in enumerate(mine) if e.op.kind == OP_B)
            last_f = max(i for i, e in enumerate(mine) if e.op.kind == OP_F)
            for a, b_ in zip(mine[first_b:last_f], mine[first_b + 1:last_f + 1]):
                assert b_.start == a.end, (S, s, a, b_)
                assert a.op.kind != b_.op.kind                  # strict alternation
        # and the whole run takes 2*M + 2*(S-1) unit slots: fill + drain only
        assert max(e.end for e in ev) == 2 * M + 2 * (S - 1)


def test_model_parallel_timeline():
    # one active minibatch: at most one stage busy at a time (Section 3.1)
    ev = [e for e in simulate(4, 1, 3) if e.op.kind != OP_U]
    ev.sort(key=lambda e: e.start)
    for a, b_ in zip(ev, ev[1:]):
        assert b_.start >= a.end
