"""Integer side of the oracle: NOAM, in-flight depth, the 1F1B op list, the simulator.

Test infrastructure only (see package docstring).  Conventions: stages s = 0..S-1
(the paper counts from 1), minibatches i = 0..M-1 (the paper's "minibatch 5" is
i = 4), version v = number of updates already applied to the stage's weights.
"""
from __future__ import annotations

import math
from typing import List, NamedTuple

OP_F, OP_B, OP_U = 0, 1, 2


class Op(NamedTuple):
    kind: int      # OP_F / OP_B / OP_U
    mb: int        # minibatch id
    version: int   # F, B: weight version read; U: weight version produced
    slot: int      # ring slot of that version = version mod depth


def noam(num_machines: int, input_stage_machines: int) -> int:
    """NUM_OPT_ACTIVE_MINIBATCHES (Section 3.2, end): ceil(machines / machines of the input stage)."""
    return math.ceil(num_machines / input_stage_machines)


def in_flight_depth(num_stages: int, noam_: int, stage: int) -> int:
    """How many minibatches stage ``stage`` may hold between their F and their B
    (also the number of weight versions it keeps: the depth of its version ring).

    The input stage admits NOAM (Section 3.3); the output stage holds one
    (Section 3.5); the worked example of Section 3.4 (4 stages: three, two, one,
    zero interleaved updates from stage 1 to stage 4) fixes the values between as
    NOAM - s, never below 1.  (A stream shorter than this simply never fills it.)
    """
    if not (0 <= stage < num_stages):
        raise ValueError("stage out of range")
    return max(1, noam_ - stage)


def schedule_1f1b(num_stages: int, noam_: int, num_minibatches: int, stage: int,
                  depth_override: int = 0, vertical_sync: bool = False) -> List[Op]:
    """The static op list of one stage, built by walking the policy of Section 3.3.

    Start-up: forwards until ``depth`` minibatches are in flight.  Then the stage
    alternates, starting with the backward of the oldest in-flight minibatch; each
    backward is followed at once by its update (Section 4, "Parameter State"); at
    the end of the stream the remaining backwards drain in arrival order.
    Versions are produced by carrying the stage's ``latest`` counter through the
    walk, as the runtime would, not from a formula.

    ``vertical_sync`` (Section 3.4): a minibatch is tagged with the version the INPUT
    stage's forward read, and every stage uses that version of its own weights for
    the minibatch's forward and backward pass.  The op order is unchanged; only the
    versions of F and B differ, and a stage then has to keep as many versions as
    the input stage (its ring has the input stage's depth, which sets ``slot``).
    """
    M = num_minibatches
    depth = depth_override if depth_override > 0 else in_flight_depth(num_stages, noam_, stage)
    if vertical_sync:
        ring = depth_override if depth_override > 0 else in_flight_depth(num_stages, noam_, 0)
        tags = {o.mb: o.version for o in schedule_1f1b(num_stages, noam_, M, 0, depth_override) if o.kind == OP_F}
        out = []
        for o in schedule_1f1b(num_stages, noam_, M, stage, depth_override):
            v = o.version if o.kind == OP_U else tags[o.mb]
            out.append(Op(o.kind, o.mb, v, v % ring))
        return out
    ops: List[Op] = []
    latest = 0
    stashed = {}          # mb -> version its forward used
    next_f = 0
    next_b = 0
    while next_b < M:
        if next_f < M and len(stashed) < depth:
            stashed[next_f] = latest                         # forward reads the latest version
            ops.append(Op(OP_F, next_f, latest, latest % depth))
            next_f += 1
            continue
        v = stashed.pop(next_b)                              # backward reads what its forward read
        ops.append(Op(OP_B, next_b, v, v % depth))
        latest += 1                                          # update goes onto the latest weights
        ops.append(Op(OP_U, next_b, latest, latest % depth))
        next_b += 1
    return ops


def stashed_version_closed_form(mb: int, depth: int) -> int:
    """Version a minibatch sees in steady state, read off the staleness equation of
    Section 3.4: a stage with ``depth`` minibatches in flight computes minibatch t's
    gradient on weights depth-1 updates old; the start-up clamp at 0 is ours."""
    return max(0, mb - depth + 1)


class Event(NamedTuple):
    stage: int
    op: Op
    start: float
    end: float


def simulate(num_stages: int, noam_: int, num_minibatches: int,
             t_forward: float = 1.0, t_backward: float = 1.0) -> List[Event]:
    """Event-driven run of all stages (Section 3.3): each stage executes its own
    static list and only waits for data -- F(i,s) for F(i,s-1)'s output, B(i,s)
    for B(i,s+1)'s input gradient (the last stage's B needs only its own F).
    The update is folded into its backward's time slot.  Returns events in a valid
    global execution order; raises if the system cannot make progress.
    """
    S, M = num_stages, num_minibatches
    lists = [schedule_1f1b(S, noam_, M, s) for s in range(S)]
    pos = [0] * S
    clock = [0.0] * S
    f_done = {}   # (mb, stage) -> finish time
    b_done = {}
    out: List[Event] = []
    remaining = sum(len(l) for l in lists)
    while remaining:
        progressed = False
        for s in range(S):
            while pos[s] < len(lists[s]):
                op = lists[s][pos[s]]
                if op.kind == OP_F:
                    ready = 0.0 if s == 0 else f_done.get((op.mb, s - 1))
                    dur = t_forward
                elif op.kind == OP_B:
                    ready = f_done.get((op.mb, s)) if s == S - 1 else b_done.get((op.mb, s + 1))
                    dur = t_backward
                else:
                    ready, dur = clock[s], 0.0
                if ready is None:
                    break
                start = max(clock[s], ready)
                end = start + dur
                clock[s] = end
                if op.kind == OP_F:
                    f_done[(op.mb, s)] = end
                elif op.kind == OP_B:
                    b_done[(op.mb, s)] = end
                out.append(Event(s, op, start, end))
                pos[s] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("pipeline deadlock: no stage can run its next op")
    return out
