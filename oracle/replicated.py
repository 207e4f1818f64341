"""A stage replicated over several machines (Section 3.3, round-robin routing; Section 4, "Data Parallelism").

Test infrastructure only (see package docstring).

What the paper fixes: minibatches are dealt to the replicas of a stage round-robin by their id, so the backward
pass of a minibatch runs where its forward pass ran (Section 3.3); the replicas' weight gradients go to a
parameter server, which hands out new parameters once the updates of ALL replicas have been aggregated
(Section 4); plain data-parallel training is the special case of one stage holding every layer (Section 4).

Reading taken where it is silent (written out here so that it can be checked by eye):
  * replica of minibatch i:  q = i mod r;  its position in that replica's own stream ("round"):  k = i div r.
    Every replica follows the ordinary 1F1B list of the stage over its rounds.
  * aggregation = SUM of the replicas' gradients of one round (each the gradient of its own minibatch-mean loss),
    so a minibatch moves the weights by lr * g exactly as it does in a stage that is not replicated.
  * one update per round, applied by every replica to its own full copy of the parameters (the copies therefore
    stay identical), after the backward passes of that round on all replicas and before any replica's next
    forward pass: replicas run in lock step, weight version = rounds completed.
  * a last round that not every replica takes part in (the stream ran out) sums over those that do; the
    others still receive the new parameters.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

from .pipeline import Stage
from .schedule import OP_B, OP_F, OP_U, Op, schedule_1f1b


def route(mb: int, replicas: int) -> Tuple[int, int]:
    """(replica, round) of minibatch ``mb`` (Section 3.3: deterministic round-robin by minibatch id)."""
    return mb % replicas, mb // replicas


def rounds_of(replica: int, replicas: int, num_minibatches: int) -> int:
    """How many minibatches of a stream of ``num_minibatches`` land on ``replica``."""
    return len(range(replica, num_minibatches, replicas))


class ReplicatedStage:
    """``replicas`` machines, each a complete Stage with its own copy of the parameters and its own stash."""

    def __init__(self, layers, params_fp32, depth: int, replicas: int, mode: str = "f32", lr: float = 0.01,
                 momentum: float = 0.9, optimizer: str = "sgd", eps: float = 1.0):
        if replicas < 1:
            raise ValueError("a stage has at least one replica")
        self.r = int(replicas)
        self.rep = [Stage(layers, params_fp32, depth, mode, lr, momentum, optimizer=optimizer, eps=eps)
                    for _ in range(self.r)]
        self.trace: List[Tuple[int, Op]] = []        # (replica, op); the joint update is listed under replica -1

    @property
    def latest(self) -> int:
        return self.rep[0].latest

    def forward(self, mb: int, x, labels=None):
        q, k = route(mb, self.r)
        out = self.rep[q].forward(k, x, labels)
        self.trace.append((q, self.rep[q].trace[-1]))
        return out

    def backward(self, mb: int, dy=None, need_dx: bool = True):
        q, k = route(mb, self.r)
        dx = self.rep[q].backward(k, dy, need_dx)
        self.trace.append((q, self.rep[q].trace[-1]))
        return dx

    def update(self, round_: int = -1):
        """The parameter server's step: sum what the replicas of this round computed, update every copy."""
        have = [s for s in self.rep if s.grad is not None]
        if not have:
            raise RuntimeError("update without a pending gradient on any replica")
        g = have[0].grad.copy()
        for s in have[1:]:                              # replica order: fixes the rounding order of the sum
            g = g + s.grad
        for s in self.rep:
            s.grad = g.copy()
            s.update(round_)
        self.trace.append((-1, self.rep[0].trace[-1]))


def run_replicated_pipeline(stage_layers: Sequence, stage_params: Sequence, replicas: Sequence[int], inputs, labels,
                            depths: Sequence[int], mode: str = "f32", lr: float = 0.01, momentum: float = 0.9,
                            order: Optional[list] = None, keep_log: bool = False):
    """A pipeline whose stage s has ``replicas[s]`` replicas and per-replica in-flight depth ``depths[s]``.

    Every replica walks the stage's static 1F1B list over its own rounds (Section 3.3: both policies are static);
    an F waits for the previous stage's output of that minibatch, a B for the next stage's input gradient, and an
    update for the backward passes of its round on every replica that has a minibatch in it.  ``order`` receives
    (stage, replica, kind, minibatch-or-round) in execution order.  Returns (stages, losses).
    """
    S, M = len(stage_layers), len(inputs)
    stages = [ReplicatedStage(stage_layers[s], stage_params[s], depths[s], replicas[s], mode, lr, momentum)
              for s in range(S)]
    if keep_log:
        for st in stages:
            for rp in st.rep:
                rp.log = {}
    # per (stage, replica): its list over rounds k; global minibatch id = k * r + q
    lists = [[schedule_1f1b(1, 1, rounds_of(q, replicas[s], M), 0, depth_override=depths[s])
              for q in range(replicas[s])] for s in range(S)]
    pos = [[0] * replicas[s] for s in range(S)]
    act, grad = {}, {}
    losses: List[Optional[float]] = [None] * M
    remaining = sum(len(l) for ls in lists for l in ls)
    while remaining:
        progressed = False
        for s in range(S):
            r = replicas[s]
            st = stages[s]
            for q in range(r):
                while pos[s][q] < len(lists[s][q]):
                    op = lists[s][q][pos[s][q]]
                    mb = op.mb * r + q
                    if op.kind == OP_F:
                        if s > 0 and (mb, s - 1) not in act:
                            break
                        x = inputs[mb] if s == 0 else act.pop((mb, s - 1))
                        y, loss = st.forward(mb, x, labels[mb] if (s == S - 1 and labels is not None) else None)
                        if s == S - 1:
                            losses[mb] = loss
                        else:
                            act[(mb, s)] = y
                        if order is not None:
                            order.append((s, q, OP_F, mb))
                    elif op.kind == OP_B:
                        if s < S - 1 and (mb, s + 1) not in grad:
                            break
                        dy = None if s == S - 1 else grad.pop((mb, s + 1))
                        dx = st.backward(mb, dy, need_dx=s > 0)
                        if s > 0:
                            grad[(mb, s)] = dx
                        if order is not None:
                            order.append((s, q, OP_B, mb))
                    else:
                        # joint update of round op.mb: every replica with a minibatch in this round must be here
                        peers = [p for p in range(r) if rounds_of(p, r, M) > op.mb]
                        ready = all(pos[s][p] < len(lists[s][p]) and lists[s][p][pos[s][p]].kind == OP_U
                                    and lists[s][p][pos[s][p]].mb == op.mb for p in peers)
                        if not ready:
                            break
                        st.update(op.mb)
                        if order is not None:
                            order.append((s, -1, OP_U, op.mb))
                        for p in peers:
                            if p != q:
                                pos[s][p] += 1
                                remaining -= 1
                    pos[s][q] += 1
                    remaining -= 1
                    progressed = True
        if not progressed:
            raise RuntimeError("pipeline deadlock")
    return stages, losses
