"""Stage state and the 1F1B weight-stashed step, in the paper's order (Sections 3.3-3.5, 4).

Test infrastructure only (see package docstring).

A stage keeps: ``latest`` (updates applied so far), every weight version it has
produced (the paper keeps a version until no in-flight minibatch needs it,
Section 4 "Parameter State"; keeping all of them gives the same numbers and lets
tests inspect history -- ring-slot reuse is asserted separately), one momentum
buffer, and a stash per in-flight minibatch holding the version id and the
layer inputs/outputs its backward needs (Section 4 "Intermediate State").

Update rule (the paper states SGD, momentum 0.9, lr 0.01 in Section 5.1 and the
plain-SGD equation in Section 3.4; the momentum form is the common one):
    m <- mu * m + g ;  w_latest <- w_latest - lr * m
with g the gradient of the minibatch-mean loss, applied once per backward pass to
the latest weights (not to the stashed ones).
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from . import layers as L
from .schedule import OP_B, OP_F, OP_U, Op, in_flight_depth, schedule_1f1b


def _split_params(layers, flat):
    """Views (W, b) per parametrised layer into a flat vector laid out layer by layer, W then b."""
    out, o = [], 0
    for ly in layers:
        if ly[0] == "linear":
            n_in, n_out = ly[1], ly[2]
            W = flat[o:o + n_in * n_out].reshape(n_out, n_in); o += n_in * n_out
            b = flat[o:o + n_out]; o += n_out
            out.append((W, b))
        elif ly[0] == "conv2d":
            c_in, c_out, kh, kw = ly[1], ly[2], ly[3], ly[4]
            n = c_out * kh * kw * c_in
            W = flat[o:o + n].reshape(c_out, kh, kw, c_in); o += n
            b = flat[o:o + c_out]; o += c_out
            out.append((W, b))
        elif ly[0] == "lstm":
            I, H = ly[1], ly[2]
            W_ih = flat[o:o + 4 * H * I].reshape(4 * H, I); o += 4 * H * I
            W_hh = flat[o:o + 4 * H * H].reshape(4 * H, H); o += 4 * H * H
            b = flat[o:o + 4 * H]; o += 4 * H
            out.append((W_ih, W_hh, b))
        elif ly[0] == "concat":                      # branches in order, each a layer list of its own
            views = []
            for br in ly[1]:
                n = _count(br)
                views.append(_split_params(br, flat[o:o + n])); o += n
            out.append(views)
        else:
            out.append(None)
    assert o == flat.size, "parameter vector does not match the layer list"
    return out


def _count(layers):
    n = 0
    for ly in layers:
        if ly[0] == "linear":
            n += ly[1] * ly[2] + ly[2]
        elif ly[0] == "conv2d":
            n += ly[2] * ly[3] * ly[4] * ly[1] + ly[2]
        elif ly[0] == "lstm":
            n += 4 * ly[2] * (ly[1] + ly[2]) + 4 * ly[2]
        elif ly[0] == "concat":
            n += sum(_count(br) for br in ly[1])
    return n


_LSTM_CACHE = {}   # id(stored h sequence) -> gate/cell values of its forward pass, until its backward
_BLOCK_CACHE = {}  # id(stored block output) -> per branch, the stored activations [input, layer outputs...]


def _layer_forward(layers, li, p, a, q):
    """Stored output of layer li for stored input a (loss layers are handled by the caller).
    A Linear after an LSTM acts on every time step: rows = T*B of the time-major sequence."""
    ly = layers[li]
    if ly[0] == "linear":
        if li > 0 and layers[li - 1][0] == "lstm":
            a = a.reshape(-1, a.shape[-1])
        elif a.ndim > 2:
            a = a.reshape(a.shape[0], -1)          # NHWC flatten
        return L.linear_forward(a, p[0], p[1], ly[3], _out_quantiser(layers, li, q))
    if ly[0] == "lstm":
        h, cache = L.lstm_forward(a, p[0], p[1], p[2], q)
        _LSTM_CACHE[id(h)] = cache
        return h
    if ly[0] == "conv2d":
        return L.conv2d_forward(a, p[0], p[1], ly[5], ly[6], ly[7], ly[8], q)
    if ly[0] == "maxpool2d":
        return L.maxpool2d_forward(a, ly[1], ly[2])
    if ly[0] == "avgpool2d":
        return L.avgpool2d_forward(a, ly[1], ly[2], ly[3], q)
    if ly[0] == "concat":
        per_branch = []
        for br, bp in zip(ly[1], p):
            acts = [a]
            for si in range(len(br)):
                acts.append(_layer_forward(br, si, bp[si], acts[-1], q))
            per_branch.append(acts)
        y = np.concatenate([acts[-1] for acts in per_branch], axis=-1)
        _BLOCK_CACHE[id(y)] = per_branch
        return y
    raise NotImplementedError(ly[0])


def _layer_backward(layers, li, p, x, y, d, need_dx, q):
    """(dx, dW, db) of layer li; dW/db are None for layers without parameters."""
    ly = layers[li]
    if ly[0] == "lstm":
        cache = _LSTM_CACHE.pop(id(y))
        dx, dWi, dWh, db = L.lstm_backward(x, p[0], p[1], cache, d.reshape(y.shape), need_dx, q)
        return dx, (dWi, dWh), db
    if ly[0] == "linear":
        x2 = x.reshape(-1, x.shape[-1]) if (li > 0 and layers[li - 1][0] == "lstm") else x.reshape(x.shape[0], -1)
        dx, dW, db = L.linear_backward(x2, p[0], y, d, ly[3], need_dx, q)
        if dx is not None:
            dx = dx.reshape(x.shape)
        return dx, dW, db
    if ly[0] == "conv2d":
        return L.conv2d_backward(x, p[0], y, d, ly[5], ly[6], ly[7], ly[8], need_dx, q)
    if ly[0] == "maxpool2d":
        return (q(L.maxpool2d_backward(x, y, d, ly[1], ly[2])) if need_dx else None), None, None
    if ly[0] == "avgpool2d":
        return (L.avgpool2d_backward(x.shape, d, ly[1], ly[2], ly[3], q) if need_dx else None), None, None
    if ly[0] == "concat":
        per_branch = _BLOCK_CACHE.pop(id(y))
        d = d.reshape(y.shape)
        grads, dx_sum, c0 = [], None, 0
        for br, bp, acts in zip(ly[1], p, per_branch):
            c1 = c0 + acts[-1].shape[-1]
            db_ = d[..., c0:c1]                          # this branch's channel slice of dL/d(output)
            c0 = c1
            g = [None] * len(br)
            for si in range(len(br) - 1, -1, -1):
                dx_b, dW, db = _layer_backward(br, si, bp[si], acts[si], acts[si + 1], db_, need_dx or si > 0, q)
                g[si] = None if dW is None else (dW, db)
                db_ = dx_b
            grads.append(g)
            if need_dx:                                  # each branch's input gradient is a stored tensor
                dx_sum = db_ if dx_sum is None else dx_sum + db_
        return (q(dx_sum) if need_dx else None), grads, None
    raise NotImplementedError(ly[0])


def _store_grad(views, dW, db):
    if isinstance(dW, list):           # concat block: per branch, per layer (dW, db) or None
        for bviews, bgrads in zip(views, dW):
            for v, g in zip(bviews, bgrads):
                if g is not None:
                    _store_grad(v, g[0], g[1])
        return
    if isinstance(dW, tuple):          # LSTM: (dW_ih, dW_hh), bias last
        views[0][...] = dW[0]
        views[1][...] = dW[1]
        views[2][...] = db
    else:
        views[0][...] = dW
        views[1][...] = db


def _out_quantiser(layers, li, q):
    """Rounding applied to layer li's stored output: logits that go straight into the
    loss stay in accumulator precision (the loss is computed unrounded); everything else
    is an activation handed on in the storage type."""
    feeds_loss = li + 1 < len(layers) and layers[li + 1][0] == "softmax_xent"
    return (lambda a: a) if feeds_loss else q


class Stage:
    def __init__(self, layers, params_fp32, depth: int, mode: str = "f32",
                 lr: float = 0.01, momentum: float = 0.9, stashing: bool = True, ring_depth: int = 0,
                 optimizer: str = "sgd", eps: float = 1.0):
        self.layers = list(layers)
        self.depth = int(depth)
        self.ring = int(ring_depth) if ring_depth else self.depth   # versions kept (vertical sync: the input stage's)
        self.mode = mode
        self.q = L.quantiser(mode)
        self.lr, self.mu = float(lr), float(momentum)
        # "sgd": momentum SGD (Section 5.1, VGG16 and S2VT).  "rmsprop" (Section 5.1, Inception-v3; the paper names
        # the optimiser and its learning rate only): the common library form, with `momentum` as the decay a --
        #     v <- a v + (1 - a) g^2 ;  w <- w - lr g / (sqrt(v) + eps)
        # one state buffer per stage either way (self.mom holds v)
        self.optimizer, self.eps = optimizer, float(eps)
        self.stashing = stashing              # False = the naive pipeline of Section 3.4 (negative control)
        self.master = np.asarray(params_fp32, dtype=np.float64).copy()
        self.versions = [self.q(self.master)]  # versions[v] = weights as the layers read them
        self.mom = np.zeros_like(self.master)
        self.latest = 0
        self.stash = {}                       # mb -> dict(version, acts, labels, probs)
        self.grad = None                      # flat gradient of the last backward, until update() consumes it
        self.trace: List[Op] = []
        self.max_in_flight = 0
        self.log = None                       # set to {} to keep, per minibatch, the stored layer outputs
                                              # ("acts"), the incoming gradient ("dy") and the result ("dx")

    # -- F ---------------------------------------------------------------------
    def forward(self, mb: int, x, labels=None, version: Optional[int] = None):
        if len(self.stash) >= self.depth:
            raise RuntimeError("more minibatches in flight than the stage's depth")
        # default semantics: the latest version available; vertical sync (Section 3.4): the version the
        # minibatch was tagged with at the input stage, which this stage must still hold
        v = self.latest if version is None else version
        if not (self.latest - self.ring < v <= self.latest):
            raise RuntimeError("requested weight version is not held by the stage")
        P = _split_params(self.layers, self.versions[v])
        acts = [self.q(x)]
        loss, probs = None, None
        for li, (ly, p) in enumerate(zip(self.layers, P)):
            if ly[0] == "softmax_xent":
                loss, probs = L.softmax_xent_forward(acts[-1], labels)
            else:
                acts.append(_layer_forward(self.layers, li, p, acts[-1], self.q))
        self.stash[mb] = dict(version=v, acts=acts, labels=labels, probs=probs)
        if self.log is not None:
            # "flat": the stored output of every compute layer in description order, a block contributing its
            # branch layers (branch 0 first) and then its concatenated output
            flat, k = [], 1
            for ly in self.layers:
                if ly[0] == "softmax_xent":
                    continue
                if ly[0] == "concat":
                    for bacts in _BLOCK_CACHE[id(acts[k])]:
                        flat.extend(bacts[1:])
                flat.append(acts[k])
                k += 1
            self.log[mb] = dict(version=v, acts=acts, loss=loss, flat=flat)
        self.max_in_flight = max(self.max_in_flight, len(self.stash))
        self.trace.append(Op(OP_F, mb, v, v % self.ring))
        return acts[-1], loss

    # -- B ---------------------------------------------------------------------
    def backward(self, mb: int, dy=None, need_dx: bool = True):
        if mb != min(self.stash):
            raise RuntimeError("backward must take the oldest in-flight minibatch")
        st = self.stash.pop(mb)                                   # releases the stash (Section 4)
        v = st["version"] if self.stashing else self.latest       # same version as the forward
        P = _split_params(self.layers, self.versions[v])
        g = np.zeros_like(self.master)
        G = _split_params(self.layers, g)
        acts = st["acts"]
        d = None if dy is None else self.q(dy)
        k = len(acts) - 1                                         # index of the current layer's output
        for li in range(len(self.layers) - 1, -1, -1):
            ly = self.layers[li]
            if ly[0] == "softmax_xent":
                d = L.softmax_xent_backward(st["probs"], st["labels"], self.q)
            else:
                first = li == 0
                dx, dW, db = _layer_backward(self.layers, li, P[li], acts[k - 1], acts[k], d,
                                             need_dx or not first, self.q)
                if dW is not None:
                    _store_grad(G[li], dW, db)
                d = dx
                k -= 1
        self.grad = g
        self.trace.append(Op(OP_B, mb, v, v % self.ring))
        if self.log is not None:
            self.log[mb]["dx"] = d
        return d

    # -- U ---------------------------------------------------------------------
    def update(self, mb: int = -1):
        if self.grad is None:
            raise RuntimeError("update without a pending gradient")
        if self.optimizer == "sgd":
            self.mom = self.mu * self.mom + self.grad
            self.master = self.master - self.lr * self.mom        # onto the latest weights
        elif self.optimizer == "rmsprop":
            self.mom = self.mu * self.mom + (1.0 - self.mu) * self.grad * self.grad
            self.master = self.master - self.lr * self.grad / (np.sqrt(self.mom) + self.eps)
        else:
            raise ValueError(self.optimizer)
        self.grad = None
        self.latest += 1
        self.versions.append(self.q(self.master))
        self.trace.append(Op(OP_U, mb, self.latest, self.latest % self.ring))

    def live_versions(self):
        """Versions some in-flight minibatch still needs, plus the latest."""
        return sorted({st["version"] for st in self.stash.values()} | {self.latest})


def run_pipeline(stage_layers: Sequence, stage_params: Sequence, inputs, labels, noam_: int,
                 mode: str = "f32", lr: float = 0.01, momentum: float = 0.9,
                 stashing: bool = True, depth_override: int = 0, keep_log: bool = False,
                 out_grads=None, order: Optional[list] = None, input_grad: bool = False,
                 vertical_sync: bool = False, optimizer: str = "sgd", eps: float = 1.0,
                 stages: Optional[list] = None):
    """All stages, each following its own static op list, run as soon as their data exists.

    inputs[i] / labels[i] belong to minibatch i.  Returns (stages, losses).  Any
    order that respects the data dependencies gives the same numbers, because each
    stage's own order is fixed (Section 3.3: the policy is static).

    ``out_grads[i]``: dL/d(output) of the last stage for minibatch i when that stage
    does not end in the loss (a stage or sub-pipeline studied on its own).  ``order``,
    if a list, receives the (stage, Op) pairs in the order they were executed.
    ``input_grad``: also form dL/d(input) of stage 0 (only visible through the log).
    ``vertical_sync`` (Section 3.4): the version the input stage's forward read travels with the
    minibatch, and every later stage uses that version of its own weights instead of its latest.
    ``stages``: drained Stage objects of an earlier call to continue with (weights, momentum and version
    counters carry over; ``stage_params`` is then ignored and minibatch ids are relative to this call).
    """
    S, M = len(stage_layers), len(inputs)
    depths = [depth_override or in_flight_depth(S, noam_, s) for s in range(S)]
    if stages is None:
        stages = [Stage(stage_layers[s], stage_params[s], depths[s], mode, lr, momentum, stashing,
                        ring_depth=depths[0] if vertical_sync else 0, optimizer=optimizer, eps=eps)
                  for s in range(S)]
    assert all(not st.stash and st.grad is None for st in stages), "continue only from a drained pipeline"
    base = [st.latest for st in stages]   # versions in the static lists count from the start of this call
    if keep_log:
        for st in stages:
            st.log = {}
    lists = [schedule_1f1b(S, noam_, M, s, depth_override, vertical_sync) for s in range(S)]
    pos = [0] * S
    tag = {}     # vertical sync: mb -> version read by the input stage's forward, carried with the activation
    act = {}     # (mb, producing stage) -> activation for the next stage
    grad = {}    # (mb, producing stage) -> gradient for the previous stage
    losses: List[Optional[float]] = [None] * M
    remaining = sum(len(l) for l in lists)
    while remaining:
        progressed = False
        for s in range(S):
            while pos[s] < len(lists[s]):
                op = lists[s][pos[s]]
                st = stages[s]
                if op.kind == OP_F:
                    if s > 0 and (op.mb, s - 1) not in act:
                        break
                    x = inputs[op.mb] if s == 0 else act.pop((op.mb, s - 1))
                    y, loss = st.forward(op.mb, x, labels[op.mb] if (s == S - 1 and labels is not None) else None,
                                         version=tag[op.mb] + base[s] if (vertical_sync and s > 0) else None)
                    if s == 0:
                        tag[op.mb] = st.trace[-1].version - base[0]
                    if s == S - 1:
                        losses[op.mb] = loss
                    else:
                        act[(op.mb, s)] = y
                elif op.kind == OP_B:
                    if s < S - 1 and (op.mb, s + 1) not in grad:
                        break
                    if s == S - 1:
                        dy = None if out_grads is None else out_grads[op.mb]
                    else:
                        dy = grad.pop((op.mb, s + 1))
                    dx = st.backward(op.mb, dy, need_dx=(s > 0 or input_grad))
                    if s > 0:
                        grad[(op.mb, s)] = dx
                else:
                    st.update(op.mb)
                # the stage really did what its static list said, version included
                # (with stashing off, B deliberately reads another version than listed)
                want = Op(op.kind, op.mb, op.version + base[s], (op.version + base[s]) % st.ring)
                assert st.trace[-1] == want or (not stashing and op.kind == OP_B), (st.trace[-1], want)
                if order is not None:
                    order.append((s, op))
                pos[s] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("pipeline deadlock")
    return stages, losses


def flat_loop(stage_layers: Sequence, stage_params: Sequence, inputs, labels, depths: Sequence[int],
              mode: str = "f32", lr: float = 0.01, momentum: float = 0.9):
    """The staleness equation of Section 3.4 as a loop, with no schedule at all.

    For t = 0..M-1: every stage s contributes its weights as they were after
    max(0, t - depth_s + 1) updates; an ordinary whole-model forward and backward of
    minibatch t runs on that composite; then every stage takes one momentum-SGD
    step from its *current* weights.  (The clamp at 0 covers start-up, which the
    equation leaves out.)  Returns (history[s][t], losses).
    """
    S, M = len(stage_layers), len(inputs)
    q = L.quantiser(mode)
    master = [np.asarray(p, dtype=np.float64).copy() for p in stage_params]
    hist = [[q(master[s])] for s in range(S)]
    mom = [np.zeros_like(m) for m in master]
    losses = []
    for t in range(M):
        W = [hist[s][max(0, t - depths[s] + 1)] for s in range(S)]
        # whole-model forward
        acts_all, a = [], q(inputs[t])
        loss = probs = None
        for s in range(S):
            P = _split_params(stage_layers[s], W[s])
            acts = [a]
            for li, (ly, p) in enumerate(zip(stage_layers[s], P)):
                if ly[0] == "softmax_xent":
                    loss, probs = L.softmax_xent_forward(acts[-1], labels[t])
                else:
                    acts.append(_layer_forward(stage_layers[s], li, p, acts[-1], q))
            acts_all.append(acts)
            a = acts[-1]
        losses.append(loss)
        # whole-model backward
        d = None
        for s in range(S - 1, -1, -1):
            P = _split_params(stage_layers[s], W[s])
            g = np.zeros_like(master[s])
            G = _split_params(stage_layers[s], g)
            acts = acts_all[s]
            k = len(acts) - 1
            for li in range(len(stage_layers[s]) - 1, -1, -1):
                ly = stage_layers[s][li]
                if ly[0] == "softmax_xent":
                    d = L.softmax_xent_backward(probs, labels[t], q)
                else:
                    need_dx = not (s == 0 and li == 0)
                    dx, dW, db = _layer_backward(stage_layers[s], li, P[li], acts[k - 1], acts[k], d, need_dx, q)
                    if dW is not None:
                        _store_grad(G[li], dW, db)
                    d = dx
                    k -= 1
            mom[s] = momentum * mom[s] + g
            master[s] = master[s] - lr * mom[s]
            hist[s].append(q(master[s]))
    return hist, losses
