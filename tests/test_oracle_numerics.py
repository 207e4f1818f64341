"""Pins for the floating-point side of the oracle (layers, stashing, SGD-momentum).

None of these re-type the oracle's formulas: they use torch autograd / torch.optim.SGD
(library routines), finite differences, closed forms, and the paper's invariants.
"""
import numpy as np
import pytest
import torch

import pd_inputs as gen
from oracle import layers as L
from oracle.pipeline import Stage, flat_loop, run_pipeline
from oracle.schedule import OP_B, OP_F, in_flight_depth

SEED = gen.BASE_SEED


def _mlp(hidden=12, classes=5, stages=4):
    return gen.config1_mlp(hidden, classes, stages)


def _data(M, B, hidden, classes, seed=SEED):
    xs = [gen.normal(seed, f"x{i}", (B, hidden)).astype(np.float64) for i in range(M)]
    ys = [gen.labels(seed, f"y{i}", (B,), classes) for i in range(M)]
    return xs, ys


def _params(stage_layers, seed=SEED):
    ps = [gen.init_params(seed, f"stage{s}", ly).astype(np.float64) for s, ly in enumerate(stage_layers)]
    # non-zero biases so that a dropped bias term is visible
    out = []
    for s, (p, ly) in enumerate(zip(ps, stage_layers)):
        p = p + 0.05 * gen.normal(seed, f"pert{s}", p.shape).astype(np.float64)
        out.append(p)
    return out


# ---- bf16 rounding -----------------------------------------------------------

def test_round_bf16_matches_torch_and_ties_to_even():
    x = gen.normal(SEED, "r", (4096,)).astype(np.float32) * np.float32(37.0)
    ours = L.round_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ours, ref)
    # exact ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert L.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert L.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert L.round_bf16(np.array([-0.0, 0.0, 256.0, 1e-30])).tolist()[:3] == [0.0, 0.0, 256.0]


# ---- layer maths against autograd and finite differences ----------------------

def _torch_model_loss(params, stage_layers, x, y):
    a = x
    for p, layers in zip(params, stage_layers):
        o = 0
        for ly in layers:
            if ly[0] == "linear":
                W = p[o:o + ly[1] * ly[2]].view(ly[2], ly[1]); o += ly[1] * ly[2]
                b = p[o:o + ly[2]]; o += ly[2]
                a = torch.nn.functional.linear(a, W, b)
                if ly[3]:
                    a = torch.relu(a)
            elif ly[0] == "softmax_xent":
                return torch.nn.functional.cross_entropy(a, y, reduction="mean")
    raise AssertionError


def test_single_stage_gradients_match_autograd():
    layers = [("linear", 7, 6, True), ("linear", 6, 5, True), ("linear", 5, 4, False), ("softmax_xent", 4)]
    p0 = _params([layers])[0]
    x = gen.normal(SEED, "gx", (9, 7)).astype(np.float64)
    y = gen.labels(SEED, "gy", (9,), 4)
    st = Stage(layers, p0, depth=1)
    _, loss = st.forward(0, x, y)
    dx = st.backward(0, None, need_dx=True)
    tp = torch.tensor(p0, requires_grad=True)
    tx = torch.tensor(x, requires_grad=True)
    tl = _torch_model_loss([tp], [layers], tx, torch.tensor(y, dtype=torch.long))
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    assert np.allclose(st.grad, tp.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_finite_differences():
    layers = [("linear", 5, 3, True), ("linear", 3, 4, False), ("softmax_xent", 4)]
    p0 = _params([layers], seed=SEED + 3)[0]
    x = gen.normal(SEED, "fx", (6, 5)).astype(np.float64)
    y = gen.labels(SEED, "fy", (6,), 4)

    def loss_at(p):
        st = Stage(layers, p, depth=1)
        return st.forward(0, x, y)[1]

    st = Stage(layers, p0, depth=1)
    st.forward(0, x, y)
    st.backward(0, None)
    h = 1e-6
    for k in range(p0.size):
        e = np.zeros_like(p0); e[k] = h
        fd = (loss_at(p0 + e) - loss_at(p0 - e)) / (2 * h)
        assert abs(fd - st.grad[k]) < 1e-7 * max(1.0, abs(fd)), k


def test_softmax_xent_closed_forms():
    # uniform logits: loss = log(C), gradient = (1/C - onehot)/rows
    C, R = 7, 3
    z = np.full((R, C), 2.5)
    y = np.array([0, 3, 6])
    loss, p = L.softmax_xent_forward(z, y)
    assert abs(loss - np.log(C)) < 1e-14
    d = L.softmax_xent_backward(p, y, L.quantiser("f32"))
    assert np.allclose(d.sum(axis=1), 0.0, atol=1e-15)
    assert np.allclose(d[0], (np.full(C, 1 / C) - np.eye(C)[0]) / R)
    # huge logits do not overflow (max subtraction)
    z = np.array([[1000.0, 0.0], [0.0, 1000.0]])
    loss, _ = L.softmax_xent_forward(z, np.array([0, 1]))
    assert abs(loss) < 1e-12


# ---- S = 1 / NOAM = 1 reduce to sequential minibatch SGD (library routine) ----

def _torch_sequential_sgd(stage_layers, params, xs, ys, lr, mu):
    tps = [torch.tensor(p, requires_grad=True) for p in params]
    opt = torch.optim.SGD(tps, lr=lr, momentum=mu)
    losses = []
    for x, y in zip(xs, ys):
        opt.zero_grad()
        l = _torch_model_loss(tps, stage_layers, torch.tensor(x), torch.tensor(y, dtype=torch.long))
        l.backward()
        opt.step()
        losses.append(l.item())
    return [p.detach().numpy() for p in tps], losses


@pytest.mark.parametrize("S,NOAM", [(1, 1), (4, 1), (3, 1)])
def test_reduces_to_sequential_sgd(S, NOAM):
    sl = _mlp(stages=S) if S > 1 else [[("linear", 12, 12, True), ("linear", 12, 5, False), ("softmax_xent", 5)]]
    params = _params(sl)
    xs, ys = _data(10, 6, 12, 5)
    stages, losses = run_pipeline(sl, params, xs, ys, NOAM, lr=0.05, momentum=0.9)
    ref_p, ref_l = _torch_sequential_sgd(sl, params, xs, ys, 0.05, 0.9)
    assert np.allclose(losses, ref_l, rtol=1e-11)
    for st, rp in zip(stages, ref_p):
        assert np.allclose(st.master, rp, rtol=1e-10, atol=1e-13)


def test_continuing_a_drained_pipeline_keeps_weights_momentum_and_versions():
    """run_pipeline(stages=...) continues with drained stages.  Pin: with one stage (or NOAM 1) nothing is ever stale,
    so two runs of 5 minibatches back to back are the sequential momentum SGD over all 10 (torch.optim.SGD); for a
    real pipeline the second run equals a fresh run started from the first run's weights AND momentum (set by hand)."""
    sl = [[("linear", 12, 12, True), ("linear", 12, 5, False), ("softmax_xent", 5)]]
    params = _params(sl)
    xs, ys = _data(10, 6, 12, 5)
    st, l1 = run_pipeline(sl, params, xs[:5], ys[:5], 1, lr=0.05, momentum=0.9)
    st, l2 = run_pipeline(sl, None, xs[5:], ys[5:], 1, lr=0.05, momentum=0.9, stages=st)
    ref_p, ref_l = _torch_sequential_sgd(sl, params, xs, ys, 0.05, 0.9)
    assert np.allclose(list(l1) + list(l2), ref_l, rtol=1e-11)
    assert np.allclose(st[0].master, ref_p[0], rtol=1e-10, atol=1e-13) and st[0].latest == 10
    assert [o.version for o in st[0].trace if o.kind == OP_F] == list(range(10))
    sl = _mlp(stages=3)
    params = _params(sl)
    a, _ = run_pipeline(sl, params, xs[:5], ys[:5], 3, lr=0.05, momentum=0.9)
    w, m = [x.master.copy() for x in a], [x.mom.copy() for x in a]
    a, la = run_pipeline(sl, None, xs[5:], ys[5:], 3, lr=0.05, momentum=0.9, stages=a)
    fresh = [Stage(sl[s], w[s], in_flight_depth(3, 3, s), "f32", 0.05, 0.9) for s in range(3)]
    for f, mm in zip(fresh, m):
        f.mom = mm
    b, lb = run_pipeline(sl, None, xs[5:], ys[5:], 3, lr=0.05, momentum=0.9, stages=fresh)
    assert la == lb
    for x, y in zip(a, b):
        assert np.array_equal(x.master, y.master) and np.array_equal(x.mom, y.mom) and x.latest == y.latest + 5


# ---- the staleness equation as an independent flat loop (autograd layers) -----

def _torch_flat_loop(stage_layers, params, xs, ys, depths, lr, mu):
    S = len(stage_layers)
    cur = [torch.tensor(p) for p in params]
    hist = [[c.clone()] for c in cur]
    mom = [torch.zeros_like(c) for c in cur]
    losses = []
    for t, (x, y) in enumerate(zip(xs, ys)):
        comp = [hist[s][max(0, t - depths[s] + 1)].clone().requires_grad_(True) for s in range(S)]
        l = _torch_model_loss(comp, stage_layers, torch.tensor(x), torch.tensor(y, dtype=torch.long))
        l.backward()
        losses.append(l.item())
        for s in range(S):
            mom[s] = mu * mom[s] + comp[s].grad
            cur[s] = cur[s] - lr * mom[s]
            hist[s].append(cur[s].clone())
    return [c.numpy() for c in cur], losses


@pytest.mark.parametrize("S,NOAM", [(4, 4), (3, 3), (4, 2), (2, 2)])
def test_event_driven_equals_staleness_equation(S, NOAM):
    sl = _mlp(stages=S)
    params = _params(sl)
    M = 14
    xs, ys = _data(M, 6, 12, 5)
    depths = [in_flight_depth(S, NOAM, s) for s in range(S)]
    stages, losses = run_pipeline(sl, params, xs, ys, NOAM, lr=0.05, momentum=0.9)
    # (a) torch autograd, no schedule, composite weights from history
    ref_p, ref_l = _torch_flat_loop(sl, params, xs, ys, depths, 0.05, 0.9)
    assert np.allclose(losses, ref_l, rtol=1e-11)
    for st, rp in zip(stages, ref_p):
        assert np.allclose(st.master, rp, rtol=1e-10, atol=1e-13)
    # (b) the oracle's own flat loop (same layer routines): identical to the last bit
    hist, l2 = flat_loop(sl, params, xs, ys, depths, lr=0.05, momentum=0.9)
    assert l2 == losses
    for s, st in enumerate(stages):
        assert len(hist[s]) == M + 1 == len(st.versions)
        for a, b in zip(hist[s], st.versions):
            assert np.array_equal(a, b)


def test_bf16_mode_flat_loop_bit_identical_and_close_to_f32():
    sl = _mlp(stages=4)
    params = _params(sl)
    M = 10
    xs, ys = _data(M, 6, 12, 5)
    depths = [in_flight_depth(4, 4, s) for s in range(4)]
    st_b, loss_b = run_pipeline(sl, params, xs, ys, 4, mode="bf16")
    hist, l2 = flat_loop(sl, params, xs, ys, depths, mode="bf16")
    assert l2 == loss_b
    for s in range(4):
        assert np.array_equal(hist[s][-1], st_b[s].versions[-1])
        # every stored version is exactly representable in bfloat16
        v = st_b[s].versions[-1]
        assert np.array_equal(v, L.round_bf16(v))
    st_f, loss_f = run_pipeline(sl, params, xs, ys, 4, mode="f32")
    assert np.allclose(loss_b, loss_f, rtol=2e-2)


# ---- weight stashing: same version for F and B; negative control ---------------

def test_same_version_invariant_and_bounds():
    sl = _mlp(stages=4)
    params = _params(sl)
    xs, ys = _data(12, 6, 12, 5)
    stages, _ = run_pipeline(sl, params, xs, ys, 4)
    for s, st in enumerate(stages):
        f = {o.mb: o.version for o in st.trace if o.kind == OP_F}
        b = {o.mb: o.version for o in st.trace if o.kind == OP_B}
        assert f == b
        assert st.max_in_flight == 4 - s               # input stage NOAM, output stage 1 (Section 3.5)
        assert st.latest == 12 and not st.stash


def test_without_stashing_differs_and_breaks_invariant():
    sl = _mlp(stages=4)
    params = _params(sl)
    xs, ys = _data(12, 6, 12, 5)
    on, l_on = run_pipeline(sl, params, xs, ys, 4, stashing=True)
    off, l_off = run_pipeline(sl, params, xs, ys, 4, stashing=False)
    for s in range(3):       # stages with interleaved updates
        f = {o.mb: o.version for o in off[s].trace if o.kind == OP_F}
        b = {o.mb: o.version for o in off[s].trace if o.kind == OP_B}
        assert any(f[i] != b[i] for i in f)
        assert not np.allclose(on[s].master, off[s].master, rtol=1e-6)
    # the output stage has no interleaved update: its first gradient is the same either way
    assert l_on[0] == l_off[0]


def test_update_applies_to_latest_not_stashed():
    # one stage with depth 2 (forced): after F0 F1 B0 U, B1 computes its gradient on version 0,
    # but the update lands on version 1: w2 = w1 - lr*(mu*m1 + g1(w0)).
    layers = [("linear", 4, 3, False), ("softmax_xent", 3)]
    p0 = _params([layers])[0]
    xs, ys = _data(2, 5, 4, 3)
    st = Stage(layers, p0, depth=2, lr=0.1, momentum=0.5)
    st.forward(0, xs[0], ys[0]); st.forward(1, xs[1], ys[1])
    st.backward(0); g0 = st.grad.copy(); st.update()
    st.backward(1); g1 = st.grad.copy(); st.update()
    ref = Stage(layers, p0, depth=1); ref.forward(1, xs[1], ys[1]); ref.backward(1)
    assert np.array_equal(g1, ref.grad)                 # gradient at w0 (stashed)
    m1 = g0; w1 = p0 - 0.1 * m1
    m2 = 0.5 * m1 + g1; w2 = w1 - 0.1 * m2
    assert np.allclose(st.master, w2, rtol=1e-14)
    assert [o.version for o in st.trace if o.kind in (OP_F, OP_B)] == [0, 0, 0, 0]


# ---- vertical sync (Section 3.4): one version per minibatch across all stages --------------------

@pytest.mark.parametrize("S,NOAM", [(4, 4), (3, 3), (4, 2), (2, 2), (3, 1)])
def test_vertical_sync_equals_its_staleness_equation(S, NOAM):
    # with vertical sync the update uses w^(t-n+1) on EVERY stage: the flat loops with one common delay
    sl = _mlp(stages=S)
    params = _params(sl)
    M = 14
    xs, ys = _data(M, 6, 12, 5)
    common = [in_flight_depth(S, NOAM, 0)] * S
    stages, losses = run_pipeline(sl, params, xs, ys, NOAM, lr=0.05, momentum=0.9, vertical_sync=True)
    ref_p, ref_l = _torch_flat_loop(sl, params, xs, ys, common, 0.05, 0.9)
    assert np.allclose(losses, ref_l, rtol=1e-11)
    for st, rp in zip(stages, ref_p):
        assert np.allclose(st.master, rp, rtol=1e-10, atol=1e-13)
    hist, l2 = flat_loop(sl, params, xs, ys, common, lr=0.05, momentum=0.9)
    assert l2 == losses
    for s, st in enumerate(stages):
        for a, b in zip(hist[s], st.versions):
            assert np.array_equal(a, b)
    # every stage read the SAME version for a given minibatch, forward and backward
    for mb in range(M):
        seen = {o.version for st in stages for o in st.trace if o.mb == mb and o.kind in (0, 1)}
        assert len(seen) == 1
    if S > 1 and NOAM > 1:   # and it is a different iteration from plain weight stashing
        plain, _ = run_pipeline(sl, params, xs, ys, NOAM, lr=0.05, momentum=0.9)
        assert not np.allclose(plain[-1].master, stages[-1].master, rtol=1e-9, atol=0)


def test_vertical_sync_worked_example_and_ring():
    # Section 3.4's example: with vertical sync, minibatch 5 uses the parameters updated by minibatch 1
    # on all machines (4 stages, NOAM 4; 0-based: minibatch 4 reads version 1 everywhere)
    from oracle.schedule import schedule_1f1b
    S, NOAM, M = 4, 4, 12
    for s in range(S):
        ops = schedule_1f1b(S, NOAM, M, s, vertical_sync=True)
        plain = schedule_1f1b(S, NOAM, M, s)
        assert [(o.kind, o.mb) for o in ops] == [(o.kind, o.mb) for o in plain]      # same op order
        for o in ops:
            if o.kind in (0, 1):
                assert o.version == max(0, o.mb - NOAM + 1)
                if o.mb == 4:
                    assert o.version == 1
        # a ring of NOAM slots never overwrites a version that is still needed
        held = {}
        for o in ops:
            if o.kind == 2:
                held[o.version % NOAM] = o.version
            elif o.version > 0:
                assert held[o.slot] == o.version
    # the stage refuses a version it no longer holds
    sl = _mlp(stages=2)
    st = Stage(sl[0], _params(sl)[0], depth=1, ring_depth=2)
    x, _ = _data(1, 6, 12, 5)
    for mb in range(3):
        st.forward(mb, x[0])
        st.backward(mb, np.zeros((6, 12)), need_dx=False)
        st.update(mb)
    st.forward(3, x[0], version=2)
    st.backward(3, np.zeros((6, 12)), need_dx=False)
    st.update(3)
    with pytest.raises(RuntimeError):
        st.forward(4, x[0], version=2)      # latest is 4, the ring holds 3 and 4
    with pytest.raises(RuntimeError):
        st.forward(4, x[0], version=5)


# ---- RMSProp (the paper's optimiser for Inception-v3, Section 5.1): library routine on the sequential case ----

@pytest.mark.parametrize("alpha,eps", [(0.9, 1.0), (0.99, 1e-8)])
def test_rmsprop_reduces_to_the_library_routine(alpha, eps):
    sl = [[("linear", 12, 12, True), ("linear", 12, 5, False), ("softmax_xent", 5)]]
    params = _params(sl)
    xs, ys = _data(9, 6, 12, 5)
    stages, losses = run_pipeline(sl, params, xs, ys, 1, lr=0.045, momentum=alpha, optimizer="rmsprop", eps=eps)
    tps = [torch.tensor(p, requires_grad=True) for p in params]
    opt = torch.optim.RMSprop(tps, lr=0.045, alpha=alpha, eps=eps)
    ref_l = []
    for x, y in zip(xs, ys):
        opt.zero_grad()
        l = _torch_model_loss(tps, sl, torch.tensor(x), torch.tensor(y, dtype=torch.long))
        l.backward()
        opt.step()
        ref_l.append(l.item())
    assert np.allclose(losses, ref_l, rtol=1e-10)
    assert np.allclose(stages[0].master, tps[0].detach().numpy(), rtol=1e-9, atol=1e-12)
    # hand value of one step: v = (1 - a) g^2, w' = w - lr g / (sqrt(v) + eps)
    st = Stage(sl[0], params[0], depth=1, lr=0.045, momentum=alpha, optimizer="rmsprop", eps=eps)
    st.forward(0, xs[0], ys[0]); st.backward(0, None, need_dx=False)
    g = st.grad.copy()
    st.update(0)
    assert np.allclose(st.mom, (1 - alpha) * g * g, rtol=1e-15)
    assert np.allclose(st.master, params[0] - 0.045 * g / (np.sqrt((1 - alpha) * g * g) + eps), rtol=1e-14)
