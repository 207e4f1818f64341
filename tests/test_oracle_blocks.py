"""Pins for the oracle's average pooling, overlapping max pooling and branched (concatenation) blocks:
library routines with autograd in fp64, finite differences, hand cases, the bf16 rounding points."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import pd_inputs as gen
from oracle import layers as L
from oracle.pipeline import Stage, run_pipeline

SEED = gen.BASE_SEED + 4
ID = L.quantiser("f32")


def _nchw(a):
    return torch.tensor(np.ascontiguousarray(a.transpose(0, 3, 1, 2)))


def _nhwc(t):
    return t.detach().numpy().transpose(0, 2, 3, 1)


@pytest.mark.parametrize("k,stride,pad,hw", [(3, 1, 1, (7, 6)), (3, 2, 0, (9, 7)), (2, 2, 0, (8, 6)), (5, 1, 0, (5, 5)),
                                             (3, 2, 1, (8, 8))])
def test_avgpool_matches_torch(k, stride, pad, hw):
    x = gen.normal(SEED, "ax", (2, hw[0], hw[1], 3)).astype(np.float64)
    y = L.avgpool2d_forward(x, k, stride, pad, ID)
    tx = _nchw(x).requires_grad_(True)
    ty = F.avg_pool2d(tx, k, stride, pad, count_include_pad=True)
    assert np.allclose(y, _nhwc(ty), rtol=1e-13, atol=1e-13)
    dy = gen.normal(SEED, "ady", y.shape).astype(np.float64)
    ty.backward(_nchw(dy))
    assert np.allclose(L.avgpool2d_backward(x.shape, dy, k, stride, pad, ID), _nhwc(tx.grad), rtol=1e-13, atol=1e-13)


def test_avgpool_hand_cases():
    x = np.arange(16, dtype=np.float64).reshape(1, 4, 4, 1)
    # global average: one output, the mean; its gradient spreads evenly
    y = L.avgpool2d_forward(x, 4, 1, 0, ID)
    assert y.shape == (1, 1, 1, 1) and y[0, 0, 0, 0] == 7.5
    assert np.array_equal(L.avgpool2d_backward(x.shape, np.full((1, 1, 1, 1), 16.0), 4, 1, 0, ID), np.ones_like(x))
    # padding counts in the divisor: the corner window of a 3x3/pad-1 pooling sees 4 values, divides by 9
    y = L.avgpool2d_forward(x, 3, 1, 1, ID)
    assert abs(y[0, 0, 0, 0] - (0 + 1 + 4 + 5) / 9.0) < 1e-15


@pytest.mark.parametrize("k,stride,hw", [(3, 2, (9, 7)), (3, 1, (6, 6)), (2, 1, (5, 4)), (3, 2, (35, 35))])
def test_overlapping_maxpool_matches_torch(k, stride, hw):
    x = gen.normal(SEED, "mx", (2, hw[0], hw[1], 3)).astype(np.float64)      # continuous values: no ties
    y = L.maxpool2d_forward(x, k, stride)
    tx = _nchw(x).requires_grad_(True)
    ty = F.max_pool2d(tx, k, stride)
    assert np.array_equal(y, _nhwc(ty))
    dy = gen.normal(SEED, "mdy", y.shape).astype(np.float64)
    ty.backward(_nchw(dy))
    assert np.allclose(L.maxpool2d_backward(x, y, dy, k, stride), _nhwc(tx.grad), rtol=1e-13, atol=1e-13)


def test_overlapping_maxpool_sums_and_first_max():
    # 1x3 row, window 2, stride 1: the middle element is the maximum of both windows and receives both gradients
    x = np.array([1.0, 5.0, 2.0]).reshape(1, 1, 3, 1)
    x = np.concatenate([x, x - 10.0], axis=1)          # second row lower everywhere, window spans both rows
    y = L.maxpool2d_forward(x, 2, 1)
    dx = L.maxpool2d_backward(x, y, np.array([3.0, 4.0]).reshape(1, 1, 2, 1), 2, 1)
    assert dx[0, 0, 1, 0] == 7.0 and dx.sum() == 7.0
    # a tie inside one window: the first position in row-major order takes it
    x = np.zeros((1, 3, 3, 1)); x[0, 0, 2, 0] = x[0, 2, 0, 0] = 9.0
    y = L.maxpool2d_forward(x, 3, 1)
    dx = L.maxpool2d_backward(x, y, np.ones((1, 1, 1, 1)), 3, 1)
    assert dx[0, 0, 2, 0] == 1.0 and dx[0, 2, 0, 0] == 0.0


def _block_stage():
    """A small Inception-like stage: stem conv, a four-branch block (1x1 | 1x1-3x3 | 1x7-7x1 | avgpool-1x1), a
    reduction block (strided conv | 1x1-strided conv | overlapping max pool), global average, classifier."""
    blk1 = ("concat", [[("conv2d", 4, 3, 1, 1, 1, 0, 0, True)],
                       [("conv2d", 4, 2, 1, 1, 1, 0, 0, True), ("conv2d", 2, 3, 3, 3, 1, 1, 1, True)],
                       [("conv2d", 4, 2, 1, 7, 1, 0, 3, True), ("conv2d", 2, 2, 7, 1, 1, 3, 0, True)],
                       [("avgpool2d", 3, 1, 1), ("conv2d", 4, 2, 1, 1, 1, 0, 0, True)]])
    blk2 = ("concat", [[("conv2d", 10, 4, 3, 3, 2, 0, 0, True)],
                       [("conv2d", 10, 3, 1, 1, 1, 0, 0, True), ("conv2d", 3, 4, 3, 3, 2, 0, 0, True)],
                       [("maxpool2d", 3, 2)]])
    return [("conv2d", 3, 4, 3, 3, 1, 1, 1, True), blk1, blk2, ("avgpool2d", 3, 1, 0), ("linear", 18, 5, False),
            ("softmax_xent", 5)]


def _torch_layers(p, layers, a, o=0):
    """Runs `layers` on NCHW tensor `a` with parameters taken from flat vector p at offset o; returns (a, o)."""
    for ly in layers:
        if ly[0] == "conv2d":
            n = ly[2] * ly[3] * ly[4] * ly[1]
            W = p[o:o + n].view(ly[2], ly[3], ly[4], ly[1]).permute(0, 3, 1, 2); o += n
            b = p[o:o + ly[2]]; o += ly[2]
            a = F.conv2d(a, W, b, stride=ly[5], padding=(ly[6], ly[7]))
            if ly[8]:
                a = torch.relu(a)
        elif ly[0] == "maxpool2d":
            a = F.max_pool2d(a, ly[1], ly[2])
        elif ly[0] == "avgpool2d":
            a = F.avg_pool2d(a, ly[1], ly[2], ly[3], count_include_pad=True)
        elif ly[0] == "concat":
            outs = []
            for br in ly[1]:
                t, o = _torch_layers(p, br, a, o)
                outs.append(t)
            a = torch.cat(outs, dim=1)
        elif ly[0] == "linear":
            if a.dim() == 4:
                a = a.permute(0, 2, 3, 1).reshape(a.shape[0], -1)
            W = p[o:o + ly[1] * ly[2]].view(ly[2], ly[1]); o += ly[1] * ly[2]
            b = p[o:o + ly[2]]; o += ly[2]
            a = F.linear(a, W, b)
    return a, o


def _torch_loss(p, layers, x, y):
    z, o = _torch_layers(p, [l for l in layers if l[0] != "softmax_xent"], x)
    assert o == p.numel()
    return F.cross_entropy(z, y)


def _data(M, hw=7):
    layers = _block_stage()
    p0 = gen.init_params(SEED, "bp", layers).astype(np.float64)
    p0 = p0 + 0.05 * gen.normal(SEED, "bpp", p0.shape)
    assert p0.size == gen.param_count(layers)
    xs = [gen.normal(SEED, f"bx{i}", (3, hw, hw, 3)).astype(np.float64) for i in range(M)]
    ys = [gen.labels(SEED, f"by{i}", (3,), 5) for i in range(M)]
    return layers, p0, xs, ys


def test_block_stage_gradient_matches_autograd():
    layers, p0, xs, ys = _data(1)
    st = Stage(layers, p0, depth=1)
    st.log = {}
    _, loss = st.forward(0, xs[0], ys[0])
    # the block's output is the concatenation of its branch outputs, branch 0 first (3 + 3 + 2 + 2 channels)
    flat = st.log[0]["flat"]
    assert [a.shape[-1] for a in flat[1:8]] == [3, 2, 3, 2, 2, 4, 2] and flat[8].shape[-1] == 10
    assert np.array_equal(flat[8], np.concatenate([flat[1], flat[3], flat[5], flat[7]], axis=-1))
    dx = st.backward(0, None, need_dx=True)
    tp = torch.tensor(p0, requires_grad=True)
    tx = _nchw(xs[0]).requires_grad_(True)
    tl = _torch_loss(tp, layers, tx, torch.tensor(ys[0], dtype=torch.long)); tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    assert np.allclose(st.grad, tp.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(dx, _nhwc(tx.grad), rtol=1e-9, atol=1e-12)


def test_block_stage_is_sequential_sgd_at_depth_one():
    layers, p0, xs, ys = _data(4)
    stages, losses = run_pipeline([layers], [p0], xs, ys, 1, lr=0.05, momentum=0.9)
    tp = torch.tensor(p0, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=0.05, momentum=0.9)
    for i in range(4):
        opt.zero_grad()
        l = _torch_loss(tp, layers, _nchw(xs[i]), torch.tensor(ys[i], dtype=torch.long)); l.backward(); opt.step()
        assert abs(l.item() - losses[i]) < 1e-10
    assert np.allclose(stages[0].master, tp.detach().numpy(), rtol=1e-9, atol=1e-12)


def test_block_finite_differences():
    layers, p0, xs, ys = _data(1)
    st = Stage(layers, p0, depth=1); st.forward(0, xs[0], ys[0]); st.backward(0, None)
    h = 1e-6
    for k in range(0, p0.size, 7):
        e = np.zeros_like(p0); e[k] = h
        fp = Stage(layers, p0 + e, depth=1).forward(0, xs[0], ys[0])[1]
        fm = Stage(layers, p0 - e, depth=1).forward(0, xs[0], ys[0])[1]
        fd = (fp - fm) / (2 * h)
        assert abs(fd - st.grad[k]) < 5e-7 * max(1.0, abs(fd)), k


def test_block_split_across_two_stages_equals_flat_staleness_loop():
    """A block stage feeding a second stage under 1F1B with stashing equals the delayed-gradient loop."""
    from oracle.pipeline import flat_loop
    layers, p0, xs, ys = _data(6)
    s0, s1 = layers[:2], layers[2:]
    n0 = gen.param_count(s0)
    stages, losses = run_pipeline([s0, s1], [p0[:n0], p0[n0:]], xs, ys, 2, lr=0.05)
    hist, fl = flat_loop([s0, s1], [p0[:n0], p0[n0:]], xs, ys, [2, 1], lr=0.05)
    assert np.allclose(losses, fl, rtol=1e-12, atol=0)
    for s in range(2):
        assert np.allclose(stages[s].master, hist[s][-1], rtol=1e-12, atol=1e-14)


def test_block_bf16_rounding_points():
    """bf16 mode: every stored tensor of the block is representable in bfloat16, and the block's input gradient is
    the once-rounded sum of the branches' (already rounded) input gradients."""
    layers, p0, xs, ys = _data(1)
    st = Stage(layers, p0, depth=1, mode="bf16")
    st.log = {}
    st.forward(0, xs[0], ys[0])
    for a in st.log[0]["flat"][:-1]:             # all but the logits
        assert np.array_equal(a, L.round_bf16(a))
    dx = st.backward(0, None, need_dx=True)
    assert np.array_equal(dx, L.round_bf16(dx))
    # sum of two bf16 numbers that is not a bf16 number: rounded once, to nearest even
    q = L.quantiser("bf16")
    a, b = np.array([1.0]), np.array([2.0 ** -8])        # 1 + 2^-8 lies half-way between 1 and 1 + 2^-7
    assert q(a + b)[0] == 1.0
