"""Pins for the oracle's convolution and pooling (library routines, finite differences, hand cases)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import pd_inputs as gen
from oracle import layers as L
from oracle.pipeline import Stage, run_pipeline

SEED = gen.BASE_SEED + 2
ID = L.quantiser("f32")


def _nchw(a):  # NHWC numpy -> NCHW torch
    return torch.tensor(np.ascontiguousarray(a.transpose(0, 3, 1, 2)))


def _nhwc(t):
    return t.detach().numpy().transpose(0, 2, 3, 1)


@pytest.mark.parametrize("k,stride,pad,relu", [(3, 1, 1, True), (3, 1, 1, False), (1, 1, 0, True), (3, 2, 1, True),
                                               ((1, 7), 1, (0, 3), True), ((7, 1), 1, (3, 0), False)])
def test_conv2d_matches_torch(k, stride, pad, relu):
    kh, kw = (k, k) if isinstance(k, int) else k
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    N, H, Wd, Ci, Co = 2, 9, 8, 3, 5
    x = gen.normal(SEED, "x", (N, H, Wd, Ci)).astype(np.float64)
    W = gen.normal(SEED, "w", (Co, kh, kw, Ci)).astype(np.float64) * 0.3
    b = gen.normal(SEED, "b", (Co,)).astype(np.float64)
    y = L.conv2d_forward(x, W, b, stride, ph, pw, relu, ID)
    tx = _nchw(x).requires_grad_(True)
    tw = torch.tensor(np.ascontiguousarray(W.transpose(0, 3, 1, 2))).requires_grad_(True)   # [Co][Ci][kh][kw]
    tb = torch.tensor(b).requires_grad_(True)
    ty = F.conv2d(tx, tw, tb, stride=stride, padding=(ph, pw))
    if relu:
        ty = torch.relu(ty)
    assert np.allclose(y, _nhwc(ty), rtol=1e-12, atol=1e-12)
    dy = gen.normal(SEED, "dy", y.shape).astype(np.float64)
    ty.backward(_nchw(dy))
    dx, dW, db = L.conv2d_backward(x, W, y, dy, stride, ph, pw, relu, True, ID)
    assert np.allclose(dx, _nhwc(tx.grad), rtol=1e-11, atol=1e-12)
    assert np.allclose(dW, tw.grad.numpy().transpose(0, 2, 3, 1), rtol=1e-11, atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_maxpool_matches_torch_and_first_max_rule():
    x = gen.normal(SEED, "px", (2, 8, 6, 3)).astype(np.float64)
    y = L.maxpool2d_forward(x, 2, 2)
    tx = _nchw(x).requires_grad_(True)
    ty = F.max_pool2d(tx, 2, 2)
    assert np.array_equal(y, _nhwc(ty))
    dy = gen.normal(SEED, "pdy", y.shape).astype(np.float64)
    ty.backward(_nchw(dy))
    assert np.array_equal(L.maxpool2d_backward(x, y, dy, 2, 2), _nhwc(tx.grad))
    # ties: the first maximum in row-major window order takes the whole gradient
    x = np.zeros((1, 2, 2, 1)); x[0, 0, 1, 0] = 5.0; x[0, 1, 0, 0] = 5.0
    y = L.maxpool2d_forward(x, 2, 2)
    dx = L.maxpool2d_backward(x, y, np.full(y.shape, 3.0), 2, 2)
    assert y[0, 0, 0, 0] == 5.0 and dx[0, 0, 1, 0] == 3.0 and dx[0, 1, 0, 0] == 0.0 and dx.sum() == 3.0
    x = np.zeros((1, 2, 2, 1))      # all equal: position (0,0)
    dx = L.maxpool2d_backward(x, L.maxpool2d_forward(x, 2, 2), np.ones((1, 1, 1, 1)), 2, 2)
    assert dx[0, 0, 0, 0] == 1.0 and dx.sum() == 1.0


def _vgg_like():
    return [("conv2d", 3, 4, 3, 3, 1, 1, 1, True), ("conv2d", 4, 4, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2),
            ("conv2d", 4, 6, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2), ("linear", 2 * 2 * 6, 5, False),
            ("softmax_xent", 5)]


def _torch_loss(p, layers, x, y):
    a = x          # NCHW
    o = 0
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
        elif ly[0] == "linear":
            if a.dim() == 4:
                a = a.permute(0, 2, 3, 1).reshape(a.shape[0], -1)       # NHWC flatten order
            W = p[o:o + ly[1] * ly[2]].view(ly[2], ly[1]); o += ly[1] * ly[2]
            b = p[o:o + ly[2]]; o += ly[2]
            a = F.linear(a, W, b)
        elif ly[0] == "softmax_xent":
            return F.cross_entropy(a, y)


def test_conv_stage_gradients_and_sequential_sgd():
    layers = _vgg_like()
    p0 = gen.init_params(SEED, "p", layers).astype(np.float64)
    p0 = p0 + 0.05 * gen.normal(SEED, "pp", p0.shape)
    M = 4
    xs = [gen.normal(SEED, f"x{i}", (3, 8, 8, 3)).astype(np.float64) for i in range(M)]
    ys = [gen.labels(SEED, f"y{i}", (3,), 5) for i in range(M)]
    # gradient of one minibatch against autograd
    st = Stage(layers, p0, depth=1)
    _, loss = st.forward(0, xs[0], ys[0]); st.backward(0, None, need_dx=True)
    tp = torch.tensor(p0, requires_grad=True)
    tl = _torch_loss(tp, layers, _nchw(xs[0]), torch.tensor(ys[0], dtype=torch.long)); tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    assert np.allclose(st.grad, tp.grad.numpy(), rtol=1e-9, atol=1e-12)
    # one stage, depth 1: plain sequential momentum SGD
    stages, losses = run_pipeline([layers], [p0], xs, ys, 1, lr=0.05, momentum=0.9)
    tp = torch.tensor(p0, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=0.05, momentum=0.9)
    for i in range(M):
        opt.zero_grad()
        l = _torch_loss(tp, layers, _nchw(xs[i]), torch.tensor(ys[i], dtype=torch.long)); l.backward(); opt.step()
        assert abs(l.item() - losses[i]) < 1e-10
    assert np.allclose(stages[0].master, tp.detach().numpy(), rtol=1e-9, atol=1e-12)


def test_conv_finite_differences():
    layers = [("conv2d", 2, 3, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2), ("linear", 2 * 2 * 3, 3, False),
              ("softmax_xent", 3)]
    p0 = gen.init_params(SEED + 5, "p", layers).astype(np.float64) + 0.1 * gen.normal(SEED, "q", (gen.param_count(layers),))
    x = gen.normal(SEED, "fx", (2, 4, 4, 2)).astype(np.float64)
    y = gen.labels(SEED, "fy", (2,), 3)
    st = Stage(layers, p0, depth=1); st.forward(0, x, y); st.backward(0, None)
    h = 1e-6
    for k in range(0, p0.size, 3):
        e = np.zeros_like(p0); e[k] = h
        fp = Stage(layers, p0 + e, depth=1).forward(0, x, y)[1]
        fm = Stage(layers, p0 - e, depth=1).forward(0, x, y)[1]
        fd = (fp - fm) / (2 * h)
        assert abs(fd - st.grad[k]) < 2e-7 * max(1.0, abs(fd)), k


def test_sampled_patches_equal_the_whole_convolution():
    # the helpers the full-size GPU tests use to get single outputs from the oracle, against the oracle run whole
    from sampling import conv_dx_at, conv_y_at, positions
    N, H, W, ci, co = 3, 6, 7, 5, 4
    x = L.round_bf16(gen.normal(SEED, "sx", (N, H, W, ci)))
    w = L.round_bf16(gen.uniform(SEED, "sw", (co, 3, 3, ci), -0.3, 0.3))
    b = L.round_bf16(gen.normal(SEED, "sb", (co,)))
    dz = L.round_bf16(gen.normal(SEED, "sd", (N, H, W, co)))
    y = L.conv2d_forward(x, w, b, 1, 1, 1, True, L.round_bf16)
    dx, _, _ = L.conv2d_backward(x, w, np.ones_like(y), dz, 1, 1, 1, False, True, L.round_bf16)
    for n, h, ww in positions(N, H, W, 40, SEED):
        assert np.array_equal(conv_y_at(x, w, b, n, h, ww, True), y[n, h, ww])
        assert np.allclose(conv_dx_at(dz, w, n, h, ww), dx[n, h, ww], rtol=0, atol=2.0 ** -8 * np.abs(dx).max())
