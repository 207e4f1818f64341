"""Textbook layer maths in fp64, with the rounding points of the bf16 mode.

Test infrastructure only (see package docstring).  The paper delegates layer
compute to its ML worker (Section 4) and gives no formulas, so each routine is
the standard definition written out:

  Linear          y = x W^T + b,  W[out][in]
  ReLU            max(y, 0); derivative 1 where the stored output is > 0, else 0
  softmax-xent    L = mean_rows( logsumexp(z) - z[label] ),  dz = (softmax(z) - onehot) / rows
  Conv2d          cross-correlation, NHWC activations, W[c_out][kh][kw][c_in], zero padding,
                  y[n,i,j,o] = b[o] + sum_{a,b,c} x[n, i*s + a - ph, j*s + b - pw, c] W[o,a,b,c]
  MaxPool2d       window k, stride s, no padding; the gradient goes to the FIRST maximum of the
                  window in row-major order (ties do occur among bf16 values); where windows overlap
                  an input position sums what it receives
  AvgPool2d       window k, stride s, zero padding p counted in the divisor: y = (sum over the window)/k^2
  Concat block    parallel branches over one input, outputs joined along the channel axis (branch 0
                  first); dL/dx = sum over branches of each branch's input gradient
  LSTM            time-major sequences x[T][B][I] -> h[T][B][H]; gates (i, f, g, o) =
                  x_t W_ih^T + h_{t-1} W_hh^T + b with W_ih[4H][I], W_hh[4H][H]; i, f, o = sigmoid,
                  g = tanh; c_t = f c_{t-1} + i g; h_t = o tanh(c_t); h_{-1} = c_{-1} = 0; backward is
                  full back-propagation through time

Precision modes.  "f32": no rounding anywhere (pure fp64; the HIP path computes
in fp32 and is compared at 1e-4).  "bf16": tensors that the mixed-precision path
keeps in bfloat16 -- ring weights, activations handed between layers and stages,
activation gradients -- are rounded to the nearest bfloat16 (ties to even) at
the moment they are stored; sums, bias add, the logits handed to the loss (the
output of the Linear that feeds softmax cross-entropy), the loss itself, weight
gradients, master weights and momentum are not rounded.  Inside an LSTM the hidden
state h_t (an activation, and the next step's matrix operand) and the gate
pre-activation gradients (matrix operands of the backward pass) are rounded; gate
values, the cell state c_t, and the recurrent gradients dh, dc are not.
"""
from __future__ import annotations

import numpy as np


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (8 significand bits), ties to even, returned as float64.

    Goes through float32 first (as hardware that accumulates in fp32 does), then
    drops the low 16 bits with the usual add-half-then-truncate on the bit pattern.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)   # finite inputs never wrap
    out = r.view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out = np.where(nan, np.nan, out)
    return out.reshape(np.shape(x))


def quantiser(mode: str):
    if mode == "f32":
        return lambda a: np.asarray(a, dtype=np.float64)
    if mode == "bf16":
        return round_bf16
    raise ValueError("mode must be 'f32' or 'bf16'")


# ---- Linear (+ optional ReLU) ------------------------------------------------

def linear_forward(x, W, b, relu: bool, q):
    """x[rows][in], W[out][in], b[out] -> stored output y[rows][out]."""
    z = x @ W.T + b
    if relu:
        z = np.maximum(z, 0.0)
    return q(z)


def linear_backward(x, W, y, dy, relu: bool, need_dx: bool, q):
    """Gradients of a Linear(+ReLU) given its stored input x, stored output y and dL/dy.

    Returns (dx or None, dW, db).  dW and db stay unrounded; dx is an activation
    gradient and is rounded when stored.
    """
    dz = dy * (y > 0.0) if relu else dy
    dW = dz.T @ x
    db = dz.sum(axis=0)
    dx = q(dz @ W) if need_dx else None
    return dx, dW, db


# ---- softmax cross-entropy ---------------------------------------------------

def softmax_xent_forward(z, labels):
    """Mean over rows of -log softmax(z)[label]; also returns softmax(z)."""
    labels = np.asarray(labels).reshape(-1)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    ssum = e.sum(axis=1, keepdims=True)
    p = e / ssum
    rows = np.arange(z.shape[0])
    loss = float(np.mean(np.log(ssum[:, 0]) + zmax[:, 0] - z[rows, labels]))
    return loss, p


def softmax_xent_backward(p, labels, q):
    """dL/dz for the mean loss: (p - onehot) / rows, stored as an activation gradient."""
    labels = np.asarray(labels).reshape(-1)
    d = p.copy()
    d[np.arange(p.shape[0]), labels] -= 1.0
    return q(d / p.shape[0])


# ---- Conv2d (+ optional ReLU), NHWC -------------------------------------------

def _conv_out(size, k, stride, pad):
    return (size + 2 * pad - k) // stride + 1


def _tap_view(xp, a, b, ho, wo, stride):
    """The input pixels that tap (a, b) of the kernel meets, one per output pixel: [N, ho, wo, C]."""
    return xp[:, a:a + (ho - 1) * stride + 1:stride, b:b + (wo - 1) * stride + 1:stride, :]


def conv2d_forward(x, W, b, stride, pad_h, pad_w, relu: bool, q):
    """x[N][H][W][Cin], W[Cout][kh][kw][Cin], b[Cout] -> stored output [N][Ho][Wo][Cout].

    Written as the definition: one matrix product per kernel tap over the shifted input.
    """
    N, H, Wd, C = x.shape
    Co, kh, kw, _ = W.shape
    ho, wo = _conv_out(H, kh, stride, pad_h), _conv_out(Wd, kw, stride, pad_w)
    xp = np.pad(x, ((0, 0), (pad_h, pad_h), (pad_w, pad_w), (0, 0)))
    z = np.zeros((N, ho, wo, Co)) + b
    for a in range(kh):
        for c in range(kw):
            z += _tap_view(xp, a, c, ho, wo, stride) @ W[:, a, c, :].T
    if relu:
        z = np.maximum(z, 0.0)
    return q(z)


def conv2d_backward(x, W, y, dy, stride, pad_h, pad_w, relu: bool, need_dx: bool, q):
    """Returns (dx or None, dW, db) for the convolution above."""
    N, H, Wd, C = x.shape
    Co, kh, kw, _ = W.shape
    ho, wo = y.shape[1], y.shape[2]
    dz = dy * (y > 0.0) if relu else dy
    xp = np.pad(x, ((0, 0), (pad_h, pad_h), (pad_w, pad_w), (0, 0)))
    dW = np.zeros_like(W)
    dxp = np.zeros_like(xp) if need_dx else None
    dz2 = dz.reshape(-1, Co)
    for a in range(kh):
        for c in range(kw):
            xs = _tap_view(xp, a, c, ho, wo, stride)
            dW[:, a, c, :] = dz2.T @ xs.reshape(-1, C)
            if need_dx:
                _tap_view(dxp, a, c, ho, wo, stride)[...] += dz @ W[:, a, c, :]
    db = dz2.sum(axis=0)
    dx = None
    if need_dx:
        dx = q(dxp[:, pad_h:pad_h + H, pad_w:pad_w + Wd, :])
    return dx, dW, db


# ---- MaxPool2d, NHWC ----------------------------------------------------------

def maxpool2d_forward(x, k, stride):
    N, H, Wd, C = x.shape
    ho, wo = (H - k) // stride + 1, (Wd - k) // stride + 1
    y = np.full((N, ho, wo, C), -np.inf)
    for a in range(k):
        for b in range(k):
            y = np.maximum(y, x[:, a:a + (ho - 1) * stride + 1:stride, b:b + (wo - 1) * stride + 1:stride, :])
    return y


def maxpool2d_backward(x, y, dy, k, stride):
    """dL/dx: each output's gradient goes to the first position (row-major in the window) holding the maximum."""
    N, H, Wd, C = x.shape
    ho, wo = y.shape[1], y.shape[2]
    dx = np.zeros_like(x)
    taken = np.zeros(y.shape, dtype=bool)
    for a in range(k):
        for b in range(k):
            xs = x[:, a:a + (ho - 1) * stride + 1:stride, b:b + (wo - 1) * stride + 1:stride, :]
            hit = (xs == y) & ~taken
            dx[:, a:a + (ho - 1) * stride + 1:stride, b:b + (wo - 1) * stride + 1:stride, :] += np.where(hit, dy, 0.0)
            taken |= hit
    return dx


# ---- AvgPool2d, NHWC ----------------------------------------------------------

def avgpool2d_forward(x, k, stride, pad, q):
    """Mean over k x k windows; padded positions are zeros and count in the divisor."""
    N, H, Wd, C = x.shape
    ho, wo = _conv_out(H, k, stride, pad), _conv_out(Wd, k, stride, pad)
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    y = np.zeros((N, ho, wo, C))
    for a in range(k):
        for b in range(k):
            y += _tap_view(xp, a, b, ho, wo, stride)
    return q(y / (k * k))


def avgpool2d_backward(x_shape, dy, k, stride, pad, q):
    """Transpose of the averaging operator: every window spreads dy / k^2 over its positions."""
    N, H, Wd, C = x_shape
    ho, wo = dy.shape[1], dy.shape[2]
    dxp = np.zeros((N, H + 2 * pad, Wd + 2 * pad, C))
    for a in range(k):
        for b in range(k):
            _tap_view(dxp, a, b, ho, wo, stride)[...] += dy / (k * k)
    return q(dxp[:, pad:pad + H, pad:pad + Wd, :])


# ---- LSTM, time-major -----------------------------------------------------------

def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def lstm_forward(x, W_ih, W_hh, b, q):
    """x[T][B][I] -> (h[T][B][H] stored, cache for the backward pass)."""
    T, B, _ = x.shape
    H = W_hh.shape[1]
    h_prev = np.zeros((B, H))
    c_prev = np.zeros((B, H))
    hs, cs, gates = [], [], []
    for t in range(T):
        a = x[t] @ W_ih.T + h_prev @ W_hh.T + b
        i, f, g, o = _sigmoid(a[:, :H]), _sigmoid(a[:, H:2 * H]), np.tanh(a[:, 2 * H:3 * H]), _sigmoid(a[:, 3 * H:])
        c = f * c_prev + i * g
        h = q(o * np.tanh(c))
        hs.append(h); cs.append(c); gates.append((i, f, g, o))
        h_prev, c_prev = h, c
    return np.stack(hs), dict(hs=hs, cs=cs, gates=gates)


def lstm_backward(x, W_ih, W_hh, cache, dh_out, need_dx: bool, q):
    """Back-propagation through time.  dh_out[T][B][H] = dL/dh_t from the layer above.
    Returns (dx or None, dW_ih, dW_hh, db)."""
    T, B, _ = x.shape
    H = W_hh.shape[1]
    dW_ih, dW_hh, db = np.zeros_like(W_ih), np.zeros_like(W_hh), np.zeros(4 * H)
    dx = np.zeros_like(x) if need_dx else None
    dh_rec = np.zeros((B, H))
    dc_next = np.zeros((B, H))
    for t in range(T - 1, -1, -1):
        i, f, g, o = cache["gates"][t]
        c = cache["cs"][t]
        c_prev = cache["cs"][t - 1] if t > 0 else np.zeros((B, H))
        h_prev = cache["hs"][t - 1] if t > 0 else np.zeros((B, H))
        dh = dh_out[t] + dh_rec
        tc = np.tanh(c)
        dc = dc_next + dh * o * (1.0 - tc * tc)
        da = q(np.concatenate([dc * g * i * (1.0 - i), dc * c_prev * f * (1.0 - f), dc * i * (1.0 - g * g),
                               dh * tc * o * (1.0 - o)], axis=1))
        dW_ih += da.T @ x[t]
        dW_hh += da.T @ h_prev
        db += da.sum(axis=0)
        if need_dx:
            dx[t] = q(da @ W_ih)
        dh_rec = da @ W_hh
        dc_next = dc * f
    return dx, dW_ih, dW_hh, db
