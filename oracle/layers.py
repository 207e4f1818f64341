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
                  window in row-major order (ties do occur among bf16 values)

Precision modes.  "f32": no rounding anywhere (pure fp64; the HIP path computes
in fp32 and is compared at 1e-4).  "bf16": tensors that the mixed-precision path
keeps in bfloat16 -- ring weights, activations handed between layers and stages,
activation gradients -- are rounded to the nearest bfloat16 (ties to even) at
the moment they are stored; sums, bias add, the logits handed to the loss (the
output of the Linear that feeds softmax cross-entropy), the loss itself, weight
gradients, master weights and momentum are not rounded.
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
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    ssum = e.sum(axis=1, keepdims=True)
    p = e / ssum
    rows = np.arange(z.shape[0])
    loss = float(np.mean(np.log(ssum[:, 0]) + zmax[:, 0] - z[rows, labels]))
    return loss, p


def softmax_xent_backward(p, labels, q):
    """dL/dz for the mean loss: (p - onehot) / rows, stored as an activation gradient."""
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
