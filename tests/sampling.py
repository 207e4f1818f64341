"""Sampled outputs of convolutions too large for the oracle to run whole: each sample is the oracle's own routine
on the 3 x 3 neighbourhood that determines it (3 x 3 filters, stride 1, padding 1)."""
import numpy as np

import pd_inputs as gen
from oracle import layers as OL


def positions(N, H, W, count, seed):
    """(image, row, column) samples: the corners of the first and last image, some edges, then seeded random ones."""
    fixed = [(n, h, w) for n in (0, N - 1) for h in (0, H - 1) for w in (0, W - 1)]
    fixed += [(N // 2, 0, W // 2), (N // 2, H // 2, W - 1), (1 % N, H - 1, 1 % W)]
    u = gen.uniform01(seed, "pos", 3 * count).reshape(count, 3)
    return fixed + [(int(a * N), int(b * H), int(c * W)) for a, b, c in u]


def patch(t, n, h, w):
    """3 x 3 spatial patch of t[n] around (h, w), zero outside the image: [1][3][3][C] float64."""
    _, H, W, C = t.shape
    out = np.zeros((1, 3, 3, C))
    for a in range(3):
        for b in range(3):
            hh, ww = h + a - 1, w + b - 1
            if 0 <= hh < H and 0 <= ww < W:
                out[0, a, b] = t[n, hh, ww]
    return out


def conv_y_at(x, w, b, n, h, ww, relu):
    """All output channels of the 3x3/pad-1 convolution at one pixel: the oracle's forward on the input patch."""
    return OL.conv2d_forward(patch(x, n, h, ww), w, b, 1, 0, 0, relu, OL.round_bf16)[0, 0, 0]


def conv_dx_at(dz, w, n, h, ww):
    """All input channels of dL/dx at one pixel: the centre of the oracle's backward pass on the 3 x 3 patch of
    upstream gradients (pixels outside the image have none)."""
    d = patch(dz, n, h, ww)
    dx, _, _ = OL.conv2d_backward(np.zeros((1, 3, 3, w.shape[3])), w, d, d, 1, 1, 1, False, True, OL.round_bf16)
    return dx[0, 1, 1]


def close_bf16(got, ref, scale):
    return bool(np.all(np.abs(got - ref) <= 2.0 ** -7 * np.maximum(np.abs(ref), scale)))
