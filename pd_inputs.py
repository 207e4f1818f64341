"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module draws numbers and shapes them; it contains none of the method's
arithmetic (no layer maths, no schedule, no update rule).  Both sides receive
the *same host arrays* from here, so parity never depends on how the values
were drawn.

Generator: counter-based.  Element ``k`` of the sub-stream named ``name`` under
``seed`` is ``splitmix64(hash(seed, name) + k)``; uniforms take the top 53 bits,
normals use Box-Muller on two consecutive uniforms.  Being counter-based, any
element can be regenerated alone, and results do not depend on chunking.

The datasets the paper trained on (ILSVRC12 images, MSVD clips; Section 5.1,
"Datasets") are not available; the tensors produced here stand in for them with
the same shapes and N(0,1) / uniform-label statistics as the benchmark configs.
"""
from __future__ import annotations

import zlib

import numpy as np

BASE_SEED = 1806033770  # + config index

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output per 64-bit counter value (vectorised, wraps mod 2^64)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _stream_base(seed: int, name: str) -> np.uint64:
    h = zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF
    mixed = ((int(seed) & 0xFFFFFFFF) << 32) | h
    return _splitmix64(np.array([mixed], dtype=np.uint64))[0]


def uniform01(seed: int, name: str, n: int, offset: int = 0) -> np.ndarray:
    """``n`` float64 uniforms in [0, 1) from sub-stream ``name`` starting at counter ``offset``."""
    out = np.empty(n, dtype=np.float64)
    base = _stream_base(seed, name)
    chunk = 1 << 22
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        with np.errstate(over="ignore"):
            ctr = base + np.arange(offset + lo, offset + hi, dtype=np.uint64)
        bits = _splitmix64(ctr) >> np.uint64(11)
        out[lo:hi] = bits.astype(np.float64) * (1.0 / 9007199254740992.0)
    return out


def normal(seed: int, name: str, shape, dtype=np.float32) -> np.ndarray:
    """N(0,1) samples (Box-Muller; two uniforms per pair of outputs)."""
    n = int(np.prod(shape))
    m = (n + 1) // 2
    u = uniform01(seed, name, 2 * m)
    u1 = 1.0 - u[0::2]  # (0, 1]
    u2 = u[1::2]
    r = np.sqrt(-2.0 * np.log(u1))
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = r * np.cos(2.0 * np.pi * u2)
    z[1::2] = r * np.sin(2.0 * np.pi * u2)
    return z[:n].reshape(shape).astype(dtype)


def normal_bulk(seed: int, name: str, shape) -> np.ndarray:
    """N(0,1) float32 samples for tensors of 10^8 elements and more, where the element-addressable generator above
    would take minutes: numpy's Philox bit generator keyed by the same (seed, name) hash.  Seeded and reproducible,
    but not element-addressable."""
    key = int(_stream_base(seed, name))
    rng = np.random.Generator(np.random.Philox(key=key))
    return rng.standard_normal(int(np.prod(shape)), dtype=np.float32).reshape(shape)


def uniform(seed: int, name: str, shape, lo: float, hi: float, dtype=np.float32) -> np.ndarray:
    n = int(np.prod(shape))
    u = uniform01(seed, name, n)
    return (lo + (hi - lo) * u).reshape(shape).astype(dtype)


def labels(seed: int, name: str, shape, num_classes: int) -> np.ndarray:
    """Uniform integer labels in [0, num_classes) as int32."""
    n = int(np.prod(shape))
    u = uniform01(seed, name, n)
    return np.minimum((u * num_classes).astype(np.int64), num_classes - 1).astype(np.int32).reshape(shape)


# ----------------------------------------------------------------------------
# Layer lists.  A layer is a tuple whose first item names its kind; the product
# binding and the oracle each translate this neutral description on their own.
#   ("linear", in_features, out_features, relu: bool)
#   ("softmax_xent", classes)
#   ("conv2d", c_in, c_out, kh, kw, stride, pad_h, pad_w, relu: bool)   (NHWC)
#   ("maxpool2d", k, stride)
#   ("lstm", input_size, hidden, seq_len)
#   ("avgpool2d", k, stride, pad)
#   ("concat", [branch, branch, ...])   each branch a list of conv2d / maxpool2d / avgpool2d tuples over the
#                                       same input; outputs joined along the channel axis, branch 0 first
# ----------------------------------------------------------------------------

def param_count(layers) -> int:
    n = 0
    for L in layers:
        if L[0] == "linear":
            n += L[1] * L[2] + L[2]
        elif L[0] == "conv2d":
            n += L[2] * L[3] * L[4] * L[1] + L[2]
        elif L[0] == "lstm":
            n += 4 * L[2] * (L[1] + L[2]) + 4 * L[2]
        elif L[0] == "concat":
            n += sum(param_count(br) for br in L[1])
    return n


def init_params(seed: int, name: str, layers) -> np.ndarray:
    """Flat fp32 parameter vector: per layer, weight then bias.

    Weights are uniform in +-sqrt(6 / fan_in) (the "Kaiming-uniform" the
    benchmark configs name), biases start at zero.  Layout per layer:
    linear W[out][in]; conv W[c_out][kh][kw][c_in]; lstm W_ih[4H][I], W_hh[4H][H], b[4H].
    """
    parts = []
    for li, L in enumerate(layers):
        tag = f"{name}/L{li}"
        if L[0] == "linear":
            bound = float(np.sqrt(6.0 / L[1]))
            parts.append(uniform(seed, tag + "/W", (L[2] * L[1],), -bound, bound))
            parts.append(np.zeros(L[2], dtype=np.float32))
        elif L[0] == "conv2d":
            fan_in = L[1] * L[3] * L[4]
            bound = float(np.sqrt(6.0 / fan_in))
            parts.append(uniform(seed, tag + "/W", (L[2] * L[3] * L[4] * L[1],), -bound, bound))
            parts.append(np.zeros(L[2], dtype=np.float32))
        elif L[0] == "lstm":
            bound = float(np.sqrt(6.0 / L[2]))
            parts.append(uniform(seed, tag + "/Wih", (4 * L[2] * L[1],), -bound, bound))
            parts.append(uniform(seed, tag + "/Whh", (4 * L[2] * L[2],), -bound, bound))
            parts.append(np.zeros(4 * L[2], dtype=np.float32))
        elif L[0] == "concat":
            for b, br in enumerate(L[1]):
                parts.append(init_params(seed, f"{tag}/B{b}", br))
    if not parts:
        return np.zeros(0, dtype=np.float32)
    return np.concatenate(parts).astype(np.float32)


# ----------------------------------------------------------------------------
# The benchmark configurations (shapes only).
# ----------------------------------------------------------------------------

def config1_mlp(hidden: int = 256, classes: int = 10, stages: int = 4):
    """4-stage MLP: each stage one Linear hidden->hidden + ReLU; last stage Linear hidden->classes + loss."""
    st = [[("linear", hidden, hidden, True)] for _ in range(stages - 1)]
    st.append([("linear", hidden, classes, False), ("softmax_xent", classes)])
    return st


def config2_vgg_fc(in_features: int = 25088, hidden: int = 4096, classes: int = 1000):
    """VGG16's classifier as one stage: Linear-ReLU-Linear-ReLU-Linear + loss."""
    return [("linear", in_features, hidden, True),
            ("linear", hidden, hidden, True),
            ("linear", hidden, classes, False),
            ("softmax_xent", classes)]


def config3_vgg_conv(widths=(64, 128, 256)):
    """VGG16's first three convolution blocks as one stage: 3x3 convolutions (pad 1) with ReLU,
    2x2 max-pooling after each block: 64-64-pool-128-128-pool-256-256-256-pool on 3-channel images."""
    a, b, c = widths

    def conv(ci, co):
        return ("conv2d", ci, co, 3, 3, 1, 1, 1, True)

    return [conv(3, a), conv(a, a), ("maxpool2d", 2, 2), conv(a, b), conv(b, b), ("maxpool2d", 2, 2),
            conv(b, c), conv(c, c), conv(c, c), ("maxpool2d", 2, 2)]


def vgg16_full(classes: int = 1000):
    """All of VGG16 as one layer list (13 convolutions, 5 poolings, 3 Linear layers, loss) on 3x224x224 images:
    the model the layer profiler and the partitioner are run on."""
    def conv(ci, co):
        return ("conv2d", ci, co, 3, 3, 1, 1, 1, True)

    pool = ("maxpool2d", 2, 2)
    return (config3_vgg_conv() + [conv(256, 512), conv(512, 512), conv(512, 512), pool,
                                  conv(512, 512), conv(512, 512), conv(512, 512), pool] + config2_vgg_fc(classes=classes))


def config4_s2vt(input_size=4096, hidden=1000, vocab=30000, seq_len=80):
    """S2VT-shaped two-stage sequence model: stage 0 = LSTM(input -> hidden); stage 1 = LSTM(hidden -> hidden),
    vocabulary projection on every time step, softmax cross-entropy over all seq_len * minibatch tokens."""
    return [[("lstm", input_size, hidden, seq_len)],
            [("lstm", hidden, hidden, seq_len), ("linear", hidden, vocab, False), ("softmax_xent", vocab)]]


def config5_inception(classes: int = 1000, width: float = 1.0):
    """Inception-v3-shaped network on 299 x 299 x 3 images, split into four pipeline stages.

    The paper cites Inception-v3 without printing its layer table; this one is the build's own, with the
    features the benchmark configuration names: a stem of strided and unstrided 3x3 convolutions with
    overlapping 3x3/2 max pooling down to a 35 x 35 grid; blocks of parallel 1x1 | 1x1-5x5 | 1x1-3x3-3x3 |
    avgpool-1x1 branches at 35 x 35; a grid reduction to 17 x 17; blocks with factorised 1x7 / 7x1
    convolutions at 17 x 17; a reduction to 8 x 8; a block at 8 x 8 with 1x3 / 3x1 convolutions; global average
    pooling and a Linear classifier.  Convolution + bias + ReLU everywhere (no batch normalisation, no
    auxiliary head).  ``width`` scales every channel count (kept a multiple of 8) for reduced test cases.
    Returns (stages, input sizes) with input sizes (h, w, channels) per stage.
    """
    def c(n):
        return max(8, int(round(n * width / 8.0)) * 8)

    def conv(ci, co, kh, kw, stride=1, ph=0, pw=0):
        return ("conv2d", ci, co, kh, kw, stride, ph, pw, True)

    def block_a(ci, pool_proj):
        return ("concat", [[conv(ci, c(64), 1, 1)],
                           [conv(ci, c(48), 1, 1), conv(c(48), c(64), 5, 5, 1, 2, 2)],
                           [conv(ci, c(64), 1, 1), conv(c(64), c(96), 3, 3, 1, 1, 1), conv(c(96), c(96), 3, 3, 1, 1, 1)],
                           [("avgpool2d", 3, 1, 1), conv(ci, pool_proj, 1, 1)]]), c(64) + c(64) + c(96) + pool_proj

    def reduce_b(ci):
        return ("concat", [[conv(ci, c(384), 3, 3, 2)],
                           [conv(ci, c(64), 1, 1), conv(c(64), c(96), 3, 3, 1, 1, 1), conv(c(96), c(96), 3, 3, 2)],
                           [("maxpool2d", 3, 2)]]), c(384) + c(96) + ci

    def block_c(ci, m):
        return ("concat", [[conv(ci, c(192), 1, 1)],
                           [conv(ci, m, 1, 1), conv(m, m, 1, 7, 1, 0, 3), conv(m, c(192), 7, 1, 1, 3, 0)],
                           [conv(ci, m, 1, 1), conv(m, m, 7, 1, 1, 3, 0), conv(m, m, 1, 7, 1, 0, 3),
                            conv(m, m, 7, 1, 1, 3, 0), conv(m, c(192), 1, 7, 1, 0, 3)],
                           [("avgpool2d", 3, 1, 1), conv(ci, c(192), 1, 1)]]), 4 * c(192)

    def reduce_d(ci):
        return ("concat", [[conv(ci, c(192), 1, 1), conv(c(192), c(320), 3, 3, 2)],
                           [conv(ci, c(192), 1, 1), conv(c(192), c(192), 1, 7, 1, 0, 3), conv(c(192), c(192), 7, 1, 1, 3, 0),
                            conv(c(192), c(192), 3, 3, 2)],
                           [("maxpool2d", 3, 2)]]), c(320) + c(192) + ci

    def block_e(ci):
        return ("concat", [[conv(ci, c(320), 1, 1)],
                           [conv(ci, c(384), 1, 1), conv(c(384), c(384), 1, 3, 1, 0, 1)],
                           [conv(ci, c(448), 1, 1), conv(c(448), c(384), 3, 3, 1, 1, 1), conv(c(384), c(384), 3, 1, 1, 1, 0)],
                           [("avgpool2d", 3, 1, 1), conv(ci, c(192), 1, 1)]]), c(320) + 2 * c(384) + c(192)

    stem = [conv(3, c(32), 3, 3, 2), conv(c(32), c(32), 3, 3), conv(c(32), c(64), 3, 3, 1, 1, 1), ("maxpool2d", 3, 2),
            conv(c(64), c(80), 1, 1), conv(c(80), c(192), 3, 3), ("maxpool2d", 3, 2)]
    ch = c(192)
    a1, ch1 = block_a(ch, c(32))
    a2, ch2 = block_a(ch1, c(64))
    a3, ch3 = block_a(ch2, c(64))
    rb, ch4 = reduce_b(ch3)
    c1, ch5 = block_c(ch4, c(128))
    c2, ch6 = block_c(ch5, c(160))
    c3, ch7 = block_c(ch6, c(160))
    c4, ch8 = block_c(ch7, c(192))
    rd, ch9 = reduce_d(ch8)
    e1, ch10 = block_e(ch9)
    head = [("avgpool2d", 8, 1, 0), ("linear", ch10, classes, False), ("softmax_xent", classes)]
    stages = [stem, [a1, a2, a3], [rb, c1, c2], [c3, c4, rd, e1] + head]
    sizes = [(299, 299, 3), (35, 35, ch), (35, 35, ch3), (17, 17, ch6)]
    return stages, sizes


def forward_flops(layers, hwc, rows: int = 1):
    """(multiply-add flops x2 of one forward pass for `rows` images, output (h, w, c)) of a layer list."""
    h, w, ch = hwc
    total = 0

    def walk(ls, h, w, ch):
        nonlocal total
        for L in ls:
            if L[0] == "conv2d":
                h, w = (h + 2 * L[6] - L[3]) // L[5] + 1, (w + 2 * L[7] - L[4]) // L[5] + 1
                total += 2 * rows * h * w * L[2] * L[3] * L[4] * L[1]
                ch = L[2]
            elif L[0] == "maxpool2d":
                h, w = (h - L[1]) // L[2] + 1, (w - L[1]) // L[2] + 1
            elif L[0] == "avgpool2d":
                h, w = (h + 2 * L[3] - L[1]) // L[2] + 1, (w + 2 * L[3] - L[1]) // L[2] + 1
            elif L[0] == "linear":
                total += 2 * rows * L[1] * L[2]
                h, w, ch = 1, 1, L[2]
            elif L[0] == "concat":
                outs = [walk(br, h, w, ch) for br in L[1]]
                h, w, ch = outs[0][0], outs[0][1], sum(o[2] for o in outs)
        return h, w, ch

    out = walk(layers, h, w, ch)
    return total, out
