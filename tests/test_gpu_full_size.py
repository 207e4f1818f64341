"""The convolution and many-row product kernels at the full sizes and in the launch configurations that bench.py
times (VGG16 layers on 64 x 3 x 224 x 224 minibatches; the VGG16 classifier's first layer at 8192 rows), checked on
sampled outputs that the oracle computes one by one.

The oracle cannot run these sizes whole.  A sampled forward output is the oracle's convolution on the 3 x 3 input
patch around that pixel (zero beyond the image); a sampled input gradient is the centre of the oracle's backward pass
on the 3 x 3 patch of upstream gradients; sampled weight gradients are the oracle's backward pass on channel slices
of the full tensors (every pixel of every image contributes).  Samples include the image corners and edges and the
first and last images, where tile tails and padding live.

Tolerances.  Outputs stored as bf16: one rounding step of the reference value (2^-8 relative) plus the fp32
accumulation error, tested as 2^-7 relative with a floor of 2^-7 of the tensor's typical magnitude.  Weight gradients
(fp32, sums of up to 3.2 million products accumulated in fp32 in chunks): 5e-4 of the largest gradient entry.
"""
import numpy as np
import pytest
import torch

import paper_1806_03377_amd as pd
import pd_inputs as gen
from gpu_util import dev, to_dev
from parity_harness import run_case
from oracle import layers as OL
from sampling import close_bf16 as _close_bf16, conv_dx_at, conv_y_at, positions as _positions

pytestmark = pytest.mark.gpu
SEED = gen.BASE_SEED + 55


def _bf(a):
    """Nearest-even bf16 rounding of a large float32 array, kept as float32 (torch's CPU conversion: the oracle's
    round_bf16 is pinned to it bit for bit in tests/test_oracle_numerics.py, and it is several times faster)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


VGG_LAYERS = [(64, 224, 224, 3, 64), (64, 224, 224, 64, 64), (64, 112, 112, 64, 128), (64, 56, 56, 256, 256)]


@pytest.mark.parametrize("N,H,W,ci,co", VGG_LAYERS)
def test_vgg_conv_layers_full_size_sampled(N, H, W, ci, co):
    geom = (N, H, W, ci, co, 3, 3, 1, 1, 1)
    print(f"full-size conv {geom}", flush=True)
    x = _bf(gen.normal_bulk(SEED, f"x{ci}_{H}", (N, H, W, ci)))
    w = _bf(gen.uniform(SEED, f"w{ci}_{co}", (co, 3, 3, ci), -0.2, 0.2))
    b = _bf(gen.normal(SEED, f"b{co}", (co,)) * 0.1)
    dz = _bf(gen.normal_bulk(SEED, f"dz{co}_{H}", (N, H, W, co)) * np.float32(0.01))
    s = torch.cuda.current_stream().cuda_stream
    xd, wd, bd, dzd = (torch.from_numpy(a).to(dev()).to(torch.bfloat16) for a in (x, w, b, dz))
    w64 = w.astype(np.float64)
    pos = _positions(N, H, W, 150, SEED + ci)

    # forward, ReLU fused
    y = torch.empty((N, H, W, co), dtype=torch.bfloat16, device=dev())
    pd.pd_conv_fwd_bf16(s, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), geom, True)
    torch.cuda.synchronize()
    yh = y.float().cpu().numpy()
    scale = float(np.abs(yh[0]).mean())
    for n, h, ww in pos:
        ref = conv_y_at(x, w64, b.astype(np.float64), n, h, ww, True)
        assert _close_bf16(yh[n, h, ww], ref, scale), ("forward", n, h, ww)
    del y, yh

    # input gradient
    if ci >= 8:
        wt = torch.empty(w.size, dtype=torch.bfloat16, device=dev())
        dx = torch.empty((N, H, W, ci), dtype=torch.bfloat16, device=dev())
        pd.pd_conv_dgrad_bf16(s, dzd.data_ptr(), wd.data_ptr(), 0, dx.data_ptr(), wt.data_ptr(), geom)
        torch.cuda.synchronize()
        dxh = dx.float().cpu().numpy()
        scale = float(np.abs(dxh[0]).mean())
        for n, h, ww in pos:
            assert _close_bf16(dxh[n, h, ww], conv_dx_at(dz, w64, n, h, ww), scale), ("input gradient", n, h, ww)
        del dx, dxh

    # weight gradient + update (momentum starts at zero, so the state after the step IS the gradient)
    lr, mu = 1e-3, 0.9
    splits = pd.pd_conv_wgrad_splits(geom)
    part = torch.empty(splits * (w.size + co), dtype=torch.float32, device=dev())
    w32 = gen.uniform(SEED, f"m{ci}_{co}", w.shape, -0.2, 0.2)
    b32 = gen.normal(SEED, f"mb{co}", (co,)) * np.float32(0.1)
    mw, mb_ = to_dev(w32, False), to_dev(b32, False)
    sw = torch.zeros(w.shape, dtype=torch.float32, device=dev()); sb = torch.zeros(co, dtype=torch.float32, device=dev())
    rw = torch.empty(w.shape, dtype=torch.bfloat16, device=dev()); rb = torch.empty(co, dtype=torch.bfloat16, device=dev())
    pd.pd_conv_wgrad_update_bf16(s, dzd.data_ptr(), xd.data_ptr(), part.data_ptr(), mw.data_ptr(), sw.data_ptr(),
                                 rw.data_ptr(), mb_.data_ptr(), sb.data_ptr(), rb.data_ptr(), geom, lr, mu)
    torch.cuda.synchronize()
    g_gpu, gb_gpu, w_gpu = sw.cpu().numpy().astype(np.float64), sb.cpu().numpy().astype(np.float64), mw.cpu().numpy()
    cis = sorted({0, ci - 1, ci // 2})
    cos = sorted({0, co - 1, co // 3, (2 * co) // 3 + 1})
    xs = x[..., cis].astype(np.float64)
    ds = dz[..., cos].astype(np.float64)
    _, dW, db = OL.conv2d_backward(xs, np.zeros((len(cos), 3, 3, len(cis))), ds, ds, 1, 1, 1, False, False, OL.round_bf16)
    gmax = float(np.abs(g_gpu).max())
    got = g_gpu[np.ix_(cos, range(3), range(3), cis)]
    assert np.max(np.abs(got - dW)) <= 5e-4 * gmax, ("weight gradient", np.max(np.abs(got - dW)), gmax)
    assert np.max(np.abs(gb_gpu[cos] - db)) <= 5e-4 * float(np.abs(gb_gpu).max()), "bias gradient"
    # the step itself and the bf16 ring copy, on every parameter
    w_ref = w32.astype(np.float64) - lr * g_gpu
    assert np.max(np.abs(w_gpu - w_ref)) <= 1e-6 * float(np.abs(w_ref).max())
    assert torch.equal(rw, mw.to(torch.bfloat16)) and torch.equal(rb, mb_.to(torch.bfloat16))


def test_many_row_products_full_size_sampled():
    # the row-count sweep's largest case: 8192 rows through the classifier's first layer (25088 -> 4096)
    M, N, K = 8192, 4096, 25088
    print(f"full-size product {M} x {N} x {K}", flush=True)
    x = _bf(gen.normal_bulk(SEED, "lx", (M, K)))
    w = _bf(gen.normal_bulk(SEED, "lw", (N, K)) * np.float32(0.01))
    b = _bf(gen.normal(SEED, "lb", (N,)) * 0.1)
    dz = _bf(gen.normal_bulk(SEED, "ldz", (M, N)) * np.float32(0.01))
    s = torch.cuda.current_stream().cuda_stream
    xd, wd, bd, dzd = (torch.from_numpy(a).to(dev()).to(torch.bfloat16) for a in (x, w, b, dz))
    u = gen.uniform01(SEED, "lpos", 3 * 400).reshape(400, 3)
    rows = [0, M - 1] + [int(a * M) for a in u[:, 0]]
    cols_n = [0, N - 1] + [int(a * N) for a in u[:, 1]]
    cols_k = [0, K - 1] + [int(a * K) for a in u[:, 2]]

    ws_bytes = pd.pd_gemm_workspace_bytes(M, N, K)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev())
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev())
    pd.pd_linear_fwd_bf16(s, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), M, N, K, True, ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    yh = y.float().cpu().numpy()
    scale = float(np.abs(yh[:64]).mean())
    for m, n in zip(rows, cols_n):
        ref = OL.linear_forward(x[m:m + 1].astype(np.float64), w[n:n + 1].astype(np.float64), b[n:n + 1].astype(np.float64),
                                True, OL.round_bf16)[0, 0]
        assert _close_bf16(yh[m, n], ref, scale), ("forward", m, n)
    del y, yh

    dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev())
    pd.pd_linear_dgrad_bf16(s, dzd.data_ptr(), wd.data_ptr(), 0, dx.data_ptr(), M, N, K, ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    dxh = dx.float().cpu().numpy()
    scale = float(np.abs(dxh[:64]).mean())
    for m, k in zip(rows, cols_k):
        ref, _, _ = OL.linear_backward(np.zeros((1, 1)), w[:, k:k + 1].astype(np.float64), None,
                                       dz[m:m + 1].astype(np.float64), False, True, OL.round_bf16)
        assert _close_bf16(dxh[m, k], ref[0, 0], scale), ("input gradient", m, k)
    del dx, dxh

    geom = (M, 1, 1, K, N, 1, 1, 1, 0, 0)
    units = pd.pd_conv_wgrad_splits(geom)
    part = torch.empty(units * (N * K + N), dtype=torch.float32, device=dev())
    lr, mu = 1e-3, 0.9
    w32 = gen.normal_bulk(SEED, "lm", (N, K)) * np.float32(0.01)
    mw = torch.from_numpy(w32).to(dev())
    mb_ = torch.zeros(N, dtype=torch.float32, device=dev())
    sw = torch.zeros((N, K), dtype=torch.float32, device=dev()); sb = torch.zeros(N, dtype=torch.float32, device=dev())
    rw = torch.empty((N, K), dtype=torch.bfloat16, device=dev()); rb = torch.empty(N, dtype=torch.bfloat16, device=dev())
    pd.pd_conv_wgrad_update_bf16(s, dzd.data_ptr(), xd.data_ptr(), part.data_ptr(), mw.data_ptr(), sw.data_ptr(),
                                 rw.data_ptr(), mb_.data_ptr(), sb.data_ptr(), rb.data_ptr(), geom, lr, mu)
    torch.cuda.synchronize()
    g = sw.cpu().numpy()
    gmax = float(np.abs(g).max())
    for n, k in zip(cols_n, cols_k):
        _, dW, _ = OL.linear_backward(x[:, k:k + 1].astype(np.float64), np.zeros((1, 1)), None,
                                      dz[:, n:n + 1].astype(np.float64), False, False, OL.round_bf16)
        assert abs(g[n, k] - dW[0, 0]) <= 5e-4 * gmax, ("weight gradient", n, k, g[n, k], dW[0, 0])
    gb = sb.cpu().numpy()
    ref_b = dz.astype(np.float64).sum(axis=0)
    assert np.max(np.abs(gb - ref_b)) <= 5e-4 * float(np.abs(ref_b).max())
    w_ref = w32.astype(np.float64) - lr * g
    assert np.max(np.abs(mw.cpu().numpy() - w_ref)) <= 1e-6 * float(np.abs(w_ref).max())
    assert torch.equal(rw, mw.to(torch.bfloat16))


@pytest.mark.timeout(2400)
def test_config4_s2vt_full_size_two_minibatches(capsys):
    """Config 4 exactly as configured -- LSTM 4096 -> 1000 | LSTM 1000 -> 1000 + Linear 1000 -> 30000 + loss, sequence
    length 80, minibatch 64 (5120 rows through the vocabulary layer), NOAM 2 -- for two minibatches, op by op in
    lockstep with the oracle, which runs these sizes whole (about a minute per minibatch on the host): every stored
    layer output (both hidden sequences, all 5120 x 30000 logits), both losses, the input gradient handed upstream
    and, after each of the four updates, all 58 million master weights, momentum values and ring copies, at the bf16
    tolerance.  Stage 0 has two minibatches in flight, so its second backward pass reads the stashed version 0 while
    the latest is 1."""
    print("config 4 at full size (T 80, minibatch 64, vocabulary 30000): oracle + GPU, two minibatches", flush=True)
    sl = gen.config4_s2vt()
    seed, M, T, B, I, V = SEED + 4, 2, 80, 64, 4096, 30000
    params = [gen.init_params(seed, f"q{s}", ly) for s, ly in enumerate(sl)]
    xs = [gen.normal_bulk(seed, f"X{i}", (T, B, I)) for i in range(M)]
    labs = list(gen.labels(seed, "Y", (M, T, B), V))
    with capsys.disabled():      # the oracle needs minutes here: let the per-op lines through as signs of life
        print(flush=True)
        out = run_case(sl, params, xs, labs, noam=2, precision=pd.PD_BF16_F32ACC, lr=0.01, mode="forced", minibatch=B,
                       verbose=True)
    assert out["updates_compared"] == (2 * M, 2 * M), out["updates_compared"]
    assert all(np.isfinite(out["losses"])) and all(l > 5.0 for l in out["losses"]), out["losses"]   # ~ log(30000)
