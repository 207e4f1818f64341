"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars (stated by the benchmark definition): schedule order and version indices bit-exact;
fp32 mode <= 1e-4 and bf16 mode (fp32 accumulate) <= 2e-2 max-norm relative error per tensor
(max|got - ref| / max|ref|), and the same relative bound on every minibatch's loss.
"""
import numpy as np
import pytest
import torch

import paper_1806_03377_amd as pd
import pd_inputs as gen
from gpu_util import GpuStage, dev, empty_act, labels_dev, rel_err, to_dev, to_host
from parity_harness import run_case
from oracle import layers as OL
from oracle.pipeline import Stage, run_pipeline
from oracle.schedule import OP_B, OP_F, OP_U, in_flight_depth, schedule_1f1b

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2
SEED = gen.BASE_SEED


def _bf(a):
    return OL.round_bf16(np.asarray(a, dtype=np.float64))


# ---------------------------------------------------------------------------------------------
# kernels on their own (bf16 MFMA): several tiles, ragged tails in every dimension, split-K on/off
# ---------------------------------------------------------------------------------------------
SHAPES = [(64, 128, 64), (64, 256, 4096), (64, 200, 264), (40, 136, 72), (1, 8, 8), (130, 1000, 520),
          (64, 4096, 1024), (96, 24, 2048), (256, 512, 768),
          (50, 1000, 1536), (64, 72, 512), (1, 8, 1024),   # reduction a multiple of 128: the direct-to-LDS forward
          (512, 256, 256), (600, 1000, 520), (1030, 264, 136),     # >= 512 rows: the 256 x 256-tile weight gradient
          # many rows, a long reduction, too few 256 x 256 tiles to fill the chip: large tiles with a split reduction
          (600, 1000, 4096), (300, 264, 2112), (1030, 2048, 520), (257, 4096, 4096),
          # the same with an output width that is not a multiple of 32: the input gradient's split reduction ends in a
          # partial stage (16, 24 and 8 elements)
          (600, 2064, 1000), (300, 2072, 264), (520, 4104, 520),
          # a few output tiles more than a whole number of rounds of the chip (258 for the input gradient, 344 for the
          # weight gradient): the tiles of the last round are split over the idle compute units
          (600, 1024, 22016)]
# the same products forced onto the large-tile kernels (threshold 1 tile): several tiles, ragged rows/columns, a
# reduction length that is a multiple of 32, one that is not, one shorter than a stage
BIG_SHAPES = [(512, 256, 256), (600, 1000, 520), (1030, 264, 136), (300, 520, 1000), (257, 8, 24), (700, 776, 4128), (2080, 264, 136)]


@pytest.fixture
def big_tiles():
    old = pd.pd_set_big_tile_threshold(1)
    yield
    pd.pd_set_big_tile_threshold(old)


@pytest.mark.parametrize("M,N,K", BIG_SHAPES)
def test_linear_fwd_bf16_big_tiles(M, N, K, big_tiles):
    test_linear_fwd_bf16(M, N, K)


# every variant of the large-tile forward kernel (pd_set_big_gemm_waves): four / eight waves, 128- / 64-byte LDS rows;
# reductions that are a multiple of 64 (the 128-byte-row kernels), a multiple of 32 only, and ragged; ragged rows / columns
@pytest.mark.parametrize("variant", [4, 8, 104, 108])
@pytest.mark.parametrize("M,N,K", [(600, 1000, 512), (300, 520, 1088), (2080, 264, 136), (257, 8, 128), (700, 776, 4128),
                                   (512, 256, 8192 + 64)])
def test_linear_fwd_bf16_big_tile_variants(M, N, K, variant, big_tiles):
    old = pd.pd_set_big_gemm_waves(variant)
    try:
        test_linear_fwd_bf16(M, N, K)
    finally:
        pd.pd_set_big_gemm_waves(old)


@pytest.mark.parametrize("M,N,K", BIG_SHAPES)
def test_linear_dgrad_bf16_big_tiles(M, N, K, big_tiles):
    test_linear_dgrad_bf16(M, N, K)


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_fwd_bf16(M, N, K):
    x = _bf(gen.normal(SEED, "kx", (M, K)))
    w = _bf(gen.uniform(SEED, "kw", (N, K), -0.1, 0.1))
    b = _bf(gen.normal(SEED, "kb", (N,)) * 0.1)
    s = torch.cuda.current_stream().cuda_stream
    wsb = pd.pd_gemm_workspace_bytes(M, N, K)
    ws = torch.zeros(max(wsb, 16), dtype=torch.uint8, device=dev())
    xd, wd, bd = to_dev(x, True), to_dev(w, True), to_dev(b, True)
    for relu in (True, False):
        for use_ws in (True, False):
            y = empty_act(M, N, True)
            pd.pd_linear_fwd_bf16(s, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), M, N, K, relu,
                                  ws.data_ptr() if use_ws else 0, wsb if use_ws else 0)
            ref = OL.linear_forward(x, w, b, relu, OL.round_bf16)
            assert rel_err(to_host(y), ref) <= TOL_BF16, (relu, use_ws)
            # tighter: never more than one bf16 step away from the oracle's rounding
            assert np.max(np.abs(to_host(y) - ref) / np.maximum(np.abs(ref), 1e-2)) < 2 ** -6


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_dgrad_bf16(M, N, K):
    dz = _bf(gen.normal(SEED, "dz", (M, N)) * 0.01)
    w = _bf(gen.uniform(SEED, "kw", (N, K), -0.1, 0.1))
    ymask = _bf(np.maximum(gen.normal(SEED, "ym", (M, K)), 0.0))
    s = torch.cuda.current_stream().cuda_stream
    wsb = pd.pd_gemm_workspace_bytes(M, N, K)
    ws = torch.zeros(max(wsb, 16), dtype=torch.uint8, device=dev())
    dzd, wd, md = to_dev(dz, True), to_dev(w, True), to_dev(ymask, True)
    for masked in (True, False):
        for use_ws in (True, False):
            dx = empty_act(M, K, True)
            pd.pd_linear_dgrad_bf16(s, dzd.data_ptr(), wd.data_ptr(), md.data_ptr() if masked else 0, dx.data_ptr(),
                                    M, N, K, ws.data_ptr() if use_ws else 0, wsb if use_ws else 0)
            ref = OL.round_bf16(dz @ w)
            if masked:
                ref = ref * (ymask > 0)
            assert rel_err(to_host(dx), ref) <= TOL_BF16, (masked, use_ws)


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_linear_wgrad_update_bf16(M, N, K):
    dz = _bf(gen.normal(SEED, "dz", (M, N)) * 0.01)
    x = _bf(gen.normal(SEED, "kx", (M, K)))
    w = gen.uniform(SEED, "kw", (N, K), -0.1, 0.1).astype(np.float64)
    b = (gen.normal(SEED, "kb", (N,)) * 0.1).astype(np.float64)
    mw = (gen.normal(SEED, "mw", (N, K)) * 0.01).astype(np.float64)
    mb = (gen.normal(SEED, "mb", (N,)) * 0.01).astype(np.float64)
    lr, mu = 0.05, 0.9
    s = torch.cuda.current_stream().cuda_stream
    dzd, xd = to_dev(dz, True), to_dev(x, True)
    wd, bd, mwd, mbd = to_dev(w, False), to_dev(b, False), to_dev(mw, False), to_dev(mb, False)
    rw, rb = empty_act(N, K, True), empty_act(1, N, True)
    pd.pd_linear_wgrad_update_bf16(s, dzd.data_ptr(), xd.data_ptr(), wd.data_ptr(), mwd.data_ptr(), rw.data_ptr(),
                                   bd.data_ptr(), mbd.data_ptr(), rb.data_ptr(), M, N, K, lr, mu)
    # oracle: the Linear backward, then the momentum-SGD step
    _, dW, db = OL.linear_backward(x, w, None, dz, False, False, OL.round_bf16)
    w32 = w.astype(np.float32).astype(np.float64); b32 = b.astype(np.float32).astype(np.float64)
    m32 = mw.astype(np.float32).astype(np.float64); mb32 = mb.astype(np.float32).astype(np.float64)
    m_ref = mu * m32 + dW; w_ref = w32 - lr * m_ref
    mb_ref = mu * mb32 + db; b_ref = b32 - lr * mb_ref
    assert rel_err(to_host(mwd), m_ref) <= TOL_F32
    assert rel_err(to_host(wd), w_ref) <= TOL_F32
    assert rel_err(to_host(mbd), mb_ref) <= TOL_F32
    assert rel_err(to_host(bd), b_ref) <= TOL_F32
    assert rel_err(to_host(rw), OL.round_bf16(w_ref)) <= TOL_BF16
    assert rel_err(to_host(rb)[0], OL.round_bf16(b_ref)) <= TOL_BF16
    # the ring copy is exactly the rounding of the fp32 master the kernel produced
    assert torch.equal(rw, wd.to(torch.bfloat16))


# ---------------------------------------------------------------------------------------------
# stages and pipelines driven op by op through pd_forward / pd_backward / pd_update, in the
# oracle's execution order (see parity_harness for what is compared and what is left out)
# ---------------------------------------------------------------------------------------------
def _make(stage_layers, B, M, seed, with_loss=True):
    S = len(stage_layers)
    n_in = stage_layers[0][0][1]
    n_out = [l for l in stage_layers[-1] if l[0] == "linear"][-1][2]
    params = []
    for s, ly in enumerate(stage_layers):
        p = gen.init_params(seed, f"s{s}", ly)
        params.append(p + 0.01 * gen.normal(seed, f"pb{s}", p.shape))        # non-zero biases
    xs = list(gen.normal(seed, "X", (M, B, n_in)))
    labs = list(gen.labels(seed, "Y", (M, B), n_out)) if with_loss else None
    dys = None if with_loss else list(gen.normal(seed, "DY", (M, B, n_out)) * 0.01)
    return params, xs, labs, dys


def _single_stage_case(layers, B, depth, M, precision, lr=0.01, mu=0.9, seed=SEED, with_loss=True, mode=None):
    params, xs, labs, dys = _make([layers], B, M, seed, with_loss)
    assert pd.pd_schedule_1f1b_depth(depth, M) == [tuple(o) for o in schedule_1f1b(1, 1, M, 0, depth_override=depth)]
    if mode is None:   # bf16 trajectories separate by design (see parity_harness): compare op by op on synced weights
        mode = "forced" if precision == pd.PD_BF16_F32ACC else "free"
    return run_case([layers], params, xs, labs, noam=1, precision=precision, depth_override=depth,
                    out_grads=dys, lr=lr, mu=mu, mode=mode)


def test_stage_f32_small_shapes():
    layers = [("linear", 20, 33, True), ("linear", 33, 7, False), ("softmax_xent", 7)]
    _single_stage_case(layers, B=5, depth=3, M=8, precision=pd.PD_F32, lr=0.05)


def test_stage_f32_reductions_longer_than_a_kernel_step():
    # the fp32 kernel walks a reduction 128 elements at a time with the next step's loads in flight: every product
    # here has a reduction of several steps with a ragged last one (forward 300 and 150, input gradient 150 and 70,
    # weight gradient 140 rows), and ragged 32 x 32 output tiles
    layers = [("linear", 300, 150, True), ("linear", 150, 70, False), ("softmax_xent", 70)]
    _single_stage_case(layers, B=140, depth=2, M=4, precision=pd.PD_F32, lr=0.05)


def test_stage_f32_middle_stage_with_relu_output():
    layers = [("linear", 48, 40, True), ("linear", 40, 24, True)]
    _single_stage_case(layers, B=9, depth=2, M=6, precision=pd.PD_F32, lr=0.05, with_loss=False)


def test_stage_bf16_reduced_vgg_fc():
    layers = [("linear", 1096, 520, True), ("linear", 520, 264, True), ("linear", 264, 104, False),
              ("softmax_xent", 104)]
    _single_stage_case(layers, B=64, depth=4, M=10, precision=pd.PD_BF16_F32ACC)


def test_stage_bf16_free_running_short():
    # both sides on their own trajectory: every forward and backward reads version 0, four updates follow
    layers = [("linear", 1096, 520, True), ("linear", 520, 264, True), ("linear", 264, 104, False),
              ("softmax_xent", 104)]
    _single_stage_case(layers, B=64, depth=4, M=4, precision=pd.PD_BF16_F32ACC, mode="free")


def test_stage_bf16_middle_stage_ragged_rows():
    layers = [("linear", 136, 200, True), ("linear", 200, 72, True)]
    _single_stage_case(layers, B=37, depth=3, M=7, precision=pd.PD_BF16_F32ACC, with_loss=False)


def test_fewer_minibatches_than_depth():
    layers = [("linear", 16, 8, False), ("softmax_xent", 8)]
    _single_stage_case(layers, B=4, depth=4, M=2, precision=pd.PD_BF16_F32ACC)
    _single_stage_case(layers, B=4, depth=4, M=1, precision=pd.PD_F32)


@pytest.mark.timeout(1500)
def test_config2_vgg_fc_full_size():
    # the VGG16 classifier stage exactly as configured (25088-4096-4096-1000, minibatch 64, ring depth 4),
    # in the launch configuration the benchmark times; five minibatches cover start-up, a forward on a
    # fresh version, backward passes on stashed versions (B4 reads version 1 while the latest is 4), drain
    print("config 2 full size: oracle + GPU, 5 minibatches", flush=True)
    params, xs, labs, _ = _make([gen.config2_vgg_fc()], 64, 5, SEED + 1)
    out = run_case([gen.config2_vgg_fc()], params, xs, labs, noam=1, precision=pd.PD_BF16_F32ACC, depth_override=4,
                   mode="forced", verbose=True)
    print("ambiguous ReLU decisions:", out["flips"], flush=True)


def test_stage_wide_softmax_rows():
    # more than 2048 classes: the loss runs on the single-pass kernel that keeps a row in registers
    # (4104 = 1026 float4: four full rounds of 256 lanes and a ragged fifth; 32768 = the widest row it takes)
    for classes, precision in ((4104, pd.PD_F32), (4104, pd.PD_BF16_F32ACC), (32768, pd.PD_BF16_F32ACC),
                               (32776, pd.PD_BF16_F32ACC)):   # the last one is too wide: three-pass kernel
        layers = [("linear", 40, classes, False), ("softmax_xent", classes)]
        _single_stage_case(layers, B=6, depth=2, M=4, precision=precision, lr=0.05)


@pytest.mark.parametrize("precision", [pd.PD_F32, pd.PD_BF16_F32ACC])
def test_rmsprop_stages(precision):
    # RMSProp (the paper's optimiser for Inception-v3) through every update kernel: the fused minibatch-sized Linear
    # update, the partial-sum reduce + update of convolutions, the many-row product with the step in its store
    bf16 = precision == pd.PD_BF16_F32ACC
    kw = dict(optimizer="rmsprop", eps=1.0, lr=0.045, mu=0.9)
    layers = [("linear", 40, 48, True), ("linear", 48, 16, False), ("softmax_xent", 16)]
    params, xs, labs, _ = _make([layers], 8, 6, SEED + 21)
    run_case([layers], params, xs, labs, noam=1, precision=precision, depth_override=3, mode="forced" if bf16 else "free", **kw)
    if not bf16:
        return
    conv = [("conv2d", 8, 16, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2), ("conv2d", 16, 32, 1, 1, 1, 0, 0, True),
            ("linear", 4 * 4 * 32, 16, False), ("softmax_xent", 16)]
    params = [gen.init_params(SEED + 22, "rc", conv)]
    xs = list(gen.normal(SEED + 22, "X", (4, 4, 8, 8, 8)))
    labs = list(gen.labels(SEED + 22, "Y", (4, 4), 16))
    run_case([conv], params, xs, labs, noam=1, precision=precision, depth_override=2, mode="forced", in_hw=(8, 8), **kw)
    many = [("lstm", 32, 24, 24), ("linear", 24, 40, False), ("softmax_xent", 40)]   # 24 steps x 24 rows = 576 rows
    params = [gen.init_params(SEED + 23, "rl", many)]
    xs = list(gen.normal(SEED + 23, "X", (3, 24, 24, 32)))
    labs = list(gen.labels(SEED + 23, "Y", (3, 24, 24), 40))
    run_case([many], params, xs, labs, noam=1, precision=precision, depth_override=2, mode="forced", minibatch=24, **kw)


def test_learning_rate_schedule_f32():
    # the rate of a stage is changed between updates (Section 5.1: Inception-v3's rate decays per epoch); the oracle
    # stage gets the same schedule by assignment
    from gpu_util import GpuStage
    from oracle.pipeline import Stage
    layers = [("linear", 24, 32, True), ("linear", 32, 10, False), ("softmax_xent", 10)]
    p = gen.init_params(SEED + 31, "lr", layers)
    M, B = 9, 6
    xs = gen.normal(SEED + 31, "X", (M, B, 24)); labs = gen.labels(SEED + 31, "Y", (M, B), 10)
    o = Stage(layers, p, 1, "f32", 0.045, 0.9, optimizer="rmsprop", eps=1.0)
    g = GpuStage(layers, p, minibatch=B, precision=pd.PD_F32, in_flight_override=1, lr=0.045, momentum=0.9, optimizer=1, eps=1.0)
    try:
        xd, ld = to_dev(xs, False), labels_dev(labs)
        loss = torch.zeros(M, dtype=torch.float32, device=dev())
        lr = 0.045
        for i in range(M):
            if i and i % 3 == 0:                      # an "epoch" of three minibatches: decay by 0.94
                lr *= 0.94
                o.lr = lr
                pd.pd_stage_set_lr(g.h, lr)
            _, l_o = o.forward(i, xs[i].astype(np.float64), labs[i]); o.backward(i, None, need_dx=False); o.update(i)
            pd.pd_forward(g.h, i, xd[i].data_ptr(), ld[i].data_ptr(), 0, loss[i:].data_ptr())
            pd.pd_backward(g.h, i, 0, 0); pd.pd_update(g.h)
            torch.cuda.synchronize()
            assert abs(loss[i].item() - l_o) <= TOL_F32 * abs(l_o)
        assert rel_err(pd.pd_stage_get_params(g.h), o.master) <= TOL_F32
        assert rel_err(pd.pd_stage_get_momentum(g.h), o.mom) <= TOL_F32
        with pytest.raises(pd.PdError):
            pd.pd_stage_set_lr(g.h, float("nan"))
        with pytest.raises(pd.PdError):
            pd.pd_stage_set_lr(g.h, -1.0)
    finally:
        g.close()


def test_one_row_minibatch_and_depth_one():
    layers = [("linear", 24, 16, True), ("linear", 16, 8, False), ("softmax_xent", 8)]
    _single_stage_case(layers, B=1, depth=1, M=4, precision=pd.PD_BF16_F32ACC)
    _single_stage_case(layers, B=1, depth=2, M=5, precision=pd.PD_F32)


# ---------------------------------------------------------------------------------------------
# convolution and pooling kernels on their own: identical inputs on both sides, element by element
# ---------------------------------------------------------------------------------------------
CONVS = [  # N, H, W, c_in, c_out, kh, kw, stride, pad_h, pad_w
    (2, 12, 12, 3, 64, 3, 3, 1, 1, 1),      # first layer of an image network (27-wide reduction)
    (3, 10, 10, 3, 16, 3, 3, 1, 1, 1),      # same path, fewer channels, ragged pixel count
    (2, 9, 11, 16, 24, 3, 3, 1, 1, 1),      # generic path, ragged everything
    (1, 16, 16, 64, 64, 3, 3, 1, 1, 1),
    (2, 8, 8, 128, 128, 3, 3, 1, 1, 1),     # 128-wide weight-gradient tiles
    (2, 8, 8, 136, 200, 3, 3, 1, 1, 1),     # ... with ragged channel tiles
    (2, 12, 12, 32, 48, 1, 1, 1, 0, 0),     # 1x1
    (2, 17, 17, 16, 16, 1, 7, 1, 0, 3),     # 1x7
    (2, 17, 17, 16, 16, 7, 1, 1, 3, 0),     # 7x1
    (1, 40, 40, 8, 8, 3, 3, 1, 1, 1),       # many pixels, few channels
    (600, 1, 1, 136, 264, 1, 1, 1, 0, 0),   # a plain matrix product with many rows (256 x 256-tile wgrad)
    (600, 1, 1, 13312, 1280, 1, 1, 1, 0, 0),  # ... with 260 output tiles: four over a round of the chip, rows split
    # size-preserving stride-1 layers with >= 32 input channels: the all-taps-per-workgroup weight-gradient kernel
    (2, 17, 17, 32, 40, 1, 7, 1, 0, 3),     # 1x7, <= 64 output channels (pixel halves as separate partials)
    (2, 17, 17, 40, 72, 7, 1, 1, 3, 0),     # 7x1: filter rows in groups of 3, 3, 1
    (2, 9, 9, 48, 64, 5, 5, 1, 2, 2),       # 5x5: one filter row per workgroup
    (3, 8, 8, 64, 136, 1, 3, 1, 0, 1),      # 1x3, ragged output-channel tile
    (3, 8, 8, 72, 48, 3, 1, 1, 1, 0),       # 3x1, ragged input-channel tile
    (70, 4, 4, 32, 32, 1, 1, 1, 0, 0),      # images smaller than one 64-pixel stage
    (4, 35, 35, 64, 96, 3, 3, 1, 1, 1),     # several pixel ranges per tile
    (3, 20, 28, 160, 256, 3, 3, 1, 1, 1),   # several channel tiles on both sides
    # stride 1 with less than "same" padding (fewer output rows and columns than input ones): the same kernel, which
    # numbers pixels by input rows and reads dz as zero where a position has no output
    (2, 13, 13, 32, 40, 3, 3, 1, 0, 0),     # unpadded 3x3
    (1, 20, 17, 80, 192, 3, 3, 1, 0, 0),    # ... several channel tiles, ragged input-channel tile
    (5, 6, 9, 32, 32, 3, 3, 1, 0, 0),       # ... images shorter than a 64-pixel stage, several per stage
    (2, 12, 12, 32, 16, 5, 5, 1, 1, 1),     # 5x5 padded by one
    (2, 11, 10, 40, 24, 1, 7, 1, 0, 2),     # 1x7 padded by two
]


def _conv_data(geom):
    N, H, W, ci, co, kh, kw, stride, ph, pw = geom
    x = _bf(gen.normal(SEED, "cx", (N, H, W, ci)))
    w = _bf(gen.uniform(SEED, "cw", (co, kh, kw, ci), -0.2, 0.2))
    b = _bf(gen.normal(SEED, "cb", (co,)) * 0.1)
    return x, w, b


@pytest.mark.parametrize("geom", CONVS + [(2, 13, 13, 16, 32, 3, 3, 2, 1, 1), (2, 12, 12, 3, 32, 3, 3, 2, 0, 0)])
def test_conv_fwd_bf16(geom):
    N, H, W, ci, co, kh, kw, stride, ph, pw = geom
    x, w, b = _conv_data(geom)
    s = torch.cuda.current_stream().cuda_stream
    xd, wd, bd = to_dev(x, True), to_dev(w, True), to_dev(b, True)
    for relu in (True, False):
        ref = OL.conv2d_forward(x, w, b, stride, ph, pw, relu, OL.round_bf16)
        y = torch.empty(ref.shape, dtype=torch.bfloat16, device=dev())
        pd.pd_conv_fwd_bf16(s, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), geom, relu)
        assert rel_err(to_host(y), ref) <= TOL_BF16
        assert np.max(np.abs(to_host(y) - ref) / np.maximum(np.abs(ref), 1e-2)) < 2 ** -6   # at most one bf16 step


# layers with >= 256 channels on the output side of the product, forced onto the 256 x 256-tile kernel
WIDE_CONVS = [(2, 12, 12, 64, 256, 3, 3, 1, 1, 1), (1, 20, 20, 32, 768, 1, 1, 1, 0, 0), (2, 9, 9, 40, 520, 3, 3, 1, 1, 1),
              (2, 12, 12, 256, 64, 3, 3, 1, 1, 1), (2, 9, 9, 512, 48, 1, 7, 1, 0, 3)]


# 3 x 3 / stride 1 / pad 1 layers with 64-channel chunks: the kernel that keeps a tile's input and halo in LDS.  Sizes
# that are not multiples of the 8 x 32 pixel tile, one to four channel chunks, ragged output-channel tiles, several
# images; the same shapes with that kernel switched off go through the implicit-GEMM kernel
HALO_CONVS = [(2, 13, 37, 64, 64, 3, 3, 1, 1, 1), (1, 9, 40, 128, 72, 3, 3, 1, 1, 1), (3, 8, 8, 64, 136, 3, 3, 1, 1, 1),
              (1, 17, 33, 256, 128, 3, 3, 1, 1, 1), (2, 5, 70, 192, 40, 3, 3, 1, 1, 1), (1, 56, 56, 64, 256, 3, 3, 1, 1, 1),
              # 64 -> at most 64 channels: the variant whose workgroups keep the weights and walk over several tiles
              # (more tiles than compute units, so some workgroups take two; fewer filters than a tile has columns)
              (9, 72, 100, 64, 56, 3, 3, 1, 1, 1), (3, 20, 70, 64, 40, 3, 3, 1, 1, 1)]


# halo: 1 = on, 2 = on without the weights-resident variant, 0 = off
@pytest.mark.parametrize("halo", [1, 2, 0])
@pytest.mark.parametrize("geom", HALO_CONVS)
def test_conv_fwd_and_dgrad_halo_kernel(geom, halo):
    old = pd.pd_set_conv_halo(halo)
    try:
        test_conv_fwd_bf16(geom)
        test_conv_dgrad_bf16(geom)
    finally:
        pd.pd_set_conv_halo(old)


@pytest.mark.parametrize("geom", WIDE_CONVS)
def test_conv_fwd_bf16_wide_tiles(geom, big_tiles):
    test_conv_fwd_bf16(geom)


@pytest.mark.parametrize("geom", WIDE_CONVS)
def test_conv_dgrad_bf16_wide_tiles(geom, big_tiles):
    test_conv_dgrad_bf16(geom)


@pytest.mark.parametrize("geom", CONVS)
def test_conv_dgrad_bf16(geom):
    N, H, W, ci, co, kh, kw, stride, ph, pw = geom
    x, w, b = _conv_data(geom)
    y = OL.conv2d_forward(x, w, b, stride, ph, pw, False, OL.round_bf16)
    dz = _bf(gen.normal(SEED, "cdz", y.shape) * 0.01)
    xmask = _bf(np.maximum(gen.normal(SEED, "cm", x.shape), 0.0))
    s = torch.cuda.current_stream().cuda_stream
    wt = torch.empty(w.size, dtype=torch.bfloat16, device=dev())
    dzd, wd, md = to_dev(dz, True), to_dev(w, True), to_dev(xmask, True)
    for masked in (True, False):
        ref, _, _ = OL.conv2d_backward(x, w, y, dz, stride, ph, pw, False, True, OL.round_bf16)
        if masked:
            ref = ref * (xmask > 0)
        dx = torch.empty(x.shape, dtype=torch.bfloat16, device=dev())
        pd.pd_conv_dgrad_bf16(s, dzd.data_ptr(), wd.data_ptr(), md.data_ptr() if masked else 0, dx.data_ptr(),
                              wt.data_ptr(), geom)
        assert rel_err(to_host(dx), ref) <= TOL_BF16, masked


@pytest.mark.parametrize("geom", CONVS + [(2, 13, 13, 16, 32, 3, 3, 2, 1, 1)])
def test_conv_wgrad_update_bf16(geom):
    N, H, W, ci, co, kh, kw, stride, ph, pw = geom
    x, w, b = _conv_data(geom)
    y = OL.conv2d_forward(x, w, b, stride, ph, pw, False, OL.round_bf16)
    dz = _bf(gen.normal(SEED, "cdz", y.shape) * 0.01)
    w32 = gen.uniform(SEED, "cw32", w.shape, -0.2, 0.2).astype(np.float64)
    b32 = (gen.normal(SEED, "cb32", (co,)) * 0.1).astype(np.float64)
    mw = (gen.normal(SEED, "cmw", w.shape) * 0.01).astype(np.float64)
    mb = (gen.normal(SEED, "cmb", (co,)) * 0.01).astype(np.float64)
    lr, mu = 0.05, 0.9
    s = torch.cuda.current_stream().cuda_stream
    splits = pd.pd_conv_wgrad_splits(geom)
    part = torch.empty(splits * (w.size + co), dtype=torch.float32, device=dev())
    wd, bd, mwd, mbd = to_dev(w32, False), to_dev(b32, False), to_dev(mw, False), to_dev(mb, False)
    rw = torch.empty(w.shape, dtype=torch.bfloat16, device=dev()); rb = torch.empty(co, dtype=torch.bfloat16, device=dev())
    dzd, xd = to_dev(dz, True), to_dev(x, True)
    pd.pd_conv_wgrad_update_bf16(s, dzd.data_ptr(), xd.data_ptr(), part.data_ptr(),
                                 wd.data_ptr(), mwd.data_ptr(), rw.data_ptr(), bd.data_ptr(), mbd.data_ptr(),
                                 rb.data_ptr(), geom, lr, mu)
    _, dW, db = OL.conv2d_backward(x, w, y, dz, stride, ph, pw, False, False, OL.round_bf16)
    f32 = lambda a: a.astype(np.float32).astype(np.float64)
    m_ref = mu * f32(mw) + dW; w_ref = f32(w32) - lr * m_ref
    mb_ref = mu * f32(mb) + db; b_ref = f32(b32) - lr * mb_ref
    assert rel_err(to_host(mwd), m_ref) <= TOL_F32
    assert rel_err(to_host(wd), w_ref) <= TOL_F32
    assert rel_err(to_host(mbd), mb_ref) <= TOL_F32
    assert rel_err(to_host(bd), b_ref) <= TOL_F32
    assert torch.equal(rw, wd.to(torch.bfloat16)) and torch.equal(rb, bd.to(torch.bfloat16))


@pytest.mark.parametrize("N,H,W,Cn", [(2, 8, 8, 8), (3, 6, 10, 24), (1, 224, 224, 64)])
def test_maxpool2x2_bf16(N, H, W, Cn):
    # bf16 values drawn from a coarse grid so that ties inside windows are common
    x = _bf(np.round(gen.normal(SEED, "px", (N, H, W, Cn)) * 4) / 4)
    x = np.maximum(x, 0.0) if Cn == 24 else x
    s = torch.cuda.current_stream().cuda_stream
    xd = to_dev(x, True)
    y_ref = OL.maxpool2d_forward(x, 2, 2)
    y = torch.empty(y_ref.shape, dtype=torch.bfloat16, device=dev())
    pd.pd_maxpool2x2_fwd_bf16(s, xd.data_ptr(), y.data_ptr(), N, H, W, Cn)
    assert np.array_equal(to_host(y), y_ref)
    dy = _bf(gen.normal(SEED, "pdy", y_ref.shape))
    dyd = to_dev(dy, True)
    for relu_mask in (False, True):
        ref = OL.maxpool2d_backward(x, y_ref, dy, 2, 2)
        if relu_mask:
            ref = ref * (x > 0)
        dx = torch.empty(x.shape, dtype=torch.bfloat16, device=dev())
        pd.pd_maxpool2x2_bwd_bf16(s, xd.data_ptr(), y.data_ptr(), dyd.data_ptr(), dx.data_ptr(), N, H, W, Cn, relu_mask)
        assert np.array_equal(to_host(dx), ref), relu_mask       # pure routing: bit-exact
    # the pair that records the routing in the forward pass (what a stage runs): same outputs, no x or y in backward
    route = torch.zeros(N * (H // 2) * (W // 2) * (Cn // 8), dtype=torch.int32, device=dev())
    y2 = torch.empty_like(y)
    pd.pd_maxpool2x2_fwd_route_bf16(s, xd.data_ptr(), y2.data_ptr(), route.data_ptr(), N, H, W, Cn)
    assert torch.equal(y, y2)
    for relu_mask in (False, True):
        ref = OL.maxpool2d_backward(x, y_ref, dy, 2, 2)
        if relu_mask:
            ref = ref * (x > 0)
        dx = torch.full(x.shape, 7.0, dtype=torch.bfloat16, device=dev())
        pd.pd_maxpool2x2_bwd_route_bf16(s, route.data_ptr(), dyd.data_ptr(), dx.data_ptr(), N, H, W, Cn, relu_mask)
        assert np.array_equal(to_host(dx), ref), relu_mask


# ---------------------------------------------------------------------------------------------
# convolution / pooling stages (bf16): implicit-GEMM forward and dgrad, transposing wgrad with
# split pixel ranges, the small-reduction first layer, 2x2 pooling with the first-maximum rule
# ---------------------------------------------------------------------------------------------
def _image_stage_case(layers, B, hw, c_in, depth, M, seed=SEED + 2, with_loss=True, lr=0.01, mode="forced",
                      verbose=False, force_acts=False):
    p = gen.init_params(seed, "c", layers)
    params = [p + 0.01 * gen.normal(seed, "cb", p.shape)]
    xs = list(gen.normal(seed, "X", (M, B, hw[0], hw[1], c_in)))
    o_shape = None
    labs = dys = None
    if with_loss:
        classes = layers[-1][1]
        labs = list(gen.labels(seed, "Y", (M, B), classes))
    else:
        from oracle.pipeline import Stage
        probe = Stage(layers, params[0], 1, "bf16")
        o_shape = probe.forward(0, xs[0].astype(np.float64))[0].shape
        dys = list(gen.normal(seed, "DY", (M,) + tuple(o_shape)) * 0.01)
    return run_case([layers], params, xs, labs, noam=1, precision=pd.PD_BF16_F32ACC, depth_override=depth,
                    out_grads=dys, lr=lr, mode=mode, in_hw=hw, verbose=verbose, force_acts=force_acts)


def test_conv_stage_small_vgg_like():
    layers = [("conv2d", 3, 16, 3, 3, 1, 1, 1, True), ("conv2d", 16, 16, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2),
              ("conv2d", 16, 32, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2), ("linear", 3 * 3 * 32, 16, False),
              ("softmax_xent", 16)]
    _image_stage_case(layers, B=3, hw=(12, 12), c_in=3, depth=2, M=5, lr=0.05)


def test_conv_stage_wide_channels_no_loss():
    # 128-channel layers take the 128x128 weight-gradient tiles; 10x10 images give ragged pixel tiles
    layers = [("conv2d", 8, 128, 3, 3, 1, 1, 1, True), ("conv2d", 128, 128, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2),
              ("conv2d", 128, 72, 3, 3, 1, 1, 1, False)]
    _image_stage_case(layers, B=3, hw=(10, 10), c_in=8, depth=3, M=4, with_loss=False)


def test_conv_stage_free_running_short():
    layers = [("conv2d", 3, 64, 3, 3, 1, 1, 1, True), ("conv2d", 64, 64, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2)]
    _image_stage_case(layers, B=2, hw=(16, 16), c_in=3, depth=2, M=2, with_loss=False, mode="free")


@pytest.mark.timeout(1500)
def test_config3_vgg_conv_full_geometry_reduced_batch():
    # the VGG16 conv stage at its real geometry (3 x 224 x 224 images, 64-64-P-128-128-P-256x3-P) with two images
    # per minibatch, the size the oracle finishes in seconds.  Every forward pass is the GPU's own and compared in
    # full; the stored activations are then the oracle's (ten bf16 layers deep, one-ulp differences turn into
    # differing ReLU / max-pooling decisions), so every backward pass and every update must meet the tolerance
    # on every row, with no loosened branch
    print("config 3 geometry, minibatch 2: oracle + GPU", flush=True)
    out = _image_stage_case(gen.config3_vgg_conv(), B=2, hw=(224, 224), c_in=3, depth=2, M=3, with_loss=False,
                            verbose=True, force_acts=True)
    assert out["updates_compared"] == (3, 3), out["updates_compared"]


# ---------------------------------------------------------------------------------------------
# strided-convolution gradient, general pooling, branched blocks (the pieces of Inception-shaped stages)
# ---------------------------------------------------------------------------------------------
STRIDED = [(2, 13, 13, 16, 32, 3, 3, 2, 1, 1), (2, 12, 12, 8, 16, 3, 3, 2, 0, 0), (1, 35, 35, 24, 40, 3, 3, 2, 0, 0),
           (2, 9, 10, 16, 8, 1, 1, 2, 0, 0), (1, 17, 17, 136, 72, 3, 3, 2, 0, 0), (2, 11, 11, 8, 8, 5, 5, 3, 2, 2)]


@pytest.mark.parametrize("geom", STRIDED)
def test_conv_dgrad_strided_bf16(geom):
    test_conv_dgrad_bf16(geom)


@pytest.mark.parametrize("is_max,N,H,W,Cn,k,stride,pad", [
    (True, 2, 9, 7, 8, 3, 2, 0), (True, 1, 35, 35, 24, 3, 2, 0), (True, 2, 6, 6, 16, 3, 1, 0), (True, 2, 8, 8, 8, 2, 2, 0),
    (True, 1, 10, 11, 8, 3, 3, 0), (True, 3, 3, 3, 8, 3, 1, 0), (True, 2, 9, 9, 16, 4, 1, 0), (True, 1, 12, 12, 8, 5, 2, 0),
    (False, 2, 7, 6, 8, 3, 1, 1), (False, 1, 17, 17, 40, 3, 1, 1), (False, 3, 8, 8, 16, 8, 1, 0), (False, 2, 9, 9, 8, 3, 2, 1)])
def test_pool2d_bf16(is_max, N, H, W, Cn, k, stride, pad):
    # coarse grid of values so that ties inside max windows are common
    x = _bf(np.round(gen.normal(SEED, "gx", (N, H, W, Cn)) * 4) / 4)
    s = torch.cuda.current_stream().cuda_stream
    xd = to_dev(x, True)
    y_ref = OL.maxpool2d_forward(x, k, stride) if is_max else OL.avgpool2d_forward(x, k, stride, pad, OL.round_bf16)
    y = torch.empty(y_ref.shape, dtype=torch.bfloat16, device=dev())
    pg = (N, H, W, Cn, k, stride, pad)
    pd.pd_pool2d_fwd_bf16(s, is_max, xd.data_ptr(), y.data_ptr(), pg)
    if is_max:
        assert np.array_equal(to_host(y), y_ref)
    else:
        assert rel_err(to_host(y), y_ref) <= 2 ** -8
    dy = _bf(gen.normal(SEED, "gdy", y_ref.shape))
    dyd = to_dev(dy, True)
    yd = to_dev(y_ref, True)
    for relu_mask in (False, True):
        ref = (OL.round_bf16(OL.maxpool2d_backward(x, y_ref, dy, k, stride)) if is_max
               else OL.avgpool2d_backward(x.shape, dy, k, stride, pad, OL.round_bf16))
        if relu_mask:
            ref = ref * (x > 0)
        dx = torch.empty(x.shape, dtype=torch.bfloat16, device=dev())
        pd.pd_pool2d_bwd_bf16(s, is_max, xd.data_ptr(), yd.data_ptr(), dyd.data_ptr(), dx.data_ptr(), pg, relu_mask)
        got = to_host(dx)
        # routing is exact; sums of up to k*k bf16 terms may round one step apart (fp32 vs fp64 accumulation)
        if is_max:
            assert np.array_equal(got == 0, ref == 0), relu_mask
        assert np.all(np.abs(got - ref) <= 2 ** -7 * np.abs(ref) + 1e-6), relu_mask
        if is_max and k <= 4:
            # the pair that records the routing in the forward pass (what a stage runs): the same bits as the pair above
            route = torch.zeros(int(np.prod(y_ref.shape)), dtype=torch.uint8, device=dev())
            y2 = torch.empty_like(yd)
            pd.pd_pool2d_fwd_route_bf16(s, xd.data_ptr(), y2.data_ptr(), route.data_ptr(), pg)
            assert torch.equal(y2, yd)
            dx2 = torch.full(x.shape, 7.0, dtype=torch.bfloat16, device=dev())
            pd.pd_pool2d_bwd_route_bf16(s, route.data_ptr(), dyd.data_ptr(), dx2.data_ptr(), pg, relu_mask)
            assert torch.equal(dx2, dx), relu_mask


def _inception_like(c0=8):
    """Stem conv, a four-branch block (1x1 | 1x1-3x3 | 1x7-7x1 | avgpool-1x1), a reduction block (strided 3x3 |
    1x1-strided 3x3 | overlapping max pool), global average pooling, classifier."""
    blk1 = ("concat", [[("conv2d", 16, 16, 1, 1, 1, 0, 0, True)],
                       [("conv2d", 16, 8, 1, 1, 1, 0, 0, True), ("conv2d", 8, 24, 3, 3, 1, 1, 1, True)],
                       [("conv2d", 16, 8, 1, 7, 1, 0, 3, True), ("conv2d", 8, 8, 7, 1, 1, 3, 0, True)],
                       [("avgpool2d", 3, 1, 1), ("conv2d", 16, 8, 1, 1, 1, 0, 0, True)]])
    blk2 = ("concat", [[("conv2d", 56, 24, 3, 3, 2, 0, 0, True)],
                       [("conv2d", 56, 16, 1, 1, 1, 0, 0, True), ("conv2d", 16, 16, 3, 3, 2, 0, 0, True)],
                       [("maxpool2d", 3, 2)]])
    return [("conv2d", c0, 16, 3, 3, 1, 1, 1, True), blk1, blk2, ("avgpool2d", 4, 1, 0), ("linear", 96, 16, False),
            ("softmax_xent", 16)]


def test_block_stage_with_loss():
    _image_stage_case(_inception_like(), B=3, hw=(9, 9), c_in=8, depth=2, M=4, lr=0.05)


def test_block_first_in_stage_and_last_no_loss():
    # the stage starts with a block (its branches read the stage input; dL/d(input) is the sum over branches) and
    # ends with one (the output gradient is split over the branches)
    blk = ("concat", [[("conv2d", 8, 16, 1, 1, 1, 0, 0, True)],
                      [("conv2d", 8, 8, 3, 3, 1, 1, 1, True), ("conv2d", 8, 8, 3, 3, 1, 1, 1, False)],
                      [("avgpool2d", 3, 1, 1), ("conv2d", 8, 8, 1, 1, 1, 0, 0, True)]])
    blk_b = ("concat", [[("conv2d", 32, 8, 1, 1, 1, 0, 0, True)], [("maxpool2d", 3, 1), ("conv2d", 32, 16, 1, 1, 1, 1, 1, True)]])
    _image_stage_case([blk, blk_b], B=2, hw=(10, 10, 8), c_in=8, depth=3, M=4, with_loss=False)


def test_block_stage_free_running_short():
    _image_stage_case(_inception_like()[:3], B=2, hw=(9, 9), c_in=8, depth=2, M=2, with_loss=False, mode="free")


def test_inception_like_four_stage_pipeline():
    """Four image stages with blocks.  (1) Op by op in lockstep with the oracle, teacher-forced, every backward pass and
    every update -- master weights, momentum, ring copies -- at the full tolerance.  (2) The same stream through
    pd_pipeline_run on four streams, free-running: op traces and version ids equal to the oracle's, losses and final
    weights at tolerance, and everything, momentum included, bit-equal to the serialised GPU run: the kernels are
    deterministic, so a missing dependency between the streams would show."""
    full = _inception_like()
    st = [[full[0]], [full[1]], [full[2]], full[3:]]
    hws = [(9, 9, 8), (9, 9, 16), (9, 9, 56), (4, 4, 96)]
    S, B, M, seed = 4, 3, 6, SEED + 9
    params = []
    for s, ly in enumerate(st):
        p = gen.init_params(seed, f"i{s}", ly)
        params.append(p + 0.01 * gen.normal(seed, f"ib{s}", p.shape))
    xs = gen.normal(seed, "X", (M, B, 9, 9, 8))
    labs = gen.labels(seed, "Y", (M, B), 16)
    out = run_case(st, params, list(xs), list(labs), noam=S, precision=pd.PD_BF16_F32ACC, lr=0.02, mode="forced",
                   in_hw=hws, force_acts=True)
    assert out["updates_compared"] == (S * M, S * M), out["updates_compared"]
    ref = run_case(st, params, list(xs), list(labs), noam=S, precision=pd.PD_BF16_F32ACC, lr=0.02, in_hw=hws,
                   compare=False)
    streams = [torch.cuda.Stream(device=dev()) for _ in range(S)]
    gs = [GpuStage(st[s], params[s], minibatch=B, precision=pd.PD_BF16_F32ACC, stage_index=s, num_stages=S, noam=S,
                   lr=0.02, stream=streams[s], in_hw=hws[s]) for s in range(S)]
    try:
        xd = to_dev(xs.reshape(M * B, -1), True)
        ld = labels_dev(labs)
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        pd.pd_pipeline_run([g.h for g in gs], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        ost, ol = run_pipeline(st, params, [x.astype(np.float64) for x in xs], list(labs), S, mode="bf16", lr=0.02)
        for s in range(S):
            assert pd.pd_stage_trace(gs[s].h) == [tuple(t) for t in ost[s].trace]
        assert np.all(np.abs(to_host(losses) - np.array(ol)) <= TOL_BF16 * np.abs(np.array(ol)))
        assert np.array_equal(to_host(losses), ref["losses"])
        for s in range(S):
            assert rel_err(pd.pd_stage_get_params(gs[s].h), ost[s].master) <= TOL_BF16
            assert np.array_equal(pd.pd_stage_get_params(gs[s].h), ref["params"][s]), s
            assert np.array_equal(pd.pd_stage_get_momentum(gs[s].h), ref["mom"][s]), s
    finally:
        for g in gs:
            g.close()


@pytest.mark.timeout(900)
def test_config5_inception_full_geometry_reduced_batch():
    # the Inception-shaped four-stage split at its real geometry (299 x 299 images, full channel counts) with two
    # images per minibatch, the size the oracle finishes in seconds; every op compared in lockstep
    print("config 5 geometry, minibatch 2: oracle + GPU", flush=True)
    st, sizes = gen.config5_inception(1000, 1.0)
    seed, M, B = SEED + 5, 3, 2
    params = [gen.init_params(seed, f"s{s}", ly) for s, ly in enumerate(st)]
    xs = list(gen.normal(seed, "X", (M, B, 299, 299, 3)))
    labs = list(gen.labels(seed, "Y", (M, B), 1000))
    out = run_case(st, params, xs, labs, noam=4, precision=pd.PD_BF16_F32ACC, lr=1e-3, mode="forced", in_hw=sizes,
                   verbose=True, force_acts=True)
    print("ambiguous ReLU decisions:", out["flips"], "updates compared (strict, all):", out["updates_compared"], flush=True)


def test_config5_reduced_width_pipeline_run():
    """The same four stages at a quarter of the channel counts, on four streams through pd_pipeline_run, free-running
    for a short stream (bf16 trajectories separate with length): traces bit-exact, losses at tolerance."""
    st, sizes = gen.config5_inception(16, 0.25)
    S, B, M, seed = 4, 2, 3, SEED + 6
    params = [gen.init_params(seed, f"w{s}", ly) for s, ly in enumerate(st)]
    xs = gen.normal(seed, "X", (M, B, 299, 299, 3))
    labs = gen.labels(seed, "Y", (M, B), 16)
    streams = [torch.cuda.Stream(device=dev()) for _ in range(S)]
    gs = [GpuStage(st[s], params[s], minibatch=B, precision=pd.PD_BF16_F32ACC, stage_index=s, num_stages=S, noam=S,
                   lr=1e-3, stream=streams[s], in_hw=sizes[s]) for s in range(S)]
    try:
        xd = to_dev(xs.reshape(M * B, -1), True)
        ld = labels_dev(labs)
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        pd.pd_pipeline_run([g.h for g in gs], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        ost, ol = run_pipeline(st, params, [x.astype(np.float64) for x in xs], list(labs), S, mode="bf16", lr=1e-3)
        for s in range(S):
            assert pd.pd_stage_trace(gs[s].h) == [tuple(t) for t in ost[s].trace]
        assert np.all(np.abs(to_host(losses) - np.array(ol)) <= TOL_BF16 * np.abs(np.array(ol))), (to_host(losses), ol)
        for s in range(S):
            assert rel_err(pd.pd_stage_get_params(gs[s].h), ost[s].master) <= TOL_BF16
    finally:
        for g in gs:
            g.close()


# ---------------------------------------------------------------------------------------------
# LSTM stages (bf16, time-major sequences): input projection GEMM, per-step recurrent GEMM + cell kernel,
# back-propagation through time, the two weight matrices updated from dG
# ---------------------------------------------------------------------------------------------
def _seq_case(stage_layers, B, T, noam, M, seed=SEED + 3, depth_override=0, with_loss=True, lr=0.05, mode="forced",
              verbose=False):
    I = stage_layers[0][0][1]
    params = []
    for s, ly in enumerate(stage_layers):
        p = gen.init_params(seed, f"q{s}", ly)
        params.append(p + 0.01 * gen.normal(seed, f"qb{s}", p.shape))
    xs = list(gen.normal(seed, "X", (M, T, B, I)))
    labs = dys = None
    if with_loss:
        V = stage_layers[-1][-1][1]
        labs = list(gen.labels(seed, "Y", (M, T, B), V))
    else:
        Hh = stage_layers[-1][-1][2]
        dys = list(gen.normal(seed, "DY", (M, T, B, Hh)) * 0.01)
    return run_case(stage_layers, params, xs, labs, noam=noam, precision=pd.PD_BF16_F32ACC,
                    depth_override=depth_override, out_grads=dys, lr=lr, mode=mode, minibatch=B, verbose=verbose)


def test_lstm_single_stage_no_loss():
    _seq_case([[("lstm", 24, 16, 5)]], B=3, T=5, noam=1, M=4, depth_override=2, with_loss=False)


def test_lstm_stage_with_vocab_projection():
    _seq_case([[("lstm", 16, 24, 6), ("linear", 24, 40, False), ("softmax_xent", 40)]], B=4, T=6, noam=1, M=4,
              depth_override=2)


def test_lstm_two_stacked_in_one_stage_free_running():
    _seq_case([[("lstm", 16, 16, 4), ("lstm", 16, 8, 4), ("linear", 8, 16, False), ("softmax_xent", 16)]], B=2, T=4,
              noam=1, M=2, depth_override=2, mode="free")


def test_lstm_many_rows_uses_partial_sum_weight_gradient():
    # seq_len * minibatch = 512 rows: the weight gradients go through the large-reduction kernel
    _seq_case([[("lstm", 24, 16, 16), ("linear", 16, 40, False), ("softmax_xent", 40)]], B=32, T=16, noam=1, M=3,
              depth_override=2)


def test_s2vt_shaped_two_stage_pipeline():
    # the two-stage sequence model at reduced widths: ragged against every tile size
    sl = gen.config4_s2vt(input_size=136, hidden=72, vocab=200, seq_len=7)
    _seq_case(sl, B=5, T=7, noam=2, M=5)


@pytest.mark.timeout(1500)
def test_config4_s2vt_full_width_reduced_vocab_and_length():
    # hidden 1000 and input 4096 as configured, minibatch 64; vocabulary and sequence length reduced so the
    # oracle finishes in seconds
    print("config 4 widths (4096 -> 1000 -> 1000), T = 8, vocab 2000", flush=True)
    sl = gen.config4_s2vt(vocab=2000, seq_len=8)
    _seq_case(sl, B=64, T=8, noam=2, M=3, lr=0.01, verbose=True)


# ---------------------------------------------------------------------------------------------
# the whole pipeline.  First op by op against the oracle (serialised), then the same run through
# pd_pipeline_run with one stream per stage: the kernels are deterministic, so the concurrent run
# must reproduce the serialised one bit for bit -- any missing inter-stream dependency would show.
# ---------------------------------------------------------------------------------------------
def _pipeline_case(stage_layers, B, noam, M, precision, lr=0.01, mu=0.9, seed=SEED):
    bf16 = precision == pd.PD_BF16_F32ACC
    S = len(stage_layers)
    n_in = stage_layers[0][0][1]
    params, xs, labs, _ = _make(stage_layers, B, M, seed)
    if bf16:
        run_case(stage_layers, params, xs, labs, noam=noam, precision=precision, lr=lr, mu=mu, mode="forced")
        ref = run_case(stage_layers, params, xs, labs, noam=noam, precision=precision, lr=lr, mu=mu, compare=False)
    else:
        ref = run_case(stage_layers, params, xs, labs, noam=noam, precision=precision, lr=lr, mu=mu, mode="free")
    streams = [torch.cuda.Stream() for _ in range(S)]
    gs = [GpuStage(stage_layers[s], params[s], minibatch=B, precision=precision, stage_index=s, num_stages=S,
                   noam=noam, lr=lr, momentum=mu, stream=streams[s]) for s in range(S)]
    try:
        xd = to_dev(np.stack(xs).reshape(M * B, n_in), bf16)
        ld = labels_dev(np.stack(labs))
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        pd.pd_pipeline_run([g.h for g in gs], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        assert np.array_equal(to_host(losses), ref["losses"])
        for s in range(S):
            assert pd.pd_stage_trace(gs[s].h) == pd.pd_schedule_1f1b(S, noam, M, s)
            assert np.array_equal(pd.pd_stage_get_params(gs[s].h), ref["params"][s]), s
            assert np.array_equal(pd.pd_stage_get_momentum(gs[s].h), ref["mom"][s]), s
    finally:
        for g in gs:
            g.close()


def test_config1_mlp_pipeline_f32_full():
    # the 4-stage MLP exactly as configured: 256 wide, 10 classes, minibatch 32, NOAM 4, 64 minibatches
    _pipeline_case(gen.config1_mlp(256, 10, 4), B=32, noam=4, M=64, precision=pd.PD_F32, seed=SEED + 0)


def test_pipeline_bf16_mlp():
    _pipeline_case(gen.config1_mlp(256, 16, 4), B=32, noam=4, M=24, precision=pd.PD_BF16_F32ACC)


@pytest.mark.parametrize("S,noam,M", [(1, 1, 5), (2, 2, 7), (3, 1, 4), (4, 2, 9), (3, 3, 2)])
def test_pipeline_shapes_f32(S, noam, M):
    _pipeline_case(gen.config1_mlp(40, 6, S), B=6, noam=noam, M=M, precision=pd.PD_F32, lr=0.05)


@pytest.mark.parametrize("S,noam,M,precision", [(4, 4, 12, pd.PD_F32), (3, 2, 9, pd.PD_F32), (2, 2, 5, pd.PD_F32),
                                                (3, 3, 6, pd.PD_BF16_F32ACC)])
def test_vertical_sync_pipeline(S, noam, M, precision):
    # Section 3.4, vertical sync: every stage uses the version the input stage's forward read.  Compared with the
    # oracle's pipeline in the same mode: op traces bit for bit, numbers within the precision's tolerance.
    bf16 = precision == pd.PD_BF16_F32ACC
    width, classes, B = (64, 16, 8) if bf16 else (40, 6, 6)
    sl = gen.config1_mlp(width, classes, S)
    params = [gen.init_params(SEED + 9, f"v{s}", ly) for s, ly in enumerate(sl)]
    xs = gen.normal(SEED + 9, "X", (M, B, width)); labs = gen.labels(SEED + 9, "Y", (M, B), classes)
    ref = None
    if bf16:
        # bf16 trajectories of two correct implementations separate (ReLU decisions next to zero), so the numbers are
        # compared op by op in lockstep, teacher-forced, momentum included, at the full tolerance; the free-running
        # driver below must then reproduce the serialised GPU run bit for bit
        out = run_case(sl, params, list(xs), list(labs), noam=noam, precision=precision, lr=0.05, mode="forced",
                       vertical_sync=True, force_acts=True)
        assert out["updates_compared"] == (S * M, S * M), out["updates_compared"]
        ref = run_case(sl, params, list(xs), list(labs), noam=noam, precision=precision, lr=0.05, compare=False,
                       vertical_sync=True)
    ostages, olosses = run_pipeline(sl, params, [x.astype(np.float64) for x in xs], list(labs), noam,
                                    mode="bf16" if bf16 else "f32", lr=0.05, momentum=0.9, vertical_sync=True)
    gs = [GpuStage(sl[s], params[s], minibatch=B, precision=precision, stage_index=s, num_stages=S, noam=noam, lr=0.05,
                   momentum=0.9, stream=torch.cuda.Stream(), vertical_sync=True) for s in range(S)]
    try:
        xd = to_dev(xs.reshape(M * B, width), bf16); ld = labels_dev(labs)
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        pd.pd_pipeline_run([g.h for g in gs], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        tol = TOL_BF16 if bf16 else TOL_F32
        lg = to_host(losses)
        for i in range(M):
            assert abs(lg[i] - olosses[i]) <= tol * abs(olosses[i]), i
        ring = max(1, noam)
        for s in range(S):
            assert pd.pd_stage_ring_depth(gs[s].h) == ring and pd.pd_stage_depth(gs[s].h)[0] == max(1, noam - s)
            trace = pd.pd_stage_trace(gs[s].h)
            assert trace == pd.pd_schedule_1f1b_vertical_sync(S, noam, M, s)
            assert trace == [tuple(o) for o in ostages[s].trace]
            assert rel_err(pd.pd_stage_get_params(gs[s].h), ostages[s].master) <= tol, s
            if ref is None:
                assert rel_err(pd.pd_stage_get_momentum(gs[s].h), ostages[s].mom) <= tol, s
            else:
                assert np.array_equal(pd.pd_stage_get_params(gs[s].h), ref["params"][s]), s
                assert np.array_equal(pd.pd_stage_get_momentum(gs[s].h), ref["mom"][s]), s
        if ref is not None:
            assert np.array_equal(lg, ref["losses"])
    finally:
        for g in gs:
            g.close()


def test_forward_versioned_protocol():
    layers = [("linear", 16, 16, True)]
    g = GpuStage(layers, gen.init_params(SEED, "pv", layers), minibatch=4, precision=pd.PD_F32, stage_index=1,
                 num_stages=2, noam=3, vertical_sync=True)   # in-flight depth 2, ring of 3 versions
    try:
        assert pd.pd_stage_depth(g.h)[0] == 2 and pd.pd_stage_ring_depth(g.h) == 3
        x = torch.zeros(4, 16, device=dev()); dy = torch.zeros(4, 16, device=dev())
        for mb in range(4):                                  # four updates: versions 2, 3, 4 are held
            pd.pd_forward_versioned(g.h, mb, -1, x.data_ptr())
            pd.pd_backward(g.h, mb, dy.data_ptr(), 0)
            pd.pd_update(g.h)
        for bad in (1, 5):
            with pytest.raises(pd.PdError) as e:
                pd.pd_forward_versioned(g.h, 4, bad, x.data_ptr())
            assert e.value.status == pd.PD_ESTATE
        pd.pd_forward_versioned(g.h, 4, 2, x.data_ptr())     # the oldest one still in the ring
        assert pd.pd_stage_version(g.h, 4) == 2 and pd.pd_stage_trace(g.h)[-1] == (pd.PD_OP_F, 4, 2, 2)
        pd.pd_backward(g.h, 4, dy.data_ptr(), 0)
        assert pd.pd_stage_trace(g.h)[-1] == (pd.PD_OP_B, 4, 2, 2)
        pd.pd_update(g.h)
        # slot safety of the version ring: versions 3, 4, 5 are held.  Two minibatches read version 3; after the first
        # one's backward pass the update to version 6 would land in version 3's slot while the second still needs it
        pd.pd_forward_versioned(g.h, 5, 3, x.data_ptr())
        pd.pd_forward_versioned(g.h, 6, 3, x.data_ptr())
        pd.pd_backward(g.h, 5, dy.data_ptr(), 0)
        with pytest.raises(pd.PdError) as e:
            pd.pd_update(g.h)
        assert e.value.status == pd.PD_ESTATE and "ring slot" in str(e.value)
        assert pd.pd_stage_version(g.h) == 5 and pd.pd_stage_version(g.h, 6) == 3      # nothing was changed
        # the record of executed ops is bounded
        pd.pd_stage_set_trace_limit(g.h, 4)
        assert pd.pd_stage_trace(g.h) == [(pd.PD_OP_U, 4, 5, 2), (pd.PD_OP_F, 5, 3, 0), (pd.PD_OP_F, 6, 3, 0), (pd.PD_OP_B, 5, 3, 0)]
        pd.pd_stage_set_trace_limit(g.h, 0)
        assert pd.pd_stage_trace(g.h) == []
    finally:
        g.close()


def test_pipeline_run_twice_continues_ids():
    sl = gen.config1_mlp(32, 8, 3)
    B, M = 4, 5
    params = [gen.init_params(SEED, f"s{s}", ly) for s, ly in enumerate(sl)]
    xs = gen.normal(SEED, "X", (2 * M, B, 32)); labs = gen.labels(SEED, "Y", (2 * M, B), 8)
    gs = [GpuStage(sl[s], params[s], minibatch=B, precision=pd.PD_F32, stage_index=s, num_stages=3, noam=3,
                   stream=torch.cuda.Stream()) for s in range(3)]
    try:
        xd = to_dev(xs.reshape(2 * M * B, 32), False); ld = labels_dev(labs)
        losses = torch.zeros(2 * M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        hs = [g.h for g in gs]
        pd.pd_pipeline_run(hs, M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
        pd.pd_pipeline_run(hs, M, xd[M * B:].data_ptr(), ld[M:].data_ptr(), losses[M:].data_ptr())
        torch.cuda.synchronize()
        # reference: two drained runs back to back; the second continues with the first one's weights, momentum
        # and version counters, as the GPU stages do
        o1, l1 = run_pipeline(sl, params, [x.astype(np.float64) for x in xs[:M]], list(labs[:M]), 3)
        o2, l2 = run_pipeline(sl, None, [x.astype(np.float64) for x in xs[M:]], list(labs[M:]), 3, stages=o1)
        lg = to_host(losses)
        for i, l_o in enumerate(list(l1) + list(l2)):
            assert abs(lg[i] - l_o) <= TOL_F32 * abs(l_o), i
        for s in range(3):
            assert rel_err(pd.pd_stage_get_params(hs[s]), o2[s].master) <= TOL_F32, s
            assert rel_err(pd.pd_stage_get_momentum(hs[s]), o2[s].mom) <= TOL_F32, s
            got = pd.pd_stage_trace(hs[s])
            assert [(k, v) for k, _, v, _ in got] == [(o.kind, o.version) for o in o2[s].trace], s
        assert [pd.pd_stage_version(h) for h in hs] == [2 * M] * 3
    finally:
        for g in gs:
            g.close()


# ---------------------------------------------------------------------------------------------
# protocol errors come back as status codes and leave the stage usable
# ---------------------------------------------------------------------------------------------
def test_master_weights_as_ring_copy_plus_remainder_round_trip():
    """The fp32 master weights of a bf16 stage's Linear layers are stored as the latest ring copy plus the low 16 bits
    of their fp32 pattern.  What pd_stage_set_params / pd_stage_overwrite_latest store, pd_stage_get_params must
    return bit for bit -- except a tie that rounds DOWN to even (low half 0x8000, upper half even), which comes back
    one fp32 unit in the last place lower -- and the ring copy must be the round-to-nearest-even bf16 of the value."""
    layers = [("linear", 64, 48, True), ("linear", 48, 16, False)]
    n = sum(l[1] * l[2] + l[2] for l in layers)
    rng = np.random.default_rng(SEED)
    bits = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
    bits &= np.uint32(0xBFFFFFFF)                      # exponent below 2: finite, no NaN / Inf
    # special patterns: zeros of both signs, denormals, ties in both directions, low halves around 0x8000
    special = np.array([0x00000000, 0x80000000, 0x00000001, 0x00008000, 0x00018000, 0x3F808000, 0x3F818000,
                        0x3F807FFF, 0x3F808001, 0xBF808000, 0xBF818000, 0x3F80FFFF, 0x3F7F8000, 0x3F7FFFFF],
                       dtype=np.uint32)
    bits[:special.size] = special
    params = bits.view(np.float32).copy()
    g = GpuStage(layers, params, minibatch=8, precision=pd.PD_BF16_F32ACC)
    try:
        def expected(b):
            lo, up = b & np.uint32(0xFFFF), b >> np.uint32(16)
            tie_down = (lo == 0x8000) & ((up & 1) == 0)
            return np.where(tie_down, b - np.uint32(1), b)
        def rne(b):
            b64 = b.astype(np.uint64)
            return (((b64 + 0x7FFF + ((b64 >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint32)
        # which entries are Linear weights (the biases keep a plain fp32 master: returned exactly)
        is_w = np.zeros(n, dtype=bool)
        o = 0
        for (_, i_, o_, _) in layers:
            is_w[o:o + i_ * o_] = True
            o += i_ * o_ + o_
        want = np.where(is_w, expected(bits), bits)
        for setter in ("set", "overwrite"):
            if setter == "overwrite":
                pd.pd_stage_overwrite_latest(g.h, params, None)
            got = pd.pd_stage_get_params(g.h, -1, False).view(np.uint32)
            assert np.array_equal(got, want), setter
            ring = pd.pd_stage_get_params(g.h, -1, True).view(np.uint32)   # the bf16 ring copy, widened
            assert np.array_equal(ring >> np.uint32(16), rne(bits)), setter
            assert np.all((ring & np.uint32(0xFFFF)) == 0)
        assert int(np.sum(want != bits)) >= 3          # the planted round-down ties are in the sample
    finally:
        g.close()


def test_protocol_errors():
    layers = [("linear", 16, 8, False), ("softmax_xent", 8)]
    params = gen.init_params(SEED, "p", layers)
    g = GpuStage(layers, params, minibatch=4, precision=pd.PD_F32, in_flight_override=2)
    try:
        x = to_dev(gen.normal(SEED, "x", (4, 16)), False); lab = labels_dev(gen.labels(SEED, "y", (4,), 8))
        dx = empty_act(4, 16, False)

        def status(fn, *a):
            with pytest.raises(pd.PdError) as e:
                fn(*a)
            return e.value.status

        assert status(pd.pd_update, g.h) == pd.PD_ESTATE                      # nothing pending
        assert status(pd.pd_backward, g.h, 0, 0, dx.data_ptr()) == pd.PD_ESTATE  # nothing in flight
        assert status(pd.pd_forward, g.h, 0, x.data_ptr(), 0, 0, 0) == pd.PD_EINVAL  # labels missing
        pd.pd_forward(g.h, 0, x.data_ptr(), lab.data_ptr())
        assert status(pd.pd_forward, g.h, 2, x.data_ptr(), lab.data_ptr()) == pd.PD_ESTATE  # ids consecutive
        pd.pd_forward(g.h, 1, x.data_ptr(), lab.data_ptr())
        assert status(pd.pd_forward, g.h, 2, x.data_ptr(), lab.data_ptr()) == pd.PD_ESTATE  # depth reached
        assert status(pd.pd_backward, g.h, 1, 0, dx.data_ptr()) == pd.PD_ESTATE  # not the oldest
        assert status(pd.pd_backward, g.h, 0, x.data_ptr(), dx.data_ptr()) == pd.PD_EINVAL  # dy on a loss stage
        pd.pd_backward(g.h, 0, 0, dx.data_ptr())
        assert status(pd.pd_forward, g.h, 2, x.data_ptr(), lab.data_ptr()) == pd.PD_ESTATE  # update first
        assert status(pd.pd_backward, g.h, 1, 0, dx.data_ptr()) == pd.PD_ESTATE
        pd.pd_update(g.h)
        assert status(pd.pd_update, g.h) == pd.PD_ESTATE
        assert status(pd.pd_stage_get_params, g.h, 5) == pd.PD_ESTATE           # version not in the ring
        assert pd.pd_stage_version(g.h) == 1 and pd.pd_stage_version(g.h, 1) == 0
        assert status(pd.pd_stage_version, g.h, 0) == pd.PD_ESTATE
        pd.pd_forward(g.h, 2, x.data_ptr(), lab.data_ptr())
        assert pd.pd_stage_version(g.h, 2) == 1
        # arena too small
        cfg = pd.make_config(layers, minibatch=4, precision=pd.PD_F32)
        with pytest.raises(pd.PdError) as e:
            pd.pd_stage_create(cfg, g.arena.data_ptr() // 256 * 256 + 256, 1024)
        assert e.value.status == pd.PD_ENOMEM
        torch.cuda.synchronize()
    finally:
        g.close()
