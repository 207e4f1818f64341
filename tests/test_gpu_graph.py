"""The stage step under HIP graph capture: pd_forward / pd_backward / pd_update only enqueue kernels on the stage's
stream, so one period of the 1F1B steady state (ring depth W: W times backward, update, forward) can be recorded once
and replayed.  Slots repeat with period W (ring slot = version mod W, stash slot = minibatch mod W), so a replay of the
recorded period continues the training exactly where the eager calls would.  Every replay is compared bit for bit with
an eager twin stage that ran the same ops, with eager work and synchronisation between the replays.
"""
import numpy as np
import pytest
import torch

import paper_1806_03377_amd as pd
import pd_inputs as gen
from gpu_util import GpuStage, dev, labels_dev, to_dev

pytestmark = pytest.mark.gpu
SEED = gen.BASE_SEED + 11


def _period(g, first_id, W, xs, labs, dys, dx):
    """One period of the steady state: backward and update of minibatches first_id .. first_id+W-1, each followed by
    the forward pass of the minibatch W later (which reuses the stash slot and the input of the one just retired)."""
    for j in range(W):
        i = first_id + j
        pd.pd_backward(g.h, i, dys[j].data_ptr() if dys is not None else 0, dx.data_ptr())
        pd.pd_update(g.h)
        pd.pd_forward(g.h, i + W, xs[j].data_ptr(), labs[j].data_ptr() if labs is not None else 0,
                      g.y.data_ptr() if g.y is not None else 0, g.loss.data_ptr() if labs is not None else 0)


def _graph_case(layers, B, W, x_shape, n_out, with_loss, in_hw=None, replays=3, lab_shape=None):
    bf = True
    params = gen.init_params(SEED, "g", layers)
    params = params + 0.01 * gen.normal(SEED, "gb", params.shape)
    xs = [to_dev(x, bf) for x in gen.normal(SEED, "GX", (W,) + x_shape)]
    labs = [labels_dev(l) for l in gen.labels(SEED, "GY", (W,) + (lab_shape or (B,)), n_out)] if with_loss else None
    dys = None
    stages = []
    for _ in range(2):   # [0]: eager twin, [1]: recorded and replayed
        s = torch.cuda.Stream()
        g = GpuStage(layers, params, minibatch=B, precision=pd.PD_BF16_F32ACC, in_flight_override=W, stream=s,
                     in_hw=in_hw)
        g.y = None
        stages.append(g)
    dx = [torch.empty(xs[0].shape, dtype=torch.bfloat16, device=dev()) for _ in range(2)]
    if not with_loss:
        # a middle stage: its output buffer and the gradient that arrives from downstream
        for g in stages:
            g.y = torch.empty((B, n_out), dtype=torch.bfloat16, device=dev())
        dys = [to_dev(d, bf) for d in gen.normal(SEED, "GDY", (W, B, n_out)) * 0.01]
    torch.cuda.synchronize()

    # both: warm-up forwards and one eager period (every kernel has run once before anything is recorded)
    for g, d in zip(stages, dx):
        with torch.cuda.stream(g.stream):
            for j in range(W):
                pd.pd_forward(g.h, j, xs[j].data_ptr(), labs[j].data_ptr() if labs is not None else 0,
                              g.y.data_ptr() if g.y is not None else 0, g.loss.data_ptr() if labs is not None else 0)
            _period(g, 0, W, xs, labs, dys, d)
        g.stream.synchronize()
    eager, rec = stages
    assert np.array_equal(pd.pd_stage_get_params(eager.h), pd.pd_stage_get_params(rec.h))

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=rec.stream):
        _period(rec, W, W, xs, labs, dys, dx[1])       # recorded, not executed: ids W .. 2W-1
    torch.cuda.synchronize()
    assert pd.pd_stage_version(rec.h) == 2 * W         # the host-side bookkeeping advanced at call time

    for r in range(replays):
        with torch.cuda.stream(eager.stream):
            _period(eager, W * (r + 1), W, xs, labs, dys, dx[0])
        eager.stream.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        # reading the parameters is eager work on the stage's stream (the fp32 weights are put together by a kernel)
        want, got = pd.pd_stage_get_params(eager.h), pd.pd_stage_get_params(rec.h)
        assert np.array_equal(want, got), f"replay {r}"
        assert np.array_equal(pd.pd_stage_get_momentum(eager.h), pd.pd_stage_get_momentum(rec.h)), f"replay {r}"
        assert torch.equal(dx[0], dx[1]), f"replay {r}"
        if with_loss:
            assert torch.equal(eager.loss, rec.loss) and torch.isfinite(rec.loss).all(), f"replay {r}"
        else:
            assert torch.equal(eager.y, rec.y), f"replay {r}"
    # the replays moved the weights (the comparison above is not between two idle stages)
    assert not np.array_equal(pd.pd_stage_get_params(rec.h), params.astype(np.float32))
    for g in stages:
        g.close()


def test_graph_replay_linear_stage_with_loss():
    layers = [("linear", 1024, 520, True), ("linear", 520, 264, True), ("linear", 264, 104, False), ("softmax_xent", 104)]
    _graph_case(layers, B=64, W=4, x_shape=(64, 1024), n_out=104, with_loss=True)


def test_graph_replay_middle_linear_stage_depth_two():
    layers = [("linear", 136, 200, True), ("linear", 200, 72, True)]
    _graph_case(layers, B=37, W=2, x_shape=(37, 136), n_out=72, with_loss=False)


def test_graph_replay_conv_stage_with_loss():
    # convolution forward / input gradient / partial-sum weight gradient + reduce-and-update, pooling, classifier
    layers = [("conv2d", 3, 16, 3, 3, 1, 1, 1, True), ("conv2d", 16, 16, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2),
              ("conv2d", 16, 32, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2), ("linear", 3 * 3 * 32, 16, False),
              ("softmax_xent", 16)]
    _graph_case(layers, B=3, W=2, x_shape=(3, 12, 12, 3), n_out=16, with_loss=True, in_hw=(12, 12))


def test_graph_replay_lstm_stage_with_vocab_projection():
    # the recurrence (one kernel per time step, forward and backward) and the many-row vocabulary product
    layers = [("lstm", 16, 24, 6), ("linear", 24, 40, False), ("softmax_xent", 40)]
    _graph_case(layers, B=4, W=2, x_shape=(6, 4, 16), n_out=40, with_loss=True, lab_shape=(6, 4))


def test_pipeline_drivers_refuse_stream_capture():
    """pd_pipeline_run / pd_pipeline_run_replicated join several streams by events and never join them back to one
    stream, which stream capture does not allow: while any stage stream is being captured they return PD_ESTATE and
    enqueue nothing.  The capture is begun and ended here directly on the HIP runtime (an empty capture)."""
    import ctypes
    from gpu_util import GpuReplicatedStage
    hip = ctypes.CDLL("libamdhip64.so.7")      # the runtime instance torch and libpd.so already share
    hip.hipStreamBeginCapture.argtypes = [ctypes.c_void_p, ctypes.c_int]
    hip.hipStreamEndCapture.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
    hip.hipGraphDestroy.argtypes = [ctypes.c_void_p]
    sl = gen.config1_mlp(32, 8, 2)
    B, M = 4, 5
    params = [gen.init_params(SEED, f"c{s}", ly) for s, ly in enumerate(sl)]
    xd = to_dev(gen.normal(SEED, "CX", (M * B, 32)), False)
    ld = labels_dev(gen.labels(SEED, "CY", (M, B), 8))
    losses = torch.zeros(M, dtype=torch.float32, device=dev())
    streams = [torch.cuda.Stream() for _ in range(3)]
    gs = [GpuStage(sl[s], params[s], minibatch=B, precision=pd.PD_F32, stage_index=s, num_stages=2, noam=2,
                   stream=streams[s]) for s in range(2)]
    rep = GpuReplicatedStage(sl[0], params[0], 2, minibatch=B, precision=pd.PD_F32, stage_index=0, num_stages=2, noam=2,
                             stream=streams[2])
    try:
        torch.cuda.synchronize()
        THREAD_LOCAL = 1                        # hipStreamCaptureModeThreadLocal
        assert hip.hipStreamBeginCapture(streams[1].cuda_stream, THREAD_LOCAL) == 0
        try:
            with pytest.raises(pd.PdError) as e:
                pd.pd_pipeline_run([g.h for g in gs], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
            assert e.value.status == pd.PD_ESTATE and "captured" in str(e.value)
            with pytest.raises(pd.PdError) as e:
                pd.pd_pipeline_run_replicated([rep.handles(), [gs[1].h]], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
            assert e.value.status == pd.PD_ESTATE and "captured" in str(e.value)
        finally:
            graph = ctypes.c_void_p()
            assert hip.hipStreamEndCapture(streams[1].cuda_stream, ctypes.byref(graph)) == 0
            if graph:
                hip.hipGraphDestroy(graph)
        assert all(pd.pd_stage_trace(g.h) == [] for g in gs)      # nothing was enqueued
        pd.pd_pipeline_run([g.h for g in gs], M, xd.data_ptr(), ld.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        assert [pd.pd_stage_version(g.h) for g in gs] == [M, M] and bool(torch.isfinite(losses).all())
    finally:
        rep.close()
        for g in gs:
            g.close()
