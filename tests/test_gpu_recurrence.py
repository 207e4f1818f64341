"""All time steps of an LSTM layer in one launch (the multi-step recurrence kernels) against one launch per step.

The multi-step kernels do the per-step kernels' arithmetic in the same order, so a stage run either way must give the
same bits: losses, input gradients, weights, momentum.  (The multi-step path is the default wherever a layer's grid fits the chip, so the oracle-parity tests of
test_gpu_parity.py run it; some of them are repeated here with one launch per step forced.)

The workgroups of a multi-step kernel wait for each other with a BOUNDED number of polls.  The last test makes the
workgroups withhold what their peers wait for, with a small poll limit: the launches must still end, and the stage must
report the failure at its next synchronising call.  No kernel is made to hang: giving up is the kernel's own exit path.
"""
import numpy as np
import pytest
import torch

import paper_1806_03377_amd as pd
import pd_inputs as gen
from gpu_util import GpuStage, dev, labels_dev, to_dev, to_host
from test_gpu_backward_stream import _run_stage, _same

pytestmark = pytest.mark.gpu
SEED = gen.BASE_SEED + 23


@pytest.fixture
def per_step_then_restore():
    yield
    pd.pd_set_recurrence_kernel(1, 0, 0)     # the default


def _both_ways(layers, B, T, M, depth, lane=False, with_loss=True):
    I = layers[0][1]
    p = gen.init_params(SEED, "rec", layers)
    p = p + 0.01 * gen.normal(SEED, "recb", p.shape)
    xs = list(gen.normal(SEED, "X", (M, T, B, I)))
    labs = dys = None
    if with_loss:
        labs = list(gen.labels(SEED, "Y", (M, T, B), layers[-1][1]))
    else:
        dys = list(gen.normal(SEED, "DY", (M, T, B, layers[-1][2])) * 0.01)
    kw = dict(B=B, depth=depth, precision=pd.PD_BF16_F32ACC, lane=lane)
    pd.pd_set_recurrence_kernel(0, 0, 0)
    a = _run_stage(layers, p, xs, labs, dys, **kw)
    pd.pd_set_recurrence_kernel(1, 0, 0)
    b = _run_stage(layers, p, xs, labs, dys, **kw)
    _same(a, b)
    assert np.all(np.isfinite(b[2])) and float(np.abs(b[2] - p).max()) > 0.0   # the run did train


# ragged against the 16 x 16 tile in rows and units; a reduction shorter than one wave's share; two stacked layers; a
# hidden size whose gate rows need all 8 reduction steps per wave; with and without a layer above / a loss
@pytest.mark.parametrize("I,H,B,T", [(24, 16, 3, 5), (136, 72, 5, 7), (64, 104, 17, 4), (32, 256, 64, 6), (40, 1000, 20, 3)])
def test_one_lstm_layer_same_bits(I, H, B, T, per_step_then_restore):
    _both_ways([("lstm", I, H, T)], B=B, T=T, M=4, depth=2, with_loss=False)


def test_two_stacked_layers_with_vocabulary_same_bits(per_step_then_restore):
    _both_ways([("lstm", 48, 72, 6), ("lstm", 72, 40, 6), ("linear", 40, 200, False), ("softmax_xent", 200)], B=9, T=6,
               M=5, depth=2)


def test_with_backward_stream_same_bits(per_step_then_restore):
    # forward and backward recurrences of consecutive minibatches may be in flight together: the launches are chained
    _both_ways([("lstm", 64, 128, 8), ("linear", 128, 104, False), ("softmax_xent", 104)], B=32, T=8, M=7, depth=3,
               lane=True)


def test_s2vt_widths_same_bits(per_step_then_restore):
    # hidden 1000, minibatch 64: 4 x 63 = 252 workgroups, the configuration the benchmark runs (shorter sequence)
    _both_ways([("lstm", 1000, 1000, 10)], B=64, T=10, M=3, depth=1, with_loss=False)


def test_oracle_parity_with_one_launch_per_step(per_step_then_restore):
    from test_gpu_parity import _seq_case
    pd.pd_set_recurrence_kernel(0, 0, 0)
    _seq_case([[("lstm", 16, 24, 6), ("linear", 24, 40, False), ("softmax_xent", 40)]], B=4, T=6, noam=1, M=4,
              depth_override=2)
    _seq_case([[("lstm", 24, 16, 16), ("linear", 16, 40, False), ("softmax_xent", 40)]], B=32, T=16, noam=1, M=3,
              depth_override=2)
    _seq_case(gen.config4_s2vt(input_size=136, hidden=72, vocab=200, seq_len=7), B=5, T=7, noam=2, M=5)


def test_a_wait_that_cannot_succeed_ends_and_is_reported(per_step_then_restore):
    layers = [("lstm", 32, 64, 5)]
    B, T = 24, 5
    p = gen.init_params(SEED, "fail", layers)
    x = to_dev(gen.normal(SEED, "X", (T, B, 32)), True)
    y = torch.zeros((T * B, 64), dtype=torch.bfloat16, device=dev())
    g = GpuStage(layers, p, minibatch=B, precision=pd.PD_BF16_F32ACC, in_flight_override=1, stream=torch.cuda.Stream())
    try:
        pd.pd_set_recurrence_kernel(1, 200, 1)      # nobody publishes; give up after 200 fetches
        pd.pd_forward(g.h, 0, x.data_ptr(), 0, y.data_ptr(), 0)
        pd.pd_set_recurrence_kernel(1, 0, 0)
        with pytest.raises(pd.PdError) as e:
            pd.pd_stage_check(g.h)                  # returns: the launch ended although no wait could succeed
        assert "gave up" in str(e.value) and "forward" in str(e.value)
        pd.pd_stage_check(g.h)                      # reported once, then cleared
    finally:
        g.close()
