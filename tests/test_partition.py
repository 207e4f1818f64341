"""pd_partition (host only) against the oracle's dynamic program; the on-device layer profiler (GPU)."""
import math

import numpy as np
import pytest

import paper_1806_03377_amd as pd
from oracle.partition import StageAssign, partition, pipeline_time


def _check_against_oracle(T, a, w, M, bw):
    ref_best, ref_stages, ref_noam = partition(T, a, w, M, bw)
    best, stages, noam = pd.pd_partition(T, a, w, M, bw)
    assert best == pytest.approx(ref_best, rel=1e-12, abs=0)
    # the optimum is unique, the partition reaching it need not be: check the returned one is feasible and optimal
    assert stages[0][0] == 0 and stages[-1][1] == len(T) - 1
    for p, q in zip(stages, stages[1:]):
        assert q[0] == p[1] + 1
    assert all(f <= l and r >= 1 for f, l, r in stages)
    assert sum(r for _, _, r in stages) == M
    assert pipeline_time(T, a, w, [StageAssign(*s) for s in stages], bw) == pytest.approx(ref_best, rel=1e-12)
    assert noam == math.ceil(M / stages[0][2])
    return stages, ref_stages, noam, ref_noam


@pytest.mark.parametrize("seed", range(8))
def test_partition_matches_oracle_on_random_profiles(seed):
    rng = np.random.default_rng(500 + seed)
    same = total = 0
    for N in (1, 2, 3, 5, 8, 13, 21):
        for M in (1, 2, 3, 4, 8, 16):
            T = rng.uniform(0.1, 5.0, N).tolist()
            a = (rng.uniform(0.0, 1.0, N) * rng.choice([0.05, 1.0, 30.0])).tolist()
            w = (rng.uniform(0.0, 1.0, N) * rng.choice([0.0, 0.5, 50.0])).tolist()
            bw = float(rng.choice([0.25, 1.0, 16.0]))
            stages, ref_stages, noam, ref_noam = _check_against_oracle(T, a, w, M, bw)
            total += 1
            same += [tuple(s) for s in ref_stages] == stages and noam == ref_noam
    assert same >= 0.9 * total  # ties aside, the same partition


def test_partition_hand_worked_example():
    best, stages, noam = pd.pd_partition([4.0, 2.0, 2.0], [1.0, 0.5, 0.25], [5.0, 3.0, 2.0], 2, 1.0)
    assert best == pytest.approx(4.0) and stages == [(0, 0, 1), (1, 2, 1)] and noam == 2
    best, stages, noam = pd.pd_partition([1.0, 2.0, 3.0, 2.0], [1e6] * 4, [1e-9] * 4, 4, 1.0)
    assert best == pytest.approx(2.0) and stages == [(0, 3, 4)] and noam == 1
    best, stages, noam = pd.pd_partition([1.0, 1.0, 1.0], [1e-9] * 3, [1e6] * 3, 3, 1.0)
    assert best == pytest.approx(1.0) and stages == [(0, 0, 1), (1, 1, 1), (2, 2, 1)] and noam == 3
    best, stages, noam = pd.pd_partition([1.0, 2.5, 0.5, 3.0], [9.0] * 4, [7.0] * 4, 1, 1.0)
    assert best == pytest.approx(7.0) and stages == [(0, 3, 1)] and noam == 1


def test_partition_vgg16_like_profile():
    # the shape of the problem the paper describes for VGG16 (Section 2.2 / 3.2): convolutions hold the compute and
    # large activations, the fully connected layers hold the parameters.  Values are synthetic.
    T = [8, 12, 6, 10, 10, 5, 9, 9, 9, 3, 3, 3, 2.0, 0.7, 0.2]
    a = [205, 205, 51, 103, 103, 26, 51, 51, 51, 13, 13, 13, 0.26, 0.26, 0.06]
    w = [0.007, 0.15, 0, 0.3, 0.6, 0, 1.2, 2.4, 2.4, 9.4, 9.4, 9.4, 411, 67, 16]
    for M in (2, 4, 8, 16):
        for bw in (1.0, 3.0, 100.0):
            _check_against_oracle(T, a, w, M, bw)


def test_partition_argument_errors():
    for args in (([], [], [], 2, 1.0), ([1.0], [1.0], [1.0], 0, 1.0), ([1.0], [1.0], [1.0], 1, 0.0),
                 ([1.0], [1.0], [1.0], 1, float("nan")), ([-1.0], [1.0], [1.0], 1, 1.0),
                 ([1.0], [float("inf")], [1.0], 1, 1.0)):
        with pytest.raises(pd.PdError) as e:
            pd.pd_partition(*args)
        assert e.value.status == pd.PD_EINVAL and "partition" in str(e.value)
    # capacity too small: PD_ENOMEM with the count reported
    import ctypes as C
    dbl = C.c_double * 3
    out = (pd.binding.pd_stage_assign * 1)()
    ns = C.c_size_t(0)
    rc = pd.binding._lib.pd_partition(3, 3, dbl(1, 1, 1), dbl(0, 0, 0), dbl(1e6, 1e6, 1e6), 1.0, None, out, 1,
                                      C.byref(ns), None)
    assert rc == pd.PD_ENOMEM and ns.value == 3


# ------------------------------------------------------------------------------------------------- GPU
@pytest.mark.gpu
def test_layer_profiler_units_sizes_and_times():
    import torch
    import pd_inputs as gen
    from gpu_util import GpuStage
    B = 8
    layers = [("conv2d", 8, 16, 3, 3, 1, 1, 1, True), ("maxpool2d", 2, 2),
              ("concat", [[("conv2d", 16, 8, 1, 1, 1, 0, 0, True)],
                          [("conv2d", 16, 8, 1, 1, 1, 0, 0, True), ("conv2d", 8, 16, 3, 3, 1, 1, 1, True)]]),
              ("linear", 8 * 8 * 24, 40, True), ("linear", 40, 16, False), ("softmax_xent", 16)]
    params = gen.init_params(77, "profiled", layers)
    st = GpuStage(layers, params, minibatch=B, precision=pd.PD_BF16_F32ACC, in_flight_override=2, in_hw=(16, 16))
    try:
        pd.pd_stage_profile(st.h, True)
        x = torch.randn(B, 16, 16, 8, device="cuda").to(torch.bfloat16)
        lab = torch.randint(0, 16, (B,), device="cuda", dtype=torch.int32)
        n_steps = 6
        pd.pd_forward(st.h, 0, x.data_ptr(), lab.data_ptr())
        pd.pd_forward(st.h, 1, x.data_ptr(), lab.data_ptr())
        for k in range(n_steps):
            pd.pd_backward(st.h, k)
            pd.pd_update(st.h)
            pd.pd_forward(st.h, k + 2, x.data_ptr(), lab.data_ptr())
        prof = pd.pd_stage_profile_read(st.h)
        pd.pd_stage_profile(st.h, False)
        # recording is off: further ops leave no marks, reading again gives the same numbers
        pd.pd_backward(st.h, n_steps)
        pd.pd_update(st.h)
        assert pd.pd_stage_profile_read(st.h) == prof
    finally:
        st.close()
    # units: conv, pool, the block (3 branch convolutions + the concatenation), linear, linear
    assert [(u["first_layer"], u["last_layer"]) for u in prof] == [(0, 0), (1, 1), (2, 5), (6, 6), (7, 7)]
    bf = 2
    assert [u["act_bytes"] for u in prof] == [B * 16 * 16 * 16 * bf, B * 8 * 8 * 16 * bf, B * 8 * 8 * 24 * bf,
                                              B * 40 * bf, B * 16 * 4]
    n_conv = lambda ci, co, k: co * k * k * ci + co
    assert [u["param_bytes"] for u in prof] == [4 * n_conv(8, 16, 3), 0,
                                                4 * (n_conv(16, 8, 1) * 2 + n_conv(8, 16, 3)),
                                                4 * (8 * 8 * 24 * 40 + 40), 4 * (40 * 16 + 16)]
    for u in prof:
        assert u["fwd_ms"] > 0 and u["bwd_ms"] > 0
        assert (u["upd_ms"] > 0) == (u["param_bytes"] > 0)
        assert u["fwd_ms"] + u["bwd_ms"] + u["upd_ms"] < 50.0
    # the profile feeds the partitioner; same answer as the oracle's dynamic program on the same numbers
    T = [u["fwd_ms"] + u["bwd_ms"] + u["upd_ms"] for u in prof]
    a = [u["act_bytes"] for u in prof]
    w = [u["param_bytes"] for u in prof]
    for M in (1, 2, 3, 4):
        _check_against_oracle(T, a, w, M, 1e6)
