"""pd_linear_fwd_bf16_static, the entry point that allocates nothing: its split-K partial sums live in a device array
that is part of the library image.  Checked through the C ABI against pd_linear_fwd_bf16 with a caller-supplied
workspace of the same size (same kernels, same number of partial sums: bit-equal) and against the oracle at the bf16
tolerance, on two calls in a row, the second on a smaller input (the array still holds the first call's partial sums),
then once more at the largest output the array serves."""
import numpy as np
import pytest
import torch

import paper_1806_03377_amd as pd
import pd_inputs as gen
from gpu_util import dev, empty_act, rel_err, to_dev, to_host
from oracle import layers as OL

pytestmark = pytest.mark.gpu
SEED = gen.BASE_SEED + 77
TOL_BF16 = 2e-2


def _bf(a):
    return OL.round_bf16(np.asarray(a, dtype=np.float64))


def _one(M, N, K, relu, tag):
    x = _bf(gen.normal(SEED, f"x{tag}", (M, K)))
    w = _bf(gen.uniform(SEED, f"w{tag}", (N, K), -0.1, 0.1))
    b = _bf(gen.normal(SEED, f"b{tag}", (N,)) * 0.1)
    s = torch.cuda.current_stream().cuda_stream
    xd, wd, bd = to_dev(x, True), to_dev(w, True), to_dev(b, True)
    wsb = 32 * M * N * 4
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev())
    y_ref, y = empty_act(M, N, True), empty_act(M, N, True)
    y.fill_(float("nan"))
    torch.cuda.synchronize()
    pd.pd_linear_fwd_bf16(s, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y_ref.data_ptr(), M, N, K, relu, ws.data_ptr(), wsb)
    pd.pd_linear_fwd_bf16_static(s, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), M, N, K, relu)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref), (M, N, K)
    assert rel_err(to_host(y), OL.linear_forward(x, w, b, relu, OL.round_bf16)) <= TOL_BF16, (M, N, K)


def test_static_scratch_forward_two_calls_second_smaller():
    _one(64, 1000, 1536, True, "a")      # split-K through the direct-to-LDS kernel (reduction a multiple of 128)
    _one(40, 136, 72, False, "b")        # smaller, ragged, the register-staged kernel: old partial sums stay behind it
    _one(64, 4096, 1024, True, "c")      # the largest output the array serves: 32 * 64 * 4096 * 4 bytes = 32 MiB


def test_static_scratch_rejects_what_does_not_fit():
    assert pd.pd_linear_fwd_bf16_static_max_bytes() == 32 << 20
    t = torch.zeros(16, dtype=torch.bfloat16, device=dev())
    with pytest.raises(pd.PdError) as e:
        pd.pd_linear_fwd_bf16_static(torch.cuda.current_stream().cuda_stream, t.data_ptr(), t.data_ptr(), 0, t.data_ptr(),
                                     65, 4096, 1024, True)
    assert e.value.status == pd.PD_ENOMEM and "pd_linear_fwd_bf16" in str(e.value)
    with pytest.raises(pd.PdError) as e:
        pd.pd_linear_fwd_bf16_static(torch.cuda.current_stream().cuda_stream, 0, t.data_ptr(), 0, t.data_ptr(), 8, 8, 8, True)
    assert e.value.status == pd.PD_EINVAL
