"""Pins for the oracle's LSTM: torch.nn.LSTM + autograd (library routine), finite differences,
and the two-stage sequence model reducing to sequential SGD when one minibatch is active."""
import numpy as np
import torch

import pd_inputs as gen
from oracle import layers as L
from oracle.pipeline import Stage, run_pipeline

SEED = gen.BASE_SEED + 3
ID = L.quantiser("f32")


def _torch_lstm(I, H, W_ih, W_hh, b):
    m = torch.nn.LSTM(I, H, batch_first=False).double()
    with torch.no_grad():
        m.weight_ih_l0.copy_(torch.tensor(W_ih)); m.weight_hh_l0.copy_(torch.tensor(W_hh))
        m.bias_ih_l0.copy_(torch.tensor(b)); m.bias_hh_l0.zero_()
    return m


def test_lstm_matches_torch():
    T, B, I, H = 6, 3, 5, 4
    x = gen.normal(SEED, "x", (T, B, I)).astype(np.float64)
    W_ih = gen.normal(SEED, "wi", (4 * H, I)).astype(np.float64) * 0.4
    W_hh = gen.normal(SEED, "wh", (4 * H, H)).astype(np.float64) * 0.4
    b = gen.normal(SEED, "b", (4 * H,)).astype(np.float64) * 0.2
    h, cache = L.lstm_forward(x, W_ih, W_hh, b, ID)
    m = _torch_lstm(I, H, W_ih, W_hh, b)
    tx = torch.tensor(x, requires_grad=True)
    th, _ = m(tx)
    assert np.allclose(h, th.detach().numpy(), rtol=1e-12, atol=1e-13)
    dh = gen.normal(SEED, "dh", h.shape).astype(np.float64)
    th.backward(torch.tensor(dh))
    dx, dWi, dWh, db = L.lstm_backward(x, W_ih, W_hh, cache, dh, True, ID)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(dWi, m.weight_ih_l0.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(dWh, m.weight_hh_l0.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(db, m.bias_ih_l0.grad.numpy(), rtol=1e-10, atol=1e-13)


def _s2vt_like(I=6, H=4, V=7, T=5):
    return [[("lstm", I, H, T)], [("lstm", H, H, T), ("linear", H, V, False), ("softmax_xent", V)]]


def test_lstm_stage_finite_differences():
    layers = [("lstm", 3, 3, 4), ("linear", 3, 5, False), ("softmax_xent", 5)]
    p0 = gen.init_params(SEED, "p", layers).astype(np.float64) * 0.5 + 0.05 * gen.normal(SEED, "q", (gen.param_count(layers),))
    x = gen.normal(SEED, "fx", (4, 2, 3)).astype(np.float64)
    y = gen.labels(SEED, "fy", (4, 2), 5)
    st = Stage(layers, p0, depth=1); _, loss = st.forward(0, x, y); st.backward(0, None)
    h = 1e-6
    for k in range(p0.size):
        e = np.zeros_like(p0); e[k] = h
        fd = (Stage(layers, p0 + e, 1).forward(0, x, y)[1] - Stage(layers, p0 - e, 1).forward(0, x, y)[1]) / (2 * h)
        assert abs(fd - st.grad[k]) < 2e-7 * max(1.0, abs(fd)), k


def test_two_stage_sequence_model_reduces_to_sequential_sgd():
    sl = _s2vt_like()
    T, B, I, H, V = 5, 3, 6, 4, 7
    params = [gen.init_params(SEED, f"s{s}", ly).astype(np.float64) + 0.05 * gen.normal(SEED, f"n{s}", (gen.param_count(ly),))
              for s, ly in enumerate(sl)]
    M = 4
    xs = [gen.normal(SEED, f"x{i}", (T, B, I)).astype(np.float64) for i in range(M)]
    ys = [gen.labels(SEED, f"y{i}", (T, B), V) for i in range(M)]
    stages, losses = run_pipeline(sl, params, xs, ys, 1, lr=0.05, momentum=0.9)
    # library reference: two nn.LSTM + Linear, torch.optim.SGD
    def split(p, I_, H_):
        a = 4 * H_ * I_; b_ = a + 4 * H_ * H_
        return p[:a].reshape(4 * H_, I_), p[a:b_].reshape(4 * H_, H_), p[b_:b_ + 4 * H_], p[b_ + 4 * H_:]
    wi0, wh0, b0, _ = split(params[0], I, H)
    wi1, wh1, b1, rest = split(params[1], H, H)
    l0, l1 = _torch_lstm(I, H, wi0, wh0, b0), _torch_lstm(H, H, wi1, wh1, b1)
    lin = torch.nn.Linear(H, V).double()
    with torch.no_grad():
        lin.weight.copy_(torch.tensor(rest[:V * H].reshape(V, H))); lin.bias.copy_(torch.tensor(rest[V * H:]))
    ps = [p for m in (l0, l1, lin) for n, p in m.named_parameters() if "bias_hh" not in n]
    opt = torch.optim.SGD(ps, lr=0.05, momentum=0.9)
    for i in range(M):
        opt.zero_grad()
        h0, _ = l0(torch.tensor(xs[i])); h1, _ = l1(h0)
        loss = torch.nn.functional.cross_entropy(lin(h1).reshape(T * B, V), torch.tensor(ys[i].reshape(-1), dtype=torch.long))
        loss.backward(); opt.step()
        assert abs(loss.item() - losses[i]) < 1e-10
    a = 4 * H * I
    assert np.allclose(stages[0].master[:a].reshape(4 * H, I), l0.weight_ih_l0.detach().numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(stages[1].master[-V:], lin.bias.detach().numpy(), rtol=1e-9, atol=1e-12)
    a1 = 4 * H * H
    assert np.allclose(stages[1].master[a1:2 * a1].reshape(4 * H, H), l1.weight_hh_l0.detach().numpy(), rtol=1e-9, atol=1e-12)


def test_bf16_mode_rounding_points():
    # hidden states are stored in bfloat16; the cell state is not
    T, B, I, H = 3, 2, 8, 8
    x = L.round_bf16(gen.normal(SEED, "bx", (T, B, I)))
    W_ih = L.round_bf16(gen.normal(SEED, "bwi", (4 * H, I)) * 0.3); W_hh = L.round_bf16(gen.normal(SEED, "bwh", (4 * H, H)) * 0.3)
    h, cache = L.lstm_forward(x, W_ih, W_hh, np.zeros(4 * H), L.round_bf16)
    assert np.array_equal(h, L.round_bf16(h))
    assert not np.array_equal(cache["cs"][1], L.round_bf16(cache["cs"][1]))
