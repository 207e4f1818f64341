"""Pins for the oracle's replicated stage (Section 3.3 round-robin routing, Section 4 "Data Parallelism").

Against things other than the oracle itself: torch autograd + torch.optim.SGD on the concatenated minibatch (the
paper's remark that plain data-parallel training is one stage replicated everywhere, i.e. synchronous minibatch SGD
on r minibatches at a time), a hand-worked two-round example, a torch flat loop of the staleness rule for a
replicated input stage, the routing rule, and a planted mistake that the first pin catches.
"""
import numpy as np
import pytest
import torch

import pd_inputs as gen
from oracle.pipeline import Stage, run_pipeline
from oracle.replicated import ReplicatedStage, rounds_of, route, run_replicated_pipeline
from oracle.schedule import OP_B, OP_F, OP_U
from test_oracle_numerics import _data, _params, _torch_model_loss

SEED = gen.BASE_SEED + 77


def test_routing_is_round_robin_by_minibatch_id():
    assert [route(i, 3) for i in range(7)] == [(0, 0), (1, 0), (2, 0), (0, 1), (1, 1), (2, 1), (0, 2)]
    assert [route(i, 1) for i in range(3)] == [(0, 0), (0, 1), (0, 2)]
    for r in (1, 2, 3, 5):
        for M in (0, 1, 4, 7, 10):
            assert sum(rounds_of(q, r, M) for q in range(r)) == M
            assert all(rounds_of(q, r, M) == sum(1 for i in range(M) if i % r == q) for q in range(r))


def test_hand_worked_two_rounds():
    # y = w x + b with w = 2, b = 0.5; two replicas, depth 1, lr 0.1, momentum 0.5; upstream gradients given.
    # round 0: (x, dy) = (1, 0.1) and (3, -0.2):  dW = 0.1 - 0.6 = -0.5, db = -0.1
    #          m = (-0.5, -0.1);  w = 2 + 0.05 = 2.05;  b = 0.5 + 0.01 = 0.51
    # round 1: (2, 0.3) and (-1, 0.4):  dW = 0.6 - 0.4 = 0.2, db = 0.7;  dx = dy * 2.05 = 0.615 and 0.82
    #          m = (0.5*-0.5 + 0.2, 0.5*-0.1 + 0.7) = (-0.05, 0.65);  w = 2.05 + 0.005 = 2.055;  b = 0.51 - 0.065 = 0.445
    st = ReplicatedStage([("linear", 1, 1, False)], np.array([2.0, 0.5]), depth=1, replicas=2, lr=0.1, momentum=0.5)
    ys = [st.forward(i, np.array([[x]]))[0] for i, x in ((0, 1.0), (1, 3.0))]
    assert np.allclose(np.ravel(ys), [2.5, 6.5], atol=1e-15)
    st.backward(0, np.array([[0.1]])); st.backward(1, np.array([[-0.2]]))
    st.update(0)
    for rp in st.rep:
        assert np.allclose(rp.master, [2.05, 0.51], atol=1e-15)
    st.forward(2, np.array([[2.0]])); st.forward(3, np.array([[-1.0]]))
    dx2 = st.backward(2, np.array([[0.3]])); dx3 = st.backward(3, np.array([[0.4]]))
    assert np.allclose([dx2.item(), dx3.item()], [0.615, 0.82], atol=1e-15)
    st.update(1)
    for rp in st.rep:
        assert np.allclose(rp.master, [2.055, 0.445], atol=1e-15)
    assert st.latest == 2


def _torch_bsp(layers, p0, xs, ys, r, lr, mu):
    """Synchronous SGD on r minibatches at a time: loss = sum of the r minibatch-mean losses."""
    tp = torch.tensor(p0, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=lr, momentum=mu)
    hist, losses = [], []
    for k in range(0, len(xs), r):
        opt.zero_grad()
        total = 0.0
        for x, y in zip(xs[k:k + r], ys[k:k + r]):
            l = _torch_model_loss([tp], [layers], torch.tensor(x), torch.tensor(y, dtype=torch.long))
            losses.append(l.item())
            total = total + l
        total.backward()
        opt.step()
        hist.append(tp.detach().numpy().copy())
    return hist, losses


LAYERS = [("linear", 12, 10, True), ("linear", 10, 5, False), ("softmax_xent", 5)]


@pytest.mark.parametrize("r,M", [(2, 8), (3, 9), (3, 8), (4, 5)])
def test_one_replicated_stage_is_synchronous_data_parallel_sgd(r, M):
    # Section 4: data-parallel training = one stage with every layer, replicated.  M not a multiple of r: ragged end
    p0 = _params([LAYERS], SEED)[0]
    xs, ys = _data(M, 6, 12, 5, SEED)
    st = ReplicatedStage(LAYERS, p0, depth=1, replicas=r, lr=0.05, momentum=0.9)
    losses, hist = [], []
    for k in range(0, M, r):
        for i in range(k, min(k + r, M)):
            losses.append(st.forward(i, xs[i], ys[i])[1])
        for i in range(k, min(k + r, M)):
            st.backward(i, None, need_dx=False)
        st.update(k // r)
        hist.append(st.rep[0].master.copy())
        for rp in st.rep[1:]:
            assert np.array_equal(rp.master, st.rep[0].master) and rp.latest == st.latest
    ref_hist, ref_losses = _torch_bsp(LAYERS, p0, xs, ys, r, 0.05, 0.9)
    assert np.allclose(losses, ref_losses, rtol=1e-11)
    for a, b in zip(hist, ref_hist):
        assert np.allclose(a, b, rtol=1e-10, atol=1e-13)


def test_planted_mean_instead_of_sum_is_caught():
    class Averaging(ReplicatedStage):
        def update(self, round_=-1):
            n = sum(1 for s in self.rep if s.grad is not None)
            for s in self.rep:
                if s.grad is not None:
                    s.grad = s.grad / n
            super().update(round_)
    p0 = _params([LAYERS], SEED)[0]
    xs, ys = _data(4, 6, 12, 5, SEED)
    st = Averaging(LAYERS, p0, depth=1, replicas=2, lr=0.05, momentum=0.9)
    for k in (0, 2):
        for i in (k, k + 1):
            st.forward(i, xs[i], ys[i])
        for i in (k, k + 1):
            st.backward(i, None, need_dx=False)
        st.update(k // 2)
    ref_hist, _ = _torch_bsp(LAYERS, p0, xs, ys, 2, 0.05, 0.9)
    assert not np.allclose(st.rep[0].master, ref_hist[-1], rtol=1e-6, atol=1e-9)


def test_backward_runs_where_forward_ran_and_uses_its_version():
    layers = [("linear", 6, 6, True), ("linear", 6, 4, False)]
    p0 = _params([layers], SEED)[0]
    r, W, M = 2, 2, 10
    st = ReplicatedStage(layers, p0, depth=W, replicas=r, lr=0.05)
    xs = [gen.normal(SEED, f"x{i}", (3, 6)).astype(np.float64) for i in range(M)]
    dys = [0.1 * gen.normal(SEED, f"d{i}", (3, 4)).astype(np.float64) for i in range(M)]
    for i in range(r * W):                                   # start-up: W rounds admitted on every replica
        st.forward(i, xs[i])
    for k in range(M // r):
        for q in range(r):
            st.backward(k * r + q, dys[k * r + q])
        st.update(k)
        for q in range(r):
            nf = (k + W) * r + q
            if nf < M:
                st.forward(nf, xs[nf])
    seen = {}
    for q, op in st.trace:
        if op.kind == OP_F:
            seen[(q, op.mb)] = op.version
            assert op.version == max(0, op.mb - W + 1)       # rounds completed when the forward ran
        elif op.kind == OP_B:
            assert seen[(q, op.mb)] == op.version            # same replica, same version (weight stashing)
    assert st.latest == M // r
    assert max(rp.max_in_flight for rp in st.rep) == W


def test_rows_of_a_round_act_as_one_minibatch_when_there_is_no_loss():
    # without a loss the stage is linear in the rows of dy, so the sum over replicas is the gradient of the
    # concatenated rows: the replicated stage must follow the (separately pinned) plain stage fed r minibatches at once
    layers = [("linear", 6, 8, True), ("linear", 8, 4, True)]
    p0 = _params([layers], SEED)[0]
    r, W, R = 3, 2, 5
    xs = [gen.normal(SEED, f"x{i}", (2, 6)).astype(np.float64) for i in range(r * R)]
    dys = [0.1 * gen.normal(SEED, f"d{i}", (2, 4)).astype(np.float64) for i in range(r * R)]
    a = ReplicatedStage(layers, p0, depth=W, replicas=r, lr=0.05)
    b = Stage(layers, p0, W, lr=0.05)
    cat = lambda v, k: np.concatenate(v[k * r:(k + 1) * r], axis=0)
    for k in range(W):
        for q in range(r):
            a.forward(k * r + q, xs[k * r + q])
        b.forward(k, cat(xs, k))
    for k in range(R):
        dxa = [a.backward(k * r + q, dys[k * r + q]) for q in range(r)]
        dxb = b.backward(k, cat(dys, k))
        assert np.allclose(np.concatenate(dxa, axis=0), dxb, rtol=1e-12, atol=1e-15)
        a.update(k); b.update(k)
        assert np.allclose(a.rep[0].master, b.master, rtol=1e-12, atol=1e-15)
        if k + W < R:
            for q in range(r):
                a.forward((k + W) * r + q, xs[(k + W) * r + q])
            b.forward(k + W, cat(xs, k + W))


def _torch_replicated_flat_loop(stage_layers, params, xs, ys, reps, depths, lr, mu):
    """Staleness rule of a pipeline whose stage s has reps[s] replicas, as a loop with no schedule: minibatch i sees
    stage s after max(0, i div r_s - W_s + 1) updates; a stage takes one momentum step per round of r_s minibatches,
    with the sum of the round's gradients (the last round may be incomplete)."""
    S, M = len(stage_layers), len(xs)
    cur = [torch.tensor(p) for p in params]
    hist = [[c.clone()] for c in cur]
    mom = [torch.zeros_like(c) for c in cur]
    acc = [torch.zeros_like(c) for c in cur]
    losses = []
    for i in range(M):
        comp = [hist[s][max(0, i // reps[s] - depths[s] + 1)].clone().requires_grad_(True) for s in range(S)]
        l = _torch_model_loss(comp, stage_layers, torch.tensor(xs[i]), torch.tensor(ys[i], dtype=torch.long))
        l.backward()
        losses.append(l.item())
        for s in range(S):
            acc[s] = acc[s] + comp[s].grad
            if i % reps[s] == reps[s] - 1 or i == M - 1:
                mom[s] = mu * mom[s] + acc[s]
                cur[s] = cur[s] - lr * mom[s]
                hist[s].append(cur[s].clone())
                acc[s] = torch.zeros_like(cur[s])
    return [c.numpy() for c in cur], losses


@pytest.mark.parametrize("reps,depths,M", [([2, 1], [2, 1], 12), ([2, 1], [1, 1], 7), ([3, 1], [2, 1], 11),
                                           ([1, 2], [2, 1], 9), ([2, 2, 1], [2, 2, 1], 13), ([2, 3], [2, 1], 10)])
def test_replicated_pipeline_equals_its_staleness_rule(reps, depths, M):
    S = len(reps)
    sl = [[("linear", 12, 12, True), ("linear", 12, 12, True)]] + [[("linear", 12, 12, True)] for _ in range(S - 2)] + \
         [[("linear", 12, 5, False), ("softmax_xent", 5)]]
    params = _params(sl, SEED)
    xs, ys = _data(M, 4, 12, 5, SEED)
    order = []
    stages, losses = run_replicated_pipeline(sl, params, reps, xs, ys, depths, lr=0.05, momentum=0.9, order=order)
    ref_p, ref_l = _torch_replicated_flat_loop(sl, params, xs, ys, reps, depths, 0.05, 0.9)
    assert np.allclose(losses, ref_l, rtol=1e-11)
    for s in range(S):
        assert np.allclose(stages[s].rep[0].master, ref_p[s], rtol=1e-10, atol=1e-13)
        # every op ran exactly once; one update per round
        assert sum(1 for o in order if o[0] == s and o[2] == OP_U) == -(-M // reps[s])
        assert sorted(o[3] for o in order if o[0] == s and o[2] == OP_F) == list(range(M))


def test_without_replication_it_is_the_plain_pipeline():
    sl = gen.config1_mlp(12, 5, 3)
    params = _params(sl, SEED)
    xs, ys = _data(9, 4, 12, 5, SEED)
    a, la = run_replicated_pipeline(sl, params, [1, 1, 1], xs, ys, [3, 2, 1], lr=0.05)
    b, lb = run_pipeline(sl, params, xs, ys, 3, lr=0.05)
    assert la == lb
    for x, y in zip(a, b):
        assert np.array_equal(x.rep[0].master, y.master)
