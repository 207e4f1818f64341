"""GPU parity of the replicated stage (Section 3.3 round-robin routing; Section 4: gradients of all replicas are
aggregated before new parameters are handed out) against oracle/replicated.py, through the C ABI.

Replicas run on their own HIP streams and share one parameter state; the gradient of a round is the sum over the
replicas.  fp32 runs follow their own trajectory (tolerance 1e-4); bf16 runs are compared op by op on the same weights:
after every joint update the shared parameter state is overwritten with the oracle's (oracle -> GPU only), as in
parity_harness.  The bf16 stages here have no ReLU, so no discrete decision can differ between the two sides.
"""
import numpy as np
import pytest
import torch

import paper_1806_03377_amd as pd
import pd_inputs as gen
from gpu_util import GpuReplicatedStage, GpuStage, dev, labels_dev, rel_err, to_dev, to_host
from oracle.replicated import ReplicatedStage, rounds_of, route, run_replicated_pipeline
from oracle.schedule import OP_B, OP_F, OP_U, schedule_1f1b

pytestmark = pytest.mark.gpu
SEED = gen.BASE_SEED + 91
TOL = {False: 1e-4, True: 2e-2}


def _order(r, depth, M):
    """Lock-step op order of one replicated stage: ("F"|"B", minibatch) and ("U", round)."""
    lists = [schedule_1f1b(1, 1, rounds_of(q, r, M), 0, depth_override=depth) for q in range(r)]
    pos = [0] * r
    out = []
    while any(pos[q] < len(lists[q]) for q in range(r)):
        moved = False
        for q in range(r):
            while pos[q] < len(lists[q]) and lists[q][pos[q]].kind != OP_U:
                op = lists[q][pos[q]]
                out.append(("F" if op.kind == OP_F else "B", op.mb * r + q))
                pos[q] += 1
                moved = True
        at_u = [q for q in range(r) if pos[q] < len(lists[q])]
        if at_u:
            k = lists[at_u[0]][pos[at_u[0]]].mb
            assert all(lists[q][pos[q]].kind == OP_U and lists[q][pos[q]].mb == k for q in at_u)
            out.append(("U", k))
            for q in at_u:
                pos[q] += 1
            moved = True
        assert moved
    return out


def _run_stage(layers, params, xs, labs, dys, *, r, depth, precision, lr=0.05, mu=0.9, optimizer="sgd", eps=1.0,
               in_hw=None, minibatch=None, forced=None, same_stream=False, compare_ops=True):
    bf16 = precision == pd.PD_BF16_F32ACC
    tol = TOL[bf16]
    forced = bf16 if forced is None else forced
    M = len(xs)
    B = minibatch or xs[0].shape[0]
    o = ReplicatedStage(layers, params, depth, r, "bf16" if bf16 else "f32", lr, mu, optimizer, eps)
    g = GpuReplicatedStage(layers, params, r, same_stream=same_stream, minibatch=B, precision=precision,
                           in_flight_override=depth, lr=lr, momentum=mu, in_hw=in_hw,
                           optimizer=1 if optimizer == "rmsprop" else 0, eps=eps)
    try:
        has_loss = labs is not None
        x_t = [to_dev(x, bf16) for x in xs]
        l_t = [labels_dev(l) for l in labs] if has_loss else None
        dy_t = [to_dev(d, bf16) for d in dys] if dys is not None else None
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        y_t, dx_t = {}, {}
        o_loss, o_y, o_dx = {}, {}, {}
        torch.cuda.synchronize()          # the inputs were written on torch's stream; the replicas use their own
        for kind, i in _order(r, depth, M):
            if kind == "U":
                o.update(i)
                g.update()
                for q in range(r):
                    assert pd.pd_stage_version(g.rep[q].h) == o.latest
                if compare_ops or o.latest == -(-M // r):
                    p, m = pd.pd_stage_get_params(g.h), pd.pd_stage_get_momentum(g.h)
                    ring = pd.pd_stage_get_params(g.h, -1, True)
                    ref = o.rep[0]
                    for name, got, want in (("weights", p, ref.master), ("state", m, ref.mom), ("ring", ring, ref.versions[-1])):
                        e = rel_err(got, want)
                        assert e <= tol, (name, "round", i, e)
                    # a further replica reads the same state
                    assert np.array_equal(pd.pd_stage_get_params(g.rep[-1].h, -1, True), ring)
                if forced:
                    pd.pd_stage_overwrite_latest(g.h, o.rep[0].master.astype(np.float32), o.rep[0].mom.astype(np.float32))
                continue
            q, k = pd.pd_replica_route(i, r)
            assert (q, k) == route(i, r)
            h = g.rep[q].h
            if kind == "F":
                y_o, loss_o = o.forward(i, np.asarray(xs[i], dtype=np.float64), labs[i] if has_loss else None)
                o_loss[i], o_y[i] = loss_o, y_o
                assert pd.pd_stage_version(h) == o.rep[q].trace[-1].version
                if not has_loss:
                    y_t[i] = torch.empty(y_o.shape, dtype=torch.bfloat16 if bf16 else torch.float32, device=dev())
                pd.pd_forward(h, k, x_t[i].data_ptr(), l_t[i].data_ptr() if has_loss else 0,
                              0 if has_loss else y_t[i].data_ptr(), losses[i:].data_ptr() if has_loss else 0)
                assert pd.pd_stage_version(h, k) == o.rep[q].trace[-1].version
            else:
                dx_o = o.backward(i, None if has_loss else np.asarray(dys[i], dtype=np.float64), need_dx=True)
                o_dx[i] = dx_o
                dx_t[i] = torch.empty(dx_o.shape, dtype=torch.bfloat16 if bf16 else torch.float32, device=dev())
                pd.pd_backward(h, k, 0 if has_loss else dy_t[i].data_ptr(), dx_t[i].data_ptr())
                if compare_ops:
                    torch.cuda.synchronize()
                    e = rel_err(to_host(dx_t[i]), dx_o)
                    assert e <= tol, ("input gradient", i, e)
                    if not has_loss:
                        e = rel_err(to_host(y_t[i]), o_y[i])
                        assert e <= tol, ("output", i, e)
        torch.cuda.synchronize()
        if has_loss and (compare_ops or not bf16):
            got = to_host(losses)
            for i in range(M):
                assert abs(got[i] - o_loss[i]) <= tol * abs(o_loss[i]), ("loss", i, got[i], o_loss[i])
        # each replica's own record: F and B of its rounds with the version both sides agree on, U once per round
        for q in range(r):
            want = [(op.kind, op.mb, op.version, op.slot) for op in o.rep[q].trace
                    if not (op.kind == OP_U and op.mb >= rounds_of(q, r, M))]
            assert pd.pd_stage_trace(g.rep[q].h) == want, ("trace", q)
        return pd.pd_stage_get_params(g.h)
    finally:
        g.close()


MLP = [("linear", 40, 48, True), ("linear", 48, 16, False), ("softmax_xent", 16)]


def _mlp_data(M, B, seed):
    p = gen.init_params(seed, "m", MLP)
    p = p + 0.01 * gen.normal(seed, "mb", p.shape)
    xs = list(gen.normal(seed, "X", (M, B, 40)))
    labs = list(gen.labels(seed, "Y", (M, B), 16))
    return p, xs, labs


@pytest.mark.parametrize("r,depth,M", [(2, 2, 9), (3, 1, 7), (4, 2, 16)])
def test_replicated_mlp_stage_f32(r, depth, M):
    p, xs, labs = _mlp_data(M, 8, SEED)
    _run_stage(MLP, p, xs, labs, None, r=r, depth=depth, precision=pd.PD_F32)


def test_replicated_stage_f32_free_running_without_host_synchronisation():
    # nothing is compared (and nothing read back) until the stream of ops has been enqueued: the order between the
    # replicas' streams and the joint update rests on the events inside pd_update_replicated alone
    p, xs, labs = _mlp_data(12, 8, SEED + 1)
    _run_stage(MLP, p, xs, labs, None, r=2, depth=2, precision=pd.PD_F32, compare_ops=False)
    _run_stage(MLP, p, xs, labs, None, r=2, depth=2, precision=pd.PD_F32, compare_ops=False, same_stream=True)


def test_replicated_stage_without_loss_f32():
    layers = [("linear", 24, 32, True), ("linear", 32, 16, True)]
    p = gen.init_params(SEED + 2, "n", layers)
    xs = list(gen.normal(SEED + 2, "X", (8, 6, 24)))
    dys = list(0.1 * gen.normal(SEED + 2, "D", (8, 6, 16)))
    _run_stage(layers, p, xs, None, dys, r=2, depth=2, precision=pd.PD_F32)


@pytest.mark.parametrize("optimizer", ["sgd", "rmsprop"])
def test_replicated_linear_stage_bf16(optimizer):
    # minibatch-sized rows: the fused weight-gradient kernel in its gradient-only mode
    layers = [("linear", 40, 48, False), ("linear", 48, 16, False), ("softmax_xent", 16)]
    p = gen.init_params(SEED + 3, "b", layers)
    p = p + 0.01 * gen.normal(SEED + 3, "bb", p.shape)
    xs = list(gen.normal(SEED + 3, "X", (7, 8, 40)))
    labs = list(gen.labels(SEED + 3, "Y", (7, 8), 16))
    _run_stage(layers, p, xs, labs, None, r=2, depth=2, precision=pd.PD_BF16_F32ACC, optimizer=optimizer,
               lr=0.045 if optimizer == "rmsprop" else 0.05)


def test_replicated_conv_stage_bf16():
    # the paper replicates the convolutional stage of VGG16; partial sums -> reduce kernel in gradient-only mode
    layers = [("conv2d", 8, 16, 3, 3, 1, 1, 1, False), ("maxpool2d", 2, 2), ("conv2d", 16, 32, 1, 1, 1, 0, 0, False),
              ("linear", 4 * 4 * 32, 16, False), ("softmax_xent", 16)]
    p = gen.init_params(SEED + 4, "c", layers)
    p = p + 0.01 * gen.normal(SEED + 4, "cb", p.shape)
    xs = list(gen.normal(SEED + 4, "X", (6, 4, 8, 8, 8)))
    labs = list(gen.labels(SEED + 4, "Y", (6, 4), 16))
    _run_stage(layers, p, xs, labs, None, r=3, depth=1, precision=pd.PD_BF16_F32ACC, in_hw=(8, 8))


def test_replicated_many_row_stage_bf16():
    # 24 steps x 24 sequences = 576 rows: the many-row weight-gradient product writing plain gradients
    layers = [("lstm", 32, 24, 24), ("linear", 24, 40, False), ("softmax_xent", 40)]
    p = gen.init_params(SEED + 5, "l", layers)
    xs = list(gen.normal(SEED + 5, "X", (4, 24, 24, 32)))
    labs = list(gen.labels(SEED + 5, "Y", (4, 24, 24), 40))
    _run_stage(layers, p, xs, labs, None, r=2, depth=1, precision=pd.PD_BF16_F32ACC, minibatch=24)


def test_pipeline_with_replicated_input_stage_f32():
    # the "2-1" shape of the paper's VGG16 configuration: a replicated input stage feeding one output stage
    sl = [[("linear", 24, 32, True), ("linear", 32, 32, True)], [("linear", 32, 10, False), ("softmax_xent", 10)]]
    params = [gen.init_params(SEED + 6, f"s{s}", ly) for s, ly in enumerate(sl)]
    M, B, r, depths = 11, 6, 2, [2, 1]
    xs = list(gen.normal(SEED + 6, "X", (M, B, 24)))
    labs = list(gen.labels(SEED + 6, "Y", (M, B), 10))
    order = []
    o_stages, o_losses = run_replicated_pipeline(sl, params, [r, 1], [np.asarray(x, dtype=np.float64) for x in xs], labs,
                                                 depths, lr=0.05, momentum=0.9, order=order)
    g0 = GpuReplicatedStage(sl[0], params[0], r, minibatch=B, precision=pd.PD_F32, stage_index=0, num_stages=2,
                            in_flight_override=depths[0], lr=0.05, momentum=0.9)
    g1 = GpuStage(sl[1], params[1], minibatch=B, precision=pd.PD_F32, stage_index=1, num_stages=2,
                  in_flight_override=depths[1], lr=0.05, momentum=0.9, stream=torch.cuda.Stream())
    try:
        x_t = [to_dev(x, False) for x in xs]
        l_t = [labels_dev(l) for l in labs]
        y_t = [torch.empty((B, 32), dtype=torch.float32, device=dev()) for _ in range(M)]
        d_t = [torch.empty((B, 32), dtype=torch.float32, device=dev()) for _ in range(M)]
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        for s, q, kind, i in order:
            if s == 0 and kind == OP_U:
                g0.update()
            elif s == 0:
                h, k = g0.rep[q].h, i // r
                if kind == OP_F:
                    pd.pd_forward(h, k, x_t[i].data_ptr(), 0, y_t[i].data_ptr(), 0)
                else:
                    pd.pd_backward(h, k, d_t[i].data_ptr(), 0)
            elif kind == OP_F:
                pd.pd_forward(g1.h, i, y_t[i].data_ptr(), l_t[i].data_ptr(), 0, losses[i:].data_ptr())
            elif kind == OP_B:
                pd.pd_backward(g1.h, i, 0, d_t[i].data_ptr())
            else:
                pd.pd_update(g1.h)
            torch.cuda.synchronize()      # the hand-off between the stages' streams is the test's, not the library's
        got = to_host(losses)
        for i in range(M):
            assert abs(got[i] - o_losses[i]) <= 1e-4 * abs(o_losses[i]), ("loss", i)
        assert rel_err(pd.pd_stage_get_params(g0.h), o_stages[0].rep[0].master) <= 1e-4
        assert rel_err(pd.pd_stage_get_params(g1.h), o_stages[1].rep[0].master) <= 1e-4
        assert pd.pd_stage_version(g0.h) == -(-M // r) and pd.pd_stage_version(g1.h) == M
    finally:
        g0.close()
        g1.close()


@pytest.mark.parametrize("reps,depths,M", [([2, 1], [2, 1], 11), ([3, 1], [1, 1], 7), ([1, 2], [2, 1], 9),
                                           ([2, 2, 1], [2, 2, 1], 13), ([2, 1], [1, 1], 1),
                                           # long streams: the drivers' event rings wrap many times
                                           ([2, 1], [2, 1], 150), ([1, 3], [3, 1], 140), ([2, 3, 1], [3, 2, 1], 130),
                                           ([4, 1], [1, 1], 101)])
def test_library_driven_pipeline_with_replicated_stages_f32(reps, depths, M):
    # pd_pipeline_run_replicated enqueues the whole stream with events only; nothing is read back before the end
    S, B = len(reps), 6
    sl = [[("linear", 24, 32, True)]] + [[("linear", 32, 32, True)] for _ in range(S - 2)] + \
         [[("linear", 32, 10, False), ("softmax_xent", 10)]]
    params = [gen.init_params(SEED + 8, f"s{s}", ly) for s, ly in enumerate(sl)]
    xs = gen.normal(SEED + 8, "X", (M, B, 24))
    labs = gen.labels(SEED + 8, "Y", (M, B), 10)
    o_stages, o_losses = run_replicated_pipeline(sl, params, reps, [np.asarray(x, dtype=np.float64) for x in xs],
                                                 list(labs), depths, lr=0.05, momentum=0.9)
    gs = []
    try:
        for s in range(S):
            kw = dict(minibatch=B, precision=pd.PD_F32, stage_index=s, num_stages=S, in_flight_override=depths[s],
                      lr=0.05, momentum=0.9)
            if reps[s] > 1:
                gs.append(GpuReplicatedStage(sl[s], params[s], reps[s], stream=torch.cuda.Stream(), **kw))
            else:
                gs.append(GpuStage(sl[s], params[s], stream=torch.cuda.Stream(), **kw))
        handles = [g.handles() if isinstance(g, GpuReplicatedStage) else [g.h] for g in gs]
        x_d, l_d = to_dev(xs, False), labels_dev(labs)
        losses = torch.zeros(M, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        pd.pd_pipeline_run_replicated(handles, M, x_d.data_ptr(), l_d.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        got = to_host(losses)
        for i in range(M):
            assert abs(got[i] - o_losses[i]) <= 1e-4 * abs(o_losses[i]), ("loss", i, got[i], o_losses[i])
        for s in range(S):
            h0 = handles[s][0]
            assert rel_err(pd.pd_stage_get_params(h0), o_stages[s].rep[0].master) <= 1e-4, ("weights", s)
            assert rel_err(pd.pd_stage_get_momentum(h0), o_stages[s].rep[0].mom) <= 1e-4, ("momentum", s)
            assert pd.pd_stage_version(h0) == -(-M // reps[s])
            for q, h in enumerate(handles[s]):      # every replica ran exactly its own static list
                want = [(op.kind, op.mb, op.version, op.slot) for op in o_stages[s].rep[q].trace
                        if not (op.kind == OP_U and op.mb >= rounds_of(q, reps[s], M))]
                assert pd.pd_stage_trace(h) == want, ("trace", s, q)
        with pytest.raises(pd.PdError):              # not freshly initialised any more
            pd.pd_pipeline_run_replicated(handles, M, x_d.data_ptr(), l_d.data_ptr(), losses.data_ptr())
    finally:
        for g in gs:
            g.close()


def test_replicated_protocol_errors():
    p, xs, labs = _mlp_data(2, 8, SEED + 7)
    g = GpuReplicatedStage(MLP, p, 2, minibatch=8, precision=pd.PD_F32, in_flight_override=1)
    plain = GpuStage(MLP, p, minibatch=8, precision=pd.PD_F32, in_flight_override=1)
    try:
        def status(fn, *a):
            with pytest.raises(pd.PdError) as e:
                fn(*a)
            return e.value.status
        assert status(pd.pd_update_replicated, g.handles()) == pd.PD_ESTATE          # nothing pending
        assert status(pd.pd_update_replicated, [g.rep[0].h]) == pd.PD_EINVAL          # not all replicas
        assert status(pd.pd_update_replicated, [g.rep[1].h, g.rep[0].h]) == pd.PD_EINVAL   # wrong order
        assert status(pd.pd_update_replicated, [plain.h]) == pd.PD_EINVAL             # not replicated
        assert status(pd.pd_stage_set_params, g.rep[1].h, p) == pd.PD_ESTATE          # state belongs to the primary
        assert status(pd.pd_stage_overwrite_latest, g.rep[1].h, p, None) == pd.PD_ESTATE
        assert status(pd.pd_stage_destroy, g.rep[0].h) == pd.PD_ESTATE                # further replicas first
        arena = torch.empty(pd.pd_stage_replica_query_bytes(g.rep[0].cfg) + 256, dtype=torch.uint8, device=dev())
        base = (arena.data_ptr() + 255) // 256 * 256
        assert status(pd.pd_stage_create_replica, g.rep[0].h, 0, base, arena.numel() - 256) == pd.PD_ESTATE  # has its 2
        assert status(pd.pd_stage_create_replica, plain.h, 0, base, arena.numel() - 256) == pd.PD_EINVAL
        x, l = to_dev(xs[0], False), labels_dev(labs[0])
        loss = torch.zeros(1, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()
        pd.pd_forward(g.rep[1].h, 0, x.data_ptr(), l.data_ptr(), 0, loss.data_ptr())
        pd.pd_backward(g.rep[1].h, 0, 0, 0)
        assert status(pd.pd_update, g.rep[1].h) == pd.PD_ESTATE                       # joint update only
        assert status(pd.pd_stage_overwrite_latest, g.h, p, None) == pd.PD_ESTATE     # a replica's gradient is pending
        g.update()                                                                    # a round with one replica in it
        assert [pd.pd_stage_version(h) for h in g.handles()] == [1, 1]
        assert len(pd.pd_stage_trace(g.rep[0].h)) == 0 and len(pd.pd_stage_trace(g.rep[1].h)) == 3
        pd.pd_stage_set_params(g.h, p)                                                # resets every replica
        assert [pd.pd_stage_version(h) for h in g.handles()] == [0, 0]
        assert len(pd.pd_stage_trace(g.rep[1].h)) == 0
    finally:
        g.close()
        plain.close()


def test_checkpoint_of_a_replicated_stage(tmp_path):
    # the parameter state of a replicated stage is one copy: saved from the primary after a joint update, loaded
    # into the primary of another replicated stage, which restarts every replica at the saved version
    import torch
    p, xs, labs = _mlp_data(4, 8, SEED + 9)
    path = str(tmp_path / "replicated.ckpt")
    a = GpuReplicatedStage(MLP, p, 2, minibatch=8, precision=pd.PD_BF16_F32ACC, in_flight_override=1, optimizer=1, eps=1.0,
                           lr=0.045)
    b = GpuReplicatedStage(MLP, None, 2, minibatch=8, precision=pd.PD_BF16_F32ACC, in_flight_override=1, optimizer=1,
                           eps=1.0, lr=0.045)
    try:
        x_t = [to_dev(x, True) for x in xs]
        l_t = [labels_dev(l) for l in labs]
        loss = torch.zeros(4, dtype=torch.float32, device=dev())
        torch.cuda.synchronize()

        def round_(g, k):
            for q in range(2):
                i = 2 * k + q
                pd.pd_forward(g.rep[q].h, k, x_t[i].data_ptr(), l_t[i].data_ptr(), 0, loss[i:].data_ptr())
            for q in range(2):
                pd.pd_backward(g.rep[q].h, k, 0, 0)
            g.update()

        round_(a, 0)
        with pytest.raises(pd.PdError) as e:
            pd.pd_stage_checkpoint_load(a.rep[1].h, path)          # the state belongs to the primary
        assert e.value.status in (pd.PD_ESTATE, pd.PD_EINVAL)
        pd.pd_stage_checkpoint_save(a.h, path)
        assert pd.pd_checkpoint_info(path)[1] == 1
        pd.pd_stage_checkpoint_load(b.h, path)
        assert [pd.pd_stage_version(h) for h in b.handles()] == [1, 1]
        assert np.array_equal(pd.pd_stage_get_params(b.rep[1].h), pd.pd_stage_get_params(a.h))
        assert np.array_equal(pd.pd_stage_get_momentum(b.h), pd.pd_stage_get_momentum(a.h))
        # both continue identically: a with round 1, b (fresh replicas at version 1) with its own round 0 of the same data
        round_(a, 1)
        for q in range(2):
            i = 2 + q
            pd.pd_forward(b.rep[q].h, 0, x_t[i].data_ptr(), l_t[i].data_ptr(), 0, loss[i:].data_ptr())
        for q in range(2):
            pd.pd_backward(b.rep[q].h, 0, 0, 0)
        b.update()
        assert np.array_equal(pd.pd_stage_get_params(b.h), pd.pd_stage_get_params(a.h))
        assert np.array_equal(pd.pd_stage_get_momentum(b.h), pd.pd_stage_get_momentum(a.h))
        assert pd.pd_stage_version(b.h) == 2 == pd.pd_stage_version(a.h)
    finally:
        a.close()
        b.close()
