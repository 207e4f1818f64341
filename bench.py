#!/usr/bin/env python3
"""Benchmark of the 1F1B weight-stashed stage step on one MI355X.

A *step* is one steady-state iteration of one stage: B(k), U(k), F(k + depth)
(backward of the oldest in-flight minibatch against its stashed weight version,
the momentum-SGD update into the version ring, and the forward that refills the
freed slot with the newest version).  Default workload: the VGG16 classifier as
one stage (Linear 25088-4096-4096-1000 + ReLU + softmax cross-entropy), bf16 with
fp32 accumulation, minibatch 64, ring depth 4, synthetic N(0,1) inputs already
resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "samples/sec per 1F1B stage step (bf16) + MFMA util % of MI355X peak"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK = 2.5e15
# Algorithmic HBM bytes per parameter of the fused weight-gradient + update launch.  With the fp32 master weights as an
# array of their own: read master 4 + momentum 4, write master 4 + momentum 4 + bf16 ring copy 2 = 18.  As stored
# here (master = latest ring copy + 16-bit remainder): read ring copy 2 + remainder 2 + momentum 4, write remainder 2 +
# momentum 4 + ring copy 2 = 16.  The roofline object reports the kernel against both.
SURVEY_UPDATE_BYTES_PER_PARAM = 18
STORED_UPDATE_BYTES_PER_PARAM = 16
# HBM bytes per launch of the dominant kernel at the default workload, from the rocprofv3 counter runs
# summarised in profiles/wgrad_update_vgg16fc_mb64.txt (FETCH_SIZE x 1.986 + WRITE_SIZE x 1.000)
MEASURED_TRAFFIC_BYTES = 1.988e9


def cpu_baseline(layers, params, xs, labs, depth, budget_s=12.0, max_steps=16, lr=0.01):
    """The oracle, as it stands, on the host cores: same stage, same step, a bounded number of steps (about 10 s of
    work; the oracle keeps every weight version it produces, about 1 GB each at this size, hence the step cap)."""
    import numpy as np
    from oracle.pipeline import Stage
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    st = Stage(layers, params, depth, "bf16", lr=lr)
    n = len(xs)
    for i in range(depth):
        st.forward(i, xs[i % n].astype(np.float64), labs[i % n])
    steps, t0 = 0, time.time()
    while steps < max_steps and (steps == 0 or time.time() - t0 < budget_s):
        k = steps
        st.backward(k, None, need_dx=True)
        st.update(k)
        st.forward(k + depth, xs[(k + depth) % n].astype(np.float64), labs[(k + depth) % n])
        steps += 1
    dt = time.time() - t0
    B = xs[0].shape[0]
    return {"value": steps * B / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{steps} steady-state steps (B,U,F) of the same full-size stage, fp64 numpy, {dt:.1f} s"}


def bench_conv(args, pd, gen, torch, np, dev):
    """Secondary workload: the VGG16 conv stage (64-64-P-128-128-P-256x3-P on 3x224x224 images) as the input
    stage of a pipeline: depth 4, synthetic upstream gradient, no dL/d(input)."""
    B, depth, K, W = args.minibatch, args.depth, args.steps, args.warmup
    hw = (64, 64) if args.small else (224, 224)
    layers = gen.config3_vgg_conv()
    seed = gen.BASE_SEED + 2
    params = gen.init_params(seed, "vgg_conv", layers)
    stream = torch.cuda.Stream(device=dev)
    bstream = None if _single_stream(args, True) else torch.cuda.Stream(device=dev)
    cfg = pd.make_config(layers, in_flight_override=depth, minibatch=B, precision=pd.PD_BF16_F32ACC, lr=0.01,
                         momentum=0.9, stream=stream.cuda_stream, in_hw=hw,
                         stream_backward=bstream.cuda_stream if bstream is not None else 0)
    nbytes = pd.pd_stage_query_bytes(cfg)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    h = pd.pd_stage_create(cfg, (arena.data_ptr() + 255) // 256 * 256, nbytes)
    pd.pd_stage_set_params(h, params)
    n_pool = 2
    xd = [torch.from_numpy(gen.normal(seed, f"x{i}", (B, hw[0], hw[1], 3))).to(dev).to(torch.bfloat16) for i in range(n_pool)]
    oh, ow = hw[0] // 8, hw[1] // 8
    dyd = [(torch.from_numpy(gen.normal(seed, f"dy{i}", (B, oh, ow, 256))) * 0.01).to(dev).to(torch.bfloat16) for i in range(n_pool)]
    torch.cuda.synchronize()
    mb_next = 0

    def fwd():
        nonlocal mb_next
        pd.pd_forward(h, mb_next, xd[mb_next % n_pool].data_ptr(), 0, 0, 0)
        mb_next += 1

    def step(k):
        pd.pd_backward(h, k, dyd[k % n_pool].data_ptr(), 0)
        pd.pd_update(h)
        fwd()

    for _ in range(depth):
        fwd()
    k = 0
    for _ in range(W):
        step(k); k += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step(k); k += 1
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / K
    # flops: 2 * pixels * 9 * c_in * c_out per conv forward; dgrad and wgrad the same, no dgrad for the first layer
    f, h_, w_, fl_first = 0.0, hw[0], hw[1], 0.0
    for L in layers:
        if L[0] == "conv2d":
            fl = 2.0 * B * h_ * w_ * 9 * L[1] * L[2]
            f += 3 * fl
            if L[1] == 3:
                f -= fl
        else:
            h_, w_ = h_ // 2, w_ // 2
    out = {"metric": METRIC, "value": B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": ("REDUCED " if args.small else "") + f"VGG16 conv stage 64-64-P-128-128-P-256x3-P on 3x{hw[0]}x{hw[1]} "
                      f"images, bf16 w/ fp32 accum, minibatch {B}, ring depth {depth}, step = B(k) U(k) F(k+depth)",
                      "minibatch": B, "ring_depth": depth},
           "step_gflop": f / 1e9, "mfma_util_pct": 100.0 * f / (ms * 1e-3) / MFMA_BF16_PEAK,
           "roofline": {"bound": "mfma", "kernel": "whole step (conv3x3_halo_kernel + conv_wgrad_tr_kernel dominate)",
                        "achieved": f / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                        "frac": f / (ms * 1e-3) / MFMA_BF16_PEAK, "traffic": None}}
    pd.pd_stage_destroy(h)
    return out


def bench_replicated(args, pd, gen, torch, np, dev):
    """Secondary workload: the VGG16 conv stage REPLICATED (the stage the paper replicates in its VGG16
    configuration), r replicas on r streams sharing one parameter state.  A step is one round: B on every replica,
    the joint update (gradients summed over the replicas), F of the round `depth` later on every replica.  The same
    stage without replication is timed beside it (ms per minibatch) to show what the replication machinery costs."""
    B, depth, K, W, r = args.minibatch, args.depth, args.steps, args.warmup, args.replicas
    hw = (64, 64) if args.small else (224, 224)
    layers = gen.config3_vgg_conv()
    seed = gen.BASE_SEED + 2
    params = gen.init_params(seed, "vgg_conv", layers)
    n_pool = 2
    xd = [torch.from_numpy(gen.normal(seed, f"x{i}", (B, hw[0], hw[1], 3))).to(dev).to(torch.bfloat16) for i in range(n_pool)]
    oh, ow = hw[0] // 8, hw[1] // 8
    dyd = [(torch.from_numpy(gen.normal(seed, f"dy{i}", (B, oh, ow, 256))) * 0.01).to(dev).to(torch.bfloat16) for i in range(n_pool)]

    def make(replicas):
        streams = [torch.cuda.Stream(device=dev) for _ in range(max(1, replicas))]
        cfg = pd.make_config(layers, in_flight_override=depth, minibatch=B, precision=pd.PD_BF16_F32ACC, lr=0.01,
                             momentum=0.9, stream=streams[0].cuda_stream, in_hw=hw, replicas=replicas)
        arenas, hs = [], []
        n = pd.pd_stage_query_bytes(cfg)
        arenas.append(torch.empty(n + 256, dtype=torch.uint8, device=dev))
        hs.append(pd.pd_stage_create(cfg, (arenas[0].data_ptr() + 255) // 256 * 256, n))
        pd.pd_stage_set_params(hs[0], params)
        for q in range(1, replicas):
            n = pd.pd_stage_replica_query_bytes(cfg)
            arenas.append(torch.empty(n + 256, dtype=torch.uint8, device=dev))
            torch.cuda.synchronize()
            hs.append(pd.pd_stage_create_replica(hs[0], streams[q].cuda_stream, (arenas[q].data_ptr() + 255) // 256 * 256, n))
        return hs, arenas, streams, cfg

    def run(hs):
        n = len(hs)
        nxt = 0

        def fwd_round():
            nonlocal nxt
            for q, h in enumerate(hs):
                pd.pd_forward(h, nxt, xd[(nxt + q) % n_pool].data_ptr(), 0, 0, 0)
            nxt += 1

        def step(k):
            for q, h in enumerate(hs):
                pd.pd_backward(h, k, dyd[(k + q) % n_pool].data_ptr(), 0)
            if n > 1:
                pd.pd_update_replicated(hs)
            else:
                pd.pd_update(hs[0])
            fwd_round()

        for _ in range(depth):
            fwd_round()
        k = 0
        for _ in range(W):
            step(k); k += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            step(k); k += 1
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / K

    torch.cuda.synchronize()
    hs1, a1, s1, _ = make(0)
    ms_single = run(hs1)
    pd.pd_stage_destroy(hs1[0])
    del a1
    hs, arenas, streams, cfg = make(r)
    ms = run(hs)
    P = pd.pd_stage_num_params(hs[0])
    for h in reversed(hs):
        pd.pd_stage_destroy(h)
    f, h_, w_ = 0.0, hw[0], hw[1]
    for L in layers:
        if L[0] == "conv2d":
            fl = 2.0 * B * h_ * w_ * 9 * L[1] * L[2]
            f += 3 * fl
            if L[1] == 3:
                f -= fl
        else:
            h_, w_ = h_ // 2, w_ // 2
    f *= r
    out = {"metric": METRIC, "value": r * B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": ("REDUCED " if args.small else "") + f"VGG16 conv stage on 3x{hw[0]}x{hw[1]} images replicated x{r} "
                      f"({r} streams, one parameter state), bf16 w/ fp32 accum, minibatch {B} per replica, depth {depth}; "
                      f"step = one round: B on every replica, summed update, F on every replica",
                      "minibatch": B, "replicas": r, "ring_depth": depth, "params": P},
           "ms_per_minibatch": ms / r, "ms_per_minibatch_unreplicated": ms_single,
           "replication_overhead": ms / r / ms_single - 1.0,
           "step_gflop": f / 1e9, "mfma_util_pct": 100.0 * f / (ms * 1e-3) / MFMA_BF16_PEAK,
           "roofline": {"bound": "mfma", "kernel": "whole round (the convolution kernels dominate; the summed update "
                        f"streams {4 * r + 18} bytes per parameter)",
                        "achieved": f / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                        "frac": f / (ms * 1e-3) / MFMA_BF16_PEAK, "traffic": None}}
    return out


def bench_vgg16_pipeline(args, pd, gen, torch, np, dev):
    """Secondary workload: ALL of VGG16 (13 convolutions, 5 poolings, 3 Linear layers, loss) as the paper's kind of
    configuration for it, a replicated convolutional stage feeding one classifier stage (its Table 1 lists 15-1 on 16
    machines; here r-1 on one GPU, every replica and the classifier on a stream of its own), run by
    pd_pipeline_run_replicated.  NOAM = ceil((r + 1) / r) = 2 for r >= 1: depth 2 on the input stage, 1 on the output stage.
    The unreplicated 1-1 pipeline is timed beside it."""
    B, K, W, r = args.minibatch, args.steps, args.warmup, args.replicas
    hw = (64, 64) if args.small else (224, 224)
    full = gen.vgg16_full()
    n_conv = len(gen.config3_vgg_conv()) + 8          # the conv/pool part (18 layers)
    conv, fc = full[:n_conv], full[n_conv:]
    if args.small:
        fc = gen.config2_vgg_fc((hw[0] // 32) * (hw[1] // 32) * 512)
    seed = gen.BASE_SEED + 6
    LR = 1e-4   # (N(0,1) pixels through 16 unnormalised layers: the paper's 0.01 diverges on such inputs)
    p_conv, p_fc = gen.init_params(seed, "conv", conv), gen.init_params(seed, "fc", fc)
    M = max(K, 2)
    x = torch.from_numpy(gen.normal_bulk(seed, "x", (M, B, hw[0], hw[1], 3))).to(dev).to(torch.bfloat16)
    lab = torch.from_numpy(gen.labels(seed, "y", (M, B), 1000)).to(dev)
    losses = torch.zeros(M, dtype=torch.float32, device=dev)

    def build(reps):
        keep, handles = [], []
        def arena(n):
            t = torch.empty(n + 256, dtype=torch.uint8, device=dev); keep.append(t)
            return (t.data_ptr() + 255) // 256 * 256
        streams = [torch.cuda.Stream(device=dev) for _ in range(reps + 1)]; keep.append(streams)
        c0 = pd.make_config(conv, stage_index=0, num_stages=2, noam=2, minibatch=B, precision=pd.PD_BF16_F32ACC, lr=LR,
                            momentum=0.9, stream=streams[0].cuda_stream, in_hw=hw, replicas=reps if reps > 1 else 0)
        n = pd.pd_stage_query_bytes(c0)
        h0 = pd.pd_stage_create(c0, arena(n), n)
        hs0 = [h0]
        for q in range(1, reps):
            n = pd.pd_stage_replica_query_bytes(c0)
            a = arena(n)
            torch.cuda.synchronize()
            hs0.append(pd.pd_stage_create_replica(h0, streams[q].cuda_stream, a, n))
        c1 = pd.make_config(fc, stage_index=1, num_stages=2, noam=2, minibatch=B, precision=pd.PD_BF16_F32ACC, lr=LR,
                            momentum=0.9, stream=streams[reps].cuda_stream)
        n = pd.pd_stage_query_bytes(c1)
        h1 = pd.pd_stage_create(c1, arena(n), n)
        return [hs0, [h1]], keep

    def run(handles, m):
        pd.pd_stage_set_params(handles[0][0], p_conv)     # (also resets every replica: the driver wants fresh stages)
        pd.pd_stage_set_params(handles[1][0], p_fc)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pd.pd_pipeline_run_replicated(handles, m, x.data_ptr(), lab.data_ptr(), losses.data_ptr())
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    res = {}
    for reps in (1, r):
        handles, keep = build(reps)
        run(handles, max(2, min(W, M)))
        res[reps] = run(handles, M)
        for hs in reversed(handles):
            for h in reversed(hs):
                pd.pd_stage_destroy(h)
        del keep
    ms = res[r] / M
    P = int(p_conv.size + p_fc.size)
    out = {"metric": METRIC, "value": B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": M, "warmup": W,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": ("REDUCED " if args.small else "") + f"VGG16 (all 16 weight layers) on 3x{hw[0]}x{hw[1]} images as a "
                      f"{r}-1 pipeline: convolutional stage replicated x{r} + classifier stage, {r + 1} streams, "
                      f"bf16 w/ fp32 accum, minibatch {B}, NOAM 2; step = one minibatch through the whole pipeline "
                      f"(wall time of {M} minibatches incl. start-up and drain)",
                      "minibatch": B, "replicas": r, "params": P},
           "ms_per_minibatch_1_1_pipeline": res[1] / M, "first_loss": float(losses[0].item()),
           "final_loss": float(losses[-1].item())}
    return out


def bench_s2vt(args, pd, gen, torch, np, dev):
    """Secondary workload: the S2VT-shaped model (LSTM 4096->1000 | LSTM 1000->1000 + vocab 30000 + loss), seq 80,
    minibatch 64, as a 2-stage pipeline on two streams (pd_pipeline_run, NOAM 2).  A step = one minibatch through
    both stages (F, B, U on each)."""
    B, K, W = args.minibatch, args.steps, args.warmup
    T, I, H, V = (8, 256, 128, 1000) if args.small else (80, 4096, 1000, 30000)
    sl = gen.config4_s2vt(I, H, V, T)
    seed = gen.BASE_SEED + 3
    streams = [torch.cuda.Stream(device=dev) for _ in range(2)]
    bstreams = [None if _single_stream(args, False) else torch.cuda.Stream(device=dev) for _ in range(2)]
    hs, arenas = [], []
    for s in range(2):
        cfg = pd.make_config(sl[s], stage_index=s, num_stages=2, noam=2, minibatch=B, precision=pd.PD_BF16_F32ACC,
                             lr=0.01, momentum=0.9, stream=streams[s].cuda_stream,
                             stream_backward=bstreams[s].cuda_stream if bstreams[s] is not None else 0)
        nbytes = pd.pd_stage_query_bytes(cfg)
        arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        h = pd.pd_stage_create(cfg, (arena.data_ptr() + 255) // 256 * 256, nbytes)
        pd.pd_stage_set_params(h, gen.init_params(seed, f"s{s}", sl[s]))
        hs.append(h); arenas.append(arena)
    M = W + K
    n_pool = 2
    x1 = torch.from_numpy(gen.normal(seed, "x", (n_pool, T, B, I))).to(dev).to(torch.bfloat16)
    l1 = torch.from_numpy(gen.labels(seed, "y", (n_pool, T, B), V)).to(dev)
    xs = x1.repeat((M + n_pool - 1) // n_pool, 1, 1, 1)[:M].contiguous()
    ls = l1.repeat((M + n_pool - 1) // n_pool, 1, 1)[:M].contiguous()
    losses = torch.zeros(M, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    if W:
        pd.pd_pipeline_run(hs, W, xs.data_ptr(), ls.data_ptr(), losses.data_ptr())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pd.pd_pipeline_run(hs, K, xs[W:].data_ptr(), ls[W:].data_ptr(), losses[W:].data_ptr())
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / K
    rows = T * B
    f = 6.0 * rows * (4 * H * I + 4 * H * H) + 6.0 * rows * (4 * H * H + 4 * H * H) + 6.0 * rows * H * V
    f -= 2.0 * rows * 4 * H * I   # no dL/d(input) on the input stage
    out = {"metric": METRIC, "value": B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": ("REDUCED " if args.small else "") + f"S2VT-shaped 2-stage pipeline: LSTM {I}->{H} | LSTM {H}->{H} + "
                      f"Linear {H}->{V} + softmax-xent, seq {T}, minibatch {B}, NOAM 2, two streams; step = one minibatch "
                      "through both stages (drained pipeline of `steps` minibatches)", "minibatch": B},
           "step_gflop": f / 1e9, "mfma_util_pct": 100.0 * f / (ms * 1e-3) / MFMA_BF16_PEAK,
           "roofline": {"bound": "mfma", "kernel": "whole step", "achieved": f / (ms * 1e-3) / 1e12,
                        "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": f / (ms * 1e-3) / MFMA_BF16_PEAK,
                        "traffic": None},
           "final_loss": float(losses[-1].item())}
    for h in hs:
        pd.pd_stage_destroy(h)
    return out


def bench_inception(args, pd, gen, torch, np, dev):
    """Secondary workload: the Inception-shaped network (299 x 299 images, blocks of parallel 1x1 / 3x3 / 5x5 /
    1x7 / 7x1 / pooling branches joined by channel concatenation) split into four stages on four streams
    (pd_pipeline_run, NOAM 4).  A step = one minibatch through all four stages (F, B, U on each)."""
    B, K, W = args.minibatch, args.steps, args.warmup
    width, classes = (0.25, 16) if args.small else (1.0, 1000)
    sl, sizes = gen.config5_inception(classes, width)
    S = len(sl)
    seed = gen.BASE_SEED + 4
    streams = [torch.cuda.Stream(device=dev) for _ in range(S)]
    bstreams = [None if _single_stream(args, True) else torch.cuda.Stream(device=dev) for _ in range(S)]
    hs, arenas = [], []
    fwd = []
    for s in range(S):
        cfg = pd.make_config(sl[s], stage_index=s, num_stages=S, noam=S, minibatch=B, precision=pd.PD_BF16_F32ACC,
                             lr=1e-3, momentum=0.9, stream=streams[s].cuda_stream, in_hw=sizes[s],
                             stream_backward=bstreams[s].cuda_stream if bstreams[s] is not None else 0)
        nbytes = pd.pd_stage_query_bytes(cfg)
        arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        h = pd.pd_stage_create(cfg, (arena.data_ptr() + 255) // 256 * 256, nbytes)
        pd.pd_stage_set_params(h, gen.init_params(seed, f"s{s}", sl[s]))
        hs.append(h); arenas.append(arena)
        fwd.append(gen.forward_flops(sl[s], sizes[s], B)[0])
    M = W + K
    n_pool = 2
    x1 = torch.from_numpy(gen.normal(seed, "x", (n_pool, B, 299, 299, 3))).to(dev).to(torch.bfloat16)
    l1 = torch.from_numpy(gen.labels(seed, "y", (n_pool, B), classes)).to(dev)
    xs = x1.repeat((M + n_pool - 1) // n_pool, 1, 1, 1, 1)[:M].contiguous()
    ls = l1.repeat((M + n_pool - 1) // n_pool, 1)[:M].contiguous()
    losses = torch.zeros(M, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    if W:
        pd.pd_pipeline_run(hs, W, xs.data_ptr(), ls.data_ptr(), losses.data_ptr())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pd.pd_pipeline_run(hs, K, xs[W:].data_ptr(), ls[W:].data_ptr(), losses[W:].data_ptr())
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / K
    # forward + weight gradient + input gradient; the first convolution needs no input gradient
    first = 2.0 * B * 149 * 149 * sl[0][0][2] * 27
    f = 3.0 * sum(fwd) - first
    out = {"metric": METRIC, "value": B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": ("REDUCED " if args.small else "") + f"Inception-shaped 4-stage pipeline on 3x299x299 images (width x{width}, "
                      f"{classes} classes), bf16 w/ fp32 accum, minibatch {B}, NOAM 4, four streams; step = one minibatch "
                      "through all stages (drained pipeline of `steps` minibatches)", "minibatch": B,
                      "stage_forward_gflop": [round(v / 1e9, 1) for v in fwd],
                      "stage_params": [gen.param_count(l) for l in sl]},
           "step_gflop": f / 1e9, "mfma_util_pct": 100.0 * f / (ms * 1e-3) / MFMA_BF16_PEAK,
           "roofline": {"bound": "mfma", "kernel": "whole step", "achieved": f / (ms * 1e-3) / 1e12,
                        "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": f / (ms * 1e-3) / MFMA_BF16_PEAK,
                        "traffic": None},
           "final_loss": float(losses[-1].item())}
    for h in hs:
        pd.pd_stage_destroy(h)
    return out


def bench_mlp4(args, pd, gen, torch, np, dev):
    """Config 1, the parity configuration: 4-stage MLP in fp32 (Linear 256->256 + ReLU per stage, the last stage
    Linear 256->10 + loss), minibatch 32, NOAM 4, 64 minibatches through pd_pipeline_run on four streams.  The
    work per op is tiny (12.6 MFLOP per hidden stage and step): this measures launch and event latency, so the
    result is reported as microseconds per op, not against a roofline."""
    B, M = 32, 64
    reps = max(1, min(args.steps, 50))
    sl = gen.config1_mlp(256, 10, 4)
    S = len(sl)
    seed = gen.BASE_SEED + 0
    streams = [torch.cuda.Stream(device=dev) for _ in range(S)]
    bstreams = [None if _single_stream(args, False) else torch.cuda.Stream(device=dev) for _ in range(S)]
    hs, arenas = [], []
    for s in range(S):
        cfg = pd.make_config(sl[s], stage_index=s, num_stages=S, noam=4, minibatch=B, precision=pd.PD_F32, lr=0.01,
                             momentum=0.9, stream=streams[s].cuda_stream,
                             stream_backward=bstreams[s].cuda_stream if bstreams[s] is not None else 0)
        nbytes = pd.pd_stage_query_bytes(cfg)
        arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        hs.append(pd.pd_stage_create(cfg, (arena.data_ptr() + 255) // 256 * 256, nbytes)); arenas.append(arena)
        pd.pd_stage_set_params(hs[-1], gen.init_params(seed, f"s{s}", sl[s]))
    xs = torch.from_numpy(gen.normal(seed, "X", (M, B, 256))).to(dev)
    ls = torch.from_numpy(gen.labels(seed, "Y", (M, B), 10)).to(dev)
    losses = torch.zeros(M, dtype=torch.float32, device=dev)
    for _ in range(max(1, min(args.warmup, 3))):
        pd.pd_pipeline_run(hs, M, xs.data_ptr(), ls.data_ptr(), losses.data_ptr())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        pd.pd_pipeline_run(hs, M, xs.data_ptr(), ls.data_ptr(), losses.data_ptr())
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / (reps * M)   # per minibatch through all four stages
    ops = 3 * S                                          # F, B, U on each stage
    out = {"metric": METRIC, "value": B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": reps * M, "warmup": M,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": "4-stage MLP (Linear 256->256 + ReLU x3, Linear 256->10 + loss), fp32, minibatch 32, NOAM 4, "
                      "64 minibatches per pipeline run on four streams; step = one minibatch through all stages",
                      "minibatch": B, "minibatches_per_run": M},
           "us_per_op": 1e3 * ms / ops, "ops_per_minibatch": ops,
           "roofline": {"bound": "latency", "kernel": "none dominates: 12 ops of a few microseconds per minibatch",
                        "achieved": None, "peak": None, "unit": None, "frac": None, "traffic": None},
           "final_loss": float(losses[-1].item())}
    for h in hs:
        pd.pd_stage_destroy(h)
    return out


def bench_gemm_sweep(args, pd, gen, torch, np, dev):
    """The stage's three contractions on their own at the VGG16 classifier's K, N with the row count M swept from
    the configured minibatch (64, HBM-bound) into the compute-bound regime: achieved TFLOP/s and % of the bf16
    MFMA peak per kernel.  One JSON line; `value` is the best forward figure."""
    s = torch.cuda.current_stream().cuda_stream
    shapes = [(4096, 4096)] if args.small else [(4096, 25088), (4096, 4096)]
    rows_list = [64, 256, 1024] if args.small else [64, 128, 256, 512, 1024, 2048, 4096, 8192]
    if getattr(args, "rows", None):
        rows_list = list(args.rows)

    def timeit(fn, n=11):
        # three untimed launches first: the chip's clock under matrix load settles over milliseconds, and the figure
        # of a short burst depends on what ran before it (44-56 % of peak for one and the same launch)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record(); fn(); b.record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in evs)[n // 2] * 1e-3

    table = []
    for (N, K) in shapes:
        w = (torch.randn(N, K, device=dev) * 0.02).to(torch.bfloat16)
        b = torch.zeros(N, device=dev, dtype=torch.bfloat16)
        mw = torch.randn(N, K, device=dev) * 0.02; mm = torch.zeros(N, K, device=dev)
        mb_ = torch.zeros(N, device=dev); mmb = torch.zeros(N, device=dev)
        rw = torch.empty(N, K, device=dev, dtype=torch.bfloat16); rb = torch.empty(N, device=dev, dtype=torch.bfloat16)
        wt = torch.empty(N * K, device=dev, dtype=torch.bfloat16)
        for M in rows_list:
            x = torch.randn(M, K, device=dev).to(torch.bfloat16); dz = (torch.randn(M, N, device=dev) * 0.01).to(torch.bfloat16)
            y = torch.empty(M, N, device=dev, dtype=torch.bfloat16); dx = torch.empty(M, K, device=dev, dtype=torch.bfloat16)
            wsb = pd.pd_gemm_workspace_bytes(M, N, K)
            ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
            geom = (M, 1, 1, K, N, 1, 1, 1, 0, 0)
            part = torch.empty(pd.pd_conv_wgrad_splits(geom) * (N * K + N), dtype=torch.float32, device=dev)
            fl = 2.0 * M * N * K
            tf = timeit(lambda: pd.pd_linear_fwd_bf16(s, x.data_ptr(), w.data_ptr(), b.data_ptr(), y.data_ptr(), M, N, K, True, ws.data_ptr(), wsb))
            td = timeit(lambda: pd.pd_linear_dgrad_bf16(s, dz.data_ptr(), w.data_ptr(), 0, dx.data_ptr(), M, N, K, ws.data_ptr(), wsb))
            if M >= 512:
                tw = timeit(lambda: pd.pd_conv_wgrad_update_bf16(s, dz.data_ptr(), x.data_ptr(), part.data_ptr(), mw.data_ptr(), mm.data_ptr(), rw.data_ptr(), mb_.data_ptr(), mmb.data_ptr(), rb.data_ptr(), geom, 0.01, 0.9))
            else:
                tw = timeit(lambda: pd.pd_linear_wgrad_update_bf16(s, dz.data_ptr(), x.data_ptr(), mw.data_ptr(), mm.data_ptr(), rw.data_ptr(), mb_.data_ptr(), mmb.data_ptr(), rb.data_ptr(), M, N, K, 0.01, 0.9))
            row = {"N": N, "K": K, "M": M}
            for name, t in (("fwd", tf), ("dgrad", td), ("wgrad_update", tw)):
                row[name + "_us"] = round(t * 1e6, 1)
                row[name + "_tflops"] = round(fl / t / 1e12, 1)
                row[name + "_mfma_pct"] = round(100 * fl / t / MFMA_BF16_PEAK, 2)
            if M >= 1024 and not getattr(args, "no_library_reference", False):
                # Context, not a target and not part of the product: the vendor library's plain products (torch.mm ->
                # hipBLASLt) on the same operands, and both forward products on all-zero operands -- the chip lowers
                # its clock under matrix load, and by how much depends on the data the multipliers see.
                row["lib_fwd_us"] = round(timeit(lambda: torch.mm(x, w.t())) * 1e6, 1)
                row["lib_dgrad_us"] = round(timeit(lambda: torch.mm(dz, w)) * 1e6, 1)
                row["lib_wgrad_us"] = round(timeit(lambda: torch.mm(dz.t(), x)) * 1e6, 1)
                for k in ("fwd", "dgrad", "wgrad"):
                    row["lib_" + k + "_mfma_pct"] = round(100 * fl / (row["lib_" + k + "_us"] * 1e-6) / MFMA_BF16_PEAK, 2)
                if M >= 8192:
                    xz = torch.zeros_like(x); wz = torch.zeros_like(w)
                    tz = timeit(lambda: pd.pd_linear_fwd_bf16(s, xz.data_ptr(), wz.data_ptr(), b.data_ptr(), y.data_ptr(), M, N, K, True, ws.data_ptr(), wsb))
                    tlz = timeit(lambda: torch.mm(xz, wz.t()))
                    row["fwd_zero_operands_mfma_pct"] = round(100 * fl / tz / MFMA_BF16_PEAK, 2)
                    row["lib_fwd_zero_operands_mfma_pct"] = round(100 * fl / tlz / MFMA_BF16_PEAK, 2)
                    del xz, wz
            table.append(row)
            print("# " + json.dumps(row), file=sys.stderr, flush=True)
            del x, dz, y, dx, ws, part
        del w, mw, mm, rw, wt
    best = max(r["fwd_tflops"] for r in table)
    out = {"metric": METRIC, "value": best, "unit": "TFLOP/s (best forward GEMM of the sweep)", "n_gpus": 1, "steps": 11,
           "warmup": 3, "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "row-count sweep of the Linear kernels at the VGG16 classifier's K, N"},
           "roofline": {"bound": "mfma", "achieved": best, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                        "frac": best * 1e12 / MFMA_BF16_PEAK, "traffic": None}, "sweep": table}
    return out


def bench_partition(args, pd, gen, torch, np, dev):
    """The step before the pipeline: profile every layer of VGG16 (minibatch 64, the build's own kernels), then run
    the partitioner for several worker counts and link bandwidths.  Prints the profile and the chosen stages."""
    B, K, W = args.minibatch, min(args.steps, 20), min(args.warmup, 3)
    hw = (64, 64) if args.small else (224, 224)
    layers = gen.vgg16_full()
    if args.small:
        layers = [("linear", 2 * 2 * 512, L[2], L[3]) if (L[0] == "linear" and L[1] == 25088) else L for L in layers]
    seed = gen.BASE_SEED + 6
    params = gen.init_params(seed, "vgg16", layers)
    stream = torch.cuda.Stream(device=dev)
    cfg = pd.make_config(layers, in_flight_override=1, minibatch=B, precision=pd.PD_BF16_F32ACC, lr=0.01,
                         momentum=0.9, stream=stream.cuda_stream, in_hw=hw)
    nbytes = pd.pd_stage_query_bytes(cfg)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    h = pd.pd_stage_create(cfg, (arena.data_ptr() + 255) // 256 * 256, nbytes)
    pd.pd_stage_set_params(h, params)
    x = torch.from_numpy(gen.normal(seed, "x", (B, hw[0], hw[1], 3))).to(dev).to(torch.bfloat16)
    lab = torch.from_numpy(gen.labels(seed, "y", (B,), 1000)).to(dev)
    mb = 0

    def step():
        nonlocal mb
        pd.pd_forward(h, mb, x.data_ptr(), lab.data_ptr(), 0, 0)
        pd.pd_backward(h, mb, 0, 0)
        pd.pd_update(h)
        mb += 1

    for _ in range(W):
        step()
    torch.cuda.synchronize()
    pd.pd_stage_profile(h, True)
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / K
    prof = pd.pd_stage_profile_read(h)
    pd.pd_stage_profile(h, False)
    pd.pd_stage_destroy(h)
    compute = [L for L in layers if L[0] != "softmax_xent"]
    T = [u["fwd_ms"] + u["bwd_ms"] + u["upd_ms"] for u in prof]
    a = [u["act_bytes"] for u in prof]
    w = [u["param_bytes"] for u in prof]
    links = {"10 Gbit/s Ethernet": 1.25e6, "25 Gbit/s Ethernet": 3.125e6, "one xGMI link (153 GB/s)": 1.53e8}  # bytes per ms
    parts = []
    for name, bw in links.items():
        for M in (4, 8, 16):
            best, stages, noam = pd.pd_partition(T, a, w, M, bw)
            parts.append({"link": name, "workers": M, "slowest_stage_ms": best, "noam": noam,
                          "config": "-".join(str(r) for _, _, r in stages),
                          "stages": [{"layers": [f, l], "replicas": r} for f, l, r in stages],
                          "samples_per_s": B / (best * 1e-3)})
    out = {"metric": "layer profile + partition (Section 3.2)", "unit": "ms", "n_gpus": 1, "steps": K, "warmup": W,
           "value": sum(T), "ms_per_step": ms, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": ("REDUCED " if args.small else "") + f"VGG16 (13 conv, 5 pool, 3 Linear) on 3x{hw[0]}x{hw[1]} "
                      f"images, minibatch {B}, one stage of depth 1 with the layer profiler on"},
           "profile": [{"layer": compute[u["first_layer"]][0] + (f" {compute[u['first_layer']][1]}->{compute[u['first_layer']][2]}"
                                                                 if compute[u["first_layer"]][0] != "maxpool2d" else ""),
                        "T_ms": round(t, 4), "fwd_ms": round(u["fwd_ms"], 4), "bwd_ms": round(u["bwd_ms"], 4),
                        "upd_ms": round(u["upd_ms"], 4), "a_bytes": u["act_bytes"], "w_bytes": u["param_bytes"]}
                       for u, t in zip(prof, T)],
           "partitions": parts}
    return out


def _single_stream(args, default_on):
    """Whether the workload runs WITHOUT backward streams."""
    return args.backward_streams == "off" or (args.backward_streams == "auto" and not default_on)


def bench_vgg16_fc(args, pd, gen, torch, np, dev):
    """The metric's workload (config 2): the VGG16 classifier as one stage, bf16 with fp32 accumulation, minibatch
    64, weight-version ring depth 4.  Step = B(k) U(k) F(k + depth).

    Inputs are NOT recycled: every minibatch of the run is a distinct synthetic one (64 x 25088 N(0,1) values and 64
    labels), resident in HBM before the timed region starts.  The stage is configured as the second stage of a two-
    stage pipeline, as the classifier is in the paper's VGG16 configurations, so its input ring has depth + 1 slots;
    a producer stream plays the upstream stage and copies minibatch k + depth + 1 into the free slot while step k runs
    (event-ordered after the update that last read that slot), exactly the hand-off pd_pipeline_run performs between
    stages.  pd_forward then reads its input in place.

    Timing: `--repetitions` (5) repetitions of `--steps` steps each, every repetition bracketed by a device
    synchronisation on both sides (wall clock) and by HIP events recorded on the stage's stream; ms_per_step is the
    MEDIAN repetition's wall-clock time per step, the spread of all repetitions is reported beside it.  Events recorded
    between the ops give the time of each op and of the dominant kernel's launch (pd_update is exactly one launch)."""
    B, depth, K, W, reps = args.minibatch, args.depth, args.steps, args.warmup, args.repetitions
    single = _single_stream(args, True)
    layers = gen.config2_vgg_fc(1024, 512, 104) if args.small else gen.config2_vgg_fc()
    n_in, classes = layers[0][1], layers[-1][1]
    seed = gen.BASE_SEED + 1
    params = gen.init_params(seed, "vgg_fc", layers)
    P = int(params.size)
    stream = torch.cuda.Stream(device=dev)
    producer = torch.cuda.Stream(device=dev)
    # the backward passes on a stream of their own: B(k + 1) then runs next to F(k + depth) instead of behind it
    stream_b = stream if single else torch.cuda.Stream(device=dev)
    cfg = pd.make_config(layers, stage_index=1, num_stages=2, noam=2, in_flight_override=depth, minibatch=B,
                         precision=pd.PD_BF16_F32ACC, lr=args.lr, momentum=0.9, stream=stream.cuda_stream,
                         stream_backward=0 if single else stream_b.cuda_stream)
    nbytes = pd.pd_stage_query_bytes(cfg)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    base = (arena.data_ptr() + 255) // 256 * 256
    h = pd.pd_stage_create(cfg, base, nbytes)
    pd.pd_stage_set_params(h, params)
    in_ring = pd.pd_stage_depth(h)[1]
    assert in_ring == depth + 1
    n_steps = max(W, in_ring) + reps * K
    n_mb = n_steps + depth                          # distinct minibatches of the whole run
    x_all = torch.from_numpy(gen.normal_bulk(seed, "x", (n_mb, B, n_in))).to(dev).to(torch.bfloat16)
    lab_all = torch.from_numpy(gen.labels(seed, "y", (n_mb, B), classes)).to(dev)
    dx = torch.empty((B, n_in), dtype=torch.bfloat16, device=dev)
    losses = torch.zeros(n_mb, dtype=torch.float32, device=dev)
    off0 = pd.pd_stage_input_slot(h, 0) - arena.data_ptr()
    slot_view = [arena[off0 + j * B * n_in * 2: off0 + (j + 1) * B * n_in * 2].view(torch.bfloat16).view(B, n_in)
                 for j in range(in_ring)]          # (slot of minibatch i = i mod in_ring, contiguous from slot 0)
    assert all(pd.pd_stage_input_slot(h, j) == slot_view[j].data_ptr() for j in range(in_ring))
    filled = [torch.cuda.Event() for _ in range(in_ring)]      # producer: slot j holds its next minibatch
    freed = [torch.cuda.Event() for _ in range(in_ring)]       # stage: the update that last read slot j is done
    torch.cuda.synchronize()

    def produce(i, wait_free):
        """The upstream stage's part: minibatch i goes into its input slot on the producer stream."""
        j = i % in_ring
        with torch.cuda.stream(producer):
            if wait_free:
                producer.wait_event(freed[j])
            slot_view[j].copy_(x_all[i], non_blocking=True)
            filled[j].record(producer)

    def fwd(i):
        stream.wait_event(filled[i % in_ring])
        pd.pd_forward(h, i, pd.pd_stage_input_slot(h, i), lab_all[i].data_ptr(), 0, losses[i:].data_ptr())

    def step(k, ev=None):
        # B(k), U(k), F(k + depth); meanwhile the producer refills the slot that U(k) frees with minibatch k + in_ring.
        # With a backward stream, B(k) starts when U(k - 2) is done (the gradient buffers exist twice) and runs next to
        # U(k - 1) and F(k - 1 + depth), enqueued by the previous step.  The events bracket each op on the stream it runs
        # on, behind the same dependencies the library inserts itself (B after the update before the last, U after B),
        # so that no waiting is counted as work.
        if ev is not None:
            if k > 1:
                stream_b.wait_event(freed[(k - 2) % in_ring])
            ev[0].record(stream_b)
        pd.pd_backward(h, k, 0, dx.data_ptr())
        if ev is not None:
            ev[1].record(stream_b)
            stream.wait_event(ev[1])
            ev[2].record(stream)
        pd.pd_update(h)
        if ev is not None:
            ev[3].record(stream)
        freed[k % in_ring].record(stream)
        if k + in_ring < n_mb:
            produce(k + in_ring, True)
        fwd(k + depth)
        if ev is not None:
            ev[4].record(stream)

    for i in range(in_ring):
        produce(i, False)
    for i in range(depth):
        fwd(i)
    k = 0
    for _ in range(max(W, in_ring)):
        step(k)
        k += 1
    rep_wall, rep_evt, ops = [], [], {"B": [], "U": [], "F": []}
    for _ in range(reps):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for j in range(K):
            step(k, evs[j])
            k += 1
        torch.cuda.synchronize()
        rep_wall.append((time.perf_counter() - t0) * 1e3 / K)
        rep_evt.append(evs[0][4].elapsed_time(evs[-1][4]) / (K - 1) if K > 1 else float("nan"))  # end of F to end of F
        for e in evs:
            ops["B"].append(e[0].elapsed_time(e[1])); ops["U"].append(e[2].elapsed_time(e[3])); ops["F"].append(e[3].elapsed_time(e[4]))
    ms_per_step = float(np.median(rep_wall))
    upd_ms_avg = float(np.mean(ops["U"]))
    lh = losses.cpu().numpy()
    first_loss, final_loss = float(lh[0]), float(lh[k + depth - 1])
    # sanity of the timed trajectory: fresh minibatches with random labels cannot be memorised, so the loss stays near
    # log(classes); a loss kernel that wrote nothing, dead units or a diverged run would all show here
    assert np.all(np.isfinite(lh[:k + depth])) and final_loss > 0.1 and float(lh[:k + depth].min()) > 0.1, (first_loss, final_loss)

    lin = [L for L in layers if L[0] == "linear"]
    flops = 6.0 * B * sum(L[1] * L[2] for L in lin)
    value = B / (ms_per_step * 1e-3)
    survey, stored = SURVEY_UPDATE_BYTES_PER_PARAM, STORED_UPDATE_BYTES_PER_PARAM
    ach = survey * P / (upd_ms_avg * 1e-3) / 1e9
    ach_stored = stored * P / (upd_ms_avg * 1e-3) / 1e9
    out = {
        "metric": METRIC, "value": value, "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": max(W, in_ring),
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": ("REDUCED " if args.small else "") +
                   f"VGG16-FC-shaped stage: Linear {n_in}-{layers[0][2]}-{layers[1][2]}-{classes} + ReLU + "
                   f"softmax-xent, bf16 w/ fp32 accum, minibatch {B}, weight-version ring depth {depth}, "
                   f"step = B(k) U(k) F(k+depth); {n_mb} distinct minibatches resident in HBM, handed into the stage's "
                   "input ring by a producer stream as an upstream stage would",
                   "params": P, "minibatch": B, "ring_depth": depth, "lr": args.lr},
        "repetitions": reps,
        "ms_per_step_repetitions_wall": [round(v, 5) for v in rep_wall],
        "backward_stream": not single,
        "ms_per_step_repetitions_hip_events": [round(v, 5) for v in rep_evt],
        "ms_per_step_spread": {"min": min(rep_wall), "median": ms_per_step, "max": max(rep_wall)},
        "per_op_ms": {name: {"mean": float(np.mean(v)), "median": float(np.median(v)), "min": float(np.min(v)),
                             "max": float(np.max(v))} for name, v in ops.items()},
        "mfma_util_pct": 100.0 * flops / (ms_per_step * 1e-3) / MFMA_BF16_PEAK,
        "step_gflop": flops / 1e9,
        # the whole step against its HBM bound: 22 B/param with an fp32 master array (2 forward + 2 input gradient +
        # 18 update), 20 B/param as stored here
        "step_roofline": {"bound": "hbm", "bytes_per_param_survey": 22, "bytes_per_param_stored": 20,
                          "frac_survey": 22.0 * P / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "frac_stored": 20.0 * P / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "kernel": "wgrad_update_kernel (dW = dZ^T X fused with momentum-SGD into the ring)",
                     "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "bytes_per_param_survey": survey, "bytes_per_param_stored": stored,
                     "achieved_stored": ach_stored, "frac_stored": ach_stored / HBM_PEAK_GBS,
                     "traffic": (MEASURED_TRAFFIC_BYTES if (not args.small and B == 64) else None),
                     "traffic_source": "profiles/wgrad_update_vgg16fc_mb64.txt", "launches_per_step": 1,
                     "avg_launch_ms": upd_ms_avg, "launch_ms_median": float(np.median(ops["U"])),
                     "bytes_per_launch": survey * P, "bytes_per_launch_stored": stored * P},
        "first_loss": first_loss, "final_loss": final_loss,
        "loss_range": [float(lh[:k + depth].min()), float(lh[:k + depth].max())],
    }
    pd.pd_stage_destroy(h)
    del arena, slot_view, x_all
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        xs = list(gen.normal_bulk(seed, "cx", (depth + 1, B, n_in)))
        labs = list(gen.labels(seed, "cy", (depth + 1, B), classes))
        out["cpu_baseline"] = cpu_baseline(layers, params, xs, labs, depth, lr=args.lr)
    return out


def _oracle_steps(stage_layers, params, xs, labs, dys, noam, budget_s, what, minibatch):
    """The oracle's pipeline on a bounded sample: whole minibatches through all stages until the budget is used."""
    import numpy as np
    from oracle.pipeline import run_pipeline
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    n, t0 = 0, time.time()
    while n == 0 or time.time() - t0 < budget_s:
        run_pipeline(stage_layers, params, [x.astype(np.float64) for x in xs], labs, noam, mode="bf16", out_grads=dys)
        n += len(xs)
    dt = time.time() - t0
    return {"value": n * minibatch / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{what}: {n} minibatches of {minibatch} in {dt:.1f} s, fp64 numpy"}


def run_extras(args, pd, gen, torch, np, dev):
    """The secondary workloads, each timed briefly in the same run (configs 1, 3, 4, 5 and the compute-bound end of
    the row-count sweep), each with its own roofline object and the oracle timed beside it at a reduced size."""
    import copy
    extras = {}

    def sub(**kw):
        a = copy.copy(args)
        for k_, v in kw.items():
            setattr(a, k_, v)
        return a

    def note(name, t0):
        print(f"# extra workload {name}: {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    t0 = time.time()
    e = bench_conv(sub(steps=10, warmup=3), pd, gen, torch, np, dev)
    if not args.no_cpu_baseline:
        layers = gen.config3_vgg_conv()
        p = gen.init_params(gen.BASE_SEED + 2, "vgg_conv", layers)
        xs = [gen.normal(gen.BASE_SEED + 2, "cx", (2, 56, 56, 3))]
        dys = [gen.normal(gen.BASE_SEED + 2, "cdy", (2, 7, 7, 256)) * 0.01]
        e["cpu_baseline"] = _oracle_steps([layers], [p], xs, None, dys, 1, 3.0, "REDUCED: the same stage on 56 x 56 images, minibatch 2", 2)
    extras["vgg16_conv"] = e
    torch.cuda.empty_cache(); note("vgg16_conv", t0)

    t0 = time.time()
    e = bench_s2vt(sub(steps=8, warmup=2), pd, gen, torch, np, dev)
    if not args.no_cpu_baseline:
        sl = gen.config4_s2vt(256, 128, 1000, 8)
        ps = [gen.init_params(gen.BASE_SEED + 3, f"c{s_}", ly) for s_, ly in enumerate(sl)]
        xs = [gen.normal(gen.BASE_SEED + 3, "cx", (8, 16, 256))]
        labs = [gen.labels(gen.BASE_SEED + 3, "cy", (8, 16), 1000)]
        e["cpu_baseline"] = _oracle_steps(sl, ps, xs, labs, None, 2, 3.0, "REDUCED: LSTM 256->128 | LSTM 128->128 + vocabulary 1000, seq 8, minibatch 16", 16)
    extras["s2vt"] = e
    torch.cuda.empty_cache(); note("s2vt", t0)

    t0 = time.time()
    e = bench_inception(sub(steps=6, warmup=2), pd, gen, torch, np, dev)
    if not args.no_cpu_baseline:
        sl, sizes = gen.config5_inception(16, 0.25)
        ps = [gen.init_params(gen.BASE_SEED + 4, f"c{s_}", ly) for s_, ly in enumerate(sl)]
        xs = [gen.normal(gen.BASE_SEED + 4, "cx", (1, 299, 299, 3))]
        labs = [gen.labels(gen.BASE_SEED + 4, "cy", (1,), 16)]
        e["cpu_baseline"] = _oracle_steps(sl, ps, xs, labs, None, 4, 3.0, "REDUCED: a quarter of the channel counts, 16 classes, minibatch 1, 299 x 299 images", 1)
    extras["inception"] = e
    torch.cuda.empty_cache(); note("inception", t0)

    t0 = time.time()
    e = bench_mlp4(sub(steps=10, warmup=2), pd, gen, torch, np, dev)
    if not args.no_cpu_baseline:
        sl = gen.config1_mlp(256, 10, 4)
        ps = [gen.init_params(gen.BASE_SEED, f"s{s_}", ly) for s_, ly in enumerate(sl)]
        xs = list(gen.normal(gen.BASE_SEED, "X", (64, 32, 256)))
        labs = list(gen.labels(gen.BASE_SEED, "Y", (64, 32), 10))
        import numpy as _np
        from oracle.pipeline import run_pipeline
        t1 = time.time()
        run_pipeline(sl, ps, [x.astype(_np.float64) for x in xs], labs, 4, mode="f32")
        dt = time.time() - t1
        e["cpu_baseline"] = {"value": 64 * 32 / dt, "unit": "samples/s", "cores": os.cpu_count() or 1, "kind": "oracle",
                             "sample": f"the same configuration in full: 64 minibatches of 32 in {dt:.2f} s, fp64 numpy"}
    extras["mlp4"] = e
    torch.cuda.empty_cache(); note("mlp4", t0)

    t0 = time.time()
    e = bench_gemm_sweep(sub(rows=[8192]), pd, gen, torch, np, dev)
    extras["gemm_sweep_peak_rows"] = e
    torch.cuda.empty_cache(); note("gemm_sweep", t0)
    return extras


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--minibatch", type=int, default=64)
    ap.add_argument("--depth", type=int, default=4)
    ap.add_argument("--repetitions", type=int, default=5, help="default workload: repetitions of --steps steps (median reported)")
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--backward-streams", choices=["auto", "on", "off"], default="auto",
                    help="run every stage's backward passes on a stream of their own (pd_stage_config.stream_backward); auto: "
                         "on for the VGG16 classifier stage (0.531 -> 0.500 ms per step), the VGG16 convolution stage (4.76 -> 4.55 ms) "
                         "and the Inception-shaped pipeline (11.35 -> 10.43 ms), off for the LSTM pipeline (no gain) and the fp32 MLP "
                         "pipeline (0.12 -> 0.18 ms: every extra event hop costs more than its tiny kernels)")
    ap.add_argument("--recurrence", choices=["per-step", "multi-step"], default="multi-step",
                    help="LSTM layers: all time steps of a pass in one launch (default) or one launch per time step "
                         "(bit-identical results; a single LSTM stage 1.29 vs 1.65 ms, the S2VT pipeline 4.15 ms either way)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="default workload only: skip the secondary workloads appended under `extra`")
    ap.add_argument("--rows", type=int, nargs="+", default=None, help="gemm_sweep: the row counts to run (default: 64 ... 8192)")
    ap.add_argument("--no-library-reference", action="store_true",
                    help="gemm_sweep: leave out the vendor library's timings of the same products (context only)")
    ap.add_argument("--small", action="store_true", help="reduced widths (debugging only; result is not the metric)")
    ap.add_argument("--workload", default="vgg16_fc", choices=["vgg16_fc", "vgg16_conv", "s2vt", "inception", "gemm_sweep", "partition", "mlp4", "replicated", "vgg16_pipeline"],
                    help="vgg16_fc (default, the metric's workload); secondary: vgg16_conv (the conv stage), "
                         "s2vt (the two LSTM stages as a 2-stream pipeline), inception (four stages of branched "
                         "convolution blocks as a 4-stream pipeline), gemm_sweep (the Linear kernels over row counts), "
                         "partition (layer profile of all of VGG16 on the device, then the partitioner), mlp4 (the 4-stage fp32 MLP, "
                         "a launch-latency case), replicated (the VGG16 conv stage as --replicas replicas on as many streams), vgg16_pipeline (all of VGG16 as "
                         "an r-1 pipeline: replicated conv stage + classifier stage)")
    ap.add_argument("--replicas", type=int, default=2, help="workload replicated: replicas of the stage (2..8)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs all pipeline stages on ONE GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1806_03377_amd as pd
    pd.pd_set_recurrence_kernel(1 if args.recurrence == "multi-step" else 0, 0, 0)
    import pd_inputs as gen

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible (the HIP path has no CPU fallback)", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    B, depth, K, W = args.minibatch, args.depth, args.steps, args.warmup
    if args.workload == "vgg16_conv":
        return print(json.dumps(bench_conv(args, pd, gen, torch, np, dev)))
    if args.workload == "s2vt":
        return print(json.dumps(bench_s2vt(args, pd, gen, torch, np, dev)))
    if args.workload == "inception":
        return print(json.dumps(bench_inception(args, pd, gen, torch, np, dev)))
    if args.workload == "gemm_sweep":
        return print(json.dumps(bench_gemm_sweep(args, pd, gen, torch, np, dev)))
    if args.workload == "partition":
        return print(json.dumps(bench_partition(args, pd, gen, torch, np, dev)))
    if args.workload == "mlp4":
        return print(json.dumps(bench_mlp4(args, pd, gen, torch, np, dev)))
    if args.workload == "replicated":
        return print(json.dumps(bench_replicated(args, pd, gen, torch, np, dev)))
    if args.workload == "vgg16_pipeline":
        return print(json.dumps(bench_vgg16_pipeline(args, pd, gen, torch, np, dev)))
    out = bench_vgg16_fc(args, pd, gen, torch, np, dev)
    if not args.no_extra and not args.small:
        out["extra"] = run_extras(args, pd, gen, torch, np, dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
