"""Helpers for the GPU tests: device buffers via torch, stage creation through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_1806_03377_amd as pd


def dev():
    return torch.device("cuda:0")


def to_dev(a: np.ndarray, bf16: bool) -> torch.Tensor:
    """Host array -> device tensor in the stage's element type (bf16 = round-to-nearest-even)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev())
    return t.to(torch.bfloat16).contiguous() if bf16 else t.contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def labels_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev())


def empty_act(rows: int, cols: int, bf16: bool) -> torch.Tensor:
    return torch.empty((rows, cols), dtype=torch.bfloat16 if bf16 else torch.float32, device=dev())


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Max-norm relative error of a tensor: max|got-ref| / max|ref|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


class GpuStage:
    """One stage created through pd_stage_create on an arena owned by a torch tensor."""

    def __init__(self, layers, params, *, minibatch, precision, stage_index=0, num_stages=1, noam=1,
                 in_flight_override=0, lr=0.01, momentum=0.9, stream=None, in_hw=None, vertical_sync=False,
                 optimizer=0, eps=0.0, replicas=0, stream_backward=None):
        self.bf16 = precision == pd.PD_BF16_F32ACC
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self.stream_backward = stream_backward    # a torch stream for the kernels of pd_backward, or None
        self.cfg = pd.make_config(layers, stage_index=stage_index, num_stages=num_stages, noam=noam,
                                  in_flight_override=in_flight_override, minibatch=minibatch, precision=precision,
                                  lr=lr, momentum=momentum, stream=self.stream.cuda_stream, in_hw=in_hw,
                                  vertical_sync=vertical_sync, optimizer=optimizer, eps=eps, replicas=replicas,
                                  stream_backward=stream_backward.cuda_stream if stream_backward is not None else 0)
        self.bytes = pd.pd_stage_query_bytes(self.cfg)
        self.arena = torch.empty(self.bytes + 256, dtype=torch.uint8, device=dev())
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self.h = pd.pd_stage_create(self.cfg, base, self.bytes)
        if params is not None:
            pd.pd_stage_set_params(self.h, params)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev())

    def close(self):
        if self.h:
            self.stream.synchronize()
            if self.stream_backward is not None:
                self.stream_backward.synchronize()
            pd.pd_stage_destroy(self.h)
            self.h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class GpuReplica:
    """A further replica of a replicated stage (pd_stage_create_replica): own arena and stream, shared parameters."""

    def __init__(self, primary: GpuStage, stream=None):
        self.bf16 = primary.bf16
        self.stream = stream if stream is not None else torch.cuda.Stream()
        self.bytes = pd.pd_stage_replica_query_bytes(primary.cfg)
        self.arena = torch.empty(self.bytes + 256, dtype=torch.uint8, device=dev())
        base = (self.arena.data_ptr() + 255) // 256 * 256
        torch.cuda.synchronize()
        self.h = pd.pd_stage_create_replica(primary.h, self.stream.cuda_stream, base, self.bytes)

    def close(self):
        if self.h:
            self.stream.synchronize()
            pd.pd_stage_destroy(self.h)
            self.h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class GpuReplicatedStage:
    """Primary + further replicas; `rep[q].h` are the handles in replica order."""

    def __init__(self, layers, params, replicas, *, same_stream=False, **kw):
        self.r = replicas
        first = GpuStage(layers, params, replicas=replicas, **kw)
        self.rep = [first] + [GpuReplica(first, first.stream if same_stream else None) for _ in range(replicas - 1)]
        self.h = first.h
        self.bf16 = first.bf16

    def handles(self):
        return [g.h for g in self.rep]

    def update(self):
        pd.pd_update_replicated(self.handles())

    def close(self):
        for g in reversed(self.rep):     # further replicas first
            g.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
