"""ctypes binding of libpd.so: same names as include/pd.h and include/pd_debug.h, argument marshalling only.

Device pointers are passed as integers (``tensor.data_ptr()``), streams as
``torch.cuda.Stream.cuda_stream``.  Every call raises ``PdError`` on a non-zero status.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence, Tuple

import numpy as np
import torch  # noqa: F401  -- must come first: libpd.so then binds to the HIP runtime torch has already loaded
                #           (same soname), so both share one runtime, one context and the same streams

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: build it first (python -m paper_1806_03377_amd.build); "
                      "there is no fallback path")
_lib = C.CDLL(LIB_PATH)

PD_OK, PD_EINVAL, PD_ESTATE, PD_ENOMEM, PD_EHIP = 0, -1, -2, -3, -4
PD_F32, PD_BF16_F32ACC = 0, 1
PD_OP_F, PD_OP_B, PD_OP_U = 0, 1, 2
PD_OPT_SGD_MOMENTUM, PD_OPT_RMSPROP = 0, 1
PD_LINEAR, PD_SOFTMAX_XENT, PD_CONV2D, PD_MAXPOOL2D, PD_LSTM = 0, 1, 2, 3, 4
PD_AVGPOOL2D, PD_CONCAT_BEGIN, PD_BRANCH, PD_CONCAT_END = 5, 6, 7, 8


class PdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pd status {status}: {message}")
        self.status = status


class pd_op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mb_id", C.c_int32), ("version", C.c_int32), ("slot", C.c_int32)]


class pd_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("p", C.c_int32 * 12)]


class pd_layer_profile(C.Structure):
    _fields_ = [("first_layer", C.c_int32), ("last_layer", C.c_int32), ("fwd_ms", C.c_double),
                ("bwd_ms", C.c_double), ("upd_ms", C.c_double), ("act_bytes", C.c_double),
                ("param_bytes", C.c_double)]


class pd_stage_assign(C.Structure):
    _fields_ = [("first_layer", C.c_int32), ("last_layer", C.c_int32), ("replicas", C.c_int32)]


class pd_stage_config(C.Structure):
    _fields_ = [("stage_index", C.c_int32), ("num_stages", C.c_int32), ("noam", C.c_int32),
                ("in_flight_override", C.c_int32), ("minibatch", C.c_int32), ("precision", C.c_int32),
                ("lr", C.c_float), ("momentum", C.c_float), ("n_layers", C.c_int32),
                ("layers", C.POINTER(pd_layer_desc)), ("stream", C.c_void_p), ("vertical_sync", C.c_int32),
                ("optimizer", C.c_int32), ("eps", C.c_float), ("replicas", C.c_int32), ("stream_backward", C.c_void_p)]


_vp, _sz, _i32, _f32 = C.c_void_p, C.c_size_t, C.c_int32, C.c_float
_SIGS = {
    "pd_schedule_1f1b": [_i32, _i32, _i32, _i32, C.POINTER(pd_op), _sz, C.POINTER(_sz)],
    "pd_schedule_1f1b_depth": [_i32, _i32, C.POINTER(pd_op), _sz, C.POINTER(_sz)],
    "pd_schedule_1f1b_vertical_sync": [_i32, _i32, _i32, _i32, C.POINTER(pd_op), _sz, C.POINTER(_sz)],
    "pd_stage_ring_depth": [_vp, C.POINTER(_i32)],
    "pd_forward_versioned": [_vp, _i32, _i32, _vp, _vp, _vp, _vp],
    "pd_stage_query_bytes": [C.POINTER(pd_stage_config), C.POINTER(_sz)],
    "pd_stage_create": [C.POINTER(pd_stage_config), _vp, _sz, C.POINTER(_vp)],
    "pd_stage_destroy": [_vp],
    "pd_replica_route": [_i32, _i32, C.POINTER(_i32), C.POINTER(_i32)],
    "pd_stage_replica_query_bytes": [C.POINTER(pd_stage_config), C.POINTER(_sz)],
    "pd_stage_create_replica": [_vp, _vp, _vp, _sz, C.POINTER(_vp)],
    "pd_update_replicated": [C.POINTER(_vp), _i32],
    "pd_stage_num_params": [_vp, C.POINTER(_sz)],
    "pd_stage_depth": [_vp, C.POINTER(_i32), C.POINTER(_i32)],
    "pd_stage_set_params": [_vp, _vp, _sz],
    "pd_stage_get_params": [_vp, _i32, _i32, _vp, _sz],
    "pd_stage_set_momentum": [_vp, _vp, _sz],
    "pd_stage_set_lr": [_vp, _f32],
    "pd_stage_get_momentum": [_vp, _vp, _sz],
    "pd_stage_overwrite_latest": [_vp, _vp, _vp, _sz],
    "pd_stage_version": [_vp, _i32, C.POINTER(_i32)],
    "pd_stage_check": [_vp],
    "pd_stage_trace": [_vp, C.POINTER(pd_op), _sz, C.POINTER(_sz)],
    "pd_stage_set_trace_limit": [_vp, _sz],
    "pd_stage_input_slot": [_vp, _i32, C.POINTER(_vp)],
    "pd_stage_grad_slot": [_vp, _i32, C.POINTER(_vp)],
    "pd_stage_debug_read": [_vp, _i32, _i32, _i32, _vp, _sz],
    "pd_stage_debug_write": [_vp, _i32, _i32, _i32, _vp, _sz],
    "pd_forward": [_vp, _i32, _vp, _vp, _vp, _vp],
    "pd_backward": [_vp, _i32, _vp, _vp],
    "pd_update": [_vp],
    "pd_pipeline_run": [C.POINTER(_vp), _i32, _i32, _vp, _vp, _vp],
    "pd_pipeline_run_replicated": [C.POINTER(_vp), C.POINTER(_i32), _i32, _i32, _vp, _vp, _vp],
    "pd_stage_checkpoint_save": [_vp, C.c_char_p],
    "pd_stage_checkpoint_load": [_vp, C.c_char_p],
    "pd_checkpoint_info": [C.c_char_p, C.POINTER(_sz), C.POINTER(_i32), C.POINTER(_i32)],
    "pd_stage_profile": [_vp, _i32],
    "pd_stage_profile_read": [_vp, C.POINTER(pd_layer_profile), _sz, C.POINTER(_sz)],
    "pd_partition": [_i32, _i32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_double,
                     C.POINTER(C.c_double), C.POINTER(pd_stage_assign), _sz, C.POINTER(_sz), C.POINTER(_i32)],
    "pd_linear_fwd_bf16": [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _sz],
    "pd_linear_fwd_bf16_static": [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32],
    "pd_linear_dgrad_bf16": [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _sz],
    "pd_linear_wgrad_update_bf16": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _f32, _f32],
    "pd_conv_wgrad_splits": [C.POINTER(_i32), C.POINTER(_i32)],
    "pd_conv_fwd_bf16": [_vp, _vp, _vp, _vp, _vp, C.POINTER(_i32), _i32],
    "pd_conv_dgrad_bf16": [_vp, _vp, _vp, _vp, _vp, _vp, C.POINTER(_i32)],
    "pd_conv_wgrad_update_bf16": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, C.POINTER(_i32), _f32, _f32],
    "pd_maxpool2x2_fwd_bf16": [_vp, _vp, _vp, _i32, _i32, _i32, _i32],
    "pd_maxpool2x2_bwd_bf16": [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32],
    "pd_maxpool2x2_fwd_route_bf16": [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32],
    "pd_maxpool2x2_bwd_route_bf16": [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32],
    "pd_pool2d_fwd_bf16": [_vp, _i32, _vp, _vp, C.POINTER(_i32)],
    "pd_pool2d_bwd_bf16": [_vp, _i32, _vp, _vp, _vp, _vp, C.POINTER(_i32), _i32],
    "pd_pool2d_fwd_route_bf16": [_vp, _vp, _vp, _vp, C.POINTER(_i32)],
    "pd_pool2d_bwd_route_bf16": [_vp, _vp, _vp, _vp, C.POINTER(_i32), _i32],
}
for _name, _args in _SIGS.items():
    _f = getattr(_lib, _name)
    _f.argtypes = _args
    _f.restype = C.c_int
_lib.pd_last_error.restype = C.c_char_p
_lib.pd_last_error.argtypes = []
_lib.pd_gemm_workspace_bytes.restype = _sz
_lib.pd_gemm_workspace_bytes.argtypes = [_i32, _i32, _i32]
_lib.pd_linear_fwd_bf16_static_max_bytes.restype = _sz
_lib.pd_linear_fwd_bf16_static_max_bytes.argtypes = []
_lib.pd_set_conv_halo.restype = C.c_int
_lib.pd_set_conv_halo.argtypes = [_i32]
_lib.pd_set_recurrence_kernel.restype = C.c_int
_lib.pd_set_recurrence_kernel.argtypes = [_i32, C.c_uint32, C.c_uint32]
_lib.pd_set_big_gemm_waves.restype = C.c_int
_lib.pd_set_big_gemm_waves.argtypes = [_i32]
_lib.pd_set_big_tile_threshold.restype = C.c_int
_lib.pd_set_big_tile_threshold.argtypes = [_i32]

EXPORTED = sorted(list(_SIGS) + ["pd_last_error", "pd_gemm_workspace_bytes", "pd_set_big_tile_threshold",
                                 "pd_linear_fwd_bf16_static_max_bytes", "pd_set_big_gemm_waves", "pd_set_conv_halo", "pd_set_recurrence_kernel"])


def pd_last_error() -> str:
    return _lib.pd_last_error().decode()


def _check(rc: int):
    if rc != PD_OK:
        raise PdError(rc, pd_last_error())


def _ops(arr, n) -> List[Tuple[int, int, int, int]]:
    return [(arr[i].kind, arr[i].mb_id, arr[i].version, arr[i].slot) for i in range(n)]


def pd_schedule_1f1b(num_stages: int, noam: int, num_minibatches: int, stage_index: int):
    cap = max(1, 3 * max(0, num_minibatches))
    arr = (pd_op * cap)()
    n = _sz(0)
    _check(_lib.pd_schedule_1f1b(num_stages, noam, num_minibatches, stage_index, arr, cap, C.byref(n)))
    return _ops(arr, n.value)


def pd_schedule_1f1b_vertical_sync(num_stages: int, noam: int, num_minibatches: int, stage_index: int):
    cap = max(1, 3 * max(0, num_minibatches))
    arr = (pd_op * cap)()
    n = _sz(0)
    _check(_lib.pd_schedule_1f1b_vertical_sync(num_stages, noam, num_minibatches, stage_index, arr, cap, C.byref(n)))
    return _ops(arr, n.value)


def pd_schedule_1f1b_depth(depth: int, num_minibatches: int):
    cap = max(1, 3 * max(0, num_minibatches))
    arr = (pd_op * cap)()
    n = _sz(0)
    _check(_lib.pd_schedule_1f1b_depth(depth, num_minibatches, arr, cap, C.byref(n)))
    return _ops(arr, n.value)


def layer_descs(layers: Sequence[tuple], in_hw=None):
    """Translate the neutral layer tuples of pd_inputs into pd_layer_desc records.

    ``in_hw`` = (height, width) of the stage's input images, needed when the stage has
    convolution or pooling layers (their descriptors carry the input size); a stage that starts with
    a pooling layer or a block whose branch starts with one also needs ``in_hw`` = (h, w, channels)."""
    recs = []
    state = {"hw": tuple(in_hw[:2]) if in_hw else None, "ch": (in_hw[2] if in_hw and len(in_hw) > 2 else None)}

    def emit(kind, *vals):
        recs.append((kind, [int(v) for v in vals]))

    def one(L):
        hw, ch = state["hw"], state["ch"]
        if L[0] == "linear":
            emit(PD_LINEAR, L[1], L[2], int(bool(L[3])))
        elif L[0] == "softmax_xent":
            emit(PD_SOFTMAX_XENT, L[1])
        elif L[0] == "conv2d":
            if hw is None:
                raise ValueError("in_hw is required for stages with convolutions")
            _, c_in, c_out, kh, kw, stride, ph, pw, relu = L
            emit(PD_CONV2D, c_in, c_out, kh, kw, stride, ph, pw, int(bool(relu)), hw[0], hw[1])
            state["hw"] = ((hw[0] + 2 * ph - kh) // stride + 1, (hw[1] + 2 * pw - kw) // stride + 1)
            state["ch"] = c_out
        elif L[0] == "maxpool2d":
            if hw is None or ch is None:
                raise ValueError("a pooling layer needs the input size and channel count (in_hw = (h, w, c))")
            emit(PD_MAXPOOL2D, L[1], L[2], ch, hw[0], hw[1])
            state["hw"] = ((hw[0] - L[1]) // L[2] + 1, (hw[1] - L[1]) // L[2] + 1)
        elif L[0] == "avgpool2d":
            if hw is None or ch is None:
                raise ValueError("a pooling layer needs the input size and channel count (in_hw = (h, w, c))")
            k, stride, pad = L[1], L[2], L[3]
            emit(PD_AVGPOOL2D, k, stride, pad, ch, hw[0], hw[1])
            state["hw"] = ((hw[0] + 2 * pad - k) // stride + 1, (hw[1] + 2 * pad - k) // stride + 1)
        elif L[0] == "concat":
            emit(PD_CONCAT_BEGIN)
            start = dict(state)
            total = 0
            for br in L[1]:
                emit(PD_BRANCH)
                state.update(start)
                for sub in br:
                    one(sub)
                total += state["ch"]
            emit(PD_CONCAT_END)
            state["ch"] = total
        elif L[0] == "lstm":
            emit(PD_LSTM, L[1], L[2], L[3])
        else:
            raise ValueError(f"layer kind {L[0]!r} is not supported by this build")

    for L in layers:
        one(L)
    arr = (pd_layer_desc * len(recs))()
    for i, (kind, vals) in enumerate(recs):
        arr[i].kind = kind
        for j, v in enumerate(vals):
            arr[i].p[j] = v
    return arr


def make_config(layers, *, stage_index=0, num_stages=1, noam=1, in_flight_override=0, minibatch=1,
                precision=PD_F32, lr=0.01, momentum=0.9, stream=0, in_hw=None, vertical_sync=False,
                optimizer=PD_OPT_SGD_MOMENTUM, eps=0.0, replicas=0, stream_backward=0):
    descs = layer_descs(layers, in_hw)
    cfg = pd_stage_config(stage_index, num_stages, noam, in_flight_override, minibatch, precision, lr, momentum,
                          len(descs), descs, stream, 1 if vertical_sync else 0, optimizer, eps, replicas,
                          stream_backward or None)
    cfg._keepalive = descs
    return cfg


def pd_stage_query_bytes(cfg) -> int:
    n = _sz(0)
    _check(_lib.pd_stage_query_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def pd_stage_create(cfg, device_arena: int, arena_bytes: int) -> int:
    h = _vp(0)
    _check(_lib.pd_stage_create(C.byref(cfg), device_arena, arena_bytes, C.byref(h)))
    return h.value


def pd_stage_destroy(stage: int):
    _check(_lib.pd_stage_destroy(stage))


def pd_replica_route(mb_id: int, n_replicas: int) -> Tuple[int, int]:
    """(replica, round) of a minibatch of a replicated stage."""
    q, k = _i32(0), _i32(0)
    _check(_lib.pd_replica_route(mb_id, n_replicas, C.byref(q), C.byref(k)))
    return q.value, k.value


def pd_stage_replica_query_bytes(cfg) -> int:
    n = _sz(0)
    _check(_lib.pd_stage_replica_query_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def pd_stage_create_replica(primary: int, stream: int, device_arena: int, arena_bytes: int) -> int:
    h = _vp(0)
    _check(_lib.pd_stage_create_replica(primary, stream, device_arena, arena_bytes, C.byref(h)))
    return h.value


def pd_update_replicated(replicas):
    arr = (_vp * len(replicas))(*replicas)
    _check(_lib.pd_update_replicated(arr, len(replicas)))


def pd_stage_num_params(stage: int) -> int:
    n = _sz(0)
    _check(_lib.pd_stage_num_params(stage, C.byref(n)))
    return n.value


def pd_stage_depth(stage: int) -> Tuple[int, int]:
    d, i = _i32(0), _i32(0)
    _check(_lib.pd_stage_depth(stage, C.byref(d), C.byref(i)))
    return d.value, i.value


def _host_f32(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def pd_stage_set_params(stage: int, params: np.ndarray):
    a = _host_f32(params)
    _check(_lib.pd_stage_set_params(stage, a.ctypes.data, a.size))


def pd_stage_get_params(stage: int, version: int = -1, ring_copy: bool = False) -> np.ndarray:
    out = np.empty(pd_stage_num_params(stage), dtype=np.float32)
    _check(_lib.pd_stage_get_params(stage, version, int(ring_copy), out.ctypes.data, out.size))
    return out


def pd_stage_set_momentum(stage: int, mom: np.ndarray):
    a = _host_f32(mom)
    _check(_lib.pd_stage_set_momentum(stage, a.ctypes.data, a.size))


def pd_stage_set_lr(stage: int, lr: float):
    _check(_lib.pd_stage_set_lr(stage, lr))


def pd_stage_get_momentum(stage: int) -> np.ndarray:
    out = np.empty(pd_stage_num_params(stage), dtype=np.float32)
    _check(_lib.pd_stage_get_momentum(stage, out.ctypes.data, out.size))
    return out


def pd_stage_overwrite_latest(stage: int, params=None, mom=None):
    a = _host_f32(params) if params is not None else None
    b = _host_f32(mom) if mom is not None else None
    n = a.size if a is not None else (b.size if b is not None else 0)
    _check(_lib.pd_stage_overwrite_latest(stage, a.ctypes.data if a is not None else None,
                                          b.ctypes.data if b is not None else None, n))


def pd_stage_version(stage: int, mb_id: int = -1) -> int:
    v = _i32(0)
    _check(_lib.pd_stage_version(stage, mb_id, C.byref(v)))
    return v.value


def pd_set_conv_halo(on: int) -> int:
    return int(_lib.pd_set_conv_halo(on))


def pd_set_recurrence_kernel(multi_step: int, spin_limit: int = 0, starve: int = 0) -> int:
    return int(_lib.pd_set_recurrence_kernel(multi_step, spin_limit, starve))


def pd_stage_check(stage: int):
    _check(_lib.pd_stage_check(stage))


def pd_set_big_gemm_waves(waves: int) -> int:
    return int(_lib.pd_set_big_gemm_waves(waves))


def pd_stage_set_trace_limit(stage: int, max_ops: int):
    _check(_lib.pd_stage_set_trace_limit(stage, max_ops))


def pd_stage_trace(stage: int):
    n = _sz(0)
    rc = _lib.pd_stage_trace(stage, None, 0, C.byref(n))
    if n.value == 0:
        _check(rc)
        return []
    arr = (pd_op * n.value)()
    _check(_lib.pd_stage_trace(stage, arr, n.value, C.byref(n)))
    return _ops(arr, n.value)


def pd_stage_input_slot(stage: int, mb_id: int) -> int:
    p = _vp(0)
    _check(_lib.pd_stage_input_slot(stage, mb_id, C.byref(p)))
    return p.value


def pd_stage_grad_slot(stage: int, mb_id: int) -> int:
    p = _vp(0)
    _check(_lib.pd_stage_grad_slot(stage, mb_id, C.byref(p)))
    return p.value


def pd_stage_debug_read(stage: int, what: int, mb_id: int, layer: int, shape) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _check(_lib.pd_stage_debug_read(stage, what, mb_id, layer, out.ctypes.data, out.size))
    return out


def pd_stage_debug_write(stage: int, what: int, mb_id: int, layer: int, values: np.ndarray):
    a = _host_f32(values)
    _check(_lib.pd_stage_debug_write(stage, what, mb_id, layer, a.ctypes.data, a.size))


def pd_forward(stage: int, mb_id: int, x_dev: int, labels_dev: int = 0, y_dev: int = 0, loss_dev: int = 0):
    _check(_lib.pd_forward(stage, mb_id, x_dev, labels_dev or None, y_dev or None, loss_dev or None))


def pd_forward_versioned(stage: int, mb_id: int, version: int, x_dev: int, labels_dev: int = 0, y_dev: int = 0,
                         loss_dev: int = 0):
    _check(_lib.pd_forward_versioned(stage, mb_id, version, x_dev, labels_dev, y_dev, loss_dev))


def pd_stage_ring_depth(stage: int) -> int:
    d = _i32(0)
    _check(_lib.pd_stage_ring_depth(stage, C.byref(d)))
    return d.value


def pd_backward(stage: int, mb_id: int, dy_dev: int = 0, dx_dev: int = 0):
    _check(_lib.pd_backward(stage, mb_id, dy_dev or None, dx_dev or None))


def pd_update(stage: int):
    _check(_lib.pd_update(stage))


def pd_pipeline_run(stages: Sequence[int], num_minibatches: int, inputs_dev: int, labels_dev: int,
                    losses_dev: int = 0):
    arr = (_vp * len(stages))(*stages)
    _check(_lib.pd_pipeline_run(arr, len(stages), num_minibatches, inputs_dev, labels_dev, losses_dev or None))


def pd_pipeline_run_replicated(replicas_by_stage: Sequence[Sequence[int]], num_minibatches: int, inputs_dev: int,
                               labels_dev: int, losses_dev: int = 0):
    """replicas_by_stage[s] = the handles of stage s, primary first."""
    flat = [h for st in replicas_by_stage for h in st]
    arr = (_vp * len(flat))(*flat)
    per = (_i32 * len(replicas_by_stage))(*[len(st) for st in replicas_by_stage])
    _check(_lib.pd_pipeline_run_replicated(arr, per, len(replicas_by_stage), num_minibatches, inputs_dev, labels_dev,
                                           losses_dev or None))


def pd_stage_checkpoint_save(stage: int, path: str):
    _check(_lib.pd_stage_checkpoint_save(stage, os.fsencode(path)))


def pd_stage_checkpoint_load(stage: int, path: str):
    _check(_lib.pd_stage_checkpoint_load(stage, os.fsencode(path)))


def pd_checkpoint_info(path: str):
    """(n_params, version, precision) of a checkpoint file; raises PdError if the file does not verify."""
    n, v, p = _sz(0), _i32(0), _i32(0)
    _check(_lib.pd_checkpoint_info(os.fsencode(path), C.byref(n), C.byref(v), C.byref(p)))
    return n.value, v.value, p.value


def pd_stage_profile(stage: int, enable: bool):
    _check(_lib.pd_stage_profile(stage, 1 if enable else 0))


def pd_stage_profile_read(stage: int):
    """One dict per profile unit: first_layer, last_layer, fwd_ms, bwd_ms, upd_ms, act_bytes, param_bytes."""
    n = _sz(0)
    rc = _lib.pd_stage_profile_read(stage, None, 0, C.byref(n))
    if rc != PD_ENOMEM:
        _check(rc)
    arr = (pd_layer_profile * max(1, n.value))()
    _check(_lib.pd_stage_profile_read(stage, arr, n.value, C.byref(n)))
    return [{name: getattr(arr[i], name) for name, _ in pd_layer_profile._fields_} for i in range(n.value)]


def pd_partition(t_layer, act_bytes, param_bytes, n_machines: int, bandwidth: float):
    """Returns (slowest stage time, [(first_layer, last_layer, replicas), ...], NOAM)."""
    n = len(t_layer)
    dbl = C.c_double * max(1, n)
    t, a, w = dbl(*map(float, t_layer)), dbl(*map(float, act_bytes)), dbl(*map(float, param_bytes))
    cap = max(1, min(n, int(n_machines)))
    out = (pd_stage_assign * cap)()
    best, ns, noam = C.c_double(0), _sz(0), _i32(0)
    _check(_lib.pd_partition(n, n_machines, t, a, w, bandwidth, C.byref(best), out, cap, C.byref(ns), C.byref(noam)))
    return best.value, [(out[k].first_layer, out[k].last_layer, out[k].replicas) for k in range(ns.value)], noam.value


def pd_set_big_tile_threshold(min_tiles: int) -> int:
    return _lib.pd_set_big_tile_threshold(min_tiles)


def pd_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return _lib.pd_gemm_workspace_bytes(M, N, K)


def pd_linear_fwd_bf16(stream, x, w, b, y, M, N, K, relu, ws=0, ws_bytes=0):
    _check(_lib.pd_linear_fwd_bf16(stream, x, w, b or None, y, M, N, K, int(relu), ws or None, ws_bytes))


def pd_linear_fwd_bf16_static_max_bytes() -> int:
    return int(_lib.pd_linear_fwd_bf16_static_max_bytes())


def pd_linear_fwd_bf16_static(stream, x, w, b, y, M, N, K, relu):
    _check(_lib.pd_linear_fwd_bf16_static(stream, x, w, b or None, y, M, N, K, int(relu)))


def pd_linear_dgrad_bf16(stream, dz, w, mask, dx, M, N, K, ws=0, ws_bytes=0):
    _check(_lib.pd_linear_dgrad_bf16(stream, dz, w, mask or None, dx, M, N, K, ws or None, ws_bytes))


def pd_linear_wgrad_update_bf16(stream, dz, x, master_w, mom_w, ring_w, master_b, mom_b, ring_b, M, N, K, lr, mu):
    _check(_lib.pd_linear_wgrad_update_bf16(stream, dz, x, master_w, mom_w, ring_w, master_b or None, mom_b or None,
                                            ring_b or None, M, N, K, lr, mu))


def _geom(N, H, W, c_in, c_out, kh, kw, stride, pad_h, pad_w):
    return (_i32 * 10)(N, H, W, c_in, c_out, kh, kw, stride, pad_h, pad_w)


def pd_conv_wgrad_splits(geom) -> int:
    n = _i32(0)
    _check(_lib.pd_conv_wgrad_splits(_geom(*geom), C.byref(n)))
    return n.value


def pd_conv_fwd_bf16(stream, x, w, b, y, geom, relu):
    _check(_lib.pd_conv_fwd_bf16(stream, x, w, b or None, y, _geom(*geom), int(relu)))


def pd_conv_dgrad_bf16(stream, dz, w, mask, dx, wt_scratch, geom):
    _check(_lib.pd_conv_dgrad_bf16(stream, dz, w, mask or None, dx, wt_scratch, _geom(*geom)))


def pd_conv_wgrad_update_bf16(stream, dz, x, part, master_w, mom_w, ring_w, master_b, mom_b, ring_b, geom, lr, mu):
    _check(_lib.pd_conv_wgrad_update_bf16(stream, dz, x, part, master_w, mom_w, ring_w, master_b, mom_b, ring_b,
                                          _geom(*geom), lr, mu))


def pd_maxpool2x2_fwd_bf16(stream, x, y, N, H, W, Cn):
    _check(_lib.pd_maxpool2x2_fwd_bf16(stream, x, y, N, H, W, Cn))


def pd_maxpool2x2_bwd_bf16(stream, x, y, dy, dx, N, H, W, Cn, relu_mask):
    _check(_lib.pd_maxpool2x2_bwd_bf16(stream, x, y, dy, dx, N, H, W, Cn, int(relu_mask)))


def pd_maxpool2x2_fwd_route_bf16(stream, x, y, route, N, H, W, Cn):
    _check(_lib.pd_maxpool2x2_fwd_route_bf16(stream, x, y, route, N, H, W, Cn))


def pd_maxpool2x2_bwd_route_bf16(stream, route, dy, dx, N, H, W, Cn, relu_mask):
    _check(_lib.pd_maxpool2x2_bwd_route_bf16(stream, route, dy, dx, N, H, W, Cn, int(relu_mask)))


def _pgeom(N, H, W, Cn, k, stride, pad):
    return (_i32 * 7)(N, H, W, Cn, k, stride, pad)


def pd_pool2d_fwd_bf16(stream, is_max, x, y, pgeom):
    _check(_lib.pd_pool2d_fwd_bf16(stream, int(is_max), x, y, _pgeom(*pgeom)))


def pd_pool2d_bwd_bf16(stream, is_max, x, y, dy, dx, pgeom, relu_mask):
    _check(_lib.pd_pool2d_bwd_bf16(stream, int(is_max), x, y, dy, dx, _pgeom(*pgeom), int(relu_mask)))


def pd_pool2d_fwd_route_bf16(stream, x, y, route, pgeom):
    _check(_lib.pd_pool2d_fwd_route_bf16(stream, x, y, route, _pgeom(*pgeom)))


def pd_pool2d_bwd_route_bf16(stream, route, dy, dx, pgeom, relu_mask):
    _check(_lib.pd_pool2d_bwd_route_bf16(stream, route, dy, dx, _pgeom(*pgeom), int(relu_mask)))
