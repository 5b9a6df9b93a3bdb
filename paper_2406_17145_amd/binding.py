"""ctypes binding of libgpp.so: the C ABI's functions under their own names, plus
`Stage`, a marshalling helper (device buffers through PyTorch, padded parameter
layout, dtype conversion).  No step of the stage's arithmetic runs here: every
forward/backward operation is a HIP kernel inside the library.

The library must have been built (`python -m paper_2406_17145_amd.build`);
`load()` raises if it is missing -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgpp.so")

GPP_OK = 0
STATUS_NAMES = ["GPP_OK", "GPP_ERR_INVALID_ARG", "GPP_ERR_BAD_GRAPH", "GPP_ERR_SHAPE", "GPP_ERR_UNSUPPORTED",
                "GPP_ERR_WORKSPACE", "GPP_ERR_ORDER", "GPP_ERR_INDEX", "GPP_ERR_DEVICE"]
(GPP_ERR_INVALID_ARG, GPP_ERR_BAD_GRAPH, GPP_ERR_SHAPE, GPP_ERR_UNSUPPORTED, GPP_ERR_WORKSPACE, GPP_ERR_ORDER,
 GPP_ERR_INDEX, GPP_ERR_DEVICE) = range(1, 9)
DTYPES = {"f32": 0, "bf16": 1, "i32": 2}
KINDS = {"input": 0, "linear": 1, "layernorm": 2, "attention": 3, "add": 4, "meanpool": 5, "concat": 6,
         "embedding_bag_sum": 7, "dot_interact": 8, "loss_mse": 9, "loss_ce": 10, "loss_bce": 11,
         "embedding_bag_concat": 12}
ACTS = {"none": 0, "relu": 1, "gelu": 2}
FLAG_FORCE_GENERIC_GEMM = 1
FLAG_SPLIT_K = 2
FLAG_GROUPED_DW = 4
FLAG_SIDE_STREAM = 8
FLAG_SHARED_GPU = 16


def flag_group_launches(lanes):
    """Stage flag bits 8-11: group launches for `lanes` streams per direction."""
    return (int(lanes) & 15) << 8


class OpDesc(C.Structure):
    _fields_ = [
        ("kind", C.c_int32), ("n_in", C.c_int32), ("in_", C.POINTER(C.c_int32)), ("branch", C.c_int32),
        ("in_features", C.c_int64), ("out_features", C.c_int64), ("act", C.c_int32), ("has_bias", C.c_int32),
        ("heads", C.c_int32), ("seq_len", C.c_int32), ("rows_extra", C.c_int32), ("requires_grad", C.c_int32),
        ("num_rows", C.c_int64), ("bag_size", C.c_int64), ("eps", C.c_double), ("loss_scale", C.c_double),
        ("dtype", C.c_int32), ("param_dtype", C.c_int32), ("param", C.c_void_p * 2), ("grad", C.c_void_p * 2),
    ]


class StageDesc(C.Structure):
    _fields_ = [("n_ops", C.c_int32), ("ops", C.POINTER(OpDesc)), ("micro_batch", C.c_int64),
                ("in_flight_slots", C.c_int32), ("flags", C.c_int32)]


EXPORTS = [
    "gpp_ld", "gpp_stage_workspace_bytes", "gpp_stage_create", "gpp_stage_create_static", "gpp_stage_forward", "gpp_stage_backward",
    "gpp_stage_grad_reset", "gpp_stage_sync_status", "gpp_stage_destroy", "gpp_stage_num_inputs",
    "gpp_stage_num_outputs", "gpp_stage_input_op", "gpp_stage_output_op", "gpp_stage_num_launches",
    "gpp_stage_embedding_sort_result", "gpp_last_error", "gpp_stage_profile_enable", "gpp_stage_profile_read",
    "gpp_profile_tag_name", "gpp_compute_in_flight", "gpp_assign_schedules", "gpp_schedule_tasks",
    "gpp_stage_run_schedule", "gpp_stage_memory", "gpp_stage_backward_weights", "gpp_stage_info", "gpp_stage_io_info",
    "gpp_stage_run_schedule_lanes", "gpp_stage_lanes", "gpp_stage_group_launches",
    "gpp_partition", "gpp_partition_search", "gpp_pipeline_workspace_bytes", "gpp_pipeline_create", "gpp_pipeline_run", "gpp_pipeline_destroy",
]
GPP_PROFILE_TAGS = 32

class MicrobatchIO(C.Structure):
    _fields_ = [("inputs", C.POINTER(C.c_void_p)), ("outputs", C.POINTER(C.c_void_p)), ("loss_out", C.c_void_p),
                ("grad_outputs", C.POINTER(C.c_void_p)), ("grad_inputs", C.POINTER(C.c_void_p))]


class PipelineEdge(C.Structure):
    _fields_ = [("from_stage", C.c_int32), ("from_output", C.c_int32), ("to_stage", C.c_int32), ("to_input", C.c_int32)]


_lib = None
_hip = None


def load():
    """Loads libgpp.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2406_17145_amd.build` "
                           "(there is no fallback implementation)")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 (same SONAME as the system
    # one).  Loading it first makes the dynamic linker bind libgpp.so to that copy, so device
    # pointers and streams created by PyTorch are valid inside the library.
    import torch  # noqa: F401
    global _hip
    _hip = C.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"), mode=C.RTLD_GLOBAL)
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.gpp_ld.restype, lib.gpp_ld.argtypes = i64, [i64]
    lib.gpp_stage_workspace_bytes.restype = i32
    lib.gpp_stage_workspace_bytes.argtypes = [C.POINTER(StageDesc), C.POINTER(C.c_size_t)]
    lib.gpp_stage_create.restype = i32
    lib.gpp_stage_create.argtypes = [C.POINTER(StageDesc), vp, C.c_size_t, C.POINTER(vp)]
    lib.gpp_stage_create_static.restype = i32
    lib.gpp_stage_create_static.argtypes = [C.POINTER(StageDesc), C.POINTER(vp)]
    lib.gpp_stage_forward.restype = i32
    lib.gpp_stage_forward.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), vp, vp]
    lib.gpp_stage_backward.restype = i32
    lib.gpp_stage_backward.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), vp]
    lib.gpp_stage_grad_reset.restype, lib.gpp_stage_grad_reset.argtypes = i32, [vp, vp]
    lib.gpp_stage_sync_status.restype, lib.gpp_stage_sync_status.argtypes = i32, [vp, vp]
    lib.gpp_stage_backward_weights.restype, lib.gpp_stage_backward_weights.argtypes = i32, [vp, vp]
    lib.gpp_stage_destroy.restype, lib.gpp_stage_destroy.argtypes = i32, [vp]
    for name in ("gpp_stage_num_inputs", "gpp_stage_num_outputs"):
        getattr(lib, name).restype, getattr(lib, name).argtypes = i32, [vp]
    for name in ("gpp_stage_input_op", "gpp_stage_output_op", "gpp_stage_num_launches"):
        getattr(lib, name).restype, getattr(lib, name).argtypes = i32, [vp, i32]
    lib.gpp_stage_embedding_sort_result.restype = i32
    lib.gpp_stage_embedding_sort_result.argtypes = [vp, i32] + [C.POINTER(vp)] * 4
    lib.gpp_last_error.restype, lib.gpp_last_error.argtypes = C.c_char_p, []
    lib.gpp_stage_profile_enable.restype, lib.gpp_stage_profile_enable.argtypes = i32, [vp, i32]
    lib.gpp_stage_profile_read.restype = i32
    lib.gpp_stage_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
    lib.gpp_profile_tag_name.restype, lib.gpp_profile_tag_name.argtypes = C.c_char_p, [i32]
    lib.gpp_compute_in_flight.restype = i32
    lib.gpp_compute_in_flight.argtypes = [i64] * 5 + [C.POINTER(i64)]
    lib.gpp_assign_schedules.restype = i32
    lib.gpp_assign_schedules.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), C.POINTER(i32),
                                         C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.gpp_schedule_tasks.restype, lib.gpp_schedule_tasks.argtypes = i32, [i64, i64, i64, i64, C.POINTER(i32)]
    lib.gpp_stage_run_schedule.restype = i32
    lib.gpp_stage_run_schedule.argtypes = [vp, C.POINTER(i32), i64, C.POINTER(MicrobatchIO), i64, vp, vp]
    lib.gpp_stage_run_schedule_lanes.restype = i32
    lib.gpp_stage_run_schedule_lanes.argtypes = [vp, C.POINTER(i32), i64, C.POINTER(MicrobatchIO), i64, C.POINTER(vp), i32,
                                                 C.POINTER(vp), i32]
    lib.gpp_stage_lanes.restype, lib.gpp_stage_lanes.argtypes = i32, [vp, C.POINTER(i32), C.POINTER(i32)]
    lib.gpp_stage_group_launches.restype, lib.gpp_stage_group_launches.argtypes = i32, [vp, C.POINTER(i32), C.POINTER(i32)]
    lib.gpp_stage_memory.restype, lib.gpp_stage_memory.argtypes = i32, [vp] + [C.POINTER(C.c_size_t)] * 3
    lib.gpp_stage_info.restype = i32
    lib.gpp_stage_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
    lib.gpp_stage_io_info.restype = i32
    lib.gpp_stage_io_info.argtypes = [vp, i32, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
    pipe_args = [i32, C.POINTER(vp), i32, C.POINTER(PipelineEdge), C.POINTER(i64), C.POINTER(i64)]
    lib.gpp_pipeline_workspace_bytes.restype = i32
    lib.gpp_pipeline_workspace_bytes.argtypes = pipe_args + [C.POINTER(C.c_size_t)]
    lib.gpp_pipeline_create.restype = i32
    lib.gpp_pipeline_create.argtypes = pipe_args + [vp, C.c_size_t, C.POINTER(vp)]
    lib.gpp_pipeline_run.restype = i32
    lib.gpp_pipeline_run.argtypes = [vp, i64, C.POINTER(C.POINTER(MicrobatchIO)), C.POINTER(vp), C.POINTER(vp)]
    lib.gpp_pipeline_destroy.restype, lib.gpp_pipeline_destroy.argtypes = i32, [vp]
    dp = C.POINTER(C.c_double)
    lib.gpp_partition.restype = i32
    lib.gpp_partition.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32), dp, dp, dp, i32, i64, C.c_double, C.c_double, i64,
                                  C.c_double, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), dp, C.POINTER(i64)]
    _lib = lib
    return lib


class GppError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status


def _check(status):
    if status != GPP_OK:
        raise GppError(status, load().gpp_last_error().decode())


def gpp_ld(features):
    return int(load().gpp_ld(int(features)))


def build_desc(ops, micro_batch, slots=1, flags=0, param_ptrs=None, grad_ptrs=None):
    """ops: list of op dicts (see workloads.py).  Returns (StageDesc, keepalive)."""
    n = len(ops)
    arr = (OpDesc * n)()
    keep = [arr]
    for i, op in enumerate(ops):
        d = arr[i]
        d.kind = KINDS[op["kind"]]
        ins = (C.c_int32 * max(1, len(op["inputs"])))(*op["inputs"])
        keep.append(ins)
        d.n_in = len(op["inputs"])
        d.in_ = C.cast(ins, C.POINTER(C.c_int32))
        d.branch = op.get("branch", -1)
        d.in_features = op.get("in_features", 0)
        d.out_features = op.get("out_features", 0)
        d.act = ACTS[op.get("act", "none")]
        d.has_bias = 1 if op.get("bias", False) else 0
        d.heads = op.get("heads", 0)
        d.seq_len = op.get("seq_len", 1)
        d.rows_extra = op.get("rows_extra", 0)
        d.requires_grad = 1 if (op["kind"] == "input" and op.get("role", "data") == "data"
                                and op.get("dtype") != "i32") else 0
        d.num_rows = op.get("num_rows", 0)
        d.bag_size = op.get("bag_size", 0)
        d.eps = op.get("eps", 0.0)
        d.loss_scale = op.get("loss_scale", 0.0)
        d.dtype = DTYPES[op.get("out_dtype", op.get("dtype", "f32"))]
        d.param_dtype = DTYPES[op.get("dtype", "f32")]
        for k in range(2):
            d.param[k] = (param_ptrs or {}).get(i, [None, None])[k]
            d.grad[k] = (grad_ptrs or {}).get(i, [None, None])[k]
    sd = StageDesc(n, C.cast(arr, C.POINTER(OpDesc)), int(micro_batch), int(slots), int(flags))
    return sd, keep


def gpp_stage_workspace_bytes(desc):
    out = C.c_size_t(0)
    _check(load().gpp_stage_workspace_bytes(C.byref(desc), C.byref(out)))
    return out.value


def gpp_stage_create(desc, workspace_ptr, workspace_bytes):
    h = C.c_void_p()
    _check(load().gpp_stage_create(C.byref(desc), workspace_ptr, workspace_bytes, C.byref(h)))
    return h


def gpp_stage_create_static(desc):
    h = C.c_void_p()
    _check(load().gpp_stage_create_static(C.byref(desc), C.byref(h)))
    return h


def _ptr_array(ptrs):
    arr = (C.c_void_p * max(1, len(ptrs)))(*ptrs)
    return arr


def gpp_stage_forward(handle, slot, input_ptrs, output_ptrs, loss_ptr, stream):
    _check(load().gpp_stage_forward(handle, slot, _ptr_array(input_ptrs),
                                    _ptr_array(output_ptrs) if output_ptrs is not None else None,
                                    loss_ptr, stream))


def gpp_stage_backward(handle, slot, grad_output_ptrs, grad_input_ptrs, stream):
    _check(load().gpp_stage_backward(handle, slot,
                                     _ptr_array(grad_output_ptrs) if grad_output_ptrs is not None else None,
                                     _ptr_array(grad_input_ptrs) if grad_input_ptrs is not None else None, stream))


def gpp_stage_backward_weights(handle, stream):
    _check(load().gpp_stage_backward_weights(handle, stream))


def gpp_stage_grad_reset(handle, stream):
    _check(load().gpp_stage_grad_reset(handle, stream))


def gpp_stage_sync_status(handle, stream):
    _check(load().gpp_stage_sync_status(handle, stream))


def gpp_compute_in_flight(k_x, b_x, k_y, b_y, i_y):
    out = C.c_int64()
    _check(load().gpp_compute_in_flight(k_x, b_x, k_y, b_y, i_y, C.byref(out)))
    return out.value


def gpp_assign_schedules(n_stages, edges, b, k_candidates):
    """edges: (x, y) pairs, S_x feeds S_y; returns (i, k) lists, one entry per stage."""
    n_e = len(edges)
    ef = (C.c_int32 * max(1, n_e))(*[e[0] for e in edges])
    et = (C.c_int32 * max(1, n_e))(*[e[1] for e in edges])
    kb, kv = [0], []
    for ks in k_candidates:
        kv += list(ks)
        kb.append(len(kv))
    i_out, k_out = (C.c_int64 * n_stages)(), (C.c_int64 * n_stages)()
    _check(load().gpp_assign_schedules(n_stages, n_e, ef, et, (C.c_int64 * n_stages)(*b), (C.c_int32 * len(kb))(*kb),
                                       (C.c_int64 * max(1, len(kv)))(*kv), i_out, k_out))
    return list(i_out), list(k_out)


def gpp_schedule_tasks(n_micro, i, k, b):
    """Task codes: +(j+1) = fw_j, -(j+1) = bw_j."""
    tasks = (C.c_int32 * max(1, 2 * n_micro))()
    _check(load().gpp_schedule_tasks(n_micro, i, k, b, tasks))
    return list(tasks)[:2 * n_micro]


def gpp_stage_run_schedule(handle, tasks, io, stream_forward, stream_backward):
    """io: one (input_ptrs, output_ptrs or None, loss_ptr or None, grad_output_ptrs or None, grad_input_ptrs or None)
    per micro-batch.  Returns the marshalled arrays; keep them while a captured graph of the call may replay
    (the call itself reads them on the host only)."""
    keep = []

    def arr(ptrs):
        if ptrs is None:
            return None
        a = _ptr_array(ptrs)
        keep.append(a)
        return a
    ios = (MicrobatchIO * max(1, len(io)))()
    for m, (inp, out, loss, gout, gin) in zip(ios, io):
        m.inputs, m.outputs, m.loss_out, m.grad_outputs, m.grad_inputs = arr(inp), arr(out), loss, arr(gout), arr(gin)
    t = (C.c_int32 * max(1, len(tasks)))(*tasks)
    _check(load().gpp_stage_run_schedule(handle, t, len(tasks), ios, len(io), stream_forward, stream_backward))
    return keep


def gpp_stage_run_schedule_lanes(handle, tasks, io, streams_forward, streams_backward):
    """gpp_stage_run_schedule with lists of streams: pass j of a direction goes to stream j % len(list)."""
    keep = []
    ios = _marshal_io(io, keep)
    t = (C.c_int32 * max(1, len(tasks)))(*tasks)
    sf, sb = _ptr_array(streams_forward), _ptr_array(streams_backward)
    _check(load().gpp_stage_run_schedule_lanes(handle, t, len(tasks), ios, len(io), sf, len(streams_forward), sb,
                                               len(streams_backward)))
    return keep


def gpp_stage_lanes(handle):
    """(several forward streams allowed, several backward streams allowed)."""
    f, b = C.c_int32(), C.c_int32()
    _check(load().gpp_stage_lanes(handle, C.byref(f), C.byref(b)))
    return bool(f.value), bool(b.value)


def gpp_stage_group_launches(handle):
    """(streams per direction the group launches are set up for, most micro-batches per launch); (0, 0) = none."""
    a, b = C.c_int32(), C.c_int32()
    _check(load().gpp_stage_group_launches(handle, C.byref(a), C.byref(b)))
    return a.value, b.value


def _marshal_io(io, keep):
    def arr(ptrs):
        if ptrs is None:
            return None
        a = _ptr_array(ptrs)
        keep.append(a)
        return a
    ios = (MicrobatchIO * max(1, len(io)))()
    for m, (inp, out, loss, gout, gin) in zip(ios, io):
        m.inputs, m.outputs, m.loss_out, m.grad_outputs, m.grad_inputs = arr(inp), arr(out), loss, arr(gout), arr(gin)
    keep.append(ios)
    return ios


def _pipeline_args(stage_handles, edges, in_flight, k):
    n, ne = len(stage_handles), len(edges)
    hs = (C.c_void_p * n)(*[h.value if isinstance(h, C.c_void_p) else h for h in stage_handles])
    es = (PipelineEdge * max(1, ne))(*[PipelineEdge(*e) for e in edges])
    return [n, hs, ne, es, (C.c_int64 * n)(*in_flight), (C.c_int64 * n)(*k)]


def gpp_pipeline_workspace_bytes(stage_handles, edges, in_flight, k):
    """edges: (from_stage, from_output, to_stage, to_input) tuples; (x, -1, y, -1) is an order-only edge."""
    out = C.c_size_t(0)
    _check(load().gpp_pipeline_workspace_bytes(*_pipeline_args(stage_handles, edges, in_flight, k), C.byref(out)))
    return out.value


def gpp_pipeline_create(stage_handles, edges, in_flight, k, workspace_ptr, workspace_bytes):
    h = C.c_void_p()
    _check(load().gpp_pipeline_create(*_pipeline_args(stage_handles, edges, in_flight, k), workspace_ptr, workspace_bytes,
                                      C.byref(h)))
    return h


def gpp_pipeline_run(handle, io, streams_forward, streams_backward):
    """io[s][j]: the tuple gpp_stage_run_schedule takes, for stage s and micro-batch j."""
    keep = []
    per_stage = [_marshal_io(rows, keep) for rows in io]
    n = len(io)
    arr = (C.POINTER(MicrobatchIO) * n)(*[C.cast(a, C.POINTER(MicrobatchIO)) for a in per_stage])
    n_micro = len(io[0]) if io else 0
    _check(load().gpp_pipeline_run(handle, n_micro, arr, (C.c_void_p * n)(*streams_forward), (C.c_void_p * n)(*streams_backward)))
    return keep


def gpp_pipeline_destroy(handle):
    _check(load().gpp_pipeline_destroy(handle))


def gpp_stage_info(handle):
    """(micro-batch size, stash slots, flags)."""
    a, b, c = C.c_int64(), C.c_int32(), C.c_int32()
    _check(load().gpp_stage_info(handle, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def gpp_stage_io_info(handle, is_output, index):
    """(rows, features, dtype code, has_grad) of an input or output."""
    r, f, d, g = C.c_int64(), C.c_int64(), C.c_int32(), C.c_int32()
    _check(load().gpp_stage_io_info(handle, 1 if is_output else 0, index, C.byref(r), C.byref(f), C.byref(d), C.byref(g)))
    return r.value, f.value, d.value, bool(g.value)


def gpp_partition(n_ops, edges, t, w, a, n_devices, b, memory_bytes, sync_seconds_per_byte=0.0, mini_batch=1, eps_rel=1e-9):
    """edges: (u, v) operator pairs.  Returns None when nothing fits, else a dict: stage_of_op, devices and
    in_flight (samples) per stage, bottleneck (seconds per sample), dp_states."""
    ne = len(edges)
    ef = (C.c_int32 * max(1, ne))(*[e[0] for e in edges])
    et = (C.c_int32 * max(1, ne))(*[e[1] for e in edges])
    dbl = C.c_double * n_ops
    stage_of, ns = (C.c_int32 * n_ops)(), C.c_int32()
    dev, inf = (C.c_int32 * n_ops)(), (C.c_int64 * n_ops)()
    tps, states = C.c_double(), C.c_int64()
    _check(load().gpp_partition(n_ops, ne, ef, et, dbl(*t), dbl(*w), dbl(*a), n_devices, b, memory_bytes,
                                sync_seconds_per_byte, mini_batch, eps_rel, stage_of, C.byref(ns), dev, inf,
                                C.byref(tps), C.byref(states)))
    if ns.value == 0:
        return None
    return dict(stage_of_op=list(stage_of), devices=list(dev)[:ns.value], in_flight=list(inf)[:ns.value],
                bottleneck=tps.value, dp_states=states.value)


def gpp_partition_search(n_ops, edges, b_values, t, w, a, k_values, n_devices, memory_bytes, x=None, link_latency=0.0,
                         link_seconds_per_byte=0.0, sync_seconds_per_byte=0.0, mini_batch=1, eps_rel=1e-9):
    """t[o][j]: seconds per sample of operator o at micro-batch size b_values[j]; x[e]: bytes per sample on edge e.
    Returns None when nothing fits, else a dict as gpp_partition plus b and k per stage."""
    lib = load()
    i32, i64, dp = C.c_int32, C.c_int64, C.POINTER(C.c_double)
    lib.gpp_partition_search.restype = i32
    lib.gpp_partition_search.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32), i32, C.POINTER(i64), dp, dp, dp, i32, C.POINTER(i64),
                                         dp, C.c_double, C.c_double, i32, C.c_double, C.c_double, i64, C.c_double, C.POINTER(i32),
                                         C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), dp,
                                         C.POINTER(i64)]
    ne, nb, nk = len(edges), len(b_values), len(k_values)
    ef = (i32 * max(1, ne))(*[e[0] for e in edges])
    et = (i32 * max(1, ne))(*[e[1] for e in edges])
    flat = [float(t[o][j]) for o in range(n_ops) for j in range(nb)]
    dbl = C.c_double * n_ops
    stage_of, ns = (i32 * n_ops)(), i32()
    dev, inf, sb, sk = (i32 * n_ops)(), (i64 * n_ops)(), (i64 * n_ops)(), (i64 * n_ops)()
    tps, states = C.c_double(), i64()
    xs = None if x is None else (C.c_double * max(1, ne))(*x)
    _check(lib.gpp_partition_search(n_ops, ne, ef, et, nb, (i64 * nb)(*b_values), (C.c_double * len(flat))(*flat), dbl(*w), dbl(*a),
                                    nk, (i64 * nk)(*k_values), xs, link_latency, link_seconds_per_byte, n_devices, memory_bytes,
                                    sync_seconds_per_byte, mini_batch, eps_rel, stage_of, C.byref(ns), dev, inf, sb, sk,
                                    C.byref(tps), C.byref(states)))
    if ns.value == 0:
        return None
    n = ns.value
    return dict(stage_of_op=list(stage_of), devices=list(dev)[:n], in_flight=list(inf)[:n], b=list(sb)[:n], k=list(sk)[:n],
                bottleneck=tps.value, dp_states=states.value)


def gpp_stage_memory(handle):
    """(bytes of one stash slot, bytes shared by all slots, total workspace bytes)."""
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(load().gpp_stage_memory(handle, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def gpp_stage_destroy(handle):
    _check(load().gpp_stage_destroy(handle))


# ---------------------------------------------------------------------------
# marshalling helper
# ---------------------------------------------------------------------------
class Stage:
    """Owns the device buffers of one stage (PyTorch tensors) and marshals numpy
    arrays to and from the C ABI."""

    def __init__(self, ops, micro_batch, params, slots=1, flags=0, device="cuda:0", static_workspace=False):
        import torch
        self.torch = torch
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.ops, self.b, self.slots = ops, int(micro_batch), int(slots)
        self.grouped_dw = bool(flags & FLAG_GROUPED_DW)
        self.tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}
        self.p_t, self.g_t, pp, gp = {}, {}, {}, {}
        for i, p in params.items():
            op = ops[i]
            names = {"linear": ["W", "b"], "layernorm": ["gamma", "beta"], "embedding_bag_sum": ["table"],
                     "embedding_bag_concat": ["table"]}[op["kind"]]
            self.p_t[i], self.g_t[i] = {}, {}
            pp[i], gp[i] = [None, None], [None, None]
            for k, nm in enumerate(names):
                if nm not in p:
                    continue
                a = np.asarray(p[nm], dtype=np.float32)
                if a.ndim == 2:
                    ld = gpp_ld(a.shape[1])
                    pad = np.zeros((a.shape[0], ld), np.float32)
                    pad[:, :a.shape[1]] = a
                    a = pad
                dt = self.tdt[op["dtype"]] if nm == "W" else torch.float32
                t = torch.from_numpy(a).to(self.dev).to(dt).contiguous()
                g = torch.zeros(a.shape, dtype=torch.float32, device=self.dev)
                self.p_t[i][nm], self.g_t[i][nm] = t, g
                pp[i][k], gp[i][k] = t.data_ptr(), g.data_ptr()
        self.desc, self._keep = build_desc(ops, micro_batch, slots, flags, pp, gp)
        self.ws_bytes = gpp_stage_workspace_bytes(self.desc)
        if static_workspace:      # the library's own device array: no workspace tensor
            self.ws = None
            self.handle = gpp_stage_create_static(self.desc)
        else:
            self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.dev)
            base = (self.ws.data_ptr() + 255) // 256 * 256
            self.handle = gpp_stage_create(self.desc, base, self.ws_bytes)
        lib = load()
        self.input_ids = [lib.gpp_stage_input_op(self.handle, k) for k in range(lib.gpp_stage_num_inputs(self.handle))]
        self.output_ids = [lib.gpp_stage_output_op(self.handle, k) for k in range(lib.gpp_stage_num_outputs(self.handle))]
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.dev)
        self._held = {}

    # -- helpers --
    def stream(self):
        return self.torch.cuda.current_stream(self.dev).cuda_stream

    def _rows(self, op_id):
        op = self.ops[op_id]
        if op["kind"] == "input":
            return self.b * op.get("seq_len", 1) + op.get("rows_extra", 0)
        if op["kind"] in ("meanpool", "embedding_bag_sum", "embedding_bag_concat"):
            return self.b
        return self._rows(op["inputs"][0])

    def to_device(self, op_id, a):
        torch = self.torch
        if isinstance(a, torch.Tensor):
            return a
        op = self.ops[op_id]
        dt = self.tdt[op.get("out_dtype", op["dtype"])]
        t = torch.from_numpy(np.ascontiguousarray(a))
        if dt == torch.int32:
            t = t.to(torch.int32)
        else:
            t = t.to(torch.float32)
        return t.to(self.dev).to(dt).contiguous()

    def stage_inputs(self, inputs):
        """numpy dict -> list of device tensors in input order (marshalling, untimed)."""
        return [self.to_device(i, inputs[i]) for i in self.input_ids]

    def alloc_outputs(self):
        torch = self.torch
        return [torch.empty((self._rows(i), self.ops[i]["out_features"]),
                            dtype=self.tdt[self.ops[i].get("out_dtype", self.ops[i]["dtype"])], device=self.dev)
                for i in self.output_ids]

    def alloc_grad_inputs(self):
        torch = self.torch
        outs = []
        for i in self.input_ids:
            op = self.ops[i]
            if op.get("role", "data") == "data" and op["dtype"] != "i32":
                outs.append(torch.empty((self._rows(i), op["out_features"]), dtype=self.tdt[op["dtype"]], device=self.dev))
            else:
                outs.append(None)
        return outs

    # -- the four calls --
    def forward(self, slot, inputs, outputs=None, loss=None):
        """inputs: list of device tensors (stage_inputs) or dict of numpy arrays."""
        if isinstance(inputs, dict):
            inputs = self.stage_inputs(inputs)
        if outputs is None:
            outputs = self.alloc_outputs()
        loss = self.loss if loss is None else loss
        gpp_stage_forward(self.handle, slot, [t.data_ptr() for t in inputs], [t.data_ptr() for t in outputs],
                          loss.data_ptr(), self.stream())
        self._held[slot] = inputs
        return outputs, loss

    def backward(self, slot, grad_outputs=None, grad_inputs=None):
        if grad_outputs is not None and isinstance(grad_outputs, dict):
            grad_outputs = [self.to_device(i, grad_outputs[i]) for i in self.output_ids]
        if grad_inputs is None:
            grad_inputs = self.alloc_grad_inputs()
        gpp_stage_backward(self.handle, slot,
                           [t.data_ptr() for t in grad_outputs] if grad_outputs else None,
                           [t.data_ptr() if t is not None else None for t in grad_inputs], self.stream())
        self._held[("g", slot)] = grad_outputs
        return grad_inputs

    def backward_weights(self):
        gpp_stage_backward_weights(self.handle, self.stream())

    def grad_reset(self):
        gpp_stage_grad_reset(self.handle, self.stream())

    def sync_status(self):
        gpp_stage_sync_status(self.handle, self.stream())

    def profile_enable(self, on):
        """on: False / True, or an integer R > 1 for the timing-only mode that launches every GEMM step R times
        inside its event bracket."""
        _check(load().gpp_stage_profile_enable(self.handle, int(on)))

    def profile_read(self, reset=True):
        """{tag name: (milliseconds, kernel launches)} accumulated since the last reset."""
        ms = (C.c_double * GPP_PROFILE_TAGS)()
        ln = (C.c_int64 * GPP_PROFILE_TAGS)()
        _check(load().gpp_stage_profile_read(self.handle, ms, ln, 1 if reset else 0))
        lib = load()
        return {lib.gpp_profile_tag_name(k).decode(): (ms[k], ln[k]) for k in range(GPP_PROFILE_TAGS) if ln[k]}

    def num_launches(self, backward):
        """backward: False / 0 forward, True / 1 backward, 2 grouped weight-gradient call."""
        return load().gpp_stage_num_launches(self.handle, int(backward))

    # -- results back to numpy (unpadded) --
    def grads_numpy(self):
        self.torch.cuda.synchronize(self.dev)
        out = {}
        for i, g in self.g_t.items():
            out[i] = {}
            for nm, t in g.items():
                a = t.cpu().numpy()
                if a.ndim == 2:
                    ref_cols = {"W": self.ops[i].get("in_features"), "table": self.ops[i].get("in_features") if self.ops[i]["kind"] == "embedding_bag_concat"
                                else self.ops[i].get("out_features")}[nm]
                    a = a[:, :ref_cols]
                out[i][nm] = a
        return out

    def embedding_sort_result(self, op_id):
        torch = self.torch
        torch.cuda.synchronize(self.dev)
        ptrs = [C.c_void_p() for _ in range(4)]
        _check(load().gpp_stage_embedding_sort_result(self.handle, op_id, *[C.byref(p) for p in ptrs]))
        cap = self.b * self.ops[op_id]["bag_size"]

        def read(ptr, n):
            buf = torch.empty(n, dtype=torch.int32, device=self.dev)
            rc = _hip.hipMemcpy(C.c_void_p(buf.data_ptr()), ptr, C.c_size_t(4 * n), C.c_int(3))
            assert rc == 0, rc
            return buf.cpu().numpy()

        counts = read(ptrs[3], 2)
        n_used, n_unique = int(counts[0]), int(counts[1])
        assert 0 <= n_used <= cap and 0 <= n_unique <= n_used
        return (read(ptrs[0], cap)[:n_used], read(ptrs[1], cap)[:n_unique], read(ptrs[2], cap + 1)[:n_unique + 1])

    def close(self):
        if self.handle is not None:
            self.torch.cuda.synchronize(self.dev)
            gpp_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
