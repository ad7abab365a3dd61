"""ctypes binding of the C ABI in ``include/coopt_attn.h``: same names, argument marshalling only.

Tensors are torch CUDA(HIP) tensors used purely as device memory; every step of the path runs in
the library's own kernels on the current torch stream.  If the shared library is missing the
binding raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcoopt_attn.so")
_lib = None

COOPT_KV_FP16 = 0
COOPT_KV_E4M3 = 1

EXPORTS = [
    "coopt_kv_cache_write_fp8", "coopt_kv_cache_write_fp16", "coopt_kv_cache_write_skipset",
    "coopt_paged_gqa_decode",
    "coopt_paged_gqa_decode_step", "coopt_paged_gqa_decode_split", "coopt_paged_gqa_decode_merge",
    "coopt_decode_workspace_bytes", "coopt_set_decode_plan", "coopt_get_decode_plan", "coopt_paged_gqa_decode_partitioned",
    "coopt_paged_gqa_reduce", "coopt_paged_gqa_prefill_chunk", "coopt_gather_cached_kv",
    "coopt_decode_schedule_bytes", "coopt_decode_schedule_prepare", "coopt_paged_gqa_decode_scheduled",
    "coopt_stream_read_probe", "coopt_status_string",
]


class CooptError(RuntimeError):
    pass


class DecodePlan(ctypes.Structure):
    """Mirror of ``coopt_decode_plan``."""
    _fields_ = [("tokens_per_group", ctypes.c_int32), ("waves_per_group", ctypes.c_int32),
                ("pipeline_depth", ctypes.c_int32), ("grid_waves", ctypes.c_int32),
                ("softmax_reduction", ctypes.c_int32)]


class Shape(ctypes.Structure):
    """Mirror of ``coopt_shape``."""
    _fields_ = [("num_seqs", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32),
                ("max_blocks_per_seq", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libcoopt_attn.so (built by ``paper_2602_09323_amd.build``); raises if absent."""
    global _lib
    if _lib is None:
        path = os.environ.get("COOPT_ATTN_LIB", _LIB_PATH)   # another build of the same library
        if not os.path.exists(path):
            raise CooptError(f"{path} is not built; run `python -m paper_2602_09323_amd.build`")
        lib = ctypes.CDLL(path)
        vp, i32, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p
        shp = ctypes.POINTER(Shape)
        lib.coopt_kv_cache_write_fp8.argtypes = [vp, vp, i64p, i32, vp, vp, vp, vp, shp, vp]
        lib.coopt_kv_cache_write_fp16.argtypes = [vp, vp, i64p, i32, vp, vp, shp, vp]
        lib.coopt_kv_cache_write_skipset.argtypes = [vp, vp, i64p, vp, i32, vp, vp, vp, vp, shp, vp]
        lib.coopt_paged_gqa_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, shp, vp]
        lib.coopt_paged_gqa_decode_step.argtypes = [vp, vp, i64p, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                    ctypes.c_size_t, shp, vp]
        lib.coopt_paged_gqa_decode_split.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, shp, vp]
        lib.coopt_paged_gqa_decode_merge.argtypes = [vp, vp, ctypes.c_size_t, vp, shp, vp]
        lib.coopt_decode_workspace_bytes.argtypes = [shp]
        lib.coopt_decode_workspace_bytes.restype = ctypes.c_size_t
        lib.coopt_set_decode_plan.argtypes = [ctypes.POINTER(DecodePlan)]
        lib.coopt_get_decode_plan.argtypes = [ctypes.POINTER(DecodePlan)]
        lib.coopt_get_decode_plan.restype = None
        lib.coopt_paged_gqa_decode_partitioned.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, shp, vp]
        lib.coopt_paged_gqa_reduce.argtypes = [vp, vp, vp, vp, i32, i32, vp, shp, vp]
        lib.coopt_paged_gqa_prefill_chunk.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, shp, vp]
        lib.coopt_gather_cached_kv.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, shp, vp]
        lib.coopt_decode_schedule_bytes.argtypes = [shp]
        lib.coopt_decode_schedule_bytes.restype = ctypes.c_size_t
        lib.coopt_decode_schedule_prepare.argtypes = [vp, vp, i64p, vp, ctypes.c_size_t, shp, vp]
        lib.coopt_paged_gqa_decode_scheduled.argtypes = [vp, vp, i64p, vp, vp, vp, vp, vp, vp, vp, vp,
                                                         ctypes.c_size_t, vp, ctypes.c_size_t, shp, vp]
        lib.coopt_stream_read_probe.argtypes = [vp, ctypes.c_size_t, i32, vp, vp]
        lib.coopt_status_string.argtypes = [ctypes.c_int]
        lib.coopt_status_string.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("coopt_decode_workspace_bytes", "coopt_decode_schedule_bytes", "coopt_status_string",
                            "coopt_get_decode_plan"):
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().coopt_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise CooptError(f"{what}: status {status} ({status_string(status)})")


def _ptr(t) -> Optional[int]:
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def kv_cache_write_fp8(k, v, slot_mapping, k_cache, v_cache, k_scale, v_scale, shape: Shape,
                       stream=None) -> None:
    _check(load_library().coopt_kv_cache_write_fp8(
        _ptr(k), _ptr(v), _ptr(slot_mapping), int(slot_mapping.numel()), _ptr(k_cache),
        _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), ctypes.byref(shape), _stream(stream)),
        "coopt_kv_cache_write_fp8")


def kv_cache_write_skipset(k, v, slot_mapping, skip_set, k_cache, v_cache, k_scale, v_scale,
                           shape: Shape, stream=None) -> None:
    """skip_set: device uint32 bitmap over the call's token indices, or None."""
    _check(load_library().coopt_kv_cache_write_skipset(
        _ptr(k), _ptr(v), _ptr(slot_mapping), _ptr(skip_set), int(slot_mapping.numel()),
        _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), ctypes.byref(shape),
        _stream(stream)), "coopt_kv_cache_write_skipset")


def kv_cache_write_fp16(k, v, slot_mapping, k_cache, v_cache, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_kv_cache_write_fp16(
        _ptr(k), _ptr(v), _ptr(slot_mapping), int(slot_mapping.numel()), _ptr(k_cache),
        _ptr(v_cache), ctypes.byref(shape), _stream(stream)), "coopt_kv_cache_write_fp16")


def decode_workspace_bytes(shape: Shape) -> int:
    return int(load_library().coopt_decode_workspace_bytes(ctypes.byref(shape)))


def get_decode_plan() -> dict:
    """The plan currently in force, as a dict of the fields of ``coopt_decode_plan``."""
    p = DecodePlan()
    load_library().coopt_get_decode_plan(ctypes.byref(p))
    return {name: int(getattr(p, name)) for name, _ in DecodePlan._fields_}


def set_decode_plan(**fields) -> None:
    """Update the named fields of the plan (see ``coopt_decode_plan``); the others keep their value."""
    cur = get_decode_plan()
    for k in fields:
        if k not in cur:
            raise KeyError(k)
    cur.update(fields)
    p = DecodePlan(*[cur[name] for name, _ in DecodePlan._fields_])
    _check(load_library().coopt_set_decode_plan(ctypes.byref(p)), "coopt_set_decode_plan")


def paged_gqa_decode(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, out,
                     workspace, shape: Shape, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().coopt_paged_gqa_decode(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), _ptr(block_tables),
        _ptr(context_lens), _ptr(out), _ptr(workspace), ctypes.c_size_t(nbytes),
        ctypes.byref(shape), _stream(stream)), "coopt_paged_gqa_decode")


def paged_gqa_decode_step(k, v, slot_mapping, q, k_cache, v_cache, k_scale, v_scale, block_tables,
                          context_lens, out, workspace, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_paged_gqa_decode_step(
        _ptr(k), _ptr(v), _ptr(slot_mapping), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale),
        _ptr(v_scale), _ptr(block_tables), _ptr(context_lens), _ptr(out), _ptr(workspace),
        ctypes.c_size_t(workspace.numel() * workspace.element_size()), ctypes.byref(shape),
        _stream(stream)), "coopt_paged_gqa_decode_step")


def paged_gqa_decode_split(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                           workspace, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_paged_gqa_decode_split(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), _ptr(block_tables),
        _ptr(context_lens), _ptr(workspace),
        ctypes.c_size_t(workspace.numel() * workspace.element_size()), ctypes.byref(shape),
        _stream(stream)), "coopt_paged_gqa_decode_split")


def paged_gqa_decode_merge(context_lens, workspace, out, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_paged_gqa_decode_merge(
        _ptr(context_lens), _ptr(workspace),
        ctypes.c_size_t(workspace.numel() * workspace.element_size()), _ptr(out),
        ctypes.byref(shape), _stream(stream)), "coopt_paged_gqa_decode_merge")


def paged_gqa_decode_partitioned(q, k_cache, v_cache, k_scale, v_scale, block_tables,
                                 context_lens, partition_size: int, tmp_out, max_logits, exp_sums,
                                 max_parts: int, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_paged_gqa_decode_partitioned(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), _ptr(block_tables),
        _ptr(context_lens), int(partition_size), _ptr(tmp_out), _ptr(max_logits), _ptr(exp_sums),
        int(max_parts), ctypes.byref(shape), _stream(stream)), "coopt_paged_gqa_decode_partitioned")


def paged_gqa_reduce(tmp_out, max_logits, exp_sums, context_lens, partition_size: int,
                     max_parts: int, out, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_paged_gqa_reduce(
        _ptr(tmp_out), _ptr(max_logits), _ptr(exp_sums), _ptr(context_lens), int(partition_size),
        int(max_parts), _ptr(out), ctypes.byref(shape), _stream(stream)), "coopt_paged_gqa_reduce")


def paged_gqa_prefill_chunk(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                            query_start, num_query_rows: int, max_chunk_len: int, out,
                            shape: Shape, stream=None) -> None:
    _check(load_library().coopt_paged_gqa_prefill_chunk(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), _ptr(block_tables),
        _ptr(context_lens), _ptr(query_start), int(num_query_rows), int(max_chunk_len), _ptr(out),
        ctypes.byref(shape), _stream(stream)), "coopt_paged_gqa_prefill_chunk")


def decode_schedule_bytes(shape: Shape) -> int:
    return int(load_library().coopt_decode_schedule_bytes(ctypes.byref(shape)))


def decode_schedule_prepare(block_tables, context_lens, slot_mapping, schedule, shape: Shape,
                            stream=None) -> None:
    """Write the decode schedule (``slot_mapping`` None: plain decode; else the fused step)."""
    _check(load_library().coopt_decode_schedule_prepare(
        _ptr(block_tables), _ptr(context_lens), _ptr(slot_mapping), _ptr(schedule),
        schedule.numel() * schedule.element_size(), ctypes.byref(shape), _stream(stream)),
        "coopt_decode_schedule_prepare")


def paged_gqa_decode_scheduled(k, v, slot_mapping, q, k_cache, v_cache, k_scale, v_scale, context_lens,
                               out, workspace, schedule, shape: Shape, stream=None) -> None:
    """Decode (k, v, slot_mapping None) or fused step from a prepared schedule; ``out`` None stops
    after the partial results."""
    _check(load_library().coopt_paged_gqa_decode_scheduled(
        _ptr(k), _ptr(v), _ptr(slot_mapping), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale),
        _ptr(v_scale), _ptr(context_lens), _ptr(out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _ptr(schedule),
        schedule.numel() * schedule.element_size(), ctypes.byref(shape), _stream(stream)),
        "coopt_paged_gqa_decode_scheduled")


def stream_read_probe(buf, workgroups: int, sink, stream=None) -> None:
    """One streaming read of the whole tensor ``buf`` (measurement aid)."""
    _check(load_library().coopt_stream_read_probe(
        _ptr(buf), buf.numel() * buf.element_size(), int(workgroups), _ptr(sink), _stream(stream)),
        "coopt_stream_read_probe")


def gather_cached_kv(k_cache, v_cache, k_scale, v_scale, block_tables, seq: int, tok_begin: int,
                     tok_end: int, k_out, v_out, shape: Shape, stream=None) -> None:
    _check(load_library().coopt_gather_cached_kv(
        _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale), _ptr(block_tables), int(seq),
        int(tok_begin), int(tok_end), _ptr(k_out), _ptr(v_out), ctypes.byref(shape),
        _stream(stream)), "coopt_gather_cached_kv")
