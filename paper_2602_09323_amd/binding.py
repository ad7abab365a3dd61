"""ctypes binding of the C ABI in ``include/coopt_attn.h``: same names, argument marshalling only.

Tensors are torch CUDA(HIP) tensors used purely as device memory; every step of the path runs in
the library's own kernels on the current torch stream.  If the shared library is missing the
binding raises: there is no fallback path.

The C side takes raw pointers and cannot see a buffer's size, type or residence, so the binding
checks what it can before anything is launched: every tensor is a contiguous device tensor, index
tensors have the integer width the kernels read (int64 slots, int32 tables / lengths / row
offsets), fp16 operands have 2-byte elements, and every buffer holds at least the bytes the shape
implies.  A violation raises ``CooptError``.
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
COOPT_KV_E5M2 = 2
COOPT_SCALE_TOKEN = 0
COOPT_SCALE_BLOCK = 1
COOPT_SCALE_STATIC = 2

EXPORTS = [
    "coopt_kv_cache_write_fp8", "coopt_kv_cache_write_fp16", "coopt_kv_cache_write_skipset",
    "coopt_kv_cache_write_fp8_scaled",
    "coopt_paged_gqa_decode", "coopt_paged_gqa_decode_step", "coopt_paged_gqa_decode_split",
    "coopt_paged_gqa_decode_merge", "coopt_decode_workspace_bytes", "coopt_default_decode_plan",
    "coopt_paged_gqa_decode_partitioned", "coopt_paged_gqa_reduce", "coopt_paged_gqa_prefill_chunk",
    "coopt_gather_cached_kv", "coopt_decode_schedule_bytes", "coopt_decode_schedule_prepare",
    "coopt_paged_gqa_decode_scheduled", "coopt_status_string",
    "coopt_paged_gqa_decode_noalloc", "coopt_decode_builtin_workspace_bytes",
    "coopt_paged_gqa_prefill_chunk_ws", "coopt_prefill_workspace_bytes",
]


class CooptError(RuntimeError):
    pass


class DecodePlan(ctypes.Structure):
    """Mirror of ``coopt_decode_plan``."""
    _fields_ = [("tokens_per_group", ctypes.c_int32), ("waves_per_group", ctypes.c_int32),
                ("pipeline_depth", ctypes.c_int32), ("grid_waves", ctypes.c_int32),
                ("softmax_reduction", ctypes.c_int32)]

    def as_dict(self) -> dict:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


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
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        shp, plp = ctypes.POINTER(Shape), ctypes.POINTER(DecodePlan)
        lib.coopt_kv_cache_write_fp8.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, shp, vp]
        lib.coopt_kv_cache_write_fp8_scaled.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, shp, vp]
        lib.coopt_kv_cache_write_fp16.argtypes = [vp, vp, vp, i32, vp, vp, shp, vp]
        lib.coopt_kv_cache_write_skipset.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, shp, vp]
        lib.coopt_paged_gqa_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, plp, shp, vp]
        lib.coopt_paged_gqa_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz,
                                                    plp, shp, vp]
        lib.coopt_paged_gqa_decode_split.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, plp, shp, vp]
        lib.coopt_paged_gqa_decode_merge.argtypes = [vp, vp, sz, vp, plp, shp, vp]
        lib.coopt_decode_workspace_bytes.argtypes = [shp, plp]
        lib.coopt_decode_workspace_bytes.restype = sz
        lib.coopt_default_decode_plan.argtypes = [plp]
        lib.coopt_default_decode_plan.restype = None
        lib.coopt_paged_gqa_decode_partitioned.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp,
                                                           i32, plp, shp, vp]
        lib.coopt_paged_gqa_reduce.argtypes = [vp, vp, vp, vp, i32, i32, vp, shp, vp]
        lib.coopt_paged_gqa_prefill_chunk.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, shp, vp]
        lib.coopt_paged_gqa_prefill_chunk_ws.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, sz,
                                                         shp, vp]
        lib.coopt_prefill_workspace_bytes.argtypes = [shp, i32]
        lib.coopt_prefill_workspace_bytes.restype = sz
        lib.coopt_gather_cached_kv.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, shp, vp]
        lib.coopt_decode_schedule_bytes.argtypes = [shp, plp]
        lib.coopt_decode_schedule_bytes.restype = sz
        lib.coopt_decode_schedule_prepare.argtypes = [vp, vp, vp, vp, sz, plp, shp, vp]
        lib.coopt_paged_gqa_decode_scheduled.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz,
                                                         vp, sz, plp, shp, vp]
        lib.coopt_paged_gqa_decode_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, plp, shp, vp]
        lib.coopt_decode_builtin_workspace_bytes.argtypes = []
        lib.coopt_decode_builtin_workspace_bytes.restype = sz
        lib.coopt_status_string.argtypes = [ctypes.c_int]
        lib.coopt_status_string.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("coopt_decode_workspace_bytes", "coopt_decode_schedule_bytes",
                            "coopt_prefill_workspace_bytes",
                            "coopt_status_string", "coopt_default_decode_plan",
                            "coopt_decode_builtin_workspace_bytes"):
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().coopt_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise CooptError(f"{what}: status {status} ({status_string(status)})")


def _call(name: str, *args) -> None:
    """Enter the library: every argument has been checked and marshalled by now."""
    _check(getattr(load_library(), name)(*args), name)


# ---------------------------------------------------------------- argument checks (host, no launch)

def _nbytes(t) -> int:
    return int(t.numel()) * int(t.element_size())


def _dev(t, name: str, *, min_bytes: int = 0, elem: Optional[int] = None, dtype=None,
         optional: bool = False):
    """Pointer of a contiguous device tensor of at least ``min_bytes`` bytes, with ``elem``-byte
    elements or exactly ``dtype`` where given.  None passes as NULL only if ``optional``."""
    if t is None:
        if optional:
            return None
        raise CooptError(f"{name}: required tensor is None")
    if not getattr(t, "is_cuda", False):
        raise CooptError(f"{name}: not a device tensor")
    if not t.is_contiguous():
        raise CooptError(f"{name}: not contiguous")
    if dtype is not None and t.dtype != dtype:
        raise CooptError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if elem is not None and int(t.element_size()) != elem:
        raise CooptError(f"{name}: {t.element_size()}-byte elements, expected {elem}")
    if _nbytes(t) < min_bytes:
        raise CooptError(f"{name}: {_nbytes(t)} bytes, the shape needs {min_bytes}")
    return ctypes.c_void_p(t.data_ptr())


def _sizes(shape: Shape):
    es = 2 if shape.kv_dtype == COOPT_KV_FP16 else 1
    tiles = shape.num_blocks * shape.num_kv_heads
    return {"cache": tiles * shape.block_size * shape.head_dim * es,
            "scale": tiles * shape.block_size * 4,
            "q": shape.num_seqs * shape.num_q_heads * shape.head_dim * 2,
            "tables": shape.num_seqs * shape.max_blocks_per_seq * 4,
            "lens": shape.num_seqs * 4,
            "row": shape.num_kv_heads * shape.head_dim * 2,
            "scaled": shape.kv_dtype != COOPT_KV_FP16}


def _cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape: Shape):
    z = _sizes(shape)
    scaled = z["scaled"]
    return (_dev(k_cache, "k_cache", min_bytes=z["cache"]), _dev(v_cache, "v_cache", min_bytes=z["cache"]),
            _dev(k_scale, "k_scale", min_bytes=z["scale"], optional=not scaled),
            _dev(v_scale, "v_scale", min_bytes=z["scale"], optional=not scaled))


def _i32():
    import torch
    return torch.int32


def _i64():
    import torch
    return torch.int64


def _plan_ptr(plan: Optional[DecodePlan]):
    return None if plan is None else ctypes.byref(plan)


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _new_rows(k, v, slot_mapping, shape: Shape, what: str):
    """Pointers of new K/V rows [T][H_k][d] fp16 and their int64 slots; returns (pk, pv, ps, T)."""
    z = _sizes(shape)
    ps = _dev(slot_mapping, f"{what}: slot_mapping", dtype=_i64())
    T = int(slot_mapping.numel())
    return (_dev(k, f"{what}: k", elem=2, min_bytes=T * z["row"]),
            _dev(v, f"{what}: v", elem=2, min_bytes=T * z["row"]), ps, T)


# ---------------------------------------------------------------- plan

def default_decode_plan() -> DecodePlan:
    """The plan a call runs under when it is given none (``coopt_default_decode_plan``)."""
    p = DecodePlan()
    load_library().coopt_default_decode_plan(ctypes.byref(p))
    return p


def make_decode_plan(**fields) -> DecodePlan:
    """The default plan with the named fields of ``coopt_decode_plan`` replaced."""
    p = default_decode_plan()
    for k, val in fields.items():
        if k not in dict(DecodePlan._fields_):
            raise KeyError(k)
        setattr(p, k, int(val))
    return p


# ---------------------------------------------------------------- cache write

def kv_cache_write_fp8(k, v, slot_mapping, k_cache, v_cache, k_scale, v_scale, shape: Shape,
                       stream=None) -> None:
    pk, pv, ps, T = _new_rows(k, v, slot_mapping, shape, "kv_cache_write_fp8")
    _call("coopt_kv_cache_write_fp8",
          pk, pv, ps, T, *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape), ctypes.byref(shape),
        _stream(stream))


def kv_cache_write_fp8_scaled(k, v, slot_mapping, k_cache, v_cache, k_scale, v_scale, shape: Shape,
                              scale_mode: int, k_static=None, v_static=None, stream=None) -> None:
    """The write under another scale rule (COOPT_SCALE_*); k_static / v_static: device float32
    [H_k], required for COOPT_SCALE_STATIC only."""
    pk, pv, ps, T = _new_rows(k, v, slot_mapping, shape, "kv_cache_write_fp8_scaled")
    static = int(scale_mode) == COOPT_SCALE_STATIC
    hk = shape.num_kv_heads * 4
    _call("coopt_kv_cache_write_fp8_scaled",
          pk, pv, ps, T, *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape), int(scale_mode),
          _dev(k_static, "k_static", elem=4, min_bytes=hk, optional=not static),
          _dev(v_static, "v_static", elem=4, min_bytes=hk, optional=not static),
          ctypes.byref(shape), _stream(stream))


def kv_cache_write_skipset(k, v, slot_mapping, skip_set, k_cache, v_cache, k_scale, v_scale,
                           shape: Shape, stream=None) -> None:
    """skip_set: device uint32 bitmap over the call's token indices, or None."""
    pk, pv, ps, T = _new_rows(k, v, slot_mapping, shape, "kv_cache_write_skipset")
    pset = _dev(skip_set, "skip_set", min_bytes=(T + 31) // 32 * 4, elem=4, optional=True)
    _call("coopt_kv_cache_write_skipset",
          pk, pv, ps, pset, T, *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape),
        ctypes.byref(shape), _stream(stream))


def kv_cache_write_fp16(k, v, slot_mapping, k_cache, v_cache, shape: Shape, stream=None) -> None:
    pk, pv, ps, T = _new_rows(k, v, slot_mapping, shape, "kv_cache_write_fp16")
    pkc, pvc, _, _ = _cache_ptrs(k_cache, v_cache, None, None, shape)
    _call("coopt_kv_cache_write_fp16",
          pk, pv, ps, T, pkc, pvc, ctypes.byref(shape), _stream(stream))


# ---------------------------------------------------------------- decode

def decode_workspace_bytes(shape: Shape, plan: Optional[DecodePlan] = None) -> int:
    return int(load_library().coopt_decode_workspace_bytes(ctypes.byref(shape), _plan_ptr(plan)))


def _decode_inputs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, shape: Shape,
                   what: str):
    z = _sizes(shape)
    return (_dev(q, f"{what}: q", elem=2, min_bytes=z["q"]),
            *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape),
            _dev(block_tables, f"{what}: block_tables", dtype=_i32(), min_bytes=z["tables"]),
            _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]))


def _workspace(workspace, shape: Shape, plan, what: str, optional: bool = False):
    if workspace is None and optional:
        return None, 0
    need = decode_workspace_bytes(shape, plan)
    return _dev(workspace, f"{what}: workspace", min_bytes=need), ctypes.c_size_t(_nbytes(workspace))


def paged_gqa_decode(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, out,
                     workspace, shape: Shape, plan: Optional[DecodePlan] = None, stream=None) -> None:
    what = "paged_gqa_decode"
    ins = _decode_inputs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, shape, what)
    pws, nws = _workspace(workspace, shape, plan, what, optional=True)
    _call("coopt_paged_gqa_decode",
          *ins, _dev(out, f"{what}: out", elem=2, min_bytes=_sizes(shape)["q"]), pws, nws,
        _plan_ptr(plan), ctypes.byref(shape), _stream(stream))


def decode_builtin_workspace_bytes() -> int:
    return int(load_library().coopt_decode_builtin_workspace_bytes())


def paged_gqa_decode_noalloc(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, out,
                             shape: Shape, plan: Optional[DecodePlan] = None, stream=None) -> None:
    """``paged_gqa_decode`` through the library's built-in workspace (no allocation anywhere)."""
    what = "paged_gqa_decode_noalloc"
    ins = _decode_inputs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, shape, what)
    _call("coopt_paged_gqa_decode_noalloc",
          *ins, _dev(out, f"{what}: out", elem=2, min_bytes=_sizes(shape)["q"]), _plan_ptr(plan),
          ctypes.byref(shape), _stream(stream))


def paged_gqa_decode_step(k, v, slot_mapping, q, k_cache, v_cache, k_scale, v_scale, block_tables,
                          context_lens, out, workspace, shape: Shape,
                          plan: Optional[DecodePlan] = None, stream=None) -> None:
    what = "paged_gqa_decode_step"
    pk, pv, ps, T = _new_rows(k, v, slot_mapping, shape, what)
    if T < shape.num_seqs:
        raise CooptError(f"{what}: slot_mapping has {T} entries, the batch {shape.num_seqs} sequences")
    ins = _decode_inputs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, shape, what)
    pws, nws = _workspace(workspace, shape, plan, what)
    _call("coopt_paged_gqa_decode_step",
          pk, pv, ps, *ins, _dev(out, f"{what}: out", elem=2, min_bytes=_sizes(shape)["q"]), pws, nws,
        _plan_ptr(plan), ctypes.byref(shape), _stream(stream))


def paged_gqa_decode_split(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                           workspace, shape: Shape, plan: Optional[DecodePlan] = None,
                           stream=None) -> None:
    what = "paged_gqa_decode_split"
    ins = _decode_inputs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, shape, what)
    pws, nws = _workspace(workspace, shape, plan, what)
    _call("coopt_paged_gqa_decode_split",
          *ins, pws, nws, _plan_ptr(plan), ctypes.byref(shape), _stream(stream))


def paged_gqa_decode_merge(context_lens, workspace, out, shape: Shape,
                           plan: Optional[DecodePlan] = None, stream=None) -> None:
    what = "paged_gqa_decode_merge"
    z = _sizes(shape)
    pws, nws = _workspace(workspace, shape, plan, what)
    _call("coopt_paged_gqa_decode_merge",
          _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]), pws, nws,
        _dev(out, f"{what}: out", elem=2, min_bytes=z["q"]), _plan_ptr(plan), ctypes.byref(shape),
        _stream(stream))


def _partial_buffers(tmp_out, max_logits, exp_sums, max_parts: int, shape: Shape, what: str):
    rows = shape.num_seqs * shape.num_q_heads * int(max_parts)
    return (_dev(tmp_out, f"{what}: tmp_out", elem=4, min_bytes=rows * shape.head_dim * 4),
            _dev(max_logits, f"{what}: max_logits", elem=4, min_bytes=rows * 4),
            _dev(exp_sums, f"{what}: exp_sums", elem=4, min_bytes=rows * 4))


def paged_gqa_decode_partitioned(q, k_cache, v_cache, k_scale, v_scale, block_tables,
                                 context_lens, partition_size: int, tmp_out, max_logits, exp_sums,
                                 max_parts: int, shape: Shape, plan: Optional[DecodePlan] = None,
                                 stream=None) -> None:
    what = "paged_gqa_decode_partitioned"
    ins = _decode_inputs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, shape, what)
    _call("coopt_paged_gqa_decode_partitioned",
          *ins, int(partition_size), *_partial_buffers(tmp_out, max_logits, exp_sums, max_parts, shape, what),
        int(max_parts), _plan_ptr(plan), ctypes.byref(shape), _stream(stream))


def paged_gqa_reduce(tmp_out, max_logits, exp_sums, context_lens, partition_size: int,
                     max_parts: int, out, shape: Shape, stream=None) -> None:
    what = "paged_gqa_reduce"
    z = _sizes(shape)
    _call("coopt_paged_gqa_reduce",
          *_partial_buffers(tmp_out, max_logits, exp_sums, max_parts, shape, what),
        _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]),
        int(partition_size), int(max_parts), _dev(out, f"{what}: out", elem=2, min_bytes=z["q"]),
        ctypes.byref(shape), _stream(stream))


def paged_gqa_prefill_chunk(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                            query_start, num_query_rows: int, max_chunk_len: int, out,
                            shape: Shape, stream=None) -> None:
    what = "paged_gqa_prefill_chunk"
    z = _sizes(shape)
    rows_bytes = int(num_query_rows) * shape.num_q_heads * shape.head_dim * 2
    _call("coopt_paged_gqa_prefill_chunk",
          _dev(q, f"{what}: q", elem=2, min_bytes=rows_bytes),
        *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape),
        _dev(block_tables, f"{what}: block_tables", dtype=_i32(), min_bytes=z["tables"]),
        _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]),
        _dev(query_start, f"{what}: query_start", dtype=_i32(), min_bytes=z["lens"] + 4),
        int(num_query_rows), int(max_chunk_len),
        _dev(out, f"{what}: out", elem=2, min_bytes=rows_bytes), ctypes.byref(shape), _stream(stream))


def prefill_workspace_bytes(shape: Shape, max_chunk_len: int) -> int:
    return int(load_library().coopt_prefill_workspace_bytes(ctypes.byref(shape), int(max_chunk_len)))


def paged_gqa_prefill_chunk_ws(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                               query_start, num_query_rows: int, max_chunk_len: int, out, workspace,
                               shape: Shape, stream=None) -> None:
    """workspace: a device buffer of at least prefill_workspace_bytes(shape, max_chunk_len) bytes
    (None where that is 0)."""
    what = "paged_gqa_prefill_chunk_ws"
    z = _sizes(shape)
    rows_bytes = int(num_query_rows) * shape.num_q_heads * shape.head_dim * 2
    need = prefill_workspace_bytes(shape, max_chunk_len)
    pws, nws = (None, ctypes.c_size_t(0)) if workspace is None else (
        _dev(workspace, f"{what}: workspace", min_bytes=need), ctypes.c_size_t(_nbytes(workspace)))
    _call("coopt_paged_gqa_prefill_chunk_ws",
          _dev(q, f"{what}: q", elem=2, min_bytes=rows_bytes),
          *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape),
          _dev(block_tables, f"{what}: block_tables", dtype=_i32(), min_bytes=z["tables"]),
          _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]),
          _dev(query_start, f"{what}: query_start", dtype=_i32(), min_bytes=z["lens"] + 4),
          int(num_query_rows), int(max_chunk_len),
          _dev(out, f"{what}: out", elem=2, min_bytes=rows_bytes), pws, nws, ctypes.byref(shape),
          _stream(stream))


def decode_schedule_bytes(shape: Shape, plan: Optional[DecodePlan] = None) -> int:
    return int(load_library().coopt_decode_schedule_bytes(ctypes.byref(shape), _plan_ptr(plan)))


def decode_schedule_prepare(block_tables, context_lens, slot_mapping, schedule, shape: Shape,
                            plan: Optional[DecodePlan] = None, stream=None) -> None:
    """Write the decode schedule (``slot_mapping`` None: plain decode; else the fused step)."""
    what = "decode_schedule_prepare"
    z = _sizes(shape)
    _call("coopt_decode_schedule_prepare",
          _dev(block_tables, f"{what}: block_tables", dtype=_i32(), min_bytes=z["tables"]),
        _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]),
        _dev(slot_mapping, f"{what}: slot_mapping", dtype=_i64(), min_bytes=2 * z["lens"], optional=True),
        _dev(schedule, f"{what}: schedule", min_bytes=decode_schedule_bytes(shape, plan)),
        _nbytes(schedule), _plan_ptr(plan), ctypes.byref(shape), _stream(stream))


def paged_gqa_decode_scheduled(k, v, slot_mapping, q, k_cache, v_cache, k_scale, v_scale, context_lens,
                               out, workspace, schedule, shape: Shape,
                               plan: Optional[DecodePlan] = None, stream=None) -> None:
    """Decode (k, v, slot_mapping None) or fused step from a prepared schedule; ``out`` None stops
    after the partial results."""
    what = "paged_gqa_decode_scheduled"
    z = _sizes(shape)
    if k is None and v is None and slot_mapping is None:
        pk = pv = ps = None
    else:
        pk, pv, ps, T = _new_rows(k, v, slot_mapping, shape, what)
        if T < shape.num_seqs:
            raise CooptError(f"{what}: slot_mapping has {T} entries, the batch {shape.num_seqs} sequences")
    pws, nws = _workspace(workspace, shape, plan, what)
    _call("coopt_paged_gqa_decode_scheduled",
          pk, pv, ps, _dev(q, f"{what}: q", elem=2, min_bytes=z["q"]),
        *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape),
        _dev(context_lens, f"{what}: context_lens", dtype=_i32(), min_bytes=z["lens"]),
        _dev(out, f"{what}: out", elem=2, min_bytes=z["q"], optional=True), pws, nws,
        _dev(schedule, f"{what}: schedule", min_bytes=decode_schedule_bytes(shape, plan)),
        _nbytes(schedule), _plan_ptr(plan), ctypes.byref(shape), _stream(stream))


def gather_cached_kv(k_cache, v_cache, k_scale, v_scale, block_tables, seq: int, tok_begin: int,
                     tok_end: int, k_out, v_out, shape: Shape, stream=None) -> None:
    what = "gather_cached_kv"
    z = _sizes(shape)
    rows = max(int(tok_end) - int(tok_begin), 0) * z["row"]
    _call("coopt_gather_cached_kv",
          *_cache_ptrs(k_cache, v_cache, k_scale, v_scale, shape),
        _dev(block_tables, f"{what}: block_tables", dtype=_i32(), min_bytes=z["tables"]), int(seq),
        int(tok_begin), int(tok_end), _dev(k_out, f"{what}: k_out", elem=2, min_bytes=rows),
        _dev(v_out, f"{what}: v_out", elem=2, min_bytes=rows), ctypes.byref(shape),
        _stream(stream))
