"""ctypes front end of the float64 CPU oracle (``coopt_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's cpu_baseline leg are
the only callers.  Nothing here touches the HIP library, and the HIP library never touches
this package.  Arrays are numpy; fp16 tensors travel as ``float16`` arrays and are handed to
C as their bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "coopt_oracle.c")
_LIB = os.path.join(_HERE, "libcoopt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_f16_to_f64.restype = ctypes.c_double
        _lib.orc_f16_to_f64.argtypes = [ctypes.c_uint16]
        _lib.orc_e4m3_to_f64.restype = ctypes.c_double
        _lib.orc_e4m3_to_f64.argtypes = [ctypes.c_uint8]
        _lib.orc_f32_to_e4m3.restype = ctypes.c_uint8
        _lib.orc_f32_to_e4m3.argtypes = [ctypes.c_float]
        _lib.orc_e5m2_to_f64.restype = ctypes.c_double
        _lib.orc_e5m2_to_f64.argtypes = [ctypes.c_uint8]
        _lib.orc_f32_to_e5m2.restype = ctypes.c_uint8
        _lib.orc_f32_to_e5m2.argtypes = [ctypes.c_float]
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk_dim(d, fp8):
    """The tile layouts need whole 16-byte chunks and whole V load groups."""
    if d % (64 if fp8 else 32) != 0:
        raise ValueError(f"head_dim {d} does not fit the cache tile layout")


def _chk(a, dtype, name):
    if a.dtype != np.dtype(dtype) or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need C-contiguous {np.dtype(dtype)}, got {a.dtype}")
    return a


def num_threads() -> int:
    return int(_load().orc_num_threads())


def e4m3_decode(code: int) -> float:
    return float(_load().orc_e4m3_to_f64(int(code) & 0xFF))


def e4m3_encode(y) -> int:
    return int(_load().orc_f32_to_e4m3(ctypes.c_float(float(np.float32(y)))))


def e4m3_encode_array(y: np.ndarray) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float32)
    lib = _load()
    out = np.empty(y.shape, dtype=np.uint8)
    lib.orc_f32_to_e4m3_array(_p(y), _p(out), ctypes.c_size_t(y.size))
    return out


def e5m2_decode(code: int) -> float:
    return float(_load().orc_e5m2_to_f64(int(code) & 0xFF))


def e5m2_encode(y) -> int:
    return int(_load().orc_f32_to_e5m2(ctypes.c_float(float(np.float32(y)))))


def e5m2_encode_array(y: np.ndarray) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float32)
    out = np.empty(y.shape, dtype=np.uint8)
    _load().orc_f32_to_e5m2_array(_p(y), _p(out), ctypes.c_size_t(y.size))
    return out


KV_DTYPES = {"fp16": 0, "e4m3": 1, "e5m2": 2}
SCALE_MODES = {"token": 0, "block": 1, "static": 2}


def f16_to_f64(bits: int) -> float:
    return float(_load().orc_f16_to_f64(int(bits) & 0xFFFF))


def _skip_bitmap(skip_set, T):
    """SkipSet of Eq. 5 as the C side takes it: uint32 words, bit i%32 of word i/32 = token i."""
    if skip_set is None:
        return None
    bits = np.zeros((T + 31) // 32, dtype=np.uint32)
    for i in skip_set:
        assert 0 <= int(i) < T
        bits[int(i) >> 5] |= np.uint32(1 << (int(i) & 31))
    return bits


def kv_cache_write_fp8(k, v, slot_mapping, k_cache, v_cache, k_scale, v_scale, *, H_k, d, B,
                       skip_set=None):
    """skip_set: iterable of token indices of this call that are not to be written (Eq. 5)."""
    _chk(k, np.float16, "k"); _chk(v, np.float16, "v"); _chk(slot_mapping, np.int64, "slot_mapping")
    _chk(k_cache, np.uint8, "k_cache"); _chk(v_cache, np.uint8, "v_cache")
    _chk(k_scale, np.float32, "k_scale"); _chk(v_scale, np.float32, "v_scale")
    T = int(slot_mapping.shape[0])
    assert k.size == T * H_k * d and v.size == T * H_k * d
    _chk_dim(d, True)
    bits = _skip_bitmap(skip_set, T)
    _load().orc_kv_cache_write_fp8(_p(k), _p(v), _p(slot_mapping), _p(bits), ctypes.c_int(T),
                                   _p(k_cache), _p(v_cache), _p(k_scale), _p(v_scale),
                                   ctypes.c_int(H_k), ctypes.c_int(d), ctypes.c_int(B))


def kv_cache_write_fp8_scaled(k, v, slot_mapping, k_cache, v_cache, k_scale, v_scale, *, H_k, d, B,
                              fmt="e4m3", scale_mode="token", k_static=None, v_static=None,
                              skip_set=None):
    """The write under another code ("e4m3" / "e5m2") and scale rule ("token" / "block" / "static";
    static needs k_static, v_static: float32 [H_k])."""
    _chk(k, np.float16, "k"); _chk(v, np.float16, "v"); _chk(slot_mapping, np.int64, "slot_mapping")
    _chk(k_cache, np.uint8, "k_cache"); _chk(v_cache, np.uint8, "v_cache")
    _chk(k_scale, np.float32, "k_scale"); _chk(v_scale, np.float32, "v_scale")
    T = int(slot_mapping.shape[0])
    assert k.size == T * H_k * d and v.size == T * H_k * d
    _chk_dim(d, True)
    if scale_mode == "static":
        _chk(k_static, np.float32, "k_static"); _chk(v_static, np.float32, "v_static")
        assert k_static.size == H_k and v_static.size == H_k
    bits = _skip_bitmap(skip_set, T)
    _load().orc_kv_cache_write_fp8_scaled(
        _p(k), _p(v), _p(slot_mapping), _p(bits), ctypes.c_int(T), _p(k_cache), _p(v_cache),
        _p(k_scale), _p(v_scale), ctypes.c_int(H_k), ctypes.c_int(d), ctypes.c_int(B),
        ctypes.c_int(KV_DTYPES[fmt]), ctypes.c_int(SCALE_MODES[scale_mode]), _p(k_static), _p(v_static))


def kv_cache_write_fp16(k, v, slot_mapping, k_cache, v_cache, *, H_k, d, B, skip_set=None):
    _chk(k, np.float16, "k"); _chk(v, np.float16, "v"); _chk(slot_mapping, np.int64, "slot_mapping")
    _chk(k_cache, np.float16, "k_cache"); _chk(v_cache, np.float16, "v_cache")
    T = int(slot_mapping.shape[0])
    assert k.size == T * H_k * d and v.size == T * H_k * d
    _chk_dim(d, False)
    bits = _skip_bitmap(skip_set, T)
    _load().orc_kv_cache_write_fp16(_p(k), _p(v), _p(slot_mapping), _p(bits), ctypes.c_int(T),
                                    _p(k_cache), _p(v_cache), ctypes.c_int(H_k), ctypes.c_int(d),
                                    ctypes.c_int(B))


def _cache_args(k_cache, v_cache, k_scale, v_scale, fmt="e4m3"):
    """kv_dtype for the C side: fp16 caches by their dtype, one-byte caches by ``fmt``."""
    if k_cache.dtype == np.uint8:
        _chk(k_cache, np.uint8, "k_cache"); _chk(v_cache, np.uint8, "v_cache")
        _chk(k_scale, np.float32, "k_scale"); _chk(v_scale, np.float32, "v_scale")
        return KV_DTYPES[fmt]
    _chk(k_cache, np.float16, "k_cache"); _chk(v_cache, np.float16, "v_cache")
    return 0


def paged_gqa_decode(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, *,
                     H_q, H_k, d, B, softmax_scale, fmt="e4m3") -> np.ndarray:
    _chk(q, np.float16, "q"); _chk(block_tables, np.int32, "block_tables")
    _chk(context_lens, np.int32, "context_lens")
    kv_dtype = _cache_args(k_cache, v_cache, k_scale, v_scale, fmt)
    S = int(context_lens.shape[0])
    out = np.zeros((S, H_q, d), dtype=np.float64)
    _load().orc_paged_gqa_decode(_p(q), _p(k_cache), _p(v_cache), _p(k_scale), _p(v_scale),
                                 _p(block_tables), _p(context_lens), _p(out), ctypes.c_int(S),
                                 ctypes.c_int(H_q), ctypes.c_int(H_k), ctypes.c_int(d),
                                 ctypes.c_int(B), ctypes.c_int(block_tables.shape[1]),
                                 ctypes.c_int(kv_dtype), ctypes.c_double(float(np.float32(softmax_scale))))
    return out


def paged_gqa_decode_partitioned(q, k_cache, v_cache, k_scale, v_scale, block_tables,
                                 context_lens, partition_size, max_parts, *, H_q, H_k, d, B,
                                 softmax_scale, fmt="e4m3"):
    """Returns (tmp_out, max_logits, exp_sums); rows of unused partitions are NaN."""
    _chk(q, np.float16, "q"); _chk(block_tables, np.int32, "block_tables")
    _chk(context_lens, np.int32, "context_lens")
    kv_dtype = _cache_args(k_cache, v_cache, k_scale, v_scale, fmt)
    S = int(context_lens.shape[0])
    tmp_out = np.full((S, H_q, max_parts, d), np.nan, dtype=np.float64)
    max_logits = np.full((S, H_q, max_parts), np.nan, dtype=np.float64)
    exp_sums = np.full((S, H_q, max_parts), np.nan, dtype=np.float64)
    _load().orc_paged_gqa_decode_partitioned(
        _p(q), _p(k_cache), _p(v_cache), _p(k_scale), _p(v_scale), _p(block_tables),
        _p(context_lens), ctypes.c_int(partition_size), ctypes.c_int(max_parts), _p(tmp_out),
        _p(max_logits), _p(exp_sums), ctypes.c_int(S), ctypes.c_int(H_q), ctypes.c_int(H_k),
        ctypes.c_int(d), ctypes.c_int(B), ctypes.c_int(block_tables.shape[1]),
        ctypes.c_int(kv_dtype), ctypes.c_double(float(np.float32(softmax_scale))))
    return tmp_out, max_logits, exp_sums


def paged_gqa_reduce(tmp_out, max_logits, exp_sums, context_lens, partition_size) -> np.ndarray:
    _chk(tmp_out, np.float64, "tmp_out"); _chk(max_logits, np.float64, "max_logits")
    _chk(exp_sums, np.float64, "exp_sums"); _chk(context_lens, np.int32, "context_lens")
    S, H_q, max_parts, d = tmp_out.shape
    out = np.zeros((S, H_q, d), dtype=np.float64)
    _load().orc_paged_gqa_reduce(_p(tmp_out), _p(max_logits), _p(exp_sums), _p(context_lens),
                                 ctypes.c_int(partition_size), ctypes.c_int(max_parts), _p(out),
                                 ctypes.c_int(S), ctypes.c_int(H_q), ctypes.c_int(d))
    return out


def paged_gqa_prefill_chunk(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                            query_start, *, H_q, H_k, d, B, softmax_scale, rows=None,
                            fmt="e4m3") -> np.ndarray:
    _chk(q, np.float16, "q"); _chk(block_tables, np.int32, "block_tables")
    _chk(context_lens, np.int32, "context_lens"); _chk(query_start, np.int32, "query_start")
    kv_dtype = _cache_args(k_cache, v_cache, k_scale, v_scale, fmt)
    S = int(context_lens.shape[0])
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        n = int(rows.shape[0])
    else:
        n = int(query_start[S])
    out = np.zeros((n, H_q, d), dtype=np.float64)
    _load().orc_paged_gqa_prefill_chunk(
        _p(q), _p(k_cache), _p(v_cache), _p(k_scale), _p(v_scale), _p(block_tables),
        _p(context_lens), _p(query_start), _p(rows), ctypes.c_int(n), _p(out), ctypes.c_int(S),
        ctypes.c_int(H_q), ctypes.c_int(H_k), ctypes.c_int(d), ctypes.c_int(B),
        ctypes.c_int(block_tables.shape[1]), ctypes.c_int(kv_dtype),
        ctypes.c_double(float(np.float32(softmax_scale))))
    return out


def gather_cached_kv(k_cache, v_cache, k_scale, v_scale, block_tables, s, j0, j1, *, H_k, d, B,
                     fmt="e4m3"):
    _chk(block_tables, np.int32, "block_tables")
    kv_dtype = _cache_args(k_cache, v_cache, k_scale, v_scale, fmt)
    n = max(0, j1 - j0)
    k_out = np.zeros((n, H_k, d), dtype=np.float64)
    v_out = np.zeros((n, H_k, d), dtype=np.float64)
    _load().orc_gather_cached_kv(_p(k_cache), _p(v_cache), _p(k_scale), _p(v_scale),
                                 _p(block_tables), ctypes.c_int(s), ctypes.c_int(j0),
                                 ctypes.c_int(j1), _p(k_out), _p(v_out), ctypes.c_int(H_k),
                                 ctypes.c_int(d), ctypes.c_int(B),
                                 ctypes.c_int(block_tables.shape[1]), ctypes.c_int(kv_dtype))
    return k_out, v_out
