"""Test-side helpers.  Independent restatements used to pin the oracle live here, not in oracle/."""
import numpy as np
import torch


def e4m3_table() -> np.ndarray:
    """All 256 OCP E4M3 values as float64, decoded by torch's float8_e4m3fn (a library)."""
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def alloc_cache(w, fill_byte=None):
    """Empty paged cache for workload ``w`` in the boundary layouts (numpy, host)."""
    if w.kv_dtype == "e4m3":
        k_cache = np.zeros((w.NB, w.H_k, w.B, w.d), dtype=np.uint8)
        v_cache = np.zeros((w.NB, w.H_k, w.d, w.B), dtype=np.uint8)
        k_scale = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32)
        v_scale = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32)
        if fill_byte is not None:
            k_cache[...] = fill_byte
            v_cache[...] = fill_byte
            k_scale[...] = np.float32(np.nan)
            v_scale[...] = np.float32(np.nan)
    else:
        k_cache = np.zeros((w.NB, w.H_k, w.B, w.d), dtype=np.float16)
        v_cache = np.zeros((w.NB, w.H_k, w.d, w.B), dtype=np.float16)
        k_scale = v_scale = None
        if fill_byte is not None:
            k_cache.view(np.uint8)[...] = fill_byte
            v_cache.view(np.uint8)[...] = fill_byte
    return k_cache, v_cache, k_scale, v_scale


def oracle_fill(oracle, w, idx=None, cache=None):
    """Write tokens ``idx`` of ``w`` (default: all) through the oracle's write path."""
    if cache is None:
        cache = alloc_cache(w)
    k_cache, v_cache, k_scale, v_scale = cache
    if idx is None:
        k, v, slots = w.k_ctx, w.v_ctx, w.slots
    else:
        k = np.ascontiguousarray(w.k_ctx[idx]); v = np.ascontiguousarray(w.v_ctx[idx])
        slots = np.ascontiguousarray(w.slots[idx])
    if w.kv_dtype == "e4m3":
        oracle.kv_cache_write_fp8(k, v, slots, k_cache, v_cache, k_scale, v_scale,
                                  H_k=w.H_k, d=w.d, B=w.B)
    else:
        oracle.kv_cache_write_fp16(k, v, slots, k_cache, v_cache, H_k=w.H_k, d=w.d, B=w.B)
    return cache


def gather_dequant(w, cache, s):
    """Contiguous dequantised K, V [t, H_k, d] float64 of sequence s, by direct indexing."""
    k_cache, v_cache, k_scale, v_scale = cache
    t = int(w.context_lens[s])
    K = np.zeros((t, w.H_k, w.d)); V = np.zeros((t, w.H_k, w.d))
    table = e4m3_table()
    for j in range(t):
        pb = int(w.block_tables[s, j // w.B]); off = j % w.B
        if w.kv_dtype == "e4m3":
            K[j] = table[k_cache[pb, :, off, :]] * k_scale[pb, :, off].astype(np.float64)[:, None]
            V[j] = table[v_cache[pb, :, :, off]] * v_scale[pb, :, off].astype(np.float64)[:, None]
        else:
            K[j] = k_cache[pb, :, off, :].astype(np.float64)
            V[j] = v_cache[pb, :, :, off].astype(np.float64)
    return K, V


def softmax_attention(q, K, V, scale):
    """Textbook single-query attention, float64: q [d], K,V [t, d]."""
    z = (K @ q) * scale
    z = z - z.max()
    p = np.exp(z)
    p /= p.sum()
    return p @ V
