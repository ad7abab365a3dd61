"""Test-side helpers.  Independent restatements used to pin the oracle live here, not in oracle/."""
import numpy as np
import torch


def e4m3_table() -> np.ndarray:
    """All 256 OCP E4M3 values as float64, decoded by torch's float8_e4m3fn (a library)."""
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def k_tile_index(d, E, B=16):
    """Element offsets [tok, dim] inside a K tile: 16-byte chunks of a token's row, chunk-major
    ([d/E][B][E]); E = elements per 16 bytes.  Restated from the public header, not from the oracle."""
    tok, dim = np.meshgrid(np.arange(B), np.arange(d), indexing="ij")
    return ((dim // E) * B + tok) * E + dim % E


def v_tile_index(d, E, B=16):
    """Element offsets [tok, dim] inside a V tile ([d/(4E)][B/4][16][E/4][4], tokens innermost)."""
    tok, dim = np.meshgrid(np.arange(B), np.arange(d), indexing="ij")
    W, c, n = E // 4, dim // 16, dim % 16
    return ((((c // W) * (B // 4) + tok // 4) * 16 + n) * W + c % W) * 4 + tok % 4


def _E(w):
    return 8 if w.kv_dtype == "fp16" else 16


def k_logical(w, k_cache):
    """[NB, H_k, B, d] copy of the K cache in plain (token, dim) order."""
    return k_cache.reshape(w.NB, w.H_k, w.B * w.d)[:, :, k_tile_index(w.d, _E(w), w.B)]


def v_logical(w, v_cache):
    """[NB, H_k, B, d] copy of the V cache in plain (token, dim) order."""
    return v_cache.reshape(w.NB, w.H_k, w.B * w.d)[:, :, v_tile_index(w.d, _E(w), w.B)]


def k_store_logical(w, k_cache, logical):
    k_cache.reshape(w.NB, w.H_k, w.B * w.d)[:, :, k_tile_index(w.d, _E(w), w.B)] = logical


def v_store_logical(w, v_cache, logical):
    v_cache.reshape(w.NB, w.H_k, w.B * w.d)[:, :, v_tile_index(w.d, _E(w), w.B)] = logical


def alloc_cache(w, fill_byte=None):
    """Empty paged cache for workload ``w`` (numpy, host): tiles of B*d elements per (block, head)
    in the boundary's tile order, scales [NB, H_k, B]."""
    dt = np.float16 if w.kv_dtype == "fp16" else np.uint8
    k_cache = np.zeros((w.NB, w.H_k, w.B * w.d), dtype=dt)
    v_cache = np.zeros((w.NB, w.H_k, w.B * w.d), dtype=dt)
    k_scale = v_scale = None
    if w.kv_dtype != "fp16":
        k_scale = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32)
        v_scale = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32)
    if fill_byte is not None:
        k_cache.view(np.uint8)[...] = fill_byte
        v_cache.view(np.uint8)[...] = fill_byte
        if k_scale is not None:
            k_scale[...] = np.float32(np.nan)
            v_scale[...] = np.float32(np.nan)
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
    elif w.kv_dtype == "e5m2":
        oracle.kv_cache_write_fp8_scaled(k, v, slots, k_cache, v_cache, k_scale, v_scale,
                                         H_k=w.H_k, d=w.d, B=w.B, fmt="e5m2", scale_mode="token")
    else:
        oracle.kv_cache_write_fp16(k, v, slots, k_cache, v_cache, H_k=w.H_k, d=w.d, B=w.B)
    return cache


def gather_dequant(w, cache, s):
    """Contiguous dequantised K, V [t, H_k, d] float64 of sequence s, by direct indexing."""
    k_cache, v_cache, k_scale, v_scale = cache
    kl, vl = k_logical(w, k_cache), v_logical(w, v_cache)
    t = int(w.context_lens[s])
    K = np.zeros((t, w.H_k, w.d)); V = np.zeros((t, w.H_k, w.d))
    table = e4m3_table()
    for j in range(t):
        pb = int(w.block_tables[s, j // w.B]); off = j % w.B
        if w.kv_dtype == "e4m3":
            K[j] = table[kl[pb, :, off, :]] * k_scale[pb, :, off].astype(np.float64)[:, None]
            V[j] = table[vl[pb, :, off, :]] * v_scale[pb, :, off].astype(np.float64)[:, None]
        else:
            K[j] = kl[pb, :, off, :].astype(np.float64)
            V[j] = vl[pb, :, off, :].astype(np.float64)
    return K, V


def softmax_attention(q, K, V, scale):
    """Textbook single-query attention, float64: q [d], K,V [t, d]."""
    z = (K @ q) * scale
    z = z - z.max()
    p = np.exp(z)
    p /= p.sum()
    return p @ V
