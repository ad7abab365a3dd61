"""TEST INFRASTRUCTURE (not part of the product path): the cache-quantisation schemes the paper's
Opt-KV is set against, for measuring what its choice buys in attention error at equal cache bytes.

Opt-KV stores K/V in FP8 and dequantises on read (Eq. 6); this build reads "FP8" as OCP E4M3 with
a dynamic scale per (token, KV head).  The alternatives below quantise the same rows with
  * "static"     one scale per KV head for the whole cache, fixed in advance from a calibration
                 sample (amax of the sample / format max), so later outliers saturate;
  * "per_block"  one scale per (16-token block, KV head): amax of the block / format max;
  * "per_token"  one scale per (token, KV head): amax of the row / format max (the scheme in use);
each with E4M3 (max 448, 3 mantissa bits) or E5M2 (max 57344, 2 mantissa bits) codes.  Every
function returns the DEQUANTISED rows in float64, i.e. what attention would read; rounding is to
nearest even on the format's grid with saturation at its largest finite value.  The scale
divisions are done in binary32 like the write path's.
"""
from __future__ import annotations

import numpy as np

from . import e4m3_encode_array

E4M3_MAX = 448.0
E5M2_MAX = 57344.0


def _e4m3_table() -> np.ndarray:
    t = np.zeros(256)
    for c in range(256):
        e, m = (c >> 3) & 15, c & 7
        v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        t[c] = -v if c & 0x80 else v
    return t


def _round_e4m3(y: np.ndarray) -> np.ndarray:
    """Nearest E4M3 value (ties to even, saturating) of binary32 values, via the oracle's encoder."""
    codes = e4m3_encode_array(np.ascontiguousarray(y, dtype=np.float32).reshape(-1))
    return _e4m3_table()[codes].reshape(y.shape)


def _round_e5m2(y: np.ndarray) -> np.ndarray:
    """Nearest E5M2 value: the fp16 grid cut to 2 mantissa bits, ties to even, saturating at
    57344; below the fp16 normal range the spacing is the subnormal one (2^-16)."""
    y = np.clip(np.asarray(y, dtype=np.float64), -E5M2_MAX, E5M2_MAX)
    mag = np.abs(y)
    e = np.floor(np.log2(np.maximum(mag, 2.0 ** -14)))
    step = 2.0 ** (e - 2)
    return np.sign(y) * np.round(mag / step) * step      # np.round is round-half-even


def quantise_rows(x: np.ndarray, scheme: str, fmt: str, calib: np.ndarray | None = None,
                  block: int = 16) -> np.ndarray:
    """x: [tokens, heads, d] fp16 rows in logical order -> dequantised float64 rows."""
    fmax = np.float32(E4M3_MAX if fmt == "e4m3" else E5M2_MAX)
    rnd = _round_e4m3 if fmt == "e4m3" else _round_e5m2
    xf = x.astype(np.float32)
    T, H, d = xf.shape
    if scheme == "per_token":
        amax = np.abs(xf).max(axis=2, keepdims=True)
    elif scheme == "per_block":
        amax = np.zeros((T, H, 1), np.float32)
        for b0 in range(0, T, block):
            amax[b0:b0 + block] = np.abs(xf[b0:b0 + block]).max(axis=(0, 2), keepdims=True)
    elif scheme == "static":
        amax = np.broadcast_to(np.abs(calib.astype(np.float32)).max(axis=(0, 2), keepdims=True), (T, H, 1))
    else:
        raise ValueError(scheme)
    scale = np.where(amax == 0, np.float32(1), (amax / fmax).astype(np.float32)).astype(np.float32)
    y = np.clip((xf / scale).astype(np.float32), -fmax, fmax)
    return rnd(y) * scale.astype(np.float64)


def attention_error(q: np.ndarray, K: np.ndarray, V: np.ndarray, Kq: np.ndarray, Vq: np.ndarray,
                    G: int, softmax_scale: float) -> tuple[float, float]:
    """Max-abs and RMS difference between attention over (Kq, Vq) and over the unquantised (K, V),
    all query heads (q: [H_q, d]; K, V: [t, H_k, d]; head h reads KV head h // G)."""
    def attend(Kx, Vx):
        out = np.zeros((q.shape[0], K.shape[2]))
        for h in range(q.shape[0]):
            g = h // G
            z = (Kx[:, g, :] @ q[h].astype(np.float64)) * softmax_scale
            p = np.exp(z - z.max())
            out[h] = (p / p.sum()) @ Vx[:, g, :]
        return out
    diff = attend(Kq, Vq) - attend(K.astype(np.float64), V.astype(np.float64))
    return float(np.abs(diff).max()), float(np.sqrt(np.mean(diff ** 2)))
