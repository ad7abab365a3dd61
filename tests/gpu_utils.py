"""Helpers for the GPU parity tests: device buffers via torch, calls through the C-ABI binding."""
import numpy as np
import torch

import paper_2602_09323_amd as coopt

ABS_TOL = 2e-3      # max-abs bar for attention outputs (fp16 out vs float64 oracle)
REL_TOL = 1e-2


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def shape_of(w, num_seqs=None) -> coopt.Shape:
    return coopt.Shape(w.S if num_seqs is None else num_seqs, w.H_q, w.H_k, w.d, w.B, w.NB,
                       w.max_blocks,
                       coopt.COOPT_KV_E4M3 if w.kv_dtype == "e4m3" else coopt.COOPT_KV_FP16,
                       float(np.float32(w.softmax_scale)))


def cache_to_dev(cache):
    return tuple(None if a is None else dev(a.view(np.uint8) if a.dtype == np.uint8 else a)
                 for a in cache)


def alloc_dev_cache(w, fill_byte=0):
    """Device cache in the boundary layouts, every byte preset to fill_byte."""
    es = 1 if w.kv_dtype == "e4m3" else 2
    k_cache = torch.full((w.NB, w.H_k, w.B * w.d * es), fill_byte, dtype=torch.uint8, device="cuda")
    v_cache = torch.full((w.NB, w.H_k, w.B * w.d * es), fill_byte, dtype=torch.uint8, device="cuda")
    if w.kv_dtype == "e4m3":
        k_scale = torch.full((w.NB, w.H_k, w.B * 4), fill_byte, dtype=torch.uint8, device="cuda")
        v_scale = torch.full((w.NB, w.H_k, w.B * 4), fill_byte, dtype=torch.uint8, device="cuda")
    else:
        k_scale = v_scale = None
    return k_cache, v_cache, k_scale, v_scale


def hip_write(w, dcache, idx=None, slots=None):
    """Write tokens idx (default all) of workload w through the HIP write path."""
    k = w.k_ctx if idx is None else w.k_ctx[idx]
    v = w.v_ctx if idx is None else w.v_ctx[idx]
    s = (w.slots if idx is None else w.slots[idx]) if slots is None else slots
    dk, dv, ds = dev(k.view(np.uint16)), dev(v.view(np.uint16)), dev(s.astype(np.int64))
    shape = shape_of(w)
    if w.kv_dtype == "e4m3":
        coopt.kv_cache_write_fp8(dk, dv, ds, *dcache, shape)
    else:
        coopt.kv_cache_write_fp16(dk, dv, ds, dcache[0], dcache[1], shape)
    torch.cuda.synchronize()


def dev_cache_to_host(w, dcache):
    """Device cache -> numpy arrays typed like the oracle's host cache."""
    k_cache, v_cache, k_scale, v_scale = dcache
    if w.kv_dtype == "e4m3":
        return (k_cache.cpu().numpy(), v_cache.cpu().numpy(),
                k_scale.cpu().numpy().view(np.float32), v_scale.cpu().numpy().view(np.float32))
    return (k_cache.cpu().numpy().view(np.float16), v_cache.cpu().numpy().view(np.float16), None, None)


def hip_decode(w, dcache, *, q=None, lens=None, tables=None, split=True):
    """coopt_paged_gqa_decode on the current stream; returns float64 numpy [S, H_q, d]."""
    shape = shape_of(w)
    dq = dev((w.q if q is None else q).view(np.uint16))
    dbt = dev(w.block_tables if tables is None else tables)
    dlen = dev(w.context_lens if lens is None else lens)
    out = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    ws = None
    if split:
        ws = torch.empty(max(16, coopt.decode_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    coopt.paged_gqa_decode(dq, *dcache, dbt, dlen, out, ws, shape)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def assert_close(got: np.ndarray, ref: np.ndarray, what: str = ""):
    """The parity bar for attention outputs: |gpu - oracle| <= 2e-3 * max(1, |oracle|) for every
    element.  This is tighter than an absolute 2e-3 plus a relative 1e-2; the relative branch is
    needed because the output is fp16, whose rounding alone is up to 1.95e-3 for |x| in [4, 8).
    Returns the largest absolute error."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    bar = ABS_TOL * np.maximum(1.0, np.abs(ref))
    worst = float(err.max()) if err.size else 0.0
    bad = err > bar
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements over the bar, max-abs {worst:.3e}, "
                           f"worst ratio {float((err / bar).max()):.2f}")
    assert np.all(err <= ABS_TOL + REL_TOL * np.abs(ref))
    return worst
