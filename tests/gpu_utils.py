"""Helpers for the GPU parity tests: device buffers via torch, calls through the C-ABI binding."""
import functools

import numpy as np
import torch

import paper_2602_09323_amd as coopt

ABS_TOL = 2e-3      # max-abs bar for attention outputs (fp16 out vs float64 oracle)
REL_TOL = 1e-2
FP16_MAX_EXACT_TOL = 4.0     # below this an fp16 output is good to 2^-10: the plain bar holds
ARITH_TOL = 5e-4             # what the arithmetic may add to the output's own rounding above it


class _Planned:
    """The binding's plan-dependent calls with the test's current decode plan passed along (the
    library has no process-wide plan: every call takes it as an argument).  ``set_plan`` replaces
    the named fields of the current plan; conftest resets it to the default after every test."""
    NAMES = ("paged_gqa_decode", "paged_gqa_decode_step", "paged_gqa_decode_split",
             "paged_gqa_decode_merge", "paged_gqa_decode_partitioned", "paged_gqa_decode_scheduled",
             "decode_schedule_prepare", "decode_schedule_bytes", "decode_workspace_bytes")

    def __init__(self):
        self.plan = None

    def set_plan(self, **fields):
        cur = (self.plan or coopt.default_decode_plan()).as_dict()
        cur.update(fields)
        self.plan = coopt.make_decode_plan(**cur)

    def reset(self):
        self.plan = None

    def __getattr__(self, name):
        if name not in self.NAMES:
            raise AttributeError(name)
        return functools.partial(getattr(coopt, name), plan=self.plan)


planned = _Planned()


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def shape_of(w, num_seqs=None) -> coopt.Shape:
    return coopt.Shape(w.S if num_seqs is None else num_seqs, w.H_q, w.H_k, w.d, w.B, w.NB,
                       w.max_blocks,
                       {"e4m3": coopt.COOPT_KV_E4M3, "e5m2": coopt.COOPT_KV_E5M2,
                        "fp16": coopt.COOPT_KV_FP16}[w.kv_dtype],
                       float(np.float32(w.softmax_scale)))


def cache_to_dev(cache):
    return tuple(None if a is None else dev(a.view(np.uint8) if a.dtype == np.uint8 else a)
                 for a in cache)


def alloc_dev_cache(w, fill_byte=0):
    """Device cache in the boundary layouts, every byte preset to fill_byte."""
    es = 2 if w.kv_dtype == "fp16" else 1
    k_cache = torch.full((w.NB, w.H_k, w.B * w.d * es), fill_byte, dtype=torch.uint8, device="cuda")
    v_cache = torch.full((w.NB, w.H_k, w.B * w.d * es), fill_byte, dtype=torch.uint8, device="cuda")
    if w.kv_dtype != "fp16":
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
    if w.kv_dtype != "fp16":
        coopt.kv_cache_write_fp8(dk, dv, ds, *dcache, shape)
    else:
        coopt.kv_cache_write_fp16(dk, dv, ds, dcache[0], dcache[1], shape)
    torch.cuda.synchronize()


def dev_cache_to_host(w, dcache):
    """Device cache -> numpy arrays typed like the oracle's host cache."""
    k_cache, v_cache, k_scale, v_scale = dcache
    if w.kv_dtype != "fp16":
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
        ws = torch.empty(max(16, planned.decode_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    planned.paged_gqa_decode(dq, *dcache, dbt, dlen, out, ws, shape)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def parity_bar(ref: np.ndarray) -> np.ndarray:
    """The elementwise bar for attention outputs against the float64 oracle: max-abs 2e-3 wherever
    |oracle| < 4.  An fp16 output cannot meet that beyond: half an ulp is 1.95e-3 in [4, 8) and
    doubles with every binade, so there the bar is that half ulp -- the output's own rounding --
    plus 5e-4 for the arithmetic in front of it."""
    a = np.abs(ref)
    half_ulp = np.exp2(np.floor(np.log2(np.maximum(a, FP16_MAX_EXACT_TOL))) - 11)
    return np.where(a < FP16_MAX_EXACT_TOL, ABS_TOL, half_ulp + ARITH_TOL)


def assert_close(got: np.ndarray, ref: np.ndarray, what: str = "", record=None):
    """Every element within parity_bar (and within the looser pair 2e-3 + 1e-2 |oracle|).  Returns
    the largest absolute error; ``record`` (pytest's record_property) also gets it, with the
    largest |oracle| and the largest error among elements with |oracle| < 4."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    bar = parity_bar(ref)
    worst = float(err.max()) if err.size else 0.0
    bad = err > bar
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements over the bar, max-abs {worst:.3e}, "
                           f"worst ratio {float((err / bar).max()):.2f}, |oracle| there "
                           f"{float(np.abs(ref)[np.unravel_index(np.argmax(err / bar), err.shape)]):.3f}")
    assert np.all(err <= ABS_TOL + REL_TOL * np.abs(ref))
    if record is not None:
        small = np.abs(ref) < FP16_MAX_EXACT_TOL
        record(f"{what} max_abs_err", worst)
        record(f"{what} max_abs_oracle", float(np.abs(ref).max()) if ref.size else 0.0)
        record(f"{what} max_abs_err_below_4", float(err[small].max()) if small.any() else 0.0)
    return worst
