"""GPU: coopt_paged_gqa_decode_noalloc (the entry point for callers that cannot allocate: its
partial results go to a device array built into the library) against coopt_paged_gqa_decode with
a caller's workspace, through the C ABI: two calls in a row, the second on a smaller input, so
that what the first call left in the array is there when the second runs."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import assert_close, cache_to_dev, dev, shape_of
from helpers import oracle_fill

pytestmark = pytest.mark.gpu


def _both(orc, w, plan=None):
    """(noalloc, with workspace, oracle) outputs for workload w."""
    cache = oracle_fill(orc, w)
    ref = orc.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q, H_k=w.H_k,
                               d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    shape = shape_of(w)
    q, bt, dl = dev(w.q.view(np.uint16)), dev(w.block_tables), dev(w.context_lens)
    dcache = cache_to_dev(cache)
    out_a = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    out_b = torch.full_like(out_a, -5.0)
    coopt.paged_gqa_decode_noalloc(q, *dcache, bt, dl, out_a, shape, plan)
    torch.cuda.synchronize()
    ws = torch.empty(coopt.decode_workspace_bytes(shape, plan), dtype=torch.uint8, device="cuda")
    coopt.paged_gqa_decode(q, *dcache, bt, dl, out_b, ws, shape, plan)
    torch.cuda.synchronize()
    return out_a.cpu().numpy(), out_b.cpu().numpy(), ref


def test_two_calls_in_a_row_the_second_smaller(oracle_mod):
    big = workloads.make_custom("noalloc_big", seed=71, S=24, H_q=40, H_k=8, d=128, B=16, NB=2200,
                                context_lens=[1500, 700, 33, 1, 2048, 900] * 4, max_blocks=128)
    small = workloads.make_custom("noalloc_small", seed=72, S=3, H_q=10, H_k=2, d=64, B=16, NB=40,
                                  context_lens=[100, 17, 260], max_blocks=17, kv_dtype="fp16")
    for w in (big, small, big):
        a, b, ref = _both(oracle_mod, w)
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), f"{w.name}: not the same rows"
        assert_close(a.astype(np.float64), ref, w.name)
    # another plan lays the partials out differently in the same array
    plan = coopt.make_decode_plan(tokens_per_group=32, grid_waves=96, pipeline_depth=1)
    a, b, ref = _both(oracle_mod, small, plan)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert_close(a.astype(np.float64), ref, "small, another plan")


def test_shapes_beyond_the_array_are_refused():
    limit = coopt.decode_builtin_workspace_bytes()
    assert limit == 32 << 20
    lib = coopt.load_library()
    one = ctypes.c_void_p(256)            # never dereferenced: refused before anything is launched
    fits = coopt.Shape(4, 40, 8, 128, 16, 16384, 2048, coopt.COOPT_KV_E4M3, 0.088)
    too_big = coopt.Shape(16, 40, 8, 128, 16, 65536, 2048, coopt.COOPT_KV_E4M3, 0.088)
    assert coopt.decode_workspace_bytes(fits) <= limit < coopt.decode_workspace_bytes(too_big)
    args = [one] * 8
    assert lib.coopt_paged_gqa_decode_noalloc(*args, None, ctypes.byref(too_big), None) == -3
    assert lib.coopt_paged_gqa_decode_noalloc(*args[:7], None, None, ctypes.byref(fits), None) == -1
