"""GPU parity: chunked prefill over the paged cache and the dequantising gather."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import alloc_dev_cache, assert_close, cache_to_dev, dev, hip_write, shape_of
from helpers import oracle_fill

pytestmark = pytest.mark.gpu


def _prefill_call(with_workspace, q, dcache, bt, dl, qs, rows, max_chunk, out, shape):
    """The plain entry point, or the one that takes a workspace for the launch's last round (the
    workspace poisoned with NaN: whatever the merge reads must have been written by this call).
    Returns the workspace size the shape asks for."""
    if not with_workspace:
        coopt.paged_gqa_prefill_chunk(q, *dcache, bt, dl, qs, rows, max_chunk, out, shape)
        return 0
    need = coopt.prefill_workspace_bytes(shape, max_chunk)
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda") if need else None
    coopt.paged_gqa_prefill_chunk_ws(q, *dcache, bt, dl, qs, rows, max_chunk, out, ws, shape)
    return need


def _hip_prefill(w, dcache, lens=None, query_start=None, max_chunk=None, with_workspace=False):
    shape = shape_of(w)
    qs = w.query_start if query_start is None else query_start
    n_rows = int(qs[-1])
    out = torch.full((n_rows, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    _prefill_call(with_workspace, dev(w.q.view(np.uint16)), dcache, dev(w.block_tables),
                  dev(w.context_lens if lens is None else lens), dev(qs), n_rows,
                  w.new_per_seq if max_chunk is None else max_chunk, out, shape)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def _oracle_prefill(oracle, w, cache, rows=None):
    return oracle.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens,
                                          w.query_start, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                          softmax_scale=w.softmax_scale, rows=rows)


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
@pytest.mark.parametrize("ctx,C,H_q,H_k,d", [(40, 24, 10, 2, 128), (0, 33, 4, 2, 64), (100, 1, 5, 1, 128),
                                             (7, 130, 6, 3, 128), (256, 64, 40, 8, 128)])
def test_small_chunks(oracle_mod, kv_dtype, ctx, C, H_q, H_k, d):
    """A few workgroups only.  Through the entry point with a workspace such a launch is all "last
    round": every pair's stages are cut into up to eight runs (more runs than some of these
    streams have stages, so some parts are empty), one workgroup each, and merged."""
    w = workloads.make_custom("pf", seed=51, S=3, H_q=H_q, H_k=H_k, d=d, B=16, NB=96,
                              context_lens=[ctx + C] * 3, new_per_seq=C, kv_dtype=kv_dtype)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_prefill(oracle_mod, w, cache)
    dcache = cache_to_dev(cache)
    assert_close(_hip_prefill(w, dcache), ref, f"prefill ctx={ctx} C={C} {kv_dtype}")
    assert coopt.prefill_workspace_bytes(shape_of(w), C) > 0
    assert_close(_hip_prefill(w, dcache, with_workspace=True), ref, f"prefill ctx={ctx} C={C} {kv_dtype}, workspace")


@pytest.mark.parametrize("kv_dtype", ["e4m3", "e5m2", "fp16"])
def test_one_sequence_spread_over_the_chip(oracle_mod, kv_dtype):
    """One sequence's chunk (8 KV heads: 8 pairs of 125 tiles = 64 workgroups) over a history of
    3000 tokens: with a workspace its stages are cut into four runs per 16 tiles."""
    C, hist = 400, 3000
    w = workloads.make_custom("pf_one", seed=57, S=1, H_q=40, H_k=8, d=128, B=16, NB=230,
                              context_lens=[hist + C], new_per_seq=C, kv_dtype=kv_dtype)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens, w.query_start,
                                             H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale,
                                             fmt="e5m2" if kv_dtype == "e5m2" else "e4m3")
    shape = shape_of(w)
    # 125 tiles a pair = 8 workgroups: 64 in the launch, four parts of each fill the 256 CUs
    assert coopt.prefill_workspace_bytes(shape, C) == 8 * 125 * 4 * 16 * 130 * 4
    dcache = cache_to_dev(cache)
    assert_close(_hip_prefill(w, dcache), ref, f"one sequence {kv_dtype}")
    assert_close(_hip_prefill(w, dcache, with_workspace=True), ref, f"one sequence {kv_dtype}, workspace")


def test_chunk_written_on_device_then_attended(oracle_mod):
    w = workloads.make(4, shrink=16)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_prefill(oracle_mod, w, cache)
    devc = alloc_dev_cache(w, fill_byte=0x7F)
    hip_write(w, devc, idx=w.history_index())
    hip_write(w, devc, idx=w.new_index())
    assert_close(_hip_prefill(w, devc), ref, "cfg4/16")


@pytest.mark.parametrize("with_workspace", [False, True])
@pytest.mark.parametrize("kv_dtype,chunks", [("e4m3", [512] * 8), ("fp16", [512, 500, 17, 512, 1, 300, 512, 496]),
                                             ("e5m2", [512, 40, 512, 512, 130, 512, 3, 512])])
def test_two_launch_split_every_row(oracle_mod, kv_dtype, chunks, with_workspace):
    """As many workgroups as the full configuration (64 pairs, up to 160 tiles each), so the entry
    point splits the work into its two launches, over a short history so that the oracle can check
    every row; the other cases have a different chunk length per sequence.  With a workspace the
    second launch streams half of every pair's stages per workgroup and a third one merges the
    halves (histories of 0 to 250 tokens: halves of one to five stages, and sequences whose last
    tiles do not exist)."""
    S, H_q, H_k, d = len(chunks), 40, 8, 128
    history = [48, 0, 100, 16, 33, 64, 7, 250]
    lens = [h + c for h, c in zip(history, chunks)]
    w = workloads.make_custom("split", seed=77, S=S, H_q=H_q, H_k=H_k, d=d, B=16, NB=512,
                              context_lens=lens, kv_dtype=kv_dtype)
    query_start = np.zeros(S + 1, dtype=np.int32)
    query_start[1:] = np.cumsum(chunks)
    rows = int(query_start[-1])
    q = np.random.default_rng(78).standard_normal((rows, H_q, d), dtype=np.float32).astype(np.float16)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_prefill_chunk(q, *cache, w.block_tables, w.context_lens, query_start, H_q=H_q,
                                             H_k=H_k, d=d, B=16, softmax_scale=w.softmax_scale,
                                             fmt="e5m2" if kv_dtype == "e5m2" else "e4m3")
    out = torch.full((rows, H_q, d), -7.0, dtype=torch.float16, device="cuda")
    need = _prefill_call(with_workspace, dev(q.view(np.uint16)), cache_to_dev(cache), dev(w.block_tables),
                         dev(w.context_lens), dev(query_start), rows, max(chunks), out, shape_of(w))
    torch.cuda.synchronize()
    assert not with_workspace or need > 0          # this shape does have a partly filled last round
    assert_close(out.cpu().numpy().astype(np.float64), ref, f"two launches {kv_dtype} {chunks}")


def test_chunked_prefill_full_size(oracle_mod, record_property):
    """Full configuration in the launch shape the benchmark times.  The oracle computes every row
    of one whole sequence (512 rows x 40 heads over 8192 + 512 tokens: the stage pipeline 136
    stages deep, every tile of both launches) and, of the other sequences, a sample of rows
    (first, last, tile edges, random).  About a minute and a half of oracle time on 16 cores."""
    w = workloads.make(4)
    print(f"full cfg4: tokens={w.total_tokens}", flush=True)
    cache = oracle_fill(oracle_mod, w)
    dcache = cache_to_dev(cache)
    got = _hip_prefill(w, dcache)
    got_ws = _hip_prefill(w, dcache, with_workspace=True)
    assert np.isfinite(got).all() and np.isfinite(got_ws).all()
    rng = np.random.default_rng(0)
    C = w.new_per_seq
    local = np.array([0, 1, 15, 16, 17, C // 2, C - 2, C - 1])
    rows = np.unique(np.concatenate([local, (w.S - 1) * C + local, rng.integers(0, w.S * C, 8)])).astype(np.int32)
    ref_rows = _oracle_prefill(oracle_mod, w, cache, rows=rows)
    print("full cfg4 sample max-abs %.2e" % assert_close(got[rows], ref_rows, "cfg4 sample", record_property), flush=True)
    whole = np.arange(5 * C, 6 * C, dtype=np.int32)                  # sequence 5, every row
    ref = _oracle_prefill(oracle_mod, w, cache, rows=whole)
    print("full cfg4 sequence 5, every row: max-abs %.2e" %
          assert_close(got[whole], ref, "cfg4 whole sequence", record_property), flush=True)
    # the entry point with a workspace (the last 32 tiles of every pair in two halves + a merge):
    # the same rows of the other tiles bit for bit, every checked row within the bar
    print("full cfg4 with workspace, sequence 5: max-abs %.2e" %
          assert_close(got_ws[whole], ref, "cfg4 whole sequence, workspace", record_property), flush=True)
    assert_close(got_ws[rows], ref_rows, "cfg4 sample, workspace")
    same = (got_ws == got).all(axis=2)                         # [row, head]
    tiles_per_head = C // 16
    tile = np.arange(w.H_q)[None, :] % (w.H_q // w.H_k) * tiles_per_head + (np.arange(w.S * C)[:, None] % C) // 16
    assert same[tile < 128].all(), "rows of the first launch differ between the two entry points"


def test_gather_cached_kv(oracle_mod):
    """Bit-exact: the device rounds code * scale to fp16 once, like the oracle's exact product."""
    for kv_dtype in ("e4m3", "fp16"):
        for d, H_k in ((128, 2), (64, 3)):
            w = workloads.make_custom("ga", seed=52 + d, S=2, H_q=2 * H_k, H_k=H_k, d=d, B=16, NB=24,
                                      context_lens=[150, 25], kv_dtype=kv_dtype)
            cache = oracle_fill(oracle_mod, w)
            dcache = cache_to_dev(cache)
            for seq, lo, hi in ((0, 3, 61), (0, 0, 150), (0, 16, 144), (0, 149, 150), (1, 7, 25), (1, 0, 16)):
                kref, vref = oracle_mod.gather_cached_kv(*cache, w.block_tables, seq, lo, hi, H_k=H_k, d=d, B=16)
                k_out = torch.full((hi - lo + 2, H_k, d), 7.0, dtype=torch.float16, device="cuda")
                v_out = torch.full_like(k_out, 7.0)
                coopt.gather_cached_kv(*dcache, dev(w.block_tables), seq, lo, hi, k_out[1:-1], v_out[1:-1], shape_of(w))
                torch.cuda.synchronize()
                for got, ref in ((k_out, kref), (v_out, vref)):
                    got = got.cpu().numpy()
                    assert np.all(got[0] == 7.0) and np.all(got[-1] == 7.0)      # nothing outside the range
                    want = ref.astype(np.float16)                                  # one rounding of the exact product
                    assert np.array_equal(got[1:-1].view(np.uint16), want.view(np.uint16)), (kv_dtype, d, seq, lo, hi)
