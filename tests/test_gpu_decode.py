"""GPU parity: paged grouped-query decode attention against the float64 oracle
(Background Eq. 1; Opt-KV Eq. 6; Opt-GQA Eq. 7-8; Opt-Pa Eq. 9-10), on the same cache bytes."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import (planned, alloc_dev_cache, assert_close, cache_to_dev, dev, dev_cache_to_host,
                       hip_decode, hip_write, shape_of)
from helpers import alloc_cache, oracle_fill

pytestmark = pytest.mark.gpu


def _oracle_decode(oracle, w, cache, q=None, lens=None, tables=None):
    return oracle.paged_gqa_decode(w.q if q is None else q, *cache,
                                   w.block_tables if tables is None else tables,
                                   w.context_lens if lens is None else lens,
                                   H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale)


def test_tiny_config(oracle_mod):
    w = workloads.make(0)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    for split in (False, True):
        got = hip_decode(w, cache_to_dev(cache), split=split)
        print("tiny split=%s max-abs %.2e" % (split, assert_close(got, ref, "tiny")), flush=True)


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
@pytest.mark.parametrize("H_q,H_k,d", [(40, 8, 128), (8, 8, 128), (6, 2, 64), (16, 1, 64), (3, 3, 128)])
def test_ragged_lengths_and_group_sizes(oracle_mod, kv_dtype, H_q, H_k, d):
    lens = [1, 15, 16, 17, 255, 256, 257, 700, 33, 512]
    w = workloads.make_custom("ragged", seed=31, S=len(lens), H_q=H_q, H_k=H_k, d=d, B=16, NB=256,
                              context_lens=lens, kv_dtype=kv_dtype, max_blocks=48)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    dcache = cache_to_dev(cache)
    for split in (False, True):
        got = hip_decode(w, dcache, split=split)
        assert_close(got, ref, f"ragged {kv_dtype} {H_q}/{H_k}/{d} split={split}")
    planned.set_plan(softmax_reduction=1)      # Opt-Pa's shared-memory max / block_sum form
    assert_close(hip_decode(w, dcache, split=True), ref, f"ragged {kv_dtype} {H_q}/{H_k}/{d} block reduce")


def _plan(tokens, waves, depth, grid, reduction=0):
    return dict(tokens_per_group=tokens, waves_per_group=waves, pipeline_depth=depth,
                grid_waves=grid, softmax_reduction=reduction)


@pytest.mark.parametrize("plan", [(32, 1, 1, 64), (32, 1, 2, 2048), (64, 2, 2, 512),
                                  (128, 1, 3, 2048), (128, 8, 2, 2048), (512, 4, 3, 256),
                                  (1024, 8, 2, 2048), (256, 4, 1, 24), (128, 1, 2, 7),
                                  (32, 2, 2, 6), (128, 1, 2, 1024), (128, 1, 2, 2), (128, 1, 3, 3),
                                  (2048, 1, 1, 1024), (128, 1, 2, 1024, 1), (32, 1, 2, 9, 1)])
def test_every_launch_plan_gives_the_same_answer(oracle_mod, plan):
    lens = [300, 1, 1025, 47, 640]
    w = workloads.make_custom("plan", seed=32, S=len(lens), H_q=10, H_k=2, d=128, B=16, NB=160,
                              context_lens=lens, max_blocks=80)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    planned.set_plan(**_plan(*plan))
    dcache = cache_to_dev(cache)
    got = hip_decode(w, dcache, split=True)
    assert_close(got, ref, f"plan {plan}")


def test_empty_and_single_token_contexts(oracle_mod):
    w = workloads.make_custom("edge", seed=33, S=4, H_q=10, H_k=2, d=128, B=16, NB=16,
                              context_lens=[5, 1, 16, 3])
    cache = oracle_fill(oracle_mod, w)
    lens = np.array([0, 1, 16, 0], np.int32)
    ref = _oracle_decode(oracle_mod, w, cache, lens=lens)
    dcache = cache_to_dev(cache)
    for split in (False, True):
        got = hip_decode(w, dcache, lens=lens, split=split)
        assert np.all(got[0] == 0) and np.all(got[3] == 0)
        assert_close(got, ref, f"edge split={split}")


def test_stale_slots_and_unused_table_entries_never_read(oracle_mod):
    """Opt-Pa Eq. 9: tokens >= t and blocks >= ceil(t/B) hold NaN codes / NaN scales here."""
    lens = [37, 50, 129, 16]
    w = workloads.make_custom("poison", seed=34, S=4, H_q=10, H_k=2, d=128, B=16, NB=32,
                              context_lens=lens, max_blocks=12)
    clean = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, clean)
    poisoned = alloc_cache(w, fill_byte=0x7F)           # 0x7F = E4M3 NaN; scales NaN
    oracle_fill(oracle_mod, w, cache=poisoned)
    tables = w.block_tables.copy()
    tables[tables < 0] = 0                               # in-range but wrong: must not matter
    for split in (False, True):
        got = hip_decode(w, cache_to_dev(poisoned), tables=tables, split=split)
        assert_close(got, ref, f"poison split={split}")
    # fp16 cache: stale entries are fp16 NaN (0x7F7F)
    w16 = workloads.make_custom("poison16", seed=35, S=4, H_q=4, H_k=4, d=128, B=16, NB=32,
                                context_lens=lens, kv_dtype="fp16", max_blocks=12)
    ref16 = _oracle_decode(oracle_mod, w16, oracle_fill(oracle_mod, w16))
    p16 = alloc_cache(w16, fill_byte=0x7F)
    oracle_fill(oracle_mod, w16, cache=p16)
    for split in (False, True):
        assert_close(hip_decode(w16, cache_to_dev(p16), split=split), ref16, "poison fp16")


def test_outlier_keys_and_peaked_softmax(oracle_mod):
    w = workloads.make_custom("outlier", seed=36, S=3, H_q=10, H_k=2, d=128, B=16, NB=128,
                              context_lens=[600, 333, 90], k_outlier_frac=0.02)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    assert_close(hip_decode(w, cache_to_dev(cache)), ref, "outliers")


def test_maximum_length_fills_the_block_table(oracle_mod):
    w = workloads.make_custom("full", seed=37, S=2, H_q=10, H_k=2, d=128, B=16, NB=140,
                              context_lens=[1024, 1009], max_blocks=64)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    for split in (False, True):
        assert_close(hip_decode(w, cache_to_dev(cache), split=split), ref, "full table")


@pytest.mark.parametrize("S", [65, 150, 300])
def test_many_short_sequences(oracle_mod, S):
    """More than 64 sequences (the schedule scans the lengths in tiles of 64), many of them
    shorter than one share, some empty."""
    rng = np.random.default_rng(S)
    lens = rng.integers(1, 200, size=S)
    lens[rng.integers(0, S, size=S // 10)] = 0
    lens[S // 2] = 700
    w = workloads.make_custom("many", seed=38, S=S, H_q=8, H_k=2, d=128, B=16, NB=2600,
                              context_lens=np.maximum(lens, 1), max_blocks=44)
    cache = oracle_fill(oracle_mod, w)
    lens = lens.astype(np.int32)
    ref = _oracle_decode(oracle_mod, w, cache, lens=lens)
    dcache = cache_to_dev(cache)
    for plan in [(128, 1, 2, 1024), (32, 1, 1, 4096), (256, 4, 2, 64), (64, 1, 2, 96)]:
        planned.set_plan(**_plan(*plan))
        got = hip_decode(w, dcache, lens=lens, split=True)
        assert np.all(got[lens == 0] == 0)
        assert_close(got, ref, f"S={S} plan={plan}")


def test_split_and_merge_as_separate_calls(oracle_mod):
    w = workloads.make_custom("sm", seed=39, S=5, H_q=10, H_k=2, d=128, B=16, NB=160,
                              context_lens=[300, 1, 1025, 47, 640], max_blocks=80)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    shape = shape_of(w)
    dcache = cache_to_dev(cache)
    ws = torch.empty(planned.decode_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    out = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    dlen = dev(w.context_lens)
    planned.paged_gqa_decode_split(dev(w.q.view(np.uint16)), *dcache, dev(w.block_tables), dlen, ws, shape)
    planned.paged_gqa_decode_merge(dlen, ws, out, shape)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, "split+merge")


def test_decode_step_end_to_end_on_device(oracle_mod):
    """History written, then the step: HIP write of one token per sequence + HIP decode."""
    w = workloads.make(1, shrink=4)
    host = alloc_cache(w)
    oracle_fill(oracle_mod, w, cache=host)
    ref = _oracle_decode(oracle_mod, w, host)
    devc = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, devc, idx=w.history_index())
    hip_write(w, devc, idx=w.new_index())
    got = hip_decode(w, devc)
    assert_close(got, ref, "step")
    for a, b in zip(host, dev_cache_to_host(w, devc)):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


@pytest.mark.parametrize("cfg", [1, 2])
def test_llama13b_shapes_full_size(oracle_mod, cfg):
    """The benchmark's own configuration and launch plan, every output element."""
    w = workloads.make(cfg)
    print(f"full cfg{cfg}: tokens={w.total_tokens}", flush=True)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    got = hip_decode(w, cache_to_dev(cache), split=True)
    print("full cfg%d max-abs %.2e" % (cfg, assert_close(got, ref, f"cfg{cfg}")), flush=True)


def test_merge_refuses_partials_of_another_plan(oracle_mod):
    """The split launch stamps the workspace with the layout its plan gives the partials; a merge
    call with a plan that lays them out differently (or on a workspace no split call has written)
    writes nothing.  With the split's own plan the same workspace then merges correctly."""
    w = workloads.make_custom("tag", seed=40, S=5, H_q=10, H_k=2, d=128, B=16, NB=160,
                              context_lens=[300, 1, 1025, 47, 640], max_blocks=80)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    shape = shape_of(w)
    dcache = cache_to_dev(cache)
    dlen = dev(w.context_lens)
    plans = [dict(tokens_per_group=128, waves_per_group=1, pipeline_depth=2, grid_waves=1024, softmax_reduction=0),
             dict(tokens_per_group=64, waves_per_group=1, pipeline_depth=2, grid_waves=1024, softmax_reduction=0),
             dict(tokens_per_group=128, waves_per_group=1, pipeline_depth=2, grid_waves=96, softmax_reduction=0)]
    sizes = []
    for p in plans:
        planned.set_plan(**p)
        sizes.append(planned.decode_workspace_bytes(shape))
    ws = torch.zeros(max(sizes), dtype=torch.uint8, device="cuda")
    out = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    planned.set_plan(**plans[0])
    planned.paged_gqa_decode_merge(dlen, ws, out, shape)            # nothing has been split into it
    torch.cuda.synchronize()
    assert torch.all(out == -7.0)
    planned.paged_gqa_decode_split(dev(w.q.view(np.uint16)), *dcache, dev(w.block_tables), dlen, ws, shape)
    for other in plans[1:]:
        planned.set_plan(**other)
        planned.paged_gqa_decode_merge(dlen, ws, out, shape)
        torch.cuda.synchronize()
        assert torch.all(out == -7.0), other
    planned.set_plan(**plans[0])
    planned.paged_gqa_decode_merge(dlen, ws, out, shape)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, "merge with the split's plan")
