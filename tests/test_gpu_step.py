"""GPU parity: the fused decode step (cache write of each sequence's new token + attention in one
launch, Opt-KV Eq. 5 / Alg. 1 with Opt-GQA Eq. 7-8 and Opt-Pa Eq. 9-10) against the oracle's
write followed by the oracle's decode: cache bytes and scales bit for bit, outputs within the
attention tolerance."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import (planned, alloc_dev_cache, assert_close, cache_to_dev, dev, dev_cache_to_host,
                       hip_write, shape_of)
from helpers import oracle_fill

pytestmark = pytest.mark.gpu


def _oracle_decode(oracle, w, cache, lens=None):
    return oracle.paged_gqa_decode(w.q, *cache, w.block_tables,
                                   w.context_lens if lens is None else lens, H_q=w.H_q, H_k=w.H_k,
                                   d=w.d, B=w.B, softmax_scale=w.softmax_scale)


def _hip_step(w, dcache, slots, k_new=None, v_new=None, lens=None):
    """coopt_paged_gqa_decode_step with the workload's new tokens (or the rows given)."""
    shape = shape_of(w)
    new = w.new_index()
    k = w.k_ctx[new] if k_new is None else k_new
    v = w.v_ctx[new] if v_new is None else v_new
    out = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    ws = torch.empty(max(16, planned.decode_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    planned.paged_gqa_decode_step(dev(k.view(np.uint16)), dev(v.view(np.uint16)),
                                dev(np.asarray(slots, dtype=np.int64)), dev(w.q.view(np.uint16)),
                                *dcache, dev(w.block_tables),
                                dev(w.context_lens if lens is None else lens), out, ws, shape)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def _same_cache(w, dcache, cache, what):
    got = dev_cache_to_host(w, dcache)
    for name, g, r in zip(("k_cache", "v_cache", "k_scale", "v_scale"), got, cache):
        if r is None:
            continue
        assert np.array_equal(g.reshape(-1).view(np.uint8), r.reshape(-1).view(np.uint8)), f"{what}: {name}"


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
@pytest.mark.parametrize("H_q,H_k,d", [(40, 8, 128), (6, 2, 64), (3, 3, 128), (16, 1, 64)])
def test_step_equals_write_then_decode(oracle_mod, kv_dtype, H_q, H_k, d):
    lens = [1, 2, 16, 17, 32, 33, 255, 257, 700, 512, 31]
    w = workloads.make_custom("step", seed=61, S=len(lens), H_q=H_q, H_k=H_k, d=d, B=16, NB=256,
                              context_lens=lens, kv_dtype=kv_dtype, max_blocks=48)
    cache = oracle_fill(oracle_mod, w)                      # history and new tokens
    ref = _oracle_decode(oracle_mod, w, cache)
    for plan in [(128, 1, 2, 1024), (32, 1, 1, 5), (64, 1, 3, 64)]:
        planned.set_plan(tokens_per_group=plan[0], waves_per_group=plan[1],
                              pipeline_depth=plan[2], grid_waves=plan[3])
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        got = _hip_step(w, dcache, w.slots[w.new_index()])
        assert_close(got, ref, f"step {kv_dtype} {H_q}/{H_k}/{d} plan={plan}")
        _same_cache(w, dcache, cache, f"step {kv_dtype} plan={plan}")


def test_filtered_tokens_and_empty_sequences(oracle_mod):
    """Negative slot: nothing is written and the sequence attends to what the cache holds at its
    last position; context length 0: nothing written, zero output rows."""
    lens = np.array([40, 1, 300, 17, 64, 5], dtype=np.int32)
    w = workloads.make_custom("skip", seed=62, S=len(lens), H_q=10, H_k=2, d=128, B=16, NB=64,
                              context_lens=lens, max_blocks=20)
    cache = oracle_fill(oracle_mod, w)                      # every token, the last ones included
    new = w.new_index()
    slots = w.slots[new].copy()
    skip = np.array([False, True, True, False, False, True])
    slots[skip] = -1
    run_lens = lens.copy()
    run_lens[4] = 0                                         # an empty sequence with a valid slot
    ref = _oracle_decode(oracle_mod, w, cache, lens=run_lens)
    dcache = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, dcache)                                    # the cache already holds all tokens
    rng = np.random.default_rng(5)
    k_new = w.k_ctx[new].copy()
    v_new = w.v_ctx[new].copy()
    junk = skip | (run_lens == 0)                           # rows that must not be used or written
    k_new[junk] = rng.standard_normal(k_new[junk].shape).astype(np.float16) * 30
    v_new[junk] = rng.standard_normal(v_new[junk].shape).astype(np.float16) * 30
    got = _hip_step(w, dcache, slots, k_new=k_new, v_new=v_new, lens=run_lens)
    assert np.all(got[4] == 0)
    assert_close(got, ref, "step with filtered tokens")
    _same_cache(w, dcache, cache, "filtered tokens leave the cache alone")


def test_many_sequences_step(oracle_mod):
    rng = np.random.default_rng(7)
    S = 150
    lens = rng.integers(1, 90, S).astype(np.int32)
    w = workloads.make_custom("manystep", seed=63, S=S, H_q=8, H_k=2, d=128, B=16, NB=1200,
                              context_lens=lens, max_blocks=8)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    for grid in (1024, 96):
        planned.set_plan(tokens_per_group=64, waves_per_group=1, pipeline_depth=2, grid_waves=grid)
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        got = _hip_step(w, dcache, w.slots[w.new_index()])
        assert_close(got, ref, f"S={S} grid={grid}")
        _same_cache(w, dcache, cache, f"S={S} grid={grid}")


def test_headline_step_full_size(oracle_mod):
    w = workloads.make(1)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    dcache = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, dcache, idx=w.history_index())
    got = _hip_step(w, dcache, w.slots[w.new_index()])
    print("cfg1 fused step max-abs %.2e" % assert_close(got, ref, "cfg1 step"), flush=True)
    _same_cache(w, dcache, cache, "cfg1 step")
