"""GPU parity on a pool of more than 2 GiB per tensor: the kernels then address tiles through
per-tile buffer descriptors and 64-bit offsets instead of one descriptor per pool.  Blocks are
dealt from the whole pool, so tiles beyond the 2 GiB mark are written and read."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import planned, alloc_dev_cache, assert_close, dev, hip_decode, hip_write, shape_of
from helpers import alloc_cache, oracle_fill

pytestmark = pytest.mark.gpu

NB_BIG = 3 << 16                # x 8 KV heads x 2048 B per tile = 3 GiB per tensor


@pytest.fixture(scope="module")
def big(oracle_mod):
    lens = [300, 1025, 47, 16]
    w = workloads.make_custom("bigpool", seed=71, S=len(lens), H_q=40, H_k=8, d=128, B=16, NB=NB_BIG,
                              context_lens=lens, new_per_seq=16, max_blocks=80)
    used = w.block_tables[w.block_tables >= 0]
    assert (used.astype(np.int64) * w.H_k * 2048).max() > (1 << 31)      # tiles past the 2 GiB mark
    cache = oracle_fill(oracle_mod, w)
    dcache = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, dcache)
    return w, cache, dcache, used


def test_written_tiles_bit_exact(big):
    w, cache, dcache, used = big
    for name, host, devt in zip(("k_cache", "v_cache", "k_scale", "v_scale"), cache, dcache):
        got = devt[torch.from_numpy(used.astype(np.int64)).cuda()].cpu().numpy()
        ref = host[used]
        assert np.array_equal(got.reshape(len(used), -1).view(np.uint8),
                              ref.reshape(len(used), -1).view(np.uint8)), name


def test_decode_all_paths(big, oracle_mod):
    w, cache, dcache, _ = big
    ref = oracle_mod.paged_gqa_decode(w.q[:w.S] if w.q.shape[0] != w.S else w.q, *cache, w.block_tables,
                                      w.context_lens, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                      softmax_scale=w.softmax_scale)
    q = w.q[:w.S] if w.q.shape[0] != w.S else w.q
    for split in (True, False):
        assert_close(hip_decode(w, dcache, q=q, split=split), ref, f"big pool split={split}")
    shape = shape_of(w)
    # the same decode from a prepared schedule
    sched = torch.zeros(planned.decode_schedule_bytes(shape), dtype=torch.uint8, device="cuda")
    ws = torch.empty(max(16, planned.decode_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    outs = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    planned.decode_schedule_prepare(dev(w.block_tables), dev(w.context_lens), None, sched, shape)
    planned.paged_gqa_decode_scheduled(None, None, None, dev(q.view(np.uint16)), *dcache,
                                     dev(w.context_lens), outs, ws, sched, shape)
    torch.cuda.synchronize()
    assert_close(outs.cpu().numpy().astype(np.float64), ref, "big pool, prepared schedule")
    P, max_parts = 256, (w.max_blocks * w.B + 255) // 256
    tmp_out = torch.empty((w.S, w.H_q, max_parts, w.d), dtype=torch.float32, device="cuda")
    ml = torch.empty((w.S, w.H_q, max_parts), dtype=torch.float32, device="cuda")
    es = torch.empty_like(ml)
    out = torch.zeros((w.S, w.H_q, w.d), dtype=torch.float16, device="cuda")
    dq, dbt, dlen = dev(q.view(np.uint16)), dev(w.block_tables), dev(w.context_lens)
    planned.paged_gqa_decode_partitioned(dq, *dcache, dbt, dlen, P, tmp_out, ml, es, max_parts, shape)
    coopt.paged_gqa_reduce(tmp_out, ml, es, dlen, P, max_parts, out, shape)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, "big pool partitioned")


def test_prefill_chunk(big, oracle_mod):
    w, cache, dcache, _ = big
    ref = oracle_mod.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens, w.query_start,
                                             H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                             softmax_scale=w.softmax_scale)
    n_rows = int(w.query_start[-1])
    out = torch.zeros((n_rows, w.H_q, w.d), dtype=torch.float16, device="cuda")
    coopt.paged_gqa_prefill_chunk(dev(w.q.view(np.uint16)), *dcache, dev(w.block_tables),
                                  dev(w.context_lens), dev(w.query_start), n_rows, w.new_per_seq, out,
                                  shape_of(w))
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, "big pool prefill")


def test_gather(big, oracle_mod):
    w, cache, dcache, _ = big
    kref, vref = oracle_mod.gather_cached_kv(*cache, w.block_tables, 1, 5, 900, H_k=w.H_k, d=w.d, B=w.B)
    k_out = torch.zeros((895, w.H_k, w.d), dtype=torch.float16, device="cuda")
    v_out = torch.zeros_like(k_out)
    coopt.gather_cached_kv(*dcache, dev(w.block_tables), 1, 5, 900, k_out, v_out, shape_of(w))
    torch.cuda.synchronize()
    for got, ref in ((k_out, kref), (v_out, vref)):
        want = ref.astype(np.float16)                              # one rounding of the exact product
        assert np.array_equal(got.cpu().numpy().view(np.uint16), want.view(np.uint16))


def test_fused_step(oracle_mod):
    lens = [300, 1025, 47, 1]
    w = workloads.make_custom("bigstep", seed=72, S=len(lens), H_q=40, H_k=8, d=128, B=16, NB=NB_BIG,
                              context_lens=lens, max_blocks=80)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q, H_k=w.H_k,
                                      d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    dcache = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, dcache, idx=w.history_index())
    shape = shape_of(w)
    new = w.new_index()
    out = torch.zeros((w.S, w.H_q, w.d), dtype=torch.float16, device="cuda")
    ws = torch.empty(planned.decode_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    planned.paged_gqa_decode_step(dev(w.k_ctx[new].view(np.uint16)), dev(w.v_ctx[new].view(np.uint16)),
                                dev(w.slots[new]), dev(w.q.view(np.uint16)), *dcache, dev(w.block_tables),
                                dev(w.context_lens), out, ws, shape)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, "big pool fused step")
    used = torch.from_numpy(w.block_tables[w.block_tables >= 0].astype(np.int64)).cuda()
    for name, host, devt in zip(("k_cache", "v_cache", "k_scale", "v_scale"), cache, dcache):
        assert np.array_equal(devt[used].cpu().numpy().reshape(len(used), -1).view(np.uint8),
                              host[used.cpu().numpy()].reshape(len(used), -1).view(np.uint8)), name
