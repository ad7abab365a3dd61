"""Pins for the oracle's attention: decode, partitioned + reduce, chunked prefill, gather.

Paper: Background Eq. 1 (single-query attention), Opt-KV Eq. 6 (dequantise before attention),
Opt-GQA Eq. 7 (group map) and Alg. 2, Opt-Pa Eq. 9 (valid blocks) and Eq. 10 (stable softmax).
The comparison partners are independent of the oracle: textbook numpy attention on tensors
gathered by direct indexing, torch's scaled_dot_product_attention in float64, closed forms.
"""
import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import workloads
from helpers import (alloc_cache, gather_dequant, k_logical, k_store_logical, oracle_fill,
                     softmax_attention, v_logical, v_store_logical)


def _decode(oracle, w, cache, q=None, lens=None, tables=None):
    return oracle.paged_gqa_decode(w.q if q is None else q, *cache,
                                   w.block_tables if tables is None else tables,
                                   w.context_lens if lens is None else lens,
                                   H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale)


@settings(max_examples=25, deadline=None)
@given(S=st.integers(1, 3), H_k=st.integers(1, 3), G=st.integers(1, 4), d=st.sampled_from([64, 128]),
       seed=st.integers(0, 10_000), data=st.data())
def test_decode_equals_contiguous_attention(oracle_mod, S, H_k, G, d, seed, data):
    lens = [data.draw(st.integers(1, 50)) for _ in range(S)]
    w = workloads.make_custom("h", seed=seed, S=S, H_q=H_k * G, H_k=H_k, d=d, B=16, NB=16,
                              context_lens=lens)
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache)
    for s in range(S):
        K, V = gather_dequant(w, cache, s)
        for h in range(w.H_q):
            g = h // G
            want = softmax_attention(w.q[s, h].astype(np.float64), K[:, g], V[:, g],
                                     float(np.float32(w.softmax_scale)))
            assert np.max(np.abs(out[s, h] - want)) <= 1e-12


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
def test_decode_equals_torch_sdpa(oracle_mod, kv_dtype):
    w = workloads.make_custom("sdpa", seed=11, S=2, H_q=8, H_k=2, d=64, B=16, NB=32,
                              context_lens=[100, 77], kv_dtype=kv_dtype)
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache)
    G = w.H_q // w.H_k
    for s in range(w.S):
        K, V = gather_dequant(w, cache, s)                                   # [t, H_k, d]
        Kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)  # [H_q, t, d]
        Vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
        Q = torch.from_numpy(w.q[s].astype(np.float64)).unsqueeze(1)         # [H_q, 1, d]
        want = torch.nn.functional.scaled_dot_product_attention(
            Q, Kt, Vt, scale=float(np.float32(w.softmax_scale))).squeeze(1).numpy()
        assert np.max(np.abs(out[s] - want)) <= 1e-12


def test_group_of_one_is_mha_and_gqa_is_mha_on_repeated_heads(oracle_mod):
    """Eq. 7: head h uses KV head floor(h / (H_q/H_k))."""
    G = 3
    w = workloads.make_custom("gqa", seed=12, S=2, H_q=6, H_k=2, d=64, B=16, NB=16,
                              context_lens=[40, 23])
    cache = oracle_fill(oracle_mod, w)
    out_gqa = _decode(oracle_mod, w, cache)
    # the same cache with every KV head physically repeated G times, read as MHA (G = 1)
    k_cache, v_cache, k_scale, v_scale = cache
    rep = tuple(np.ascontiguousarray(np.repeat(a, G, axis=1)) for a in cache)
    out_mha = oracle_mod.paged_gqa_decode(w.q, *rep, w.block_tables, w.context_lens, H_q=6, H_k=6,
                                          d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    assert np.array_equal(out_gqa, out_mha)
    # and a wrong map must differ: swapping the two KV heads changes the result
    swapped = tuple(np.ascontiguousarray(a[:, ::-1]) for a in cache)
    assert not np.allclose(_decode(oracle_mod, w, swapped), out_gqa)


def test_single_token_context_returns_its_value(oracle_mod):
    w = workloads.make_custom("t1", seed=13, S=3, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[1, 1, 1])
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache)
    for s in range(3):
        _, V = gather_dequant(w, cache, s)
        for h in range(4):
            assert np.array_equal(out[s, h], V[0, h // 2])


def test_zero_query_gives_mean_of_values(oracle_mod):
    w = workloads.make_custom("q0", seed=14, S=1, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[45])
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache, q=np.zeros_like(w.q))
    _, V = gather_dequant(w, cache, 0)
    for h in range(4):
        assert np.max(np.abs(out[0, h] - V[:, h // 2].mean(axis=0))) <= 1e-13


def test_dominant_key_selects_its_value(oracle_mod):
    w = workloads.make_custom("dom", seed=15, S=1, H_q=2, H_k=1, d=64, B=16, NB=8,
                              context_lens=[40])
    jstar = 17
    w.k_ctx[:] = (w.k_ctx.astype(np.float32) * 0.01).astype(np.float16)
    w.k_ctx[jstar, 0, :] = np.float16(100.0)
    q = np.full_like(w.q, np.float16(4.0))       # z_j* = 4*100*64/8 = 3200, others ~ 0
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache, q=q)
    _, V = gather_dequant(w, cache, 0)
    assert np.array_equal(out[0, 0], V[jstar, 0]) and np.array_equal(out[0, 1], V[jstar, 0])


def test_output_within_value_hull_and_weights_sum_to_one(oracle_mod):
    w = workloads.make_custom("hull", seed=16, S=2, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[60, 31])
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache)
    for s in range(2):
        _, V = gather_dequant(w, cache, s)
        for h in range(4):
            lo, hi = V[:, h // 2].min(axis=0), V[:, h // 2].max(axis=0)
            assert np.all(out[s, h] >= lo - 1e-12) and np.all(out[s, h] <= hi + 1e-12)
    # constant V => output is that constant regardless of scores (weights sum to 1)
    w.v_ctx[:] = np.float16(0.875)          # 448 * 2^-9: the scale is an exact power of two
    cache = oracle_fill(oracle_mod, w)
    assert np.max(np.abs(_decode(oracle_mod, w, cache) - 0.875)) <= 1e-14


def test_invalid_tokens_and_blocks_never_read(oracle_mod):
    """Eq. 9: tokens >= t and blocks >= ceil(t/B) cannot influence the output."""
    w = workloads.make_custom("poison", seed=17, S=2, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[37, 50], max_blocks=6)
    cache = oracle_fill(oracle_mod, w)
    ref = _decode(oracle_mod, w, cache)
    k_cache, v_cache, k_scale, v_scale = (a.copy() for a in cache)
    used = np.zeros((w.NB, w.B), bool)
    used.reshape(-1)[w.slots] = True
    unused_scale = np.broadcast_to(~used[:, None, :], k_scale.shape)
    kl, vl = k_logical(w, k_cache), v_logical(w, v_cache)
    unused = np.broadcast_to(~used[:, None, :, None], kl.shape)
    kl[unused] = 0x7F
    vl[unused] = 0x7F
    k_store_logical(w, k_cache, kl)
    v_store_logical(w, v_cache, vl)
    k_scale[unused_scale] = np.nan
    v_scale[unused_scale] = np.nan
    tables = w.block_tables.copy()
    tables[tables < 0] = 10 ** 6                  # would fault / index out of range if read
    out = _decode(oracle_mod, w, (k_cache, v_cache, k_scale, v_scale), tables=tables)
    assert np.array_equal(out, ref)
    # shorter context_lens on the same cache == attention over the prefix
    lens = np.array([20, 16], np.int32)
    out_short = _decode(oracle_mod, w, cache, lens=lens)
    for s in range(2):
        K, V = gather_dequant(w, cache, s)
        for h in range(4):
            want = softmax_attention(w.q[s, h].astype(np.float64), K[:lens[s], h // 2],
                                     V[:lens[s], h // 2], float(np.float32(w.softmax_scale)))
            assert np.max(np.abs(out_short[s, h] - want)) <= 1e-12


def test_physical_block_choice_does_not_matter(oracle_mod):
    a = workloads.make_custom("perm", seed=18, S=2, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[40, 25])
    b = workloads.make_custom("perm", seed=18, S=2, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[40, 25])
    rng = np.random.default_rng(99)
    b.block_tables, b.slots, _ = workloads.make_paging(rng, b.context_lens, b.B, b.NB)
    assert not np.array_equal(a.block_tables, b.block_tables)
    oa = _decode(oracle_mod, a, oracle_fill(oracle_mod, a))
    ob = _decode(oracle_mod, b, oracle_fill(oracle_mod, b))
    assert np.array_equal(oa, ob)


def test_zero_length_context_gives_zero_row(oracle_mod):
    w = workloads.make_custom("z", seed=19, S=2, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[5, 9])
    cache = oracle_fill(oracle_mod, w)
    out = _decode(oracle_mod, w, cache, lens=np.array([0, 9], np.int32))
    assert np.all(out[0] == 0) and np.any(out[1] != 0)


@pytest.mark.parametrize("P", [16, 32, 512, 4096])
def test_partitioned_equals_unpartitioned(oracle_mod, P):
    w = workloads.make_custom("part", seed=20, S=3, H_q=4, H_k=2, d=64, B=16, NB=64,
                              context_lens=[300, 17, 512], k_outlier_frac=0.05)
    cache = oracle_fill(oracle_mod, w)
    ref = _decode(oracle_mod, w, cache)
    max_parts = (512 + P - 1) // P
    tmp, ml, es = oracle_mod.paged_gqa_decode_partitioned(
        w.q, *cache, w.block_tables, w.context_lens, P, max_parts, H_q=w.H_q, H_k=w.H_k, d=w.d,
        B=w.B, softmax_scale=w.softmax_scale)
    out = oracle_mod.paged_gqa_reduce(tmp, ml, es, w.context_lens, P)
    assert np.max(np.abs(out - ref)) <= 1e-12
    # partials are the attention of each token range on its own
    for s in range(w.S):
        K, V = gather_dequant(w, cache, s)
        t = int(w.context_lens[s])
        nparts = (t + P - 1) // P
        assert np.isnan(tmp[s, :, nparts:]).all()
        for p in range(nparts):
            sl = slice(p * P, min((p + 1) * P, t))
            want = softmax_attention(w.q[s, 1].astype(np.float64), K[sl, 0], V[sl, 0],
                                     float(np.float32(w.softmax_scale)))
            assert np.max(np.abs(tmp[s, 1, p] - want)) <= 1e-12
            z = (K[sl, 0] @ w.q[s, 1].astype(np.float64)) * float(np.float32(w.softmax_scale))
            assert abs(ml[s, 1, p] - z.max()) <= 1e-12
            assert abs(es[s, 1, p] - np.exp(z - z.max()).sum()) <= 1e-10


def test_reduce_closed_forms(oracle_mod):
    """Two partitions with equal maxima and sums average; a dominant one wins."""
    tmp = np.zeros((1, 1, 2, 4)); tmp[0, 0, 0] = 1.0; tmp[0, 0, 1] = 3.0
    lens = np.array([32], np.int32)
    out = oracle_mod.paged_gqa_reduce(tmp, np.array([[[0.5, 0.5]]]), np.array([[[2.0, 2.0]]]), lens, 16)
    assert np.allclose(out, 2.0, atol=1e-15)
    out = oracle_mod.paged_gqa_reduce(tmp, np.array([[[0.0, np.log(3.0)]]]), np.array([[[1.0, 1.0]]]), lens, 16)
    assert np.allclose(out, (1 * 1 + 3 * 3) / 4, atol=1e-14)
    out = oracle_mod.paged_gqa_reduce(tmp, np.array([[[900.0, 0.0]]]), np.array([[[1.0, 5.0]]]), lens, 16)
    assert np.array_equal(out, np.ones((1, 1, 4)))


def test_prefill_rows_equal_decode_at_growing_context(oracle_mod):
    C, ctx = 24, 40
    w = workloads.make_custom("pf", seed=21, S=2, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[ctx + C] * 2, new_per_seq=C)
    cache = oracle_fill(oracle_mod, w)
    out = oracle_mod.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens,
                                             w.query_start, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                             softmax_scale=w.softmax_scale)
    assert out.shape == (2 * C, 4, 64)
    for i in [0, 1, 7, C - 1]:
        lens = np.array([ctx + i + 1] * 2, np.int32)
        q_i = np.ascontiguousarray(w.q.reshape(2, C, 4, 64)[:, i])
        dec = _decode(oracle_mod, w, cache, q=q_i, lens=lens)
        assert np.array_equal(out.reshape(2, C, 4, 64)[:, i], dec)
    rows = np.array([3, C + 5, 2 * C - 1], np.int32)
    sub = oracle_mod.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens,
                                             w.query_start, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                             softmax_scale=w.softmax_scale, rows=rows)
    assert np.array_equal(sub, out[rows])


def test_prefill_without_history_is_plain_causal_attention(oracle_mod):
    C = 33
    w = workloads.make_custom("pf0", seed=22, S=1, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[C], new_per_seq=C, kv_dtype="fp16")
    cache = oracle_fill(oracle_mod, w)
    out = oracle_mod.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens,
                                             w.query_start, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                             softmax_scale=w.softmax_scale)
    K = torch.from_numpy(w.k_ctx.astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, dim=0)
    V = torch.from_numpy(w.v_ctx.astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, dim=0)
    Q = torch.from_numpy(w.q.astype(np.float64)).permute(1, 0, 2)
    want = torch.nn.functional.scaled_dot_product_attention(
        Q, K, V, is_causal=True, scale=float(np.float32(w.softmax_scale))).permute(1, 0, 2).numpy()
    assert np.max(np.abs(out - want)) <= 1e-12


def test_gather_matches_direct_indexing(oracle_mod):
    w = workloads.make_custom("ga", seed=23, S=2, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[40, 25])
    cache = oracle_fill(oracle_mod, w)
    K, V = gather_dequant(w, cache, 1)
    k, v = oracle_mod.gather_cached_kv(*cache, w.block_tables, 1, 3, 22, H_k=2, d=64, B=16)
    assert np.array_equal(k, K[3:22]) and np.array_equal(v, V[3:22])
