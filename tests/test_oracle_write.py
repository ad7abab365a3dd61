"""Pins for the oracle's cache write: dynamic scale, codes, slot/block indexing, skip rule.

Paper: Opt-KV, Eq. 5 (skip rule) and Alg. 1 phase 1 (store into the block-wise cache).
"""
import numpy as np
import pytest

import workloads
from helpers import alloc_cache, e4m3_table, k_logical, k_tile_index, oracle_fill, v_logical, v_tile_index


def _one_row(oracle, row_k, row_v=None, B=16):
    d = row_k.shape[0]
    k = np.ascontiguousarray(row_k.reshape(1, 1, d).astype(np.float16))
    v = np.ascontiguousarray((row_k if row_v is None else row_v).reshape(1, 1, d).astype(np.float16))
    k_cache = np.zeros((1, 1, B * d), np.uint8); v_cache = np.zeros((1, 1, B * d), np.uint8)
    k_scale = np.zeros((1, 1, B), np.float32); v_scale = np.zeros((1, 1, B), np.float32)
    oracle.kv_cache_write_fp8(k, v, np.array([3], np.int64), k_cache, v_cache, k_scale, v_scale,
                              H_k=1, d=d, B=B)
    return (k_cache[0, 0, k_tile_index(d, 16, B)[3]], v_cache[0, 0, v_tile_index(d, 16, B)[3]],
            k_scale[0, 0, 3], v_scale[0, 0, 3])


def test_amax_element_maps_to_448(oracle_mod):
    rng = np.random.default_rng(0)
    for trial in range(50):
        x = rng.standard_normal(64).astype(np.float16)
        kc, vc, ks, vs = _one_row(oracle_mod, x)
        i = int(np.argmax(np.abs(x.astype(np.float32))))
        assert kc[i] == (0xFE if x[i] < 0 else 0x7E)
        assert ks == np.float32(np.abs(x[i].astype(np.float32))) / np.float32(448)
        assert np.array_equal(kc, vc) and ks == vs


def test_amax_448_gives_unit_scale_and_plain_codes(oracle_mod):
    rng = np.random.default_rng(1)
    x = rng.uniform(-400, 400, 64).astype(np.float16)
    x[5] = -448.0
    kc, _, ks, _ = _one_row(oracle_mod, x)
    assert ks == np.float32(1.0)
    assert np.array_equal(kc, oracle_mod.e4m3_encode_array(x.astype(np.float32)))


def test_power_of_two_scale_roundtrips_exactly(oracle_mod):
    table = e4m3_table()
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 0x7F, 64).astype(np.uint8) | (rng.integers(0, 2, 64) << 7).astype(np.uint8)
    codes[0] = 0x7E                                     # amax = 448 * 2^-5
    x = (table[codes] * 2.0 ** -5).astype(np.float16)   # exact in fp16
    assert np.array_equal(x.astype(np.float64), table[codes] * 2.0 ** -5)
    kc, _, ks, _ = _one_row(oracle_mod, x)
    assert ks == np.float32(2.0 ** -5)
    same = (kc == codes) | ((table[kc] == 0) & (table[codes] == 0) & ((kc ^ codes) & 0x7F == 0))
    assert np.all(same)


def test_all_zero_row_and_signed_zero(oracle_mod):
    x = np.zeros(64, np.float16)
    x[1] = np.float16(-0.0)
    kc, _, ks, _ = _one_row(oracle_mod, x)
    assert ks == np.float32(1.0)
    want = np.zeros(64, np.uint8); want[1] = 0x80
    assert np.array_equal(kc, want)


def test_fp16_subnormal_rows(oracle_mod):
    x = np.zeros(64, np.float16)
    x[0] = np.uint16(0x0001).view(np.float16)    # 2^-24
    x[1] = np.uint16(0x8001).view(np.float16)
    kc, _, ks, _ = _one_row(oracle_mod, x)
    assert kc[0] == 0x7E and kc[1] == 0xFE and ks == np.float32(2.0 ** -24) / np.float32(448)


def test_quantisation_error_bound(oracle_mod):
    """|x - scale*dec(code)| <= half the local E4M3 grid step times scale (plus fp32 slack)."""
    table = e4m3_table()
    rng = np.random.default_rng(3)
    for trial in range(20):
        x = (rng.standard_normal(128) * rng.choice([0.01, 1, 30])).astype(np.float16)
        kc, _, ks, _ = _one_row(oracle_mod, x)
        y = x.astype(np.float64) / float(ks)
        deq = table[kc]
        pos = table[:0x7F]
        mag = np.minimum(np.abs(y), 448)
        hi = np.searchsorted(pos, mag, side="left").clip(1, 0x7E)
        step = pos[hi] - pos[hi - 1]
        assert np.all(np.abs(np.clip(y, -448, 448) - deq) <= step / 2 * (1 + 2.0 ** -20) + 1e-300)


def test_skip_rule_and_untouched_slots(oracle_mod):
    """Eq. 5: tokens with a negative slot write nothing; nothing else is touched either."""
    w = workloads.make_custom("skip", seed=5, S=2, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[20, 37])
    slots = w.slots.copy()
    skip = np.zeros(len(slots), bool); skip[::3] = True
    slots[skip] = -1 - np.arange(skip.sum())
    cache = alloc_cache(w, fill_byte=0xA5)
    k_cache, v_cache, k_scale, v_scale = cache
    oracle_mod.kv_cache_write_fp8(w.k_ctx, w.v_ctx, slots, k_cache, v_cache, k_scale, v_scale,
                                  H_k=w.H_k, d=w.d, B=w.B)
    written = np.zeros(w.NB * w.B, bool); written[slots[~skip]] = True
    wr = written.reshape(w.NB, w.B)
    k_cache, v_cache = k_logical(w, k_cache), v_logical(w, v_cache)
    for blk in range(w.NB):
        for off in range(w.B):
            if wr[blk, off]:
                assert not np.isnan(k_scale[blk, :, off]).any()
            else:
                assert np.all(k_cache[blk, :, off, :] == 0xA5) and np.all(v_cache[blk, :, off, :] == 0xA5)
                assert np.isnan(k_scale[blk, :, off]).all() and np.isnan(v_scale[blk, :, off]).all()


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
def test_explicit_skip_set_is_the_negative_slot_rule(oracle_mod, kv_dtype):
    """Eq. 5 with the SkipSet spelled out: leaving token indices out through the set gives the same
    cache, byte for byte, as giving those tokens a negative slot; tokens in neither are written,
    and a token index outside the set whose slot is negative is still left out."""
    w = workloads.make_custom("skipset", seed=8, S=3, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[20, 37, 45], kv_dtype=kv_dtype)
    T = w.total_tokens
    rng = np.random.default_rng(3)
    in_set = rng.random(T) < 0.3
    in_set[[0, 31, 32, 33, 63, 64, T - 1]] = [True, True, False, True, False, True, True]   # word edges
    neg = np.zeros(T, bool); neg[5] = neg[70] = True; in_set[5] = False
    by_set = alloc_cache(w, fill_byte=0xA5)
    by_slot = alloc_cache(w, fill_byte=0xA5)
    slots_a = w.slots.copy(); slots_a[neg] = -1
    slots_b = w.slots.copy(); slots_b[in_set | neg] = -7
    write = oracle_mod.kv_cache_write_fp8 if kv_dtype == "e4m3" else oracle_mod.kv_cache_write_fp16
    args = lambda c: c if kv_dtype == "e4m3" else c[:2]
    write(w.k_ctx, w.v_ctx, slots_a, *args(by_set), H_k=w.H_k, d=w.d, B=w.B, skip_set=np.nonzero(in_set)[0])
    write(w.k_ctx, w.v_ctx, slots_b, *args(by_slot), H_k=w.H_k, d=w.d, B=w.B)
    for a, b in zip(by_set, by_slot):
        if a is not None:
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    # and the set really removed something and kept something
    full = alloc_cache(w, fill_byte=0xA5)
    write(w.k_ctx, w.v_ctx, w.slots, *args(full), H_k=w.H_k, d=w.d, B=w.B)
    assert not np.array_equal(full[0].view(np.uint8), by_set[0].view(np.uint8))
    assert np.any(by_set[0].view(np.uint8) != 0xA5)
    empty = alloc_cache(w, fill_byte=0xA5)
    write(w.k_ctx, w.v_ctx, w.slots, *args(empty), H_k=w.H_k, d=w.d, B=w.B, skip_set=np.arange(T))
    assert np.all(empty[0].view(np.uint8) == 0xA5) and np.all(empty[1].view(np.uint8) == 0xA5)


def test_slot_and_block_indexing_brute_force(oracle_mod):
    """Write tokens one at a time in random order; read back through the block table."""
    w = workloads.make_custom("idx", seed=6, S=3, H_q=6, H_k=3, d=64, B=16, NB=16,
                              context_lens=[1, 33, 48])
    cache = alloc_cache(w, fill_byte=0xEE)
    order = np.random.default_rng(0).permutation(w.total_tokens)
    for i in order:
        oracle_fill(oracle_mod, w, idx=np.array([i]), cache=cache)
    k_cache, v_cache, k_scale, v_scale = cache
    k_cache, v_cache = k_logical(w, k_cache), v_logical(w, v_cache)
    rows = {}
    for s in range(w.S):
        for j in range(int(w.context_lens[s])):
            rows[(s, j)] = int(w.seq_start[s]) + j
    for (s, j), i in rows.items():
        pb = int(w.block_tables[s, j // w.B]); off = j % w.B
        assert w.slots[i] == pb * w.B + off
        for g in range(w.H_k):
            kc, vc, ks, vs = _one_row(oracle_mod, w.k_ctx[i, g], w.v_ctx[i, g])
            assert np.array_equal(k_cache[pb, g, off, :], kc)
            assert np.array_equal(v_cache[pb, g, off, :], vc)
            assert k_scale[pb, g, off] == ks and v_scale[pb, g, off] == vs


def test_fp16_write_is_a_pure_scatter(oracle_mod):
    w = workloads.make_custom("f16", seed=7, S=2, H_q=4, H_k=4, d=64, B=16, NB=8,
                              context_lens=[17, 30], kv_dtype="fp16")
    k_cache, v_cache, _, _ = oracle_fill(oracle_mod, w)
    k_cache, v_cache = k_logical(w, k_cache), v_logical(w, v_cache)
    for s in range(w.S):
        for j in range(int(w.context_lens[s])):
            i = int(w.seq_start[s]) + j
            pb = int(w.block_tables[s, j // w.B]); off = j % w.B
            assert np.array_equal(k_cache[pb, :, off, :].view(np.uint16), w.k_ctx[i].view(np.uint16))
            assert np.array_equal(v_cache[pb, :, off, :].view(np.uint16), w.v_ctx[i].view(np.uint16))
