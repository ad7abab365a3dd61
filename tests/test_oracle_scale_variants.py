"""Pins for the oracle's comparison schemes (the alternatives Opt-KV's dynamic per-token E4M3 scale
stands against): the OCP E5M2 codec and the per-block / static scale rules of
orc_kv_cache_write_fp8_scaled.

None of these re-type the oracle's formula: format landmarks from the OCP definition, torch's
float8_e5m2 / float16 as an independent library, a brute-force nearest-value search, round-trip
and closed-form invariants, the numpy restatement in oracle/variants.py (a second, independent
implementation), and the existing per-token E4M3 write as the special case."""
import os

import numpy as np
import pytest
import torch

import workloads
from helpers import alloc_cache, e4m3_table, k_logical, oracle_fill, softmax_attention, v_logical

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e5m2_landmarks.txt")


def e5m2_table() -> np.ndarray:
    """All 256 OCP E5M2 values as float64, decoded by torch's float8_e5m2 (a library)."""
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e5m2).to(torch.float64).numpy()


def _parse(v):
    if v in ("nan", "inf", "-inf"):
        return float(v)
    sign = -1.0 if v.startswith("-") else 1.0
    v = v.lstrip("-")
    if "2^" in v:
        m, e = v.split("2^")
        m = float(m.rstrip("*")) if m else 1.0
        return sign * m * 2.0 ** int(e)
    return sign * float(v)


def test_e5m2_decode_landmarks_and_library(oracle_mod):
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        want, got = _parse(val), oracle_mod.e5m2_decode(int(code, 16))
        assert (np.isnan(got) if np.isnan(want) else (got == want and np.signbit(got) == np.signbit(want))), code
    table = e5m2_table()
    for c in range(256):
        got = oracle_mod.e5m2_decode(c)
        assert (np.isnan(got) if np.isnan(table[c]) else got == table[c]), c
    # an E5M2 code is the high byte of the fp16 pattern of its value
    for c in range(256):
        h = np.array([c << 8], dtype=np.uint16).view(np.float16)[0]
        got = oracle_mod.e5m2_decode(c)
        assert (np.isnan(got) if np.isnan(h) else got == float(h)), c


def test_e5m2_encode_round_trip_nearest_and_saturation(oracle_mod):
    table = e5m2_table()
    finite = [c for c in range(256) if np.isfinite(table[c])]
    for c in finite:
        assert oracle_mod.e5m2_encode(table[c]) == c, c
    # brute force: nearest finite code, ties to the even mantissa, on every finite fp16 input
    # inside the format's range and on every midpoint of neighbouring values
    pos = np.array(sorted(table[c] for c in range(0x7C)))
    x16 = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    x16 = x16[np.isfinite(x16) & (np.abs(x16) <= 57344.0)]
    mids = (pos[1:] + pos[:-1]) / 2
    xs = np.concatenate([x16, mids, -mids])
    got = oracle_mod.e5m2_encode_array(xs.astype(np.float32))
    assert np.all(xs.astype(np.float32).astype(np.float64) == xs)          # all exact in binary32
    codes = np.arange(0x7C)
    dist = np.abs(np.abs(xs)[:, None] - table[codes][None, :])
    best = dist.min(axis=1)
    for i in np.nonzero((dist == best[:, None]).sum(axis=1) > 1)[0]:       # ties: even mantissa wins
        cands = codes[dist[i] == best[i]]
        dist[i, [c for c in cands if c & 1]] = np.inf
    want = dist.argmin(axis=1).astype(np.uint8) | np.where(np.signbit(xs), 0x80, 0).astype(np.uint8)
    assert np.array_equal(got, want)
    # library cross-check inside the range
    t = torch.from_numpy(x16.astype(np.float32)).to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(oracle_mod.e5m2_encode_array(x16.astype(np.float32)), t)
    # saturation, never an infinity: 57344 itself, the would-be tie to infinity 61440, far beyond
    for y in (57344.0, 57345.0, 61440.0, 65504.0, 1e30):
        assert oracle_mod.e5m2_encode(y) == 0x7B and oracle_mod.e5m2_encode(-y) == 0xFB
    assert oracle_mod.e5m2_encode(float("nan")) == 0x7F
    assert oracle_mod.e5m2_encode(-0.0) == 0x80


def _write(orc, w, fmt, mode, cache=None, idx=None, **kw):
    cache = alloc_cache(w) if cache is None else cache
    k, v, s = (w.k_ctx, w.v_ctx, w.slots) if idx is None else (
        np.ascontiguousarray(w.k_ctx[idx]), np.ascontiguousarray(w.v_ctx[idx]), np.ascontiguousarray(w.slots[idx]))
    orc.kv_cache_write_fp8_scaled(k, v, s, *cache, H_k=w.H_k, d=w.d, B=w.B, fmt=fmt, scale_mode=mode, **kw)
    return cache


def _dequant(w, cache, fmt):
    """[NB, H_k, B, d] float64 values of K and V by direct indexing and a library decode table."""
    table = e4m3_table() if fmt == "e4m3" else e5m2_table()
    kc, vc, ks, vs = cache
    return (table[k_logical(w, kc)] * ks.astype(np.float64)[..., None],
            table[v_logical(w, vc)] * vs.astype(np.float64)[..., None])


def test_token_mode_e4m3_is_the_method_write(oracle_mod):
    w = workloads.make_custom("sv", seed=11, S=2, H_q=4, H_k=2, d=64, B=16, NB=12, context_lens=[70, 33])
    a, b = oracle_fill(oracle_mod, w), _write(oracle_mod, w, "e4m3", "token")
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


@pytest.mark.parametrize("fmt,cmax,top", [("e4m3", 448.0, 0x7E), ("e5m2", 57344.0, 0x7B)])
def test_token_mode_closed_forms(oracle_mod, fmt, cmax, top):
    """The row's absmax element becomes +-max code; a row whose absmax is the max code has scale 1
    and codes enc(x); a power-of-two scale round-trips grid values exactly."""
    w = workloads.make_custom("cf", seed=12, S=1, H_q=2, H_k=2, d=64, B=16, NB=2, context_lens=[3])
    table = e4m3_table() if fmt == "e4m3" else e5m2_table()
    enc = oracle_mod.e4m3_encode_array if fmt == "e4m3" else oracle_mod.e5m2_encode_array
    rng = np.random.default_rng(0)
    k = rng.standard_normal((3, 2, 64)).astype(np.float16)
    k[1, 0, :] = 0
    k[1, 0, 5] = np.float16(-cmax if cmax < 60000 else -57344.0)          # absmax = the max code
    grid = table[[c for c in range(0x10, top)]]                             # exact grid values
    k[2, 1, :] = (rng.choice(grid, 64) * 2.0 ** -3).astype(np.float16)
    k[2, 1, 0] = np.float16(cmax * 2.0 ** -3)                               # scale = 2^-3 exactly
    w.k_ctx, w.v_ctx = k, k.copy()
    cache = _write(oracle_mod, w, fmt, "token")
    kl = k_logical(w, cache[0]); ks = cache[2]
    for t in range(3):
        blk, off = divmod(int(w.slots[t]), 16)
        for h in range(2):
            row = k[t, h].astype(np.float64)
            j = int(np.argmax(np.abs(row)))
            assert kl[blk, h, off, j] == (top | (0x80 if row[j] < 0 else 0))
            assert ks[blk, h, off] == np.float32(np.float32(np.abs(row).max()) / np.float32(cmax))
    blk, off = divmod(int(w.slots[1]), 16)
    assert ks[blk, 0, off] == 1.0 and np.array_equal(kl[blk, 0, off], enc(k[1, 0].astype(np.float32)))
    blk, off = divmod(int(w.slots[2]), 16)
    assert ks[blk, 1, off] == 0.125
    assert np.array_equal(table[kl[blk, 1, off]] * 0.125, k[2, 1].astype(np.float64))


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_block_and_static_scales(oracle_mod, fmt):
    cmax = 448.0 if fmt == "e4m3" else 57344.0
    w = workloads.make_custom("bs", seed=13, S=3, H_q=4, H_k=2, d=64, B=16, NB=16,
                              context_lens=[40, 16, 7], k_outlier_frac=0.1)
    # ---- block mode, everything in one call: every token of a block carries the block's scale,
    # which is the largest row absmax of the block / max code
    cache = _write(oracle_mod, w, fmt, "block")
    for name, rows, scales in (("k", w.k_ctx, cache[2]), ("v", w.v_ctx, cache[3])):
        amax = np.abs(rows.astype(np.float32)).max(axis=2)                  # [tokens, H_k]
        blocks = w.slots // 16
        for b in np.unique(blocks):
            mine = blocks == b
            want = (amax[mine].max(axis=0) / np.float32(cmax)).astype(np.float32)
            for t in np.nonzero(mine)[0]:
                assert np.array_equal(scales[b, :, int(w.slots[t]) % 16], want), (name, b)
    # values stay within half a grid step of the block scale (nothing saturates: scale covers the block)
    kd, vd = _dequant(w, cache, fmt)
    step = 2.0 ** (-3 if fmt == "e4m3" else -2)
    for t in range(w.total_tokens):
        b, off = divmod(int(w.slots[t]), 16)
        s = cache[2][b, :, off].astype(np.float64)[:, None]
        x = w.k_ctx[t].astype(np.float64)
        assert np.all(np.abs(kd[b, :, off] - x) <= np.maximum(np.abs(x) * step / 2, s * 2.0 ** -6 * (1 if fmt == "e4m3" else 2.0 ** -8)) * (1 + 1e-6) + 1e-12)
    # ---- block mode, one token per call: a block of one is the token's own scale
    one = alloc_cache(w)
    for t in range(w.total_tokens):
        _write(oracle_mod, w, fmt, "block", cache=one, idx=np.array([t]))
    tok = _write(oracle_mod, w, fmt, "token")
    for x, y in zip(one, tok):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
    # ---- two calls into one block: the rows of the first call keep their scale
    first = np.arange(0, 5); second = np.arange(5, 16)
    two = _write(oracle_mod, w, fmt, "block", idx=first)
    _write(oracle_mod, w, fmt, "block", cache=two, idx=second)
    b0 = int(w.slots[0]) // 16
    a1 = np.abs(w.k_ctx[first].astype(np.float32)).max(axis=(0, 2)) / np.float32(cmax)
    a2 = np.abs(w.k_ctx[second].astype(np.float32)).max(axis=(0, 2)) / np.float32(cmax)
    assert np.array_equal(two[2][b0, :, 0:5], np.repeat(a1.astype(np.float32)[:, None], 5, 1))
    assert np.array_equal(two[2][b0, :, 5:16], np.repeat(a2.astype(np.float32)[:, None], 11, 1))
    # ---- static mode: the given scale everywhere, rows beyond it saturate at +-max code
    k_static = np.array([0.5, 2.0 ** -9], dtype=np.float32); v_static = np.array([1.0, 0.25], dtype=np.float32)
    st = _write(oracle_mod, w, fmt, "static", k_static=k_static, v_static=v_static)
    used = np.zeros((w.NB, 16), bool); used[w.slots // 16, w.slots % 16] = True
    for h in range(2):
        assert np.all(st[2][:, h][used] == k_static[h]) and np.all(st[3][:, h][used] == v_static[h])
    kd, _ = _dequant(w, st, fmt)
    for t in range(w.total_tokens):
        b, off = divmod(int(w.slots[t]), 16)
        x = w.k_ctx[t, 1].astype(np.float64)
        big = np.abs(x) >= cmax * 2.0 ** -9
        assert np.array_equal(kd[b, 1, off][big], np.sign(x[big]) * cmax * 2.0 ** -9)     # saturated


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
@pytest.mark.parametrize("mode", ["token", "block", "static"])
def test_numpy_restatement_agrees_value_for_value(oracle_mod, fmt, mode):
    """oracle/variants.py (numpy, written separately: its own E5M2 rounding by scaling and
    np.round, its own scale rules) and the C write give the same dequantised rows."""
    from oracle import variants
    w = workloads.make_custom("nv", seed=14, S=1, H_q=4, H_k=2, d=64, B=16, NB=8,
                              context_lens=[112], k_outlier_frac=0.05)
    calib = slice(0, 32)
    kw = {}
    if mode == "static":
        kw = dict(k_static=(np.abs(w.k_ctx[calib].astype(np.float32)).max(axis=(0, 2)) /
                            np.float32(variants.E4M3_MAX if fmt == "e4m3" else variants.E5M2_MAX)).astype(np.float32),
                  v_static=(np.abs(w.v_ctx[calib].astype(np.float32)).max(axis=(0, 2)) /
                            np.float32(variants.E4M3_MAX if fmt == "e4m3" else variants.E5M2_MAX)).astype(np.float32))
    cache = _write(oracle_mod, w, fmt, mode, **kw)
    kd, vd = _dequant(w, cache, fmt)
    scheme = {"token": "per_token", "block": "per_block", "static": "static"}[mode]
    # the sequence's blocks in logical order (its tokens fill whole blocks: 112 = 7 x 16)
    order = w.block_tables[0, :7]
    K = kd[order].transpose(0, 2, 1, 3).reshape(112, 2, 64)
    V = vd[order].transpose(0, 2, 1, 3).reshape(112, 2, 64)
    assert np.array_equal(K, variants.quantise_rows(w.k_ctx, scheme, fmt, calib=w.k_ctx[calib]))
    assert np.array_equal(V, variants.quantise_rows(w.v_ctx, scheme, fmt, calib=w.v_ctx[calib]))


def test_attention_over_an_e5m2_cache(oracle_mod):
    """The read side with kv_dtype E5M2: textbook attention on rows dequantised by direct indexing
    and torch's table."""
    w = workloads.make_custom("a5", seed=15, S=2, H_q=4, H_k=2, d=64, B=16, NB=12, context_lens=[50, 17])
    cache = _write(oracle_mod, w, "e5m2", "token")
    out = oracle_mod.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q, H_k=w.H_k,
                                      d=w.d, B=w.B, softmax_scale=w.softmax_scale, fmt="e5m2")
    kd, vd = _dequant(w, cache, "e5m2")
    for s in range(w.S):
        t = int(w.context_lens[s])
        blk = w.block_tables[s, np.arange(t) // 16]; off = np.arange(t) % 16
        for h in range(w.H_q):
            g = h // (w.H_q // w.H_k)
            ref = softmax_attention(w.q[s, h].astype(np.float64), kd[blk, g, off], vd[blk, g, off], w.softmax_scale)
            assert np.max(np.abs(out[s, h] - ref)) < 1e-12
    # and it differs from reading the same bytes as E4M3 (the format argument is honoured)
    other = oracle_mod.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q, H_k=w.H_k,
                                        d=w.d, B=w.B, softmax_scale=w.softmax_scale, fmt="e4m3")
    assert np.max(np.abs(other - out)) > 1e-3
