"""Pins for the oracle's number formats (OCP E4M3 codec, fp16 decode).

None of these re-type the oracle's formula: they use the format's landmark values, torch's
float8_e4m3fn / float16 as an independent library, a brute-force nearest-value search, and
order/round-trip invariants.
"""
import os

import numpy as np
import pytest
import torch

from helpers import e4m3_table

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e4m3_landmarks.txt")


def _parse(v):
    if v == "nan":
        return float("nan")
    sign = -1.0 if v.startswith("-") else 1.0
    v = v.lstrip("-")
    if "2^" in v:
        m, e = v.split("2^")
        m = float(m.rstrip("*")) if m else 1.0
        return sign * m * 2.0 ** int(e)
    return sign * float(v)


def test_decode_landmarks(oracle_mod):
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        want = _parse(val)
        got = oracle_mod.e4m3_decode(int(code, 16))
        if np.isnan(want):
            assert np.isnan(got)
        else:
            assert got == want and np.signbit(got) == np.signbit(want), (code, got, want)


def test_decode_matches_torch_for_all_codes(oracle_mod):
    table = e4m3_table()
    for c in range(256):
        got = oracle_mod.e4m3_decode(c)
        if np.isnan(table[c]):
            assert np.isnan(got)
        else:
            assert got == table[c], c


def test_decode_monotone_and_symmetric(oracle_mod):
    vals = [oracle_mod.e4m3_decode(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))
    for c in range(0x7F):
        assert oracle_mod.e4m3_decode(c | 0x80) == -vals[c]


def test_encode_roundtrip_all_finite_codes(oracle_mod):
    table = e4m3_table()
    for c in range(256):
        if np.isnan(table[c]):
            continue
        assert oracle_mod.e4m3_encode(table[c]) == c


def _brute_encode(y: np.ndarray, table: np.ndarray) -> np.ndarray:
    """Nearest finite E4M3 value by exhaustive search; ties go to the even code; sign kept."""
    pos = table[:0x7F]                                     # 0 .. 448, increasing
    a = np.abs(y.astype(np.float64))
    dist = np.abs(a[:, None] - pos[None, :])
    best = dist.min(axis=1)
    out = np.zeros(y.shape, dtype=np.uint8)
    for i in range(y.size):
        cand = np.nonzero(dist[i] == best[i])[0]
        c = cand[0] if len(cand) == 1 else [x for x in cand if x % 2 == 0][0]
        out[i] = c
    out |= np.where(np.signbit(y), 0x80, 0).astype(np.uint8)
    return out


def test_encode_brute_force_all_fp16(oracle_mod):
    table = e4m3_table()
    bits = np.arange(65536, dtype=np.uint16)
    y = bits.view(np.float16).astype(np.float32)
    keep = np.isfinite(y)
    y = y[keep]
    got = oracle_mod.e4m3_encode_array(y)
    # saturation for |y| >= 448 (includes 464, the would-be tie, and fp16 max)
    big = np.abs(y) >= 448
    assert np.all((got[big] & 0x7F) == 0x7E)
    want = _brute_encode(y[~big], table)
    assert np.array_equal(got[~big], want)


def test_encode_midpoints_tie_to_even(oracle_mod):
    table = e4m3_table()
    pos = table[:0x7F]
    mids = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)      # exact in binary32
    assert np.array_equal(mids.astype(np.float64), (pos[:-1] + pos[1:]) / 2)
    got = oracle_mod.e4m3_encode_array(mids)
    for i, c in enumerate(got):
        assert c in (i, i + 1) and c % 2 == 0, (i, c)
    # one float below / above a midpoint goes to the nearer neighbour
    below = np.nextafter(mids, np.float32(0))
    above = np.nextafter(mids, np.float32(1000))
    assert np.array_equal(oracle_mod.e4m3_encode_array(below), np.arange(0x7E, dtype=np.uint8))
    assert np.array_equal(oracle_mod.e4m3_encode_array(above), np.arange(1, 0x7F, dtype=np.uint8))
    neg = oracle_mod.e4m3_encode_array(-mids)
    assert np.array_equal(neg, got | 0x80)


def test_encode_saturation(oracle_mod):
    for y in [448.0, 449.0, 464.0, 480.0, 1e30, 65504.0]:
        assert oracle_mod.e4m3_encode(y) == 0x7E
        assert oracle_mod.e4m3_encode(-y) == 0xFE
    assert oracle_mod.e4m3_encode(447.9) == 0x7E          # nearer to 448 than to 416
    assert oracle_mod.e4m3_encode(431.9) == 0x7D          # below the 416/448 midpoint 432
    assert oracle_mod.e4m3_encode(432.0) == 0x7E          # tie 416|448 -> even mantissa (0x7E)
    assert oracle_mod.e4m3_encode(-0.0) == 0x80 and oracle_mod.e4m3_encode(0.0) == 0x00
    assert oracle_mod.e4m3_encode(2.0 ** -10) == 0x00     # tie 0 | 2^-9 -> even (0)
    assert oracle_mod.e4m3_encode(3 * 2.0 ** -10) == 0x02  # tie 2^-9 | 2^-8 -> even (2)


def test_encode_matches_torch_in_range(oracle_mod):
    rng = np.random.default_rng(1)
    y = np.concatenate([
        rng.uniform(-448, 448, 20000), rng.normal(0, 1, 20000), rng.normal(0, 0.01, 20000),
        rng.uniform(-2.0 ** -5, 2.0 ** -5, 20000)]).astype(np.float32)
    want = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle_mod.e4m3_encode_array(y)
    assert np.array_equal(got, want)


def test_f16_decode_matches_numpy(oracle_mod):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    for b in range(0, 65536, 7):
        got = oracle_mod.f16_to_f64(b)
        if np.isnan(want[b]):
            assert np.isnan(got)
        else:
            assert got == want[b] and np.signbit(got) == np.signbit(want[b])
    for b in [0x0001, 0x03FF, 0x0400, 0x7BFF, 0x8001, 0xFBFF, 0x3C00]:
        assert oracle_mod.f16_to_f64(b) == want[b]
