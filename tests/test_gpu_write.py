"""GPU parity: quantise-on-write (Opt-KV Eq. 5, Alg. 1 phase 1) against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import workloads
from gpu_utils import alloc_dev_cache, dev_cache_to_host, hip_write
from helpers import alloc_cache, oracle_fill

pytestmark = pytest.mark.gpu


def _compare_caches(w, host, devc, what):
    names = ["k_cache", "v_cache", "k_scale", "v_scale"]
    got = dev_cache_to_host(w, devc)
    for name, a, b in zip(names, host, got):
        if a is None:
            continue
        au = (a.view(np.uint8) if a.dtype == np.uint8 else
              a.view(np.uint32 if a.dtype == np.float32 else np.uint16)).reshape(-1)
        bu = b.view(au.dtype).reshape(-1)
        bad = np.nonzero(au != bu)
        assert bad[0].size == 0, f"{what}: {name} differs at {bad[0].size} places, first {tuple(x[0] for x in bad)}"


def _roundtrip(w, slots=None, idx=None, fill=0xA5):
    host = alloc_cache(w, fill_byte=fill)
    if w.kv_dtype == "e4m3":    # alloc_cache poisons scales with NaN; use the same byte pattern as the GPU side
        host[2].view(np.uint8)[...] = fill
        host[3].view(np.uint8)[...] = fill
    devc = alloc_dev_cache(w, fill_byte=fill)
    return host, devc


@pytest.mark.parametrize("cfg,shrink", [(0, 1), (1, 8), (3, 16), (4, 8), (1, 1)])
def test_fp8_cache_bytes_and_scales_bit_exact(oracle_mod, cfg, shrink):
    w = workloads.make(cfg, shrink=shrink)
    print(f"write parity cfg={cfg} shrink={shrink} tokens={w.total_tokens}", flush=True)
    host, devc = _roundtrip(w)
    oracle_fill(oracle_mod, w, cache=host)
    hip_write(w, devc)
    _compare_caches(w, host, devc, f"cfg{cfg}/shrink{shrink}")


def test_fp16_cache_is_a_pure_scatter(oracle_mod):
    w = workloads.make(2, shrink=8)
    host, devc = _roundtrip(w)
    oracle_fill(oracle_mod, w, cache=host)
    hip_write(w, devc)
    _compare_caches(w, host, devc, "cfg2")


def test_head_dim_64_and_odd_head_counts(oracle_mod):
    for seed, (H_q, H_k, d) in enumerate([(6, 3, 64), (7, 7, 64), (12, 4, 128), (1, 1, 128)]):
        w = workloads.make_custom("w", seed=100 + seed, S=3, H_q=H_q, H_k=H_k, d=d, B=16, NB=32,
                                  context_lens=[1, 47, 130])
        host, devc = _roundtrip(w)
        oracle_fill(oracle_mod, w, cache=host)
        hip_write(w, devc)
        _compare_caches(w, host, devc, f"H_k={H_k} d={d}")


def test_skip_rule_negative_slots(oracle_mod):
    """Eq. 5: a negative slot writes nothing; untouched bytes keep their poison."""
    w = workloads.make_custom("skip", seed=5, S=2, H_q=8, H_k=2, d=128, B=16, NB=16,
                              context_lens=[70, 37])
    slots = w.slots.copy()
    slots[::3] = -1 - np.arange(len(slots[::3]))
    host, devc = _roundtrip(w)
    oracle_mod.kv_cache_write_fp8(w.k_ctx, w.v_ctx, slots, *host, H_k=w.H_k, d=w.d, B=w.B)
    hip_write(w, devc, slots=slots)
    _compare_caches(w, host, devc, "skip")
    # all-negative and empty calls are no-ops
    before = [t.clone() for t in devc]
    hip_write(w, devc, slots=np.full_like(slots, -1))
    hip_write(w, devc, idx=np.zeros(0, np.int64))
    for a, b in zip(before, devc):
        assert torch.equal(a, b)


def test_every_fp16_input_value(oracle_mod):
    """All 63488 finite fp16 values as inputs, in rows whose absmax is 448 (scale exactly 1), a
    random value, or the row's own maximum; plus all-zero and signed-zero rows."""
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16)
    finite = vals[np.isfinite(vals)]
    rng = np.random.default_rng(7)
    rows = []
    small = finite[np.abs(finite.astype(np.float32)) <= 448]
    pad = (-len(small)) % 127
    small = np.concatenate([small, np.zeros(pad, np.float16)]).reshape(-1, 127)
    rows.append(np.concatenate([np.full((len(small), 1), 448, np.float16), small], axis=1))  # scale 1
    allv = np.concatenate([finite, np.zeros((-len(finite)) % 128, np.float16)])
    rows.append(rng.permutation(allv).reshape(-1, 128))                                       # mixed
    srt = np.sort(allv.astype(np.float32)).astype(np.float16).reshape(-1, 128)               # similar magnitudes
    rows.append(srt)
    z = np.zeros((2, 128), np.float16); z[1, ::2] = np.float16(-0.0)
    rows.append(z)
    k = np.concatenate(rows)
    T = len(k)
    v = k[rng.permutation(T)]
    w = workloads.make_custom("sweep", seed=9, S=1, H_q=1, H_k=1, d=128, B=16,
                              NB=(T + 15) // 16 + 1, context_lens=[T])
    w.k_ctx = np.ascontiguousarray(k.reshape(T, 1, 128)); w.v_ctx = np.ascontiguousarray(v.reshape(T, 1, 128))
    host, devc = _roundtrip(w)
    oracle_fill(oracle_mod, w, cache=host)
    hip_write(w, devc)
    _compare_caches(w, host, devc, "fp16 sweep")


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
def test_explicit_skip_set(oracle_mod, kv_dtype):
    """Eq. 5 with the SkipSet given as a device bitmap over the call's token indices."""
    import paper_2602_09323_amd as coopt
    from gpu_utils import dev, shape_of
    w = workloads.make_custom("skipset", seed=108, S=4, H_q=10, H_k=2, d=128, B=16, NB=64,
                              context_lens=[1, 100, 257, 64], kv_dtype=kv_dtype)
    T = w.total_tokens
    rng = np.random.default_rng(4)
    in_set = rng.random(T) < 0.35
    in_set[[0, 31, 32, 33, T - 1]] = [True, False, True, True, False]
    slots = w.slots.copy()
    slots[7] = -1                                   # a negative slot outside the set still skips
    host, devc = _roundtrip(w)
    write = oracle_mod.kv_cache_write_fp8 if kv_dtype == "e4m3" else oracle_mod.kv_cache_write_fp16
    write(w.k_ctx, w.v_ctx, slots, *(host if kv_dtype == "e4m3" else host[:2]), H_k=w.H_k, d=w.d,
          B=w.B, skip_set=np.nonzero(in_set)[0])
    bits = np.zeros((T + 31) // 32, dtype=np.uint32)
    for i in np.nonzero(in_set)[0]:
        bits[i >> 5] |= np.uint32(1 << (i & 31))
    coopt.kv_cache_write_skipset(dev(w.k_ctx.view(np.uint16)), dev(w.v_ctx.view(np.uint16)), dev(slots),
                                 dev(bits), *devc, shape_of(w))
    torch.cuda.synchronize()
    _compare_caches(w, host, devc, f"skip set {kv_dtype}")
    # NULL set = the plain write
    host2, devc2 = _roundtrip(w)
    write(w.k_ctx, w.v_ctx, slots, *(host2 if kv_dtype == "e4m3" else host2[:2]), H_k=w.H_k, d=w.d, B=w.B)
    coopt.kv_cache_write_skipset(dev(w.k_ctx.view(np.uint16)), dev(w.v_ctx.view(np.uint16)), dev(slots),
                                 None, *devc2, shape_of(w))
    torch.cuda.synchronize()
    _compare_caches(w, host2, devc2, f"empty skip set {kv_dtype}")


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
@pytest.mark.parametrize("d,H_k", [(128, 2), (64, 3)])
def test_bulk_calls_with_every_slot_pattern(oracle_mod, d, H_k, kv_dtype):
    """Calls of 64 tokens and more take the bulk kernel, whose V stores depend on how four
    consecutive tokens' slots lie: aligned runs, runs that start off a multiple of four, runs cut
    by skipped tokens, slots scattered at random -- all against the oracle, and the same tokens
    again through calls small enough for the row kernel."""
    import paper_2602_09323_amd as coopt
    from gpu_utils import dev, shape_of
    T, NB = 333, 64
    w = workloads.make_custom("bulk", seed=200 + d, S=1, H_q=H_k, H_k=H_k, d=d, B=16, NB=NB,
                              context_lens=[T], kv_dtype=kv_dtype)
    rng = np.random.default_rng(d)
    fp8 = kv_dtype == "e4m3"
    o_write = oracle_mod.kv_cache_write_fp8 if fp8 else oracle_mod.kv_cache_write_fp16
    d_write = coopt.kv_cache_write_fp8 if fp8 else coopt.kv_cache_write_fp16
    patterns = {}
    patterns["aligned runs"] = np.arange(T, dtype=np.int64) + 32
    patterns["runs from an odd slot"] = np.arange(T, dtype=np.int64) + 37
    scattered = rng.permutation(NB * 16)[:T].astype(np.int64)
    patterns["scattered"] = scattered
    cut = np.arange(T, dtype=np.int64) + 48
    cut[rng.random(T) < 0.2] = -1
    patterns["runs cut by skipped tokens"] = cut
    mixed = np.arange(T, dtype=np.int64) + 16
    mixed[100:200] = scattered[:100][np.argsort(rng.random(100))] % (NB * 16 - 600) + 500   # may collide: dedupe
    _, first = np.unique(mixed, return_index=True)
    keep = np.zeros(T, bool); keep[first] = True
    mixed[~keep] = -1
    patterns["runs and scatter mixed"] = mixed
    shape = shape_of(w)
    dk, dv = dev(w.k_ctx.view(np.uint16)), dev(w.v_ctx.view(np.uint16))
    for name, slots in patterns.items():
        host, devc = _roundtrip(w)
        o_write(w.k_ctx, w.v_ctx, slots, *(host if fp8 else host[:2]), H_k=H_k, d=d, B=16)
        d_write(dk, dv, dev(slots), *(devc if fp8 else devc[:2]), shape)       # one bulk call
        torch.cuda.synchronize()
        _compare_caches(w, host, devc, f"bulk {kv_dtype} d={d}: {name}")
        _, devr = _roundtrip(w)
        ds = dev(slots)
        for i in range(0, T, 40):                                            # row kernel
            d_write(dk[i:i + 40], dv[i:i + 40], ds[i:i + 40], *(devr if fp8 else devr[:2]), shape)
        torch.cuda.synchronize()
        _compare_caches(w, host, devr, f"rows {kv_dtype} d={d}: {name}")
