"""GPU parity: decode and the fused step run from a prepared schedule (coopt_decode_schedule_prepare
+ coopt_paged_gqa_decode_scheduled) against the oracle, to the same bar as the calls that derive
the schedule inside the launch; and what happens when the schedule does not fit the launch."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import planned, alloc_dev_cache, assert_close, dev, dev_cache_to_host, hip_write, shape_of
from helpers import alloc_cache, oracle_fill

pytestmark = pytest.mark.gpu

PLANS = [(128, 1, 2, 1024, 0), (32, 1, 1, 5, 0), (64, 1, 3, 64, 0), (128, 1, 2, 1024, 1)]


def _set_plan(plan):
    planned.set_plan(tokens_per_group=plan[0], waves_per_group=plan[1], pipeline_depth=plan[2],
                          grid_waves=plan[3], softmax_reduction=plan[4])


def _oracle_decode(oracle, w, cache, lens=None):
    return oracle.paged_gqa_decode(w.q, *cache, w.block_tables,
                                   w.context_lens if lens is None else lens, H_q=w.H_q, H_k=w.H_k,
                                   d=w.d, B=w.B, softmax_scale=w.softmax_scale)


def _same_cache(w, dcache, cache, what):
    got = dev_cache_to_host(w, dcache)
    for name, g, r in zip(("k_cache", "v_cache", "k_scale", "v_scale"), got, cache):
        if r is None:
            continue
        assert np.array_equal(g.reshape(-1).view(np.uint8), r.reshape(-1).view(np.uint8)), f"{what}: {name}"


def _prepare(w, slots=None, lens=None, fill=0):
    shape = shape_of(w)
    n = planned.decode_schedule_bytes(shape)
    assert n > 0 and n % 4 == 0
    sched = torch.full((n + 64,), fill, dtype=torch.uint8, device="cuda")      # 64 guard bytes
    sched[n:] = 0xC3
    dslots = None if slots is None else dev(np.asarray(slots, dtype=np.int64))
    planned.decode_schedule_prepare(dev(w.block_tables), dev(w.context_lens if lens is None else lens),
                                  dslots, sched[:n], shape)
    torch.cuda.synchronize()
    assert bool((sched[n:] == 0xC3).all()), "prepare wrote past the schedule"
    return sched[:n]


def _run(w, dcache, sched, slots=None, k_new=None, v_new=None, lens=None, out=None):
    shape = shape_of(w)
    fused = slots is not None
    if fused:
        new = w.new_index()
        k = dev((w.k_ctx[new] if k_new is None else k_new).view(np.uint16))
        v = dev((w.v_ctx[new] if v_new is None else v_new).view(np.uint16))
        s = dev(np.asarray(slots, dtype=np.int64))
    else:
        k = v = s = None
    if out is None:
        out = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    ws = torch.empty(max(16, planned.decode_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    planned.paged_gqa_decode_scheduled(k, v, s, dev(w.q.view(np.uint16)), *dcache,
                                     dev(w.context_lens if lens is None else lens), out, ws, sched, shape)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("kv_dtype", ["e4m3", "fp16"])
@pytest.mark.parametrize("H_q,H_k,d", [(40, 8, 128), (6, 2, 64), (3, 3, 128), (16, 1, 64)])
def test_scheduled_decode_and_step(oracle_mod, kv_dtype, H_q, H_k, d):
    lens = [1, 2, 16, 17, 32, 33, 255, 257, 700, 512, 31]
    w = workloads.make_custom("sched", seed=81, S=len(lens), H_q=H_q, H_k=H_k, d=d, B=16, NB=256,
                              context_lens=lens, kv_dtype=kv_dtype, max_blocks=48)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    new_slots = w.slots[w.new_index()]
    for plan in PLANS:
        _set_plan(plan)
        # plain decode over a cache that already holds every token
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache)
        got = _run(w, dcache, _prepare(w))
        assert_close(got, ref, f"scheduled decode {kv_dtype} {H_q}/{H_k}/{d} plan={plan}")
        # fused step: history in the cache, the new tokens written by the launch
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        got = _run(w, dcache, _prepare(w, slots=new_slots), slots=new_slots)
        assert_close(got, ref, f"scheduled step {kv_dtype} {H_q}/{H_k}/{d} plan={plan}")
        _same_cache(w, dcache, cache, f"scheduled step {kv_dtype} plan={plan}")


def test_one_schedule_serves_many_layers(oracle_mod):
    """Layers share block tables and lengths, not values: one schedule, three caches."""
    lens = [300, 77, 1, 1000, 48]
    ws_ = [workloads.make_custom("layer", seed=90 + i, S=len(lens), H_q=10, H_k=2, d=128, B=16, NB=200,
                                 context_lens=lens, max_blocks=64) for i in range(3)]
    w0 = ws_[0]
    sched = _prepare(w0, slots=w0.slots[w0.new_index()])
    before = sched.clone()
    for w in ws_:
        # same tables and slots in every layer (same generator structure), other K/V/q values
        w.block_tables[...] = w0.block_tables
        w.slots[...] = w0.slots
        cache = oracle_fill(oracle_mod, w)
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        got = _run(w, dcache, sched, slots=w.slots[w.new_index()])
        assert_close(got, _oracle_decode(oracle_mod, w, cache), "layer from a shared schedule")
        _same_cache(w, dcache, cache, "layer from a shared schedule")
    assert torch.equal(sched, before), "a scheduled launch changed the schedule"


def test_filtered_tokens_and_empty_sequences(oracle_mod):
    lens = np.array([40, 1, 300, 17, 64, 5], dtype=np.int32)
    w = workloads.make_custom("sskip", seed=82, S=len(lens), H_q=10, H_k=2, d=128, B=16, NB=64,
                              context_lens=lens, max_blocks=20)
    cache = oracle_fill(oracle_mod, w)
    new = w.new_index()
    slots = w.slots[new].copy()
    skip = np.array([False, True, True, False, False, True])
    slots[skip] = -1
    run_lens = lens.copy()
    run_lens[4] = 0
    ref = _oracle_decode(oracle_mod, w, cache, lens=run_lens)
    dcache = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, dcache)
    rng = np.random.default_rng(5)
    k_new, v_new = w.k_ctx[new].copy(), w.v_ctx[new].copy()
    junk = skip | (run_lens == 0)
    k_new[junk] = rng.standard_normal(k_new[junk].shape).astype(np.float16) * 30
    v_new[junk] = rng.standard_normal(v_new[junk].shape).astype(np.float16) * 30
    sched = _prepare(w, slots=slots, lens=run_lens)
    got = _run(w, dcache, sched, slots=slots, k_new=k_new, v_new=v_new, lens=run_lens)
    assert np.all(got[4] == 0)
    assert_close(got, ref, "scheduled step with filtered tokens")
    _same_cache(w, dcache, cache, "filtered tokens leave the cache alone")
    # every sequence empty: a schedule with no work, zero rows
    zero = np.zeros_like(lens)
    got = _run(w, dcache, _prepare(w, lens=zero), lens=zero)
    assert np.all(got == 0)


def test_many_sequences(oracle_mod):
    rng = np.random.default_rng(7)
    S = 150
    lens = rng.integers(1, 90, S).astype(np.int32)
    w = workloads.make_custom("smany", seed=83, S=S, H_q=8, H_k=2, d=128, B=16, NB=1200,
                              context_lens=lens, max_blocks=8)
    cache = oracle_fill(oracle_mod, w)
    ref = _oracle_decode(oracle_mod, w, cache)
    new_slots = w.slots[w.new_index()]
    for grid in (1024, 96):
        planned.set_plan(tokens_per_group=64, waves_per_group=1, pipeline_depth=2, grid_waves=grid)
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        got = _run(w, dcache, _prepare(w, slots=new_slots), slots=new_slots)
        assert_close(got, ref, f"scheduled S={S} grid={grid}")
        _same_cache(w, dcache, cache, f"scheduled S={S} grid={grid}")


def test_schedule_that_does_not_fit_is_refused_on_the_device(oracle_mod):
    """Wrong mode, wrong plan, never prepared: the launch touches nothing but the status word."""
    lens = [100, 40, 7]
    w = workloads.make_custom("stale", seed=84, S=len(lens), H_q=4, H_k=2, d=64, B=16, NB=32,
                              context_lens=lens, max_blocks=8)
    cache = oracle_fill(oracle_mod, w)
    new_slots = w.slots[w.new_index()]

    def untouched(sched, **kw):
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        before = [None if t is None else t.clone() for t in dcache]
        got = _run(w, dcache, sched, **kw)
        assert np.all(got == -7.0)
        for a, b in zip(dcache, before):
            assert a is None or torch.equal(a, b)
        assert int(sched.view(torch.int32)[1]) == 1

    decode_sched = _prepare(w)                                   # prepared for plain decode
    assert int(decode_sched.view(torch.int32)[1]) == 0
    untouched(decode_sched, slots=new_slots)                     # ... used for the fused step
    step_sched = _prepare(w, slots=new_slots)
    untouched(step_sched)                                        # and the other way round
    n = planned.decode_schedule_bytes(shape_of(w))
    for fill in (0, 0xFF):
        untouched(torch.full((n,), fill, dtype=torch.uint8, device="cuda"))   # never prepared
    fresh = _prepare(w)
    planned.set_plan(tokens_per_group=64, waves_per_group=1, pipeline_depth=2, grid_waves=1024)
    if planned.decode_schedule_bytes(shape_of(w)) <= fresh.numel():
        untouched(fresh)                                         # prepared under another plan
    # prepared again, it works again (and the status word is back to 0)
    again = _prepare(w)
    dcache = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, dcache)
    assert_close(_run(w, dcache, again), _oracle_decode(oracle_mod, w, cache), "prepared again")
    assert int(again.view(torch.int32)[1]) == 0


def test_full_size_configs(oracle_mod):
    for cfg in (1, 2, 3):
        w = workloads.make(cfg)
        cache = oracle_fill(oracle_mod, w)
        new_slots = w.slots[w.new_index()]
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=w.history_index())
        got = _run(w, dcache, _prepare(w, slots=new_slots), slots=new_slots)
        _same_cache(w, dcache, cache, f"cfg{cfg} scheduled step")
        ref = _oracle_decode(oracle_mod, w, cache)
        print("cfg%d scheduled step max-abs %.2e" % (cfg, assert_close(got, ref, f"cfg{cfg} scheduled")), flush=True)


def test_stale_slots_are_never_read(oracle_mod):
    """Opt-Pa Eq. 9 from a prepared schedule: tokens >= t and blocks >= ceil(t/B) hold NaN codes
    and NaN scales, and the records name no tile beyond the context."""
    from gpu_utils import cache_to_dev
    lens = [37, 50, 129, 16, 1]
    for kv_dtype in ("e4m3", "fp16"):
        w = workloads.make_custom("spoison", seed=85, S=len(lens), H_q=10, H_k=2, d=128, B=16, NB=40,
                                  context_lens=lens, max_blocks=12, kv_dtype=kv_dtype)
        ref = _oracle_decode(oracle_mod, w, oracle_fill(oracle_mod, w))
        poisoned = alloc_cache(w, fill_byte=0x7F)            # E4M3 NaN / fp16 NaN; scales NaN
        oracle_fill(oracle_mod, w, cache=poisoned)
        got = _run(w, cache_to_dev(poisoned), _prepare(w))
        assert_close(got, ref, f"scheduled decode over a poisoned {kv_dtype} cache")
