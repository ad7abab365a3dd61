"""GPU parity on randomly drawn shapes: every decode entry point (plain, with and without a
workspace, from a prepared schedule, the fused step with some sequences appending nothing, fixed
partitions + reduce), the dequantising gather (bit-exact) and chunked prefill with a different
chunk length per sequence, each against the oracle on the same seeded inputs.  Head counts, head
size, cache type (E4M3, E5M2, fp16), length mix, pool size and decode plan are all drawn from the seed, and the seed is
in every failure message."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import planned, alloc_dev_cache, assert_close, cache_to_dev, dev, dev_cache_to_host, hip_write, shape_of
from helpers import oracle_fill

pytestmark = pytest.mark.gpu

PLANS = [(128, 1, 2, 1024, 0), (32, 1, 1, 5, 0), (64, 1, 3, 64, 0), (128, 1, 2, 1024, 1),
         (256, 1, 2, 333, 0), (32, 1, 3, 2048, 0), (512, 1, 2, 16, 0)]


def _set_plan(plan):
    planned.set_plan(tokens_per_group=plan[0], waves_per_group=plan[1], pipeline_depth=plan[2],
                          grid_waves=plan[3], softmax_reduction=plan[4])


def _random_lengths(rng, S, cap):
    """Block-boundary lengths, short, medium and long contexts, whole blocks, anything."""
    lens = []
    for kind in rng.integers(0, 6, size=S):
        if kind == 0:
            lens.append(int(rng.choice([1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49])))
        elif kind == 1:
            lens.append(int(rng.integers(1, 64)))
        elif kind == 2:
            lens.append(int(rng.integers(64, 600)))
        elif kind == 3:
            lens.append(int(rng.integers(min(600, cap - 1), cap)))
        elif kind == 4:
            lens.append(16 * int(rng.integers(1, cap // 16)))
        else:
            lens.append(int(rng.integers(1, cap)))
    return lens


def _same_bytes(got, want, what):
    for name, g, r in zip(("k_cache", "v_cache", "k_scale", "v_scale"), got, want):
        if r is not None:
            assert np.array_equal(g.reshape(-1).view(np.uint8), r.reshape(-1).view(np.uint8)), f"{what}: {name}"


def _decode_case(orc, seed):
    rng = np.random.default_rng(seed)
    d = int(rng.choice([64, 128]))
    kv = str(rng.choice(["e4m3", "fp16", "e5m2"]))
    H_k = int(rng.choice([1, 2, 3, 4, 8]))
    H_q = H_k * int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
    S = int(rng.integers(1, 40))
    cap = int(rng.choice([200, 1200, 3000]))
    lens = _random_lengths(rng, S, cap)
    NB = sum((t + 15) // 16 for t in lens) + int(rng.integers(0, 50))
    max_blocks = max((t + 15) // 16 for t in lens) + int(rng.integers(0, 5))
    w = workloads.make_custom("random", seed=seed, S=S, H_q=H_q, H_k=H_k, d=d, B=16, NB=NB,
                              context_lens=lens, kv_dtype=kv, max_blocks=max_blocks,
                              k_outlier_frac=float(rng.choice([0.0, 0.02])))
    plan = PLANS[int(rng.integers(0, len(PLANS)))]
    what = f"seed={seed} d={d} kv={kv} heads={H_q}/{H_k} S={S} cap={cap} NB={NB} plan={plan}"
    _set_plan(plan)
    cache = oracle_fill(orc, w)
    fmt = "e5m2" if kv == "e5m2" else "e4m3"
    ref = orc.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=H_q, H_k=H_k, d=d,
                               B=16, softmax_scale=w.softmax_scale, fmt=fmt)
    shape = shape_of(w)
    ws = torch.empty(max(16, planned.decode_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    q, bt, dl = dev(w.q.view(np.uint16)), dev(w.block_tables), dev(w.context_lens)

    def new_out():
        return torch.full((S, H_q, d), -7.0, dtype=torch.float16, device="cuda")

    def host(o):
        torch.cuda.synchronize()
        return o.cpu().numpy().astype(np.float64)

    # ---- plain decode over a cache that holds every token (unwritten bytes are arbitrary)
    full = alloc_dev_cache(w, fill_byte=int(rng.integers(0, 256)))
    hip_write(w, full)
    for workspace in (ws, None):
        out = new_out()
        planned.paged_gqa_decode(q, *full, bt, dl, out, workspace, shape)
        assert_close(host(out), ref, f"decode, workspace={workspace is not None}, {what}")
    sched = torch.zeros(planned.decode_schedule_bytes(shape), dtype=torch.uint8, device="cuda")
    planned.decode_schedule_prepare(bt, dl, None, sched, shape)
    out = new_out()
    planned.paged_gqa_decode_scheduled(None, None, None, q, *full, dl, out, ws, sched, shape)
    assert_close(host(out), ref, f"decode from a schedule, {what}")

    # ---- fused step; some sequences append nothing (their last token is already in the cache)
    new, hist = w.new_index(), w.history_index()
    drop = rng.random(S) < 0.15
    slots = w.slots[new].copy()
    slots[drop] = -1
    before = np.sort(np.concatenate([hist, new[drop]]))
    k_new, v_new = dev(w.k_ctx[new].view(np.uint16)), dev(w.v_ctx[new].view(np.uint16))
    dslots = dev(slots.astype(np.int64))
    whole = alloc_dev_cache(w, fill_byte=0)
    hip_write(w, whole)
    want_bytes = dev_cache_to_host(w, whole)
    for prepared in (False, True):
        dcache = alloc_dev_cache(w, fill_byte=0)
        hip_write(w, dcache, idx=before)
        out = new_out()
        if prepared:
            planned.decode_schedule_prepare(bt, dl, dslots, sched, shape)
            planned.paged_gqa_decode_scheduled(k_new, v_new, dslots, q, *dcache, dl, out, ws, sched, shape)
        else:
            planned.paged_gqa_decode_step(k_new, v_new, dslots, q, *dcache, bt, dl, out, ws, shape)
        assert_close(host(out), ref, f"step, prepared={prepared}, {what}")
        _same_bytes(dev_cache_to_host(w, dcache), want_bytes, f"step, prepared={prepared}, {what}")

    # ---- fixed partitions + reduce
    P = int(rng.choice([16, 64, 256, 512]))
    max_parts = (max_blocks * 16 + P - 1) // P
    tmp = torch.full((S, H_q, max_parts, d), float("nan"), dtype=torch.float32, device="cuda")
    ml = torch.full((S, H_q, max_parts), float("nan"), dtype=torch.float32, device="cuda")
    es = torch.full((S, H_q, max_parts), float("nan"), dtype=torch.float32, device="cuda")
    out = new_out()
    planned.paged_gqa_decode_partitioned(q, *full, bt, dl, P, tmp, ml, es, max_parts, shape)
    coopt.paged_gqa_reduce(tmp, ml, es, dl, P, max_parts, out, shape)
    assert_close(host(out), ref, f"partitioned P={P}, {what}")

    # ---- gather of random token ranges: one rounding of the exact product, nothing outside
    for _ in range(3):
        s = int(rng.integers(0, S))
        lo = int(rng.integers(0, lens[s]))
        hi = int(rng.integers(lo, lens[s] + 1))
        k_ref, v_ref = orc.gather_cached_kv(*cache, w.block_tables, s, lo, hi, H_k=H_k, d=d, B=16, fmt=fmt)
        k_out = torch.full((hi - lo + 2, H_k, d), 7.0, dtype=torch.float16, device="cuda")
        v_out = torch.full_like(k_out, 7.0)
        coopt.gather_cached_kv(*full, bt, s, lo, hi, k_out[1:-1], v_out[1:-1], shape)
        torch.cuda.synchronize()
        for got, want in ((k_out, k_ref), (v_out, v_ref)):
            got = got.cpu().numpy()
            assert np.all(got[0] == 7.0) and np.all(got[-1] == 7.0), f"gather wrote outside, {what}"
            assert np.array_equal(got[1:-1].view(np.uint16), want.astype(np.float16).view(np.uint16)), \
                f"gather seq {s} [{lo}, {hi}), {what}"


def _prefill_case(orc, seed):
    rng = np.random.default_rng(seed)
    d = int(rng.choice([64, 128]))
    kv = str(rng.choice(["e4m3", "fp16", "e5m2"]))
    H_k = int(rng.choice([1, 2, 3, 8]))
    H_q = H_k * int(rng.choice([1, 2, 4, 5, 8]))
    S = int(rng.integers(1, 6))
    history = [int(rng.choice([0, 1, 15, 16, 17, 100, 333, 1000])) for _ in range(S)]
    chunk = [int(rng.choice([0, 1, 2, 15, 16, 17, 31, 33, 64, 100, 129, 260])) for _ in range(S)]
    if sum(chunk) == 0:
        chunk[0] = 5
    lens = [h + c for h, c in zip(history, chunk)]
    stored = [max(1, t) for t in lens]                 # the generator wants a token per sequence
    NB = sum((t + 15) // 16 for t in stored) + int(rng.integers(0, 9))
    max_blocks = max((t + 15) // 16 for t in stored) + int(rng.integers(0, 3))
    w = workloads.make_custom("random", seed=seed, S=S, H_q=H_q, H_k=H_k, d=d, B=16, NB=NB,
                              context_lens=stored, kv_dtype=kv, max_blocks=max_blocks)
    what = f"seed={seed} d={d} kv={kv} heads={H_q}/{H_k} history={history} chunk={chunk}"
    context_lens = np.asarray(lens, dtype=np.int32)
    query_start = np.zeros(S + 1, dtype=np.int32)
    query_start[1:] = np.cumsum(chunk)
    rows = int(query_start[-1])
    q = rng.standard_normal((rows, H_q, d), dtype=np.float32).astype(np.float16)
    cache = oracle_fill(orc, w)
    ref = orc.paged_gqa_prefill_chunk(q, *cache, w.block_tables, context_lens, query_start, H_q=H_q,
                                      H_k=H_k, d=d, B=16, softmax_scale=w.softmax_scale,
                                      fmt="e5m2" if kv == "e5m2" else "e4m3")
    out = torch.full((rows, H_q, d), -7.0, dtype=torch.float16, device="cuda")
    args = (dev(q.view(np.uint16)), *cache_to_dev(cache), dev(w.block_tables), dev(context_lens),
            dev(query_start), rows, max(chunk))
    coopt.paged_gqa_prefill_chunk(*args, out, shape_of(w))
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, what)
    # the entry point with a workspace: these launches are smaller than the chip, so every pair's
    # stages are cut into parts (often more parts than stages) and merged
    need = coopt.prefill_workspace_bytes(shape_of(w), max(chunk))
    ws = torch.full((max(need, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    out.fill_(-7.0)
    coopt.paged_gqa_prefill_chunk_ws(*args, out, ws if need else None, shape_of(w))
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy().astype(np.float64), ref, what + f" workspace={need}")


@pytest.mark.parametrize("first", [2000, 2008, 2016, 2024])
def test_random_decode_shapes(oracle_mod, first):
    for seed in range(first, first + 8):
        _decode_case(oracle_mod, seed)


@pytest.mark.parametrize("first", [3000, 3010])
def test_random_prefill_shapes(oracle_mod, first):
    for seed in range(first, first + 10):
        _prefill_case(oracle_mod, seed)
