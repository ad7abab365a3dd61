#!/usr/bin/env python3
"""Benchmark of the paged FP8 GQA decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--layers L]

A "step" is one pass of the whole hot path for one layer over one synthetic batch: the cache
write of one new token per sequence (quantise-on-write) followed by paged grouped-query decode
attention (split-context kernel + cross-partition reduce).  Consecutive steps rotate over L
distinct per-layer KV pools with the same block tables, so that the 256 MB Infinity Cache cannot
serve the reads: the KV bytes of every step come from HBM.

Prints ONE JSON line.  `value` is the achieved KV throughput of the whole step (algorithmic KV
bytes of the step / mean step time); `roofline` prices the dominant kernel (the decode kernel)
against the 8 TB/s HBM peak, its duration measured here with HIP events on the launch stream;
`cpu_baseline` is the float64 oracle timed on this machine's host cores on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(w):
    """Bytes the method itself must move per step (one layer): codes + scales of the visible tokens,
    q, out, the block-table entries used, and the step's own cache write."""
    es = 1 if w.kv_dtype == "e4m3" else 2
    per_token = w.H_k * (2 * w.d * es + (8 if w.kv_dtype == "e4m3" else 0))
    tokens = int(w.context_lens.sum())
    kv = tokens * per_token
    q_out = 2 * w.S * w.H_q * w.d * 2
    tables = int(((w.context_lens + w.B - 1) // w.B).sum()) * 4 + w.S * 4
    write = w.S * w.new_per_seq * (w.H_k * 2 * w.d * 2 + per_token)
    return {"kv": kv, "q_out": q_out, "tables": tables, "write": write, "tokens": tokens,
            "per_token": per_token}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=1, choices=[0, 1, 2, 3])
    ap.add_argument("--layers", type=int, default=0, help="distinct KV pools to rotate over (0 = auto)")
    ap.add_argument("--plan", type=str, default="", help="tokens_per_group,waves,depth (tuning)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: this build has no multi-GPU path "
                 "(run with --gpus 1; how the path would shard is described in DESIGN.md)")

    import torch
    import paper_2602_09323_amd as coopt
    import workloads
    from paper_2602_09323_amd.build import build, needs_build

    if not os.path.exists(coopt.lib_path()):
        build(force=True)
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU: the HIP path has no CPU fallback")
    coopt.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.plan:
        coopt.set_decode_plan(*[int(x) for x in args.plan.split(",")])

    w = workloads.make(args.config)
    ab = algorithmic_bytes(w)
    e4m3 = w.kv_dtype == "e4m3"
    shape = coopt.Shape(w.S, w.H_q, w.H_k, w.d, w.B, w.NB, w.max_blocks,
                        coopt.COOPT_KV_E4M3 if e4m3 else coopt.COOPT_KV_FP16,
                        float(np.float32(w.softmax_scale)))
    es = 1 if e4m3 else 2
    pool_bytes = w.NB * w.H_k * w.B * (2 * w.d * es + (8 if e4m3 else 0))
    layers = args.layers or max(2, min(40, int(24e9 // pool_bytes)))

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    hist, new = w.history_index(), w.new_index()
    k_hist, v_hist = to_dev(w.k_ctx[hist].view(np.uint16)), to_dev(w.v_ctx[hist].view(np.uint16))
    s_hist = to_dev(w.slots[hist])
    k_new, v_new = to_dev(w.k_ctx[new].view(np.uint16)), to_dev(w.v_ctx[new].view(np.uint16))
    s_new = to_dev(w.slots[new])
    q, bt, lens = to_dev(w.q.view(np.uint16)), to_dev(w.block_tables), to_dev(w.context_lens)
    out = torch.zeros((w.S, w.H_q, w.d), dtype=torch.float16, device=dev)
    ws = torch.empty(max(16, coopt.decode_workspace_bytes(shape)), dtype=torch.uint8, device=dev)

    pools = []
    for _ in range(layers):
        kc = torch.zeros((w.NB, w.H_k, w.B, w.d * es), dtype=torch.uint8, device=dev)
        vc = torch.zeros((w.NB, w.H_k, w.d, w.B * es), dtype=torch.uint8, device=dev)
        ks = torch.zeros((w.NB, w.H_k, w.B), dtype=torch.float32, device=dev) if e4m3 else None
        vs = torch.zeros((w.NB, w.H_k, w.B), dtype=torch.float32, device=dev) if e4m3 else None
        if e4m3:
            coopt.kv_cache_write_fp8(k_hist, v_hist, s_hist, kc, vc, ks, vs, shape)
        else:
            coopt.kv_cache_write_fp16(k_hist, v_hist, s_hist, kc, vc, shape)
        pools.append((kc, vc, ks, vs))
    torch.cuda.synchronize()

    def step(i):
        kc, vc, ks, vs = pools[i % layers]
        if e4m3:
            coopt.kv_cache_write_fp8(k_new, v_new, s_new, kc, vc, ks, vs, shape)
        else:
            coopt.kv_cache_write_fp16(k_new, v_new, s_new, kc, vc, shape)
        coopt.paged_gqa_decode(q, kc, vc, ks, vs, bt, lens, out, ws, shape)

    # ---- whole step: W warm-up, then exactly K steps between two synchronisations
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    step_ms = e0.elapsed_time(e1) / args.steps

    # ---- dominant kernel alone (the split-context decode kernel), one event pair per launch on
    # the launch stream, same rotation over pools.  coopt_paged_gqa_decode_partitioned launches
    # exactly that kernel with the plan's token range as the partition size.
    tokens_per_group, plan_waves, plan_depth = coopt.get_decode_plan()
    parts = (w.max_blocks * w.B + tokens_per_group - 1) // tokens_per_group
    kern_us = None
    b2b_us = None
    if parts > 1:
        rows = w.S * w.H_q
        tmp = torch.empty((rows, parts, w.d), dtype=torch.float32, device=dev)
        ml = torch.empty((rows, parts), dtype=torch.float32, device=dev)
        sm = torch.empty((rows, parts), dtype=torch.float32, device=dev)

        def kern(i):
            kc, vc, ks, vs = pools[i % layers]
            coopt.paged_gqa_decode_partitioned(q, kc, vc, ks, vs, bt, lens, tokens_per_group, tmp,
                                               ml, sm, parts, shape)
        for i in range(args.warmup):
            kern(i)
        torch.cuda.synchronize()
        n = min(args.steps, 500)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(n)]
        for i, (a, b) in enumerate(evs):
            a.record()
            kern(i)
            b.record()
        torch.cuda.synchronize()
        kern_us = float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e3
        e0.record()
        for i in range(n):
            kern(i)
        e1.record()
        torch.cuda.synchronize()
        b2b_us = e0.elapsed_time(e1) / n * 1e3

    kv_gbs = ab["kv"] / (step_ms * 1e-3) / 1e9
    result = {
        "metric": "paged GQA decode: achieved KV HBM GB/s per step (us/step in ms_per_step)",
        "value": round(kv_gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(step_ms, 6),
        "us_per_step": round(step_ms * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3 cache, f16 MFMA, f32 accumulate" if e4m3 else "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": w.S, "q_heads": w.H_q, "kv_heads": w.H_k,
                   "head_dim": w.d, "block_size": w.B, "context_tokens": ab["tokens"],
                   "kv_pools_rotated": layers,
                   "decode_plan": {"tokens_per_group": tokens_per_group, "waves": plan_waves,
                                   "depth": plan_depth}, "step": "kv_cache_write + paged_gqa_decode, one layer"},
        "pct_of_hbm_peak_step": round(100 * kv_gbs / HBM_PEAK_GBS, 2),
        "wall_ms_timed_region": round(wall_ms, 2),
    }
    if kern_us:
        # algorithmic bytes of one decode-kernel launch: KV codes + scales of the visible tokens,
        # q, and the block-table entries used (partials are a by-product of the split, not counted)
        alg = ab["kv"] + ab["q_out"] // 2 + ab["tables"]
        achieved = alg / (kern_us * 1e-6) / 1e9
        result["roofline"] = {"bound": "hbm", "kernel": "paged_decode_kernel",
                              "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                              "algorithmic_bytes_per_launch": int(alg),
                              "kernel_us_event_pair_median": round(kern_us, 3),
                              "kernel_us_back_to_back_mean": round(b2b_us, 3)}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, ab)
    print(json.dumps(result), flush=True)


def cpu_baseline(w, ab):
    """The oracle as it stands, timed on the host cores: the same step (write of the new tokens +
    attention) on a bounded sample of the workload's sequences (about 10-30 s of CPU work)."""
    import oracle
    oracle.build()
    # sample: the first sequences whose context tokens sum to <= ~1/4 of the batch
    budget = max(int(w.context_lens[0]), ab["tokens"] // 4)
    n = 1
    while n < w.S and int(w.context_lens[:n + 1].sum()) <= budget:
        n += 1
    tok_end = int(w.seq_start[n])
    es = 1 if w.kv_dtype == "e4m3" else 2
    dt = np.uint8 if es == 1 else np.float16
    kc = np.zeros((w.NB, w.H_k, w.B, w.d), dtype=dt)
    vc = np.zeros((w.NB, w.H_k, w.d, w.B), dtype=dt)
    ks = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32) if es == 1 else None
    vs = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32) if es == 1 else None
    hist = np.concatenate([np.arange(w.seq_start[s], w.seq_start[s + 1] - w.new_per_seq) for s in range(n)])
    new = np.concatenate([np.arange(w.seq_start[s + 1] - w.new_per_seq, w.seq_start[s + 1]) for s in range(n)])

    def write(idx):
        k, v, s = (np.ascontiguousarray(x[idx]) for x in (w.k_ctx, w.v_ctx, w.slots))
        if es == 1:
            oracle.kv_cache_write_fp8(k, v, s, kc, vc, ks, vs, H_k=w.H_k, d=w.d, B=w.B)
        else:
            oracle.kv_cache_write_fp16(k, v, s, kc, vc, H_k=w.H_k, d=w.d, B=w.B)
    write(hist)
    best = float("inf")
    for _ in range(2):
        t0 = time.perf_counter()
        write(new)
        oracle.paged_gqa_decode(np.ascontiguousarray(w.q[:n]), kc, vc, ks, vs,
                                np.ascontiguousarray(w.block_tables[:n]),
                                np.ascontiguousarray(w.context_lens[:n]), H_q=w.H_q, H_k=w.H_k,
                                d=w.d, B=w.B, softmax_scale=w.softmax_scale)
        best = min(best, time.perf_counter() - t0)
    kv = tok_end * ab["per_token"]
    return {"value": round(kv / best / 1e9, 5), "unit": "GB/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(best, 3),
            "sample": f"first {n} of {w.S} sequences ({tok_end} of {ab['tokens']} context tokens), "
                      f"one layer, write + decode, best of 2"}


if __name__ == "__main__":
    main()
