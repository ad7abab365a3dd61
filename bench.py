#!/usr/bin/env python3
"""Benchmark of the paged FP8 GQA decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--layers L]
    python bench.py --config 3 --path partitioned     (fixed 512-token partitions + reduce)
    python bench.py --config 4 --steps 20             (chunked prefill, priced against the MFMA peak)

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
MFMA_F16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs of this script (FETCH_SIZE
# and WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for a plain
# 256 MiB device copy: FETCH_SIZE reads half the bytes, WRITE_SIZE all of them).  The summaries
# with the commands are under profiles/; the figures belong to the default decode plan.
PMC_TRAFFIC = {
    # (workload, launch mode) -> counters of the kernel that `roofline` times, and the hash of the
    # kernel sources they were measured on (kernel_sources_sha16): quoted only while that matches
    ("llama13b_gqa_fp8_decode", "fused"): {"fetch_kib": 36678.9, "fetch_scale": 2.0, "write_kib": 3152.1,
                                           "write_scale": 1.0, "sources_sha16": "f67412d6569893ab"},
    ("llama13b_gqa_fp8_decode", "plain"): {"fetch_kib": 36582.8, "fetch_scale": 2.0, "write_kib": 3152.1,
                                           "write_scale": 1.0, "sources_sha16": "f67412d6569893ab"},
}


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


def kernel_sources_sha16():
    """Hash of the sources the decode kernels are built from: counter figures in PMC_TRAFFIC are
    only quoted for the code they were measured on."""
    import hashlib
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2602_09323_amd", "csrc")
    h = hashlib.sha256()
    for name in ("common.hpp", "attn_tile.hpp", "kv_quant.hpp", "decode_internal.hpp", "decode_flat.hip"):
        with open(os.path.join(here, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=None, choices=[0, 1, 2, 3, 4],
                    help="workload (1 = LLaMa-13B GQA FP8 decode, the headline configuration; "
                         "4 = chunked prefill).  Without it the line is the headline configuration "
                         "and carries the other configurations under `all_configs`")
    ap.add_argument("--path", choices=["balanced", "partitioned"], default="balanced",
                    help="decode through coopt_paged_gqa_decode (balanced split + merge) or through "
                         "coopt_paged_gqa_decode_partitioned + coopt_paged_gqa_reduce with the "
                         "workload's partition size (512 if it names none)")
    ap.add_argument("--prefill-entry", choices=["workspace", "plain"], default="workspace",
                    help="config 4: coopt_paged_gqa_prefill_chunk_ws (a workspace for the launch's last "
                         "round) or coopt_paged_gqa_prefill_chunk")
    ap.add_argument("--prefill-seqs", type=int, default=0,
                    help="config 4 with this many sequences instead of its 8 (0 = the configuration)")
    ap.add_argument("--layers", type=int, default=0, help="distinct KV pools to rotate over (0 = auto)")
    ap.add_argument("--plan", type=str, default="",
                    help="decode plan fields in header order, comma separated (tuning)")
    ap.add_argument("--write", choices=["fused", "separate"], default="fused",
                    help="the step's cache write inside the decode launch (coopt_paged_gqa_decode_step) "
                         "or as its own kernel before coopt_paged_gqa_decode (balanced path only)")
    ap.add_argument("--schedule", choices=["prepared", "live"], default="prepared",
                    help="balanced path: 'prepared' derives the decode schedule once per rotation "
                         "over the KV pools (coopt_decode_schedule_prepare, inside the timed region: "
                         "the layers of one decoding step share block tables and lengths) and runs "
                         "the layers from it; 'live' derives it inside every launch")
    ap.add_argument("--op", choices=["step", "gather", "stream-read", "schemes"], default="step",
                    help="step: the decode / prefill step of the workload (default).  gather: "
                         "coopt_gather_cached_kv of every sequence's whole context (one launch per "
                         "sequence), reported in GB/s against the HBM peak.  stream-read: the "
                         "read-only streaming probe over 2 GiB, every launch shape it tries.  "
                         "schemes: E4M3 / E5M2 codes with a per-token, per-block or static scale on the "
                         "long-context outlier workload (config 3 unless --config names another): "
                         "step time and attention error against an fp16 cache")
    ap.add_argument("--probe-mb", type=float, default=0.0,
                    help="with --op stream-read: read buffers of this many MB instead (as many distinct "
                         "ones as fit 12 GB, at most 40, in rotation, launches back to back in HIP "
                         "graphs like the decode launches): what ONE read-only launch of a decode "
                         "launch's size reaches")
    ap.add_argument("--preroll", type=int, default=300,
                    help="untimed launches of the step before the warm-up steps, so that a short run "
                         "is not timed while the clocks are still coming up (disclosed in the line)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="headline configuration only (no `all_configs`)")
    ap.add_argument("--no-graph", action="store_true", help="eager launches instead of HIP graphs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run plain device copies of 256 MiB instead of the workload (the known "
                         "traffic that scales the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: this build has no multi-GPU path "
                 "(run with --gpus 1; the path shards by sequence or by KV head with no exchange inside attention)")

    import torch
    import paper_2602_09323_amd as coopt
    import workloads
    from paper_2602_09323_amd import probe
    from paper_2602_09323_amd.build import build

    if not os.path.exists(coopt.lib_path()) or not os.path.exists(probe.lib_path()):
        build(force=True)
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU: the HIP path has no CPU fallback")
    coopt.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    plan = None
    if args.plan:
        names = [f for f, _ in coopt.DecodePlan._fields_]
        plan = coopt.make_decode_plan(**dict(zip(names, [int(x) for x in args.plan.split(",")])))

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": src.numel(), "copies": 10}))
        return

    if args.op == "stream-read":
        if args.probe_mb > 0:
            print(json.dumps(stream_read_sized(probe, torch, dev, args.probe_mb)), flush=True)
        else:
            print(json.dumps(stream_read_ceiling(probe, torch, dev, detail=True)), flush=True)
        return
    if args.op == "schemes":
        w = workloads.make(3 if args.config is None else args.config)
        print(json.dumps(bench_schemes(args, w, coopt, torch, dev, plan)), flush=True)
        return
    cfg = 1 if args.config is None else args.config
    w = workloads.make(cfg)
    if cfg == 4 and args.prefill_seqs:
        # the named configuration's sequences, fewer of them (8192 history + 512 chunk tokens each)
        C = w.new_per_seq
        w = workloads.make_custom(w.name + "_%dseq" % args.prefill_seqs, seed=workloads.BASE_SEED + 4,
                                  S=args.prefill_seqs, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B, NB=w.NB,
                                  context_lens=[int(w.context_lens[0])] * args.prefill_seqs, new_per_seq=C,
                                  max_blocks=w.max_blocks)
    if args.op == "gather":
        print(json.dumps(bench_gather(args, w, coopt, torch, dev)), flush=True)
        return
    if cfg == 4:
        print(json.dumps(bench_prefill(args, w, coopt, torch, dev, args.steps, args.warmup,
                                       not args.no_cpu_baseline)), flush=True)
        return
    result = bench_decode(args, w, coopt, probe, torch, dev, plan, args.path, args.steps, args.warmup,
                          cpu=not args.no_cpu_baseline, stream=True)
    if args.config is None and not args.no_all_configs:
        # the other configurations, each for at least 200 steps: kernel, roofline fraction, step
        steps = max(args.steps, 200)
        rows = [compact(result, "balanced")]
        # the same step with the schedule derived inside every launch (coopt_paged_gqa_decode_step)
        live = argparse.Namespace(**vars(args))
        live.schedule = "live"
        r = bench_decode(live, w, coopt, probe, torch, dev, plan, "balanced", steps, max(args.warmup, 20),
                         cpu=False, stream=False)
        rows.append(compact(r, "balanced, schedule derived in every launch"))
        for c, path in ((2, "balanced"), (3, "balanced"), (3, "partitioned")):
            del w
            torch.cuda.empty_cache()
            w = workloads.make(c)
            r = bench_decode(args, w, coopt, probe, torch, dev, plan, path, steps, max(args.warmup, 20),
                             cpu=False, stream=False)
            rows.append(compact(r, path))
        del w
        torch.cuda.empty_cache()
        r = bench_prefill(args, workloads.make(4), coopt, torch, dev, steps, max(args.warmup, 20), False)
        rows.append(compact(r, "prefill"))
        result["all_configs"] = rows
    print(json.dumps(result), flush=True)


def compact(r, path):
    rf = r["roofline"]
    return {"workload": r["config"]["workload"], "path": path, "kernel": rf["kernel"].split(" ")[0],
            "kernel_us": rf.get("kernel_us_mean", round(rf.get("kernel_ms_mean", 0.0) * 1e3, 3)),
            "bound": rf["bound"], "achieved": rf["achieved"], "unit": rf["unit"], "frac": rf["frac"],
            "step_us": round(r["ms_per_step"] * 1e3, 3), "steps": r["steps"]}


def graph_timed(torch, fn, count, layers, eager=False):
    """Mean GPU time per call of fn(i), i = 0..count-1, in ms.  The calls are captured into HIP
    graphs of one rotation over the pools each (the step is ~2 launches of a few us, so eager
    launches from Python would measure the host, not the GPU) and replayed back to back on the
    current stream between two events."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if eager:
        e0.record()
        for i in range(count):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / count
    graphs = []
    for n_in in (layers, count % layers):
        if n_in == 0 or (n_in == layers and count < layers):
            graphs.append(None)
            continue
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n_in):
                fn(i)
        graphs.append(g)
    full, rest = graphs
    if full is not None:
        full.replay()                     # untimed: first replay uploads the graph
    if rest is not None:
        rest.replay()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(count // layers):
        full.replay()
    if rest is not None:
        rest.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / count


def bench_decode(args, w, coopt, probe, torch, dev, plan, path, steps, warmup, cpu, stream):
    """One decode workload: whole-step time over `steps` steps, the dominant kernel alone, and the
    step's output against the oracle (`cpu` = time the oracle and compare)."""
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
    ws = torch.empty(max(16, coopt.decode_workspace_bytes(shape, plan)), dtype=torch.uint8, device=dev)

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
    del k_hist, v_hist, s_hist

    partitioned = path == "partitioned"
    if partitioned:
        P = w.partition_size or 512
        max_parts = (w.max_blocks * w.B + P - 1) // P
        tmp_out = torch.empty((w.S, w.H_q, max_parts, w.d), dtype=torch.float32, device=dev)
        max_logits = torch.empty((w.S, w.H_q, max_parts), dtype=torch.float32, device=dev)
        exp_sums = torch.empty_like(max_logits)

    def attend(i, reduce=True):
        kc, vc, ks, vs = pools[i % layers]
        if not partitioned:
            coopt.paged_gqa_decode(q, kc, vc, ks, vs, bt, lens, out, ws, shape, plan)
            return
        coopt.paged_gqa_decode_partitioned(q, kc, vc, ks, vs, bt, lens, P, tmp_out, max_logits,
                                           exp_sums, max_parts, shape, plan)
        if reduce:
            coopt.paged_gqa_reduce(tmp_out, max_logits, exp_sums, lens, P, max_parts, out, shape)

    fused = args.write == "fused" and not partitioned
    prepared = args.schedule == "prepared" and not partitioned
    if prepared:
        sched = torch.zeros(coopt.decode_schedule_bytes(shape, plan), dtype=torch.uint8, device=dev)
        sched_plain = torch.zeros_like(sched)            # plain-decode schedule: the attention-only timing
        coopt.decode_schedule_prepare(bt, lens, None, sched_plain, shape, plan)

    def write_new(kc, vc, ks, vs):
        if e4m3:
            coopt.kv_cache_write_fp8(k_new, v_new, s_new, kc, vc, ks, vs, shape)
        else:
            coopt.kv_cache_write_fp16(k_new, v_new, s_new, kc, vc, shape)

    def step(i):
        kc, vc, ks, vs = pools[i % layers]
        if prepared:
            if i % layers == 0:                          # one decoding step of the model begins
                coopt.decode_schedule_prepare(bt, lens, s_new if fused else None, sched, shape, plan)
            if not fused:
                write_new(kc, vc, ks, vs)
            coopt.paged_gqa_decode_scheduled(k_new if fused else None, v_new if fused else None,
                                             s_new if fused else None, q, kc, vc, ks, vs, lens, out,
                                             ws, sched, shape, plan)
            return
        if fused:
            coopt.paged_gqa_decode_step(k_new, v_new, s_new, q, kc, vc, ks, vs, bt, lens, out, ws,
                                        shape, plan)
            return
        write_new(kc, vc, ks, vs)
        attend(i)

    def timed(fn, count):
        return graph_timed(torch, fn, count, layers, args.no_graph)

    # ---- untimed pre-roll (the first launches after idle run while the clocks come up), then W
    # warm-up steps, then exactly K steps between two synchronisations
    if args.preroll > 0:
        timed(step, args.preroll)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_ms = timed(step, steps)
    wall_ms = (time.perf_counter() - t0) * 1e3
    got = out.cpu().numpy().astype(np.float64)           # the last timed step's output rows

    # ---- dominant kernel alone: the launch the step itself runs (with a fused write, the decode
    # launch that also appends the new tokens), same rotation over pools, launches back to back on
    # the stream, one event pair around them; and the attention-only launch beside it.
    ksteps = max(steps, 200)

    def kern(i):
        if partitioned:
            return attend(i, reduce=False)
        kc, vc, ks, vs = pools[i % layers]
        if prepared:
            coopt.paged_gqa_decode_scheduled(k_new if fused else None, v_new if fused else None,
                                             s_new if fused else None, q, kc, vc, ks, vs, lens, None,
                                             ws, sched, shape, plan)
        else:
            coopt.paged_gqa_decode_split(q, kc, vc, ks, vs, bt, lens, ws, shape, plan)

    def kern_plain(i):
        kc, vc, ks, vs = pools[i % layers]
        coopt.paged_gqa_decode_scheduled(None, None, None, q, kc, vc, ks, vs, lens, None, ws,
                                         sched_plain, shape, plan)
    kern_us = timed(kern, ksteps) * 1e3
    plain_us = timed(kern_plain, ksteps) * 1e3 if (prepared and fused) else None

    # the same kernel on empty contexts: what one launch costs before any byte moves (the gap
    # between dependent launches in a stream plus the schedule prologue)
    lens_zero = torch.zeros_like(lens)
    if prepared:
        sched_empty = torch.zeros_like(sched)
        coopt.decode_schedule_prepare(bt, lens_zero, None, sched_empty, shape, plan)

    def kern_empty(i):
        kc, vc, ks, vs = pools[i % layers]
        if partitioned:
            coopt.paged_gqa_decode_partitioned(q, kc, vc, ks, vs, bt, lens_zero, P, tmp_out,
                                               max_logits, exp_sums, max_parts, shape, plan)
        elif prepared:
            coopt.paged_gqa_decode_scheduled(None, None, None, q, kc, vc, ks, vs, lens_zero, None, ws,
                                             sched_empty, shape, plan)
        else:
            coopt.paged_gqa_decode_split(q, kc, vc, ks, vs, bt, lens_zero, ws, shape, plan)
    floor_us = timed(kern_empty, 200) * 1e3

    kv_gbs = ab["kv"] / (step_ms * 1e-3) / 1e9
    plan_used = (plan or coopt.default_decode_plan()).as_dict()
    result = {
        "metric": "paged GQA decode: achieved KV HBM GB/s per step (us/step in ms_per_step)",
        "value": round(kv_gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(step_ms, 6),
        "us_per_step": round(step_ms * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3 cache, f16 MFMA, f32 accumulate" if e4m3 else "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": w.S, "q_heads": w.H_q, "kv_heads": w.H_k,
                   "head_dim": w.d, "block_size": w.B, "context_tokens": ab["tokens"],
                   "kv_pools_rotated": layers,
                   "decode_plan": plan_used,
                   "step": ("kv_cache_write + paged_gqa_decode_partitioned (P=%d) + paged_gqa_reduce, "
                            "one layer" % P) if partitioned else
                           (("paged_gqa_decode_scheduled" if prepared else "paged_gqa_decode_step") +
                            " (cache write fused into the decode launch), one layer"
                            if fused else
                            "kv_cache_write + " + ("paged_gqa_decode_scheduled" if prepared else "paged_gqa_decode") +
                            ", one layer"),
                   "schedule": ("prepared once per %d steps (one per decoding step of a %d-layer model), "
                                "inside the timed region" % (layers, layers)) if prepared else
                               ("fixed partitions" if partitioned else "derived inside every launch"),
                   "launch": "eager" if args.no_graph else "hip_graph",
                   "clock_preroll_launches": args.preroll},
        "pct_of_hbm_peak_step": round(100 * kv_gbs / HBM_PEAK_GBS, 2),
        "wall_ms_timed_region": round(wall_ms, 2),
    }
    # algorithmic bytes of one decode-kernel launch: KV codes + scales of the visible tokens,
    # q, and the block-table entries used (partials are a by-product of the split, not counted;
    # nor are the new rows a fused launch also reads and writes)
    alg = ab["kv"] + ab["q_out"] // 2 + ab["tables"]
    mode = ("fused" if fused else "plain") if prepared else "live"
    pmc = PMC_TRAFFIC.get((w.name, mode))
    traffic = None
    if pmc and not args.plan and not partitioned and pmc.get("sources_sha16") == kernel_sources_sha16():
        traffic = int((pmc["fetch_kib"] * pmc["fetch_scale"] + pmc["write_kib"] * pmc["write_scale"]) * 1024)
    achieved = alg / (kern_us * 1e-6) / 1e9
    kernel = ("paged_decode_kernel (coopt_paged_gqa_decode_partitioned)" if partitioned else
              ("flat_stream_prepared_kernel (coopt_paged_gqa_decode_scheduled%s)"
               % (", the launch of the step: attention and the new tokens' cache write" if fused else "")
               if prepared else "flat_stream_kernel (coopt_paged_gqa_decode_split)"))
    result["roofline"] = {"bound": "hbm", "kernel": kernel,
                          "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                          "algorithmic_bytes_per_launch": int(alg),
                          "kernel_us_mean": round(kern_us, 3), "kernel_launches_timed": ksteps,
                          "launch_floor_us": round(floor_us, 3),
                          "timing": "HIP events around back-to-back launches on the launch "
                                    "stream; includes the inter-launch gap (launch_floor_us), "
                                    "which a kernel trace's begin-to-end duration does not"}
    if plain_us is not None:
        result["roofline"]["attention_only_kernel_us_mean"] = round(plain_us, 3)
        result["roofline"]["attention_only_frac"] = round(alg / (plain_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
    if stream:
        sr = stream_read_ceiling(probe, torch, dev)
        result["roofline"]["stream_read_gbs"] = sr["gbs"]
        result["roofline"]["frac_of_stream_read"] = round(achieved / sr["gbs"], 4)
        # and what ONE read-only launch of this launch's own size reaches, timed the same way
        del pools
        pools = []
        torch.cuda.empty_cache()
        ro = stream_read_sized(probe, torch, dev, alg / 1e6)
        result["roofline"]["read_only_launch_us"] = ro["us_per_launch"]
        result["roofline"]["frac_of_read_only_launch"] = round(ro["us_per_launch"] / kern_us, 4)
    if cpu:
        base, ref = cpu_baseline(w, ab)
        result["cpu_baseline"] = base
        # the step's output rows (last timed step) against the oracle's, on the sampled sequences
        err = np.abs(got[:ref.shape[0]] - ref)
        result["parity"] = {"against": "oracle (float64) on the cpu_baseline sample, same inputs",
                            "sequences": int(ref.shape[0]), "elements": int(ref.size),
                            "max_abs": float(err.max()), "max_abs_oracle": float(np.abs(ref).max()),
                            "over_2e-3": int((err > 2e-3).sum()),
                            "finite": bool(np.isfinite(got).all())}
    del pools
    return result


def bench_schemes(args, w, coopt, torch, dev, plan):
    """The cache schemes that Opt-KV's choice (E4M3 codes, a scale per token and KV head computed at
    write time) stands against, on one workload: E4M3 or E5M2 codes, with a scale per token, per
    16-token block, or fixed in advance per KV head.  For each: the time of a decode step (the new
    tokens' write under that scheme + balanced decode, one layer, pools rotated) and the error of
    the attention output against the same step over an fp16 cache.  The fp16-cache rows come from
    this library's own fp16 path (which the GPU tests hold to 2e-3 of the float64 oracle, an order
    of magnitude under the differences reported here).  All schemes keep one scale entry per
    (token, KV head) in the cache, so they move the same bytes."""
    steps, layers = max(args.steps, 200), 8
    hist, new = w.history_index(), w.new_index()

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    k_hist, v_hist = to_dev(w.k_ctx[hist].view(np.uint16)), to_dev(w.v_ctx[hist].view(np.uint16))
    k_new, v_new = to_dev(w.k_ctx[new].view(np.uint16)), to_dev(w.v_ctx[new].view(np.uint16))
    s_hist, s_new = to_dev(w.slots[hist]), to_dev(w.slots[new])
    q, bt, lens = to_dev(w.q.view(np.uint16)), to_dev(w.block_tables), to_dev(w.context_lens)
    calib = 256                                          # static scales: absmax of the first tokens of sequence 0
    k_amax = np.abs(w.k_ctx[:calib].astype(np.float32)).max(axis=(0, 2))
    v_amax = np.abs(w.v_ctx[:calib].astype(np.float32)).max(axis=(0, 2))
    modes = {"token": coopt.COOPT_SCALE_TOKEN, "block": coopt.COOPT_SCALE_BLOCK, "static": coopt.COOPT_SCALE_STATIC}

    def run(codes, scale):
        fp16 = codes == "fp16"
        kv = {"fp16": coopt.COOPT_KV_FP16, "e4m3": coopt.COOPT_KV_E4M3, "e5m2": coopt.COOPT_KV_E5M2}[codes]
        shape = coopt.Shape(w.S, w.H_q, w.H_k, w.d, w.B, w.NB, w.max_blocks, kv, float(np.float32(w.softmax_scale)))
        es = 2 if fp16 else 1
        cmax = np.float32(448.0 if codes == "e4m3" else 57344.0)
        k_st = to_dev((k_amax / cmax).astype(np.float32)) if scale == "static" else None
        v_st = to_dev((v_amax / cmax).astype(np.float32)) if scale == "static" else None

        def write(k, v, s, pool):
            kc, vc, ks, vs = pool
            if fp16:
                coopt.kv_cache_write_fp16(k, v, s, kc, vc, shape)
            else:
                coopt.kv_cache_write_fp8_scaled(k, v, s, kc, vc, ks, vs, shape, modes[scale], k_st, v_st)

        pools = []
        for _ in range(layers):
            kc = torch.zeros((w.NB, w.H_k, w.B, w.d * es), dtype=torch.uint8, device=dev)
            vc = torch.zeros((w.NB, w.H_k, w.d, w.B * es), dtype=torch.uint8, device=dev)
            ks = None if fp16 else torch.zeros((w.NB, w.H_k, w.B), dtype=torch.float32, device=dev)
            vs = None if fp16 else torch.zeros((w.NB, w.H_k, w.B), dtype=torch.float32, device=dev)
            pools.append((kc, vc, ks, vs))
            write(k_hist, v_hist, s_hist, pools[-1])
        out = torch.zeros((w.S, w.H_q, w.d), dtype=torch.float16, device=dev)
        ws = torch.empty(max(16, coopt.decode_workspace_bytes(shape, plan)), dtype=torch.uint8, device=dev)

        def decode(i):
            coopt.paged_gqa_decode(q, *pools[i % layers], bt, lens, out, ws, shape, plan)

        def step(i):
            write(k_new, v_new, s_new, pools[i % layers])
            decode(i)

        graph_timed(torch, step, args.preroll, layers, args.no_graph)
        step_us = graph_timed(torch, step, steps, layers, args.no_graph) * 1e3
        decode_us = graph_timed(torch, decode, steps, layers, args.no_graph) * 1e3
        rows = out.cpu().numpy().astype(np.float64)
        del pools
        torch.cuda.empty_cache()
        return step_us, decode_us, rows

    _, _, ref = run("fp16", None)
    ref_rms = float(np.sqrt((ref ** 2).mean()))
    table = []
    for codes in ("e4m3", "e5m2"):
        for scale in ("token", "block", "static"):
            step_us, decode_us, rows = run(codes, scale)
            err = rows - ref
            table.append({"codes": codes, "scale": scale, "step_us": round(step_us, 3),
                          "decode_us": round(decode_us, 3), "max_abs_err": float(np.abs(err).max()),
                          "rms_err": float(np.sqrt((err ** 2).mean())),
                          "rel_rms_err": float(np.sqrt((err ** 2).mean())) / ref_rms,
                          "finite": bool(np.isfinite(rows).all())})
            print("# %s %s: %s" % (codes, scale, table[-1]), file=sys.stderr, flush=True)
    return {"metric": "cache schemes: decode step time and attention error against an fp16 cache",
            "workload": w.name, "steps": steps, "kv_pools_rotated": layers,
            "reference": "the same step over an fp16 cache (this library's fp16 path), rms of its rows %.4f" % ref_rms,
            "static_scale_calibration": "absmax over the first %d tokens of sequence 0, per KV head, / largest code" % calib,
            "method": {"codes": "e4m3", "scale": "token"}, "schemes": table}


def stream_read_sized(probe, torch, dev, mb):
    """The read-only probe over buffers of `mb` MB, timed like a decode launch: distinct buffers in
    rotation (so that the memory-side cache cannot serve them), launches back to back in HIP
    graphs between two events, the inter-launch gap included."""
    n = int(mb * 1e6) // 4096 * 4096
    layers = max(2, min(40, int(12e9 // n)))
    bufs = [torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(layers)]
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    shapes = {}
    for wgs in (256, 512, 1024, 2048, 4096, 8192):
        def fn(i):
            probe.stream_read_probe(bufs[i % layers], wgs, sink)
        graph_timed(torch, fn, 300, layers)
        us = graph_timed(torch, fn, 1000, layers) * 1e3
        shapes[wgs] = {"us_per_launch": round(us, 2), "gbs": round(n / us / 1e3, 1)}
    best = min(shapes, key=lambda k: shapes[k]["us_per_launch"])
    return {"metric": "read-only launch of %.1f MB (coopt_stream_read_probe), HIP-graph timing" % mb,
            "bytes": n, "buffers_rotated": layers, "launches_timed": 1000,
            "best_workgroups": best, "us_per_launch": shapes[best]["us_per_launch"], "gbs": shapes[best]["gbs"],
            "workgroups_of_256_lanes": shapes}


def stream_read_ceiling(coopt, torch, dev, detail=False):      # `coopt`: the probe's binding
    """GB/s of coopt_stream_read_probe (a kernel that only reads, 16-byte streaming loads) over a
    2 GiB buffer, far beyond the memory-side cache: the best of a few launch shapes, 10 launches
    each between two events.  What this GPU delivers when nothing but the loads is in the way."""
    buf = torch.empty(2 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    shapes = {}
    for wgs in (2048, 4096, 8192, 16384):
        for _ in range(3):
            coopt.stream_read_probe(buf, wgs, sink)
        e0.record()
        for _ in range(10):
            coopt.stream_read_probe(buf, wgs, sink)
        e1.record()
        torch.cuda.synchronize()
        shapes[wgs] = round(buf.numel() / (e0.elapsed_time(e1) / 10) / 1e6, 1)
    del buf
    best = max(shapes, key=shapes.get)
    out = {"gbs": shapes[best], "workgroups": best, "bytes": 2 << 30}
    if detail:
        out["gbs_by_workgroups"] = shapes
    return out


def bench_prefill(args, w, coopt, torch, dev, steps, warmup, cpu):
    """Config 4: a step = cache write of every sequence's chunk (quantise-on-write) + causal
    attention of the chunk rows over history and chunk.  A dense contraction: the dominant kernel
    is priced against the fp16 matrix-core peak."""
    shape = coopt.Shape(w.S, w.H_q, w.H_k, w.d, w.B, w.NB, w.max_blocks, coopt.COOPT_KV_E4M3,
                        float(np.float32(w.softmax_scale)))
    C = w.new_per_seq
    layers = args.layers or 4

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    hist, new = w.history_index(), w.new_index()
    k_hist, v_hist = to_dev(w.k_ctx[hist].view(np.uint16)), to_dev(w.v_ctx[hist].view(np.uint16))
    s_hist = to_dev(w.slots[hist])
    k_new, v_new = to_dev(w.k_ctx[new].view(np.uint16)), to_dev(w.v_ctx[new].view(np.uint16))
    s_new = to_dev(w.slots[new])
    q, bt, lens, qs = (to_dev(w.q.view(np.uint16)), to_dev(w.block_tables), to_dev(w.context_lens),
                       to_dev(w.query_start))
    n_rows = int(w.query_start[-1])
    out = torch.zeros((n_rows, w.H_q, w.d), dtype=torch.float16, device=dev)
    pools = []
    for _ in range(layers):
        kc = torch.zeros((w.NB, w.H_k, w.B * w.d), dtype=torch.uint8, device=dev)
        vc = torch.zeros_like(kc)
        ks = torch.zeros((w.NB, w.H_k, w.B), dtype=torch.float32, device=dev)
        vs = torch.zeros_like(ks)
        coopt.kv_cache_write_fp8(k_hist, v_hist, s_hist, kc, vc, ks, vs, shape)
        pools.append((kc, vc, ks, vs))
    torch.cuda.synchronize()

    # The entry point with a workspace for the launch's last, partly filled round (its tiles then run
    # as half-streams in full-size workgroups plus a merge); --prefill-entry plain times the one
    # without (half-size workgroups for those tiles).
    with_ws = args.prefill_entry == "workspace"
    ws_bytes = coopt.prefill_workspace_bytes(shape, C) if with_ws else 0
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev) if with_ws else None

    def attend_plain(i):
        coopt.paged_gqa_prefill_chunk(q, *pools[i % layers], bt, lens, qs, n_rows, C, out, shape)

    def attend(i):
        if with_ws:
            coopt.paged_gqa_prefill_chunk_ws(q, *pools[i % layers], bt, lens, qs, n_rows, C, out, ws, shape)
        else:
            attend_plain(i)

    def step(i):
        coopt.kv_cache_write_fp8(k_new, v_new, s_new, *pools[i % layers], shape)
        attend(i)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, count):                 # launches of ~1 ms: eager is fine
        e0.record()
        for i in range(count):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / count

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    steps = min(steps, 200)
    t0 = time.perf_counter()
    step_ms = timed(step, steps)
    wall_ms = (time.perf_counter() - t0) * 1e3
    kern_ms = timed(attend, steps)
    plain_ms = timed(attend_plain, steps) if with_ws else kern_ms
    attend(0)                             # the rows the parity check reads come from the timed entry point
    torch.cuda.synchronize()
    # 2 products of 2*d flops per (row, query head, visible token)
    pairs = sum(C * (int(t) - C) + C * (C + 1) // 2 for t in w.context_lens)
    flops = 4.0 * w.d * w.H_q * pairs
    result = {
        "metric": "chunked prefill attention over the paged FP8 cache: TFLOP/s per step",
        "value": round(flops / step_ms / 1e9, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(step_ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 cache, f16 MFMA, f32 accumulate", "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": w.S, "q_heads": w.H_q, "kv_heads": w.H_k,
                   "head_dim": w.d, "block_size": w.B, "history_tokens": int(w.context_lens[0]) - C,
                   "chunk_tokens": C, "kv_pools_rotated": layers,
                   "step": "kv_cache_write of the chunk + %s, one layer" %
                           ("paged_gqa_prefill_chunk_ws" if with_ws else "paged_gqa_prefill_chunk"),
                   "workspace_bytes": int(ws_bytes),
                   "launch": "eager"},
        "wall_ms_timed_region": round(wall_ms, 2),
        "roofline": {"bound": "mfma",
                     "kernel": ("prefill_chunk_kernel (coopt_paged_gqa_prefill_chunk_ws: full workgroups, then the "
                                "last tiles as half-streams in full workgroups, and the merge of the halves)")
                     if with_ws else
                     "prefill_chunk_kernel (coopt_paged_gqa_prefill_chunk: its two launches, full and half-size workgroups)",
                     "achieved": round(flops / kern_ms / 1e9, 1), "peak": MFMA_F16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(flops / kern_ms / 1e9 / MFMA_F16_PEAK_TFLOPS, 4),
                     "traffic": None, "algorithmic_flops_per_launch": flops,
                     "kernel_ms_mean": round(kern_ms, 4),
                     "without_workspace_kernel_ms_mean": round(plain_ms, 4)},
    }
    if cpu:
        base, rows, ref = cpu_baseline_prefill(w, flops)
        result["cpu_baseline"] = base
        got = out.cpu().numpy().astype(np.float64)[rows]          # sequence 0 starts at row 0
        err = np.abs(got - ref)
        result["parity"] = {"against": "oracle (float64) on the cpu_baseline sample, same inputs",
                            "rows": int(len(rows)), "elements": int(ref.size),
                            "max_abs": float(err.max()), "max_abs_oracle": float(np.abs(ref).max()),
                            "over_2e-3": int((err > 2e-3).sum()),
                            "finite": bool(np.isfinite(got).all())}
    del pools
    return result


def bench_gather(args, w, coopt, torch, dev):
    """The dequantising gather over every sequence of the workload: a step = S launches, sequence s
    reading its t_s cached tokens (codes + scales through the block table) and writing them as
    contiguous fp16.  Pure data movement, priced against the HBM peak."""
    e4m3 = w.kv_dtype == "e4m3"
    es = 1 if e4m3 else 2
    shape = coopt.Shape(w.S, w.H_q, w.H_k, w.d, w.B, w.NB, w.max_blocks,
                        coopt.COOPT_KV_E4M3 if e4m3 else coopt.COOPT_KV_FP16,
                        float(np.float32(w.softmax_scale)))
    pool_bytes = w.NB * w.H_k * w.B * (2 * w.d * es + (8 if e4m3 else 0))
    layers = args.layers or max(2, min(8, int(8e9 // pool_bytes)))

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    k_all, v_all = to_dev(w.k_ctx.view(np.uint16)), to_dev(w.v_ctx.view(np.uint16))
    slots, bt = to_dev(w.slots), to_dev(w.block_tables)
    pools = []
    for _ in range(layers):
        kc = torch.zeros((w.NB, w.H_k, w.B * w.d * es), dtype=torch.uint8, device=dev)
        vc = torch.zeros_like(kc)
        ks = torch.zeros((w.NB, w.H_k, w.B), dtype=torch.float32, device=dev) if e4m3 else None
        vs = torch.zeros_like(ks) if e4m3 else None
        if e4m3:
            coopt.kv_cache_write_fp8(k_all, v_all, slots, kc, vc, ks, vs, shape)
        else:
            coopt.kv_cache_write_fp16(k_all, v_all, slots, kc, vc, shape)
        pools.append((kc, vc, ks, vs))
    lens = [int(t) for t in w.context_lens]
    outs = [(torch.empty((t, w.H_k, w.d), dtype=torch.float16, device=dev),
             torch.empty((t, w.H_k, w.d), dtype=torch.float16, device=dev)) for t in lens]
    torch.cuda.synchronize()

    def step(i):
        pool = pools[i % layers]
        for s_, t in enumerate(lens):
            coopt.gather_cached_kv(*pool, bt, s_, 0, t, outs[s_][0], outs[s_][1], shape)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    steps = min(args.steps, 200)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    step_ms = e0.elapsed_time(e1) / steps
    # per (token, KV head): K and V codes, their two scales, and the two fp16 rows written
    per_row = 2 * w.d * es + (8 if e4m3 else 0) + 2 * 2 * w.d
    total = float(sum(lens)) * w.H_k * per_row + sum((t + w.B - 1) // w.B for t in lens) * 4.0
    gbps = total / step_ms / 1e6
    result = {
        "metric": "dequantising gather of the paged cache (gather_cached_kv): GB/s per step",
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3 -> f16" if e4m3 else "f16", "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": w.S, "kv_heads": w.H_k, "head_dim": w.d,
                   "block_size": w.B, "tokens": sum(lens), "kv_pools_rotated": layers,
                   "step": "coopt_gather_cached_kv of tokens [0, t_s) for each of the S sequences",
                   "launch": "eager, back to back on one stream"},
        "wall_ms_timed_region": round(wall_ms, 2),
        "roofline": {"bound": "hbm", "kernel": "gather_cached_kv_kernel (coopt_gather_cached_kv)",
                     "achieved": round(gbps, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": round(total / len(lens), 1),
                     "launch_us_mean": round(step_ms * 1e3 / len(lens), 2),
                     "note": "launch duration = event time of the step / launches (includes the "
                             "gap between dependent launches)"},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        dt = np.uint8 if e4m3 else np.float16
        kc = np.zeros((w.NB, w.H_k, w.B * w.d), dtype=dt)
        vc = np.zeros_like(kc)
        ks = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32) if e4m3 else None
        vs = np.zeros_like(ks) if e4m3 else None
        idx = np.arange(int(w.seq_start[1]))
        rows = (np.ascontiguousarray(w.k_ctx[idx]), np.ascontiguousarray(w.v_ctx[idx]),
                np.ascontiguousarray(w.slots[idx]))
        if e4m3:
            oracle.kv_cache_write_fp8(*rows, kc, vc, ks, vs, H_k=w.H_k, d=w.d, B=w.B)
        else:
            oracle.kv_cache_write_fp16(*rows, kc, vc, H_k=w.H_k, d=w.d, B=w.B)
        cache = (kc, vc, ks, vs)
        t0 = time.perf_counter()
        oracle.gather_cached_kv(*cache, w.block_tables, 0, 0, lens[0], H_k=w.H_k, d=w.d, B=w.B)
        sec = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(lens[0] * w.H_k * per_row / sec / 1e9, 3), "unit": "GB/s",
                                  "cores": 1, "kind": "oracle", "seconds": round(sec, 3),
                                  "sample": f"sequence 0 ({lens[0]} of {sum(lens)} tokens), all KV heads"}
    return result


def cpu_baseline_prefill(w, flops):
    """The oracle on a sample of chunk rows of the first sequence (every query head), scaled by
    flops to the whole step."""
    import oracle
    oracle.build()
    C = w.new_per_seq
    n_tok = int(w.seq_start[1])
    kc = np.zeros((w.NB, w.H_k, w.B, w.d), dtype=np.uint8)
    vc = np.zeros((w.NB, w.H_k, w.d, w.B), dtype=np.uint8)
    ks = np.zeros((w.NB, w.H_k, w.B), dtype=np.float32)
    vs = np.zeros_like(ks)
    idx = np.arange(n_tok)
    oracle.kv_cache_write_fp8(np.ascontiguousarray(w.k_ctx[idx]), np.ascontiguousarray(w.v_ctx[idx]),
                              np.ascontiguousarray(w.slots[idx]), kc, vc, ks, vs, H_k=w.H_k, d=w.d, B=w.B)
    rows = np.arange(0, C, 8, dtype=np.int32)               # 64 rows of sequence 0
    t0 = time.perf_counter()
    ref = oracle.paged_gqa_prefill_chunk(w.q, kc, vc, ks, vs, w.block_tables, w.context_lens,
                                         w.query_start, H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                         softmax_scale=w.softmax_scale, rows=rows)
    sec = time.perf_counter() - t0
    t_ctx = int(w.context_lens[0]) - C
    sample_flops = 4.0 * w.d * w.H_q * sum(t_ctx + int(r) + 1 for r in rows)
    return ({"value": round(sample_flops / sec / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
             "kind": "oracle", "seconds": round(sec, 3),
             "sample": f"{len(rows)} of {C} chunk rows of sequence 0, all {w.H_q} query heads, "
                       f"attention only ({sample_flops / flops:.2%} of the step's flops)"},
            rows, np.asarray(ref, dtype=np.float64))


def cpu_baseline(w, ab):
    """The oracle as it stands, timed on the host cores: the same step (write of the new tokens +
    attention) on a bounded sample of the workload's sequences (about 10-30 s of CPU work).
    Returns the baseline record and the oracle's output rows for the sampled sequences."""
    import oracle
    oracle.build()
    # sample: the whole batch when the oracle finishes it in about a second, else its first quarter
    budget = ab["tokens"] if w.H_q * ab["tokens"] <= 4_000_000 else ab["tokens"] // 4
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
    for _ in range(5):
        t0 = time.perf_counter()
        write(new)
        ref = oracle.paged_gqa_decode(np.ascontiguousarray(w.q[:n]), kc, vc, ks, vs,
                                np.ascontiguousarray(w.block_tables[:n]),
                                np.ascontiguousarray(w.context_lens[:n]), H_q=w.H_q, H_k=w.H_k,
                                d=w.d, B=w.B, softmax_scale=w.softmax_scale)
        best = min(best, time.perf_counter() - t0)
    kv = tok_end * ab["per_token"]
    return ({"value": round(kv / best / 1e9, 5), "unit": "GB/s", "cores": oracle.num_threads(),
             "kind": "oracle", "seconds": round(best, 3),
             "sample": f"first {n} of {w.S} sequences ({tok_end} of {ab['tokens']} context tokens), "
                       f"one layer, write + decode, best of 5"}, np.asarray(ref, dtype=np.float64))


if __name__ == "__main__":
    main()
