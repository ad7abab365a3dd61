"""GPU: the entry points under HIP graph capture.  Serving loops (and bench.py) capture the decode
step once and replay it; a replay has to give what the same calls give eagerly, on every replay,
with eager work of the same library and synchronisations in between.  Captured here: the fused
step from a prepared schedule (attention launch + merge launch, which also stores the step's new
rows into the cache), the decode that keeps its partials in the library's built-in array, and a
prefill chunk (two launches; three with a workspace).  None of them allocates, sets memory or
synchronises, so capture needs no special path -- this test is what holds them to that."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import alloc_dev_cache, assert_close, dev, hip_write, shape_of
from helpers import oracle_fill

pytestmark = pytest.mark.gpu


def _decode_inputs(w):
    new = w.new_index()
    return dict(q=dev(w.q.view(np.uint16)), bt=dev(w.block_tables), dl=dev(w.context_lens),
                k_new=dev(w.k_ctx[new].view(np.uint16)), v_new=dev(w.v_ctx[new].view(np.uint16)),
                slots=dev(w.slots[new].astype(np.int64)))


def test_replays_of_a_captured_decode_step_equal_the_eager_step(oracle_mod):
    w = workloads.make_custom("graph_step", seed=81, S=12, H_q=40, H_k=8, d=128, B=16, NB=900,
                              context_lens=[700, 33, 1, 512, 1300, 64, 17, 129, 2, 960, 48, 300],
                              max_blocks=96)
    other = workloads.make_custom("graph_other", seed=82, S=5, H_q=10, H_k=2, d=64, B=16, NB=60,
                                  context_lens=[100, 17, 260, 1, 31], max_blocks=17, kv_dtype="fp16")
    shape = shape_of(w)
    x = _decode_inputs(w)
    ref = oracle_mod.paged_gqa_decode(w.q, *oracle_fill(oracle_mod, w), w.block_tables, w.context_lens,
                                      H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    ws = torch.empty(coopt.decode_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    sched = torch.zeros(coopt.decode_schedule_bytes(shape), dtype=torch.uint8, device="cuda")
    coopt.decode_schedule_prepare(x["bt"], x["dl"], x["slots"], sched, shape)

    def history_cache():
        dcache = alloc_dev_cache(w, fill_byte=0x7F)
        hip_write(w, dcache, idx=w.history_index())
        return dcache

    def step(dcache, out_step, out_builtin):
        coopt.paged_gqa_decode_scheduled(x["k_new"], x["v_new"], x["slots"], x["q"], *dcache, x["dl"],
                                         out_step, ws, sched, shape)
        # the same attention again, now over the cache that holds the new rows
        coopt.paged_gqa_decode_noalloc(x["q"], *dcache, x["bt"], x["dl"], out_builtin, shape)

    # eager
    eager_cache = history_cache()
    eager_step = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    eager_builtin = torch.full_like(eager_step, -6.0)
    step(eager_cache, eager_step, eager_builtin)
    torch.cuda.synchronize()
    assert_close(eager_step.cpu().numpy().astype(np.float64), ref, "eager fused step")
    assert_close(eager_builtin.cpu().numpy().astype(np.float64), ref, "eager decode, built-in array")

    # captured
    graph_cache = history_cache()
    g_step = torch.full_like(eager_step, -5.0)
    g_builtin = torch.full_like(eager_step, -4.0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(graph_cache, g_step, g_builtin)
    torch.cuda.synchronize()
    for replay in range(4):
        g_step.fill_(-5.0 - replay)
        g_builtin.fill_(-4.0 - replay)
        if replay == 2:                      # the new rows are stored again by every replay
            fresh = history_cache()
            for dst, src in zip(graph_cache, fresh):
                dst.copy_(src)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_step, eager_step), f"replay {replay}: fused step differs from the eager one"
        assert torch.equal(g_builtin, eager_builtin), f"replay {replay}: built-in-array decode differs"
        for name, a, b in zip(("k_cache", "v_cache", "k_scale", "v_scale"), graph_cache, eager_cache):
            assert torch.equal(a, b), f"replay {replay}: {name} differs from the eager step's"
        # eager work of the same library between the replays: another shape, another cache type,
        # the built-in array and the workspace both reused
        oc = alloc_dev_cache(other)
        hip_write(other, oc)
        oshape = shape_of(other)
        oout = torch.zeros((other.S, other.H_q, other.d), dtype=torch.float16, device="cuda")
        coopt.paged_gqa_decode_noalloc(dev(other.q.view(np.uint16)), *oc, dev(other.block_tables),
                                       dev(other.context_lens), oout, oshape)
        torch.cuda.synchronize()
        assert torch.isfinite(oout.float()).all()


@pytest.mark.parametrize("with_workspace", [False, True])
def test_replays_of_a_captured_prefill_chunk_equal_the_eager_call(oracle_mod, with_workspace):
    """(with a workspace: three launches -- here every pair's stages in eight parts -- and the
    partial rows of one replay are overwritten by the next and by the eager call in between)"""
    S, C, hist = 3, 80, [0, 300, 1000]
    w = workloads.make_custom("graph_prefill", seed=83, S=S, H_q=10, H_k=2, d=128, B=16, NB=120,
                              context_lens=[h + C for h in hist], new_per_seq=C)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_prefill_chunk(w.q, *cache, w.block_tables, w.context_lens, w.query_start,
                                             H_q=w.H_q, H_k=w.H_k, d=w.d, B=w.B,
                                             softmax_scale=w.softmax_scale)
    shape = shape_of(w)
    dcache = alloc_dev_cache(w)
    hip_write(w, dcache)
    q, bt, dl, qs = dev(w.q.view(np.uint16)), dev(w.block_tables), dev(w.context_lens), dev(w.query_start)
    eager = torch.full((S * C, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    need = coopt.prefill_workspace_bytes(shape, C)
    assert need > 0
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")

    def call(out):
        if with_workspace:
            coopt.paged_gqa_prefill_chunk_ws(q, *dcache, bt, dl, qs, S * C, C, out, ws, shape)
        else:
            coopt.paged_gqa_prefill_chunk(q, *dcache, bt, dl, qs, S * C, C, out, shape)

    call(eager)
    torch.cuda.synchronize()
    assert_close(eager.cpu().numpy().astype(np.float64), ref, "eager prefill chunk")

    out = torch.full_like(eager, -5.0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call(out)
    torch.cuda.synchronize()
    for replay in range(3):
        out.fill_(-5.0 - replay)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {replay}: prefill chunk differs from the eager call"
        scratch = torch.full_like(eager, -1.0)          # an eager call between the replays
        ws.fill_(float("nan"))
        call(scratch)
        torch.cuda.synchronize()
        assert torch.equal(scratch, eager)
