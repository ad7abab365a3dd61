"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed);
argument validation returns error codes before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2602_09323_amd as coopt
from paper_2602_09323_amd import binding, probe
from paper_2602_09323_amd.build import build, needs_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "coopt_attn.h")
PROBE_HEADER = os.path.join(ROOT, "include", "coopt_probe.h")


@pytest.fixture(scope="module")
def lib():
    if needs_build():
        build(force=True)
    return coopt.load_library()


@pytest.fixture(scope="module")
def probe_lib(lib):
    return probe.load_library()


def _declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(coopt_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib, probe_lib):
    """Every header under include/ against the library that implements it."""
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert headers == ["coopt_attn.h", "coopt_probe.h"]
    names = _declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), f"{name} declared in the header but not exported"
    assert sorted(binding.EXPORTS) == names
    probe_names = _declared_functions(PROBE_HEADER)
    assert probe_names == sorted(probe.EXPORTS) == ["coopt_stream_read_probe"]
    for name in probe_names:
        assert hasattr(probe_lib, name)
        assert not hasattr(lib, name), "the measurement aid is no part of the product library"


def test_no_process_wide_plan(lib):
    assert not hasattr(lib, "coopt_set_decode_plan") and not hasattr(lib, "coopt_get_decode_plan")
    p = coopt.default_decode_plan().as_dict()
    assert p == dict(tokens_per_group=128, waves_per_group=1, pipeline_depth=2,
                     grid_waves=p["grid_waves"], softmax_reduction=0)
    assert p["grid_waves"] > 0 and p["grid_waves"] % 4 == 0      # one wavefront per SIMD


def _struct_fields(name):
    body = re.search(r"typedef struct %s \{(.*?)\}" % name, open(HEADER).read(), flags=re.S).group(1)
    return re.findall(r"^\s+(?:int32_t|float)\s+(\w+);", body, flags=re.M)


def test_structs_match_header():
    assert ctypes.sizeof(coopt.Shape) == 9 * 4
    assert [f[0] for f in coopt.Shape._fields_] == _struct_fields("coopt_shape")
    assert ctypes.sizeof(coopt.DecodePlan) == 5 * 4
    assert [f[0] for f in coopt.DecodePlan._fields_] == _struct_fields("coopt_decode_plan")


def test_status_strings(lib):
    for code in (0, -1, -2, -3, -4, -99):
        assert isinstance(coopt.status_string(code), str) and coopt.status_string(code)


def _shape(**kw):
    base = dict(num_seqs=2, num_q_heads=40, num_kv_heads=8, head_dim=128, block_size=16,
                num_blocks=64, max_blocks_per_seq=8, kv_dtype=1, softmax_scale=0.088)
    base.update(kw)
    return coopt.Shape(*[base[f[0]] for f in coopt.Shape._fields_])


@pytest.mark.parametrize("bad", [dict(head_dim=96), dict(block_size=32), dict(num_q_heads=41),
                                 dict(num_q_heads=8 * 17), dict(kv_dtype=3), dict(num_blocks=0),
                                 dict(num_kv_heads=0), dict(num_seqs=(1 << 20) + 1),
                                 dict(num_q_heads=8192, num_kv_heads=1024),
                                 dict(max_blocks_per_seq=(1 << 24) + 1),
                                 dict(num_blocks=1 << 29, num_kv_heads=8)])
def test_unsupported_shapes_are_refused_without_launch(lib, bad):
    sh = _shape(**bad)
    one = ctypes.c_void_p(16)          # never dereferenced: validation comes first
    assert lib.coopt_kv_cache_write_fp8(one, one, one, 1, one, one, one, one, ctypes.byref(sh), None) == -2
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, None, ctypes.c_size_t(0), None, ctypes.byref(sh), None) == -2
    assert lib.coopt_paged_gqa_reduce(one, one, one, one, 16, 1, one, ctypes.byref(sh), None) == -2
    assert lib.coopt_decode_workspace_bytes(ctypes.byref(sh), None) == 0
    assert lib.coopt_decode_schedule_bytes(ctypes.byref(sh), None) == 0


def test_null_pointers_and_bad_arguments(lib):
    # sizes go in as ctypes.c_size_t: a bare Python int is passed as a 32-bit int, and the upper
    # half of a size_t argument on the stack would be whatever was there
    sh = _shape()
    one = ctypes.c_void_p(16)
    assert lib.coopt_kv_cache_write_fp8(None, one, one, 1, one, one, one, one, ctypes.byref(sh), None) == -1
    assert lib.coopt_kv_cache_write_fp8(one, one, one, 1, one, one, None, one, ctypes.byref(sh), None) == -1
    assert lib.coopt_kv_cache_write_fp8(one, one, one, 0, one, one, one, one, ctypes.byref(sh), None) == 0
    assert lib.coopt_kv_cache_write_fp16(one, one, one, 1, one, one, ctypes.byref(sh), None) == -2  # wrong dtype
    assert lib.coopt_paged_gqa_decode(one, one, one, None, one, one, one, one, None, ctypes.c_size_t(0), None, ctypes.byref(sh), None) == -1
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, None, None, ctypes.c_size_t(0), None, ctypes.byref(sh), None) == -1
    # split decode with a workspace that is too small / misaligned
    # (every call below is refused by validation before any launch: pointers are never read)
    sh2 = _shape(max_blocks_per_seq=128)
    need2 = lib.coopt_decode_workspace_bytes(ctypes.byref(sh2), None)
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, one, ctypes.c_size_t(need2 - 1), None, ctypes.byref(sh2), None) == -3
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, ctypes.c_void_p(8), ctypes.c_size_t(need2), None, ctypes.byref(sh2), None) == -3
    assert lib.coopt_kv_cache_write_skipset(None, one, one, one, 1, one, one, one, one, ctypes.byref(sh), None) == -1
    assert lib.coopt_kv_cache_write_skipset(one, one, one, None, 0, one, one, one, one, ctypes.byref(sh), None) == 0
    assert lib.coopt_kv_cache_write_skipset(one, one, one, one, 1, one, one, one, one, None, None) == -1
    # the write under another scale rule: the mode is checked, static scales are required for it
    scaled = lib.coopt_kv_cache_write_fp8_scaled
    assert scaled(one, one, one, 1, one, one, one, one, 3, None, None, ctypes.byref(sh), None) == -2
    assert scaled(one, one, one, 1, one, one, one, one, 2, None, one, ctypes.byref(sh), None) == -1
    assert scaled(one, one, one, 1, one, one, one, None, 1, None, None, ctypes.byref(sh), None) == -1
    assert scaled(one, one, one, 0, one, one, one, one, 1, None, None, ctypes.byref(sh), None) == 0
    assert scaled(one, one, one, 1, one, one, one, one, 0, None, None, ctypes.byref(_shape(kv_dtype=0)), None) == -2
    # fused step: the new rows and a workspace are required
    assert lib.coopt_paged_gqa_decode_step(None, one, one, one, one, one, one, one, one, one, one, one, ctypes.c_size_t(need2), None, ctypes.byref(sh2), None) == -1
    assert lib.coopt_paged_gqa_decode_step(one, one, one, one, one, one, one, one, one, one, one, None, ctypes.c_size_t(need2), None, ctypes.byref(sh2), None) == -1
    assert lib.coopt_paged_gqa_decode_step(one, one, one, one, one, one, one, one, one, one, one, one, ctypes.c_size_t(need2 - 1), None, ctypes.byref(sh2), None) == -3
    # prepared schedule: buffers are required, sized and aligned; a fused call needs all three rows
    nsched = lib.coopt_decode_schedule_bytes(ctypes.byref(sh2), None)
    assert nsched > 0 and nsched % 16 == 0
    cs = ctypes.c_size_t
    assert lib.coopt_decode_schedule_prepare(one, one, None, None, cs(nsched), None, ctypes.byref(sh2), None) == -1
    assert lib.coopt_decode_schedule_prepare(None, one, None, one, cs(nsched), None, ctypes.byref(sh2), None) == -1
    assert lib.coopt_decode_schedule_prepare(one, one, None, one, cs(nsched - 1), None, ctypes.byref(sh2), None) == -3
    assert lib.coopt_decode_schedule_prepare(one, one, None, ctypes.c_void_p(8), cs(nsched), None, ctypes.byref(sh2), None) == -3
    run = lib.coopt_paged_gqa_decode_scheduled
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), None, cs(nsched), None, ctypes.byref(sh2), None) == -1
    assert run(one, None, one, one, one, one, one, one, one, one, one, cs(need2), one, cs(nsched), None, ctypes.byref(sh2), None) == -1
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2 - 1), one, cs(nsched), None, ctypes.byref(sh2), None) == -3
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), one, cs(nsched - 1), None, ctypes.byref(sh2), None) == -3
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), ctypes.c_void_p(8), cs(nsched), None, ctypes.byref(sh2), None) == -3
    assert run(None, None, None, None, one, one, one, one, one, one, one, cs(need2), one, cs(nsched), None, ctypes.byref(sh2), None) == -1
    # partitioned: partition size must be a positive multiple of 16; buffers must cover the table
    assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 24, one, one, one, 8, None, ctypes.byref(sh), None) == -2
    assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 16, one, one, one, 7, None, ctypes.byref(sh), None) == -3
    assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 16, None, one, one, 8, None, ctypes.byref(sh), None) == -1
    assert lib.coopt_gather_cached_kv(one, one, one, one, one, 5, 0, 4, one, one, ctypes.byref(sh), None) == -2
    assert lib.coopt_gather_cached_kv(one, one, one, one, one, 0, 0, 999, one, one, ctypes.byref(sh), None) == -2
    # a plan with a field out of range: refused by every entry point that takes one
    good = coopt.default_decode_plan().as_dict()
    for bad in (dict(tokens_per_group=100), dict(tokens_per_group=0), dict(waves_per_group=3),
                dict(pipeline_depth=4), dict(pipeline_depth=0), dict(grid_waves=0),
                dict(grid_waves=-5), dict(softmax_reduction=2)):
        p = coopt.make_decode_plan(**{**good, **bad})
        pp = ctypes.byref(p)
        assert lib.coopt_decode_workspace_bytes(ctypes.byref(sh2), pp) == 0
        assert lib.coopt_decode_schedule_bytes(ctypes.byref(sh2), pp) == 0
        assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, one, cs(need2), pp, ctypes.byref(sh2), None) == -2
        assert lib.coopt_paged_gqa_decode_step(one, one, one, one, one, one, one, one, one, one, one, one, cs(need2), pp, ctypes.byref(sh2), None) == -2
        assert lib.coopt_paged_gqa_decode_split(one, one, one, one, one, one, one, one, cs(need2), pp, ctypes.byref(sh2), None) == -2
        assert lib.coopt_paged_gqa_decode_merge(one, one, cs(need2), one, pp, ctypes.byref(sh2), None) == -2
        assert lib.coopt_decode_schedule_prepare(one, one, None, one, cs(nsched), pp, ctypes.byref(sh2), None) == -2
        assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), one, cs(nsched), pp, ctypes.byref(sh2), None) == -2
        assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 16, one, one, one, 8, pp, ctypes.byref(sh), None) == -2
    # the plan changes the sizes it is asked about
    small = coopt.make_decode_plan(tokens_per_group=32)
    assert lib.coopt_decode_workspace_bytes(ctypes.byref(sh2), ctypes.byref(small)) > need2


def test_probe_arguments(probe_lib):
    """The streaming-read probe: launch shape and alignment are checked before anything else."""
    one = ctypes.c_void_p(16)
    f = probe_lib.coopt_stream_read_probe
    assert f(one, ctypes.c_size_t(1 << 20), 0, one, None) == -2
    assert f(one, ctypes.c_size_t(1 << 20), (1 << 20) + 1, one, None) == -2
    assert f(ctypes.c_void_p(24), ctypes.c_size_t(1 << 20), 64, one, None) == -2
    assert f(None, ctypes.c_size_t(1 << 20), 64, one, None) == -1
    assert f(one, ctypes.c_size_t(1 << 20), 64, None, None) == -1
    assert f(None, ctypes.c_size_t(0), 64, None, None) == 0


def test_prefill_workspace_size_and_refusals(lib):
    """The workspace of coopt_paged_gqa_prefill_chunk_ws: zero where the tiles fill whole rounds
    of 256 workgroups, otherwise parts x 16 columns x (d + 2) floats per tile of the last round
    and (sequence, KV head) pair, parts (2 to 8) = the split that makes that round shortest on 256
    CUs.  Refusals come before any launch."""
    cs = ctypes.c_size_t
    one = ctypes.c_void_p(16)
    size = lib.coopt_prefill_workspace_bytes
    cfg4 = _shape(num_seqs=8, num_q_heads=40, num_kv_heads=8, head_dim=128, num_blocks=8192,
                  max_blocks_per_seq=544)
    # 64 pairs x 160 tiles = 640 workgroups of 16 tiles: two rounds of 256 and 32 tiles a pair left
    assert size(ctypes.byref(cfg4), 512) == 64 * 32 * 2 * 16 * 130 * 4
    # 5 tiles a pair: 64 workgroups, a quarter of a round, so every pair's stages are cut in four
    assert size(ctypes.byref(cfg4), 16) == 64 * 5 * 4 * 16 * 130 * 4
    one_seq = _shape(num_seqs=1, num_q_heads=40, num_kv_heads=8, head_dim=128, num_blocks=8192,
                     max_blocks_per_seq=544)
    assert size(ctypes.byref(one_seq), 16) == 8 * 5 * 7 * 16 * 130 * 4     # 8 workgroups: seven parts (at most eight)
    assert size(ctypes.byref(one_seq), 512) == 8 * 160 * 3 * 16 * 130 * 4  # 80 workgroups: three parts fill 240 CUs
    three = _shape(num_seqs=3, num_q_heads=40, num_kv_heads=8, head_dim=128, num_blocks=8192,
                   max_blocks_per_seq=544)
    assert size(ctypes.byref(three), 512) == 0          # 240 workgroups: no number of parts makes the round shorter
    assert size(ctypes.byref(cfg4), 0) == 0
    whole = _shape(num_seqs=8, num_q_heads=32, num_kv_heads=8, head_dim=128, num_blocks=8192,
                   max_blocks_per_seq=544)
    assert size(ctypes.byref(whole), 512) == 0          # 64 pairs x 8 workgroups: two whole rounds
    assert size(ctypes.byref(_shape(head_dim=96)), 512) == 0      # a shape the library refuses
    run = lib.coopt_paged_gqa_prefill_chunk_ws
    need = size(ctypes.byref(cfg4), 512)
    args = (one, one, one, one, one, one, one, one, 4096, 512, one)
    assert run(*args, None, cs(need), ctypes.byref(cfg4), None) == -1
    assert run(*args, one, cs(need - 1), ctypes.byref(cfg4), None) == -3
    assert run(*args[:-1], None, one, cs(need), ctypes.byref(cfg4), None) == -1       # out is required
    assert run(one, one, one, one, one, one, one, one, 0, 512, one, None, cs(0), ctypes.byref(cfg4), None) == -1
    assert run(one, one, one, one, one, one, one, one, 0, 0, one, None, cs(0), ctypes.byref(cfg4), None) == 0
    assert run(*args, one, cs(need), ctypes.byref(_shape(head_dim=96)), None) == -2


def test_prefill_launch_plan_over_many_shapes(lib):
    """The rule behind coopt_prefill_workspace_bytes, restated here and swept over batch sizes,
    chunk lengths and group sizes: a workgroup covers 16 tiles of a pair (8 where a pair has at
    most 8), a round is 256 workgroups, whole rounds keep whole streams, and the L workgroups of
    the last round are cut into the p in 2..8 that minimises ceil(L p / 256) / p + 0.02 (p - 1) if
    that beats ceil(L / 256)."""
    import math
    size = lib.coopt_prefill_workspace_bytes
    for H_q, H_k in ((40, 8), (32, 8), (8, 8), (64, 4)):
        for S in list(range(1, 20)) + [31, 32, 33, 64, 100]:
            for C in (1, 16, 17, 64, 128, 500, 512, 2048):
                sh = _shape(num_seqs=S, num_q_heads=H_q, num_kv_heads=H_k, head_dim=128,
                            num_blocks=1 << 16, max_blocks_per_seq=1024)
                tiles = (H_q // H_k) * ((C + 15) // 16)
                wg_tiles = 8 if tiles <= 8 else 16
                pairs8 = (S * H_k + 7) // 8 * 8
                full = (tiles + wg_tiles - 1) // wg_tiles
                W = pairs8 * full
                cand = (W // 256) * 256 // pairs8
                want = 0
                if cand < full:
                    rest = tiles - cand * wg_tiles
                    last = pairs8 * ((rest + wg_tiles - 1) // wg_tiles)
                    best, best_cost = 1, float(math.ceil(last / 256))
                    for p in range(2, 9):
                        cost = math.ceil(last * p / 256) / p + 0.02 * (p - 1)
                        if cost < best_cost:
                            best, best_cost = p, cost
                    if best >= 2:
                        want = S * H_k * rest * best * 16 * 130 * 4
                assert size(ctypes.byref(sh), C) == want, (H_q, H_k, S, C)


def test_binding_refuses_bad_tensors_before_any_launch(lib, monkeypatch):
    """The C side sees raw pointers only, so the binding checks residence, contiguity, integer
    widths and sizes against the shape; none of these calls reaches the library."""
    import torch

    class SizeQueriesOnly:
        def __getattr__(self, name):
            if name in ("coopt_decode_workspace_bytes", "coopt_decode_schedule_bytes",
                        "coopt_prefill_workspace_bytes", "coopt_status_string", "coopt_default_decode_plan"):
                return getattr(lib, name)
            raise AssertionError(f"{name} was reached: the binding did not refuse the call")

    monkeypatch.setattr(binding, "load_library", lambda: SizeQueriesOnly())

    class FakeDev:
        """A stand-in with a device tensor's attributes (no GPU here); its pointer goes nowhere
        because every call below is refused before the library is entered."""
        is_cuda = True

        def __init__(self, n, dtype, contiguous=True):
            self._t = torch.empty(n, dtype=dtype)
            self.dtype = dtype
            self._c = contiguous

        def numel(self): return self._t.numel()
        def element_size(self): return self._t.element_size()
        def is_contiguous(self): return self._c
        def data_ptr(self): return 16

    sh = _shape()
    z = binding._sizes(sh)
    f16, i32, i64, u8, f32 = torch.float16, torch.int32, torch.int64, torch.uint8, torch.float32

    def ok():
        return dict(q=FakeDev(z["q"] // 2, f16), kc=FakeDev(z["cache"], u8), vc=FakeDev(z["cache"], u8),
                    ks=FakeDev(z["scale"] // 4, f32), vs=FakeDev(z["scale"] // 4, f32),
                    bt=FakeDev(z["tables"] // 4, i32), cl=FakeDev(z["lens"] // 4, i32),
                    out=FakeDev(z["q"] // 2, f16))

    def decode(a):
        coopt.paged_gqa_decode(a["q"], a["kc"], a["vc"], a["ks"], a["vs"], a["bt"], a["cl"], a["out"],
                               None, sh)

    cases = {
        "host tensor": ("q", torch.empty(z["q"] // 2, dtype=f16)),
        "fp32 q": ("q", FakeDev(z["q"] // 2, f32)),
        "short q": ("q", FakeDev(z["q"] // 2 - 1, f16)),
        "cache too small": ("kc", FakeDev(z["cache"] - 1, u8)),
        "v cache too small": ("vc", FakeDev(z["cache"] // 2, u8)),
        "scales missing": ("ks", None),
        "scales too small": ("vs", FakeDev(z["scale"] // 4 - 1, f32)),
        "int64 block table": ("bt", FakeDev(z["tables"] // 4, i64)),
        "short block table": ("bt", FakeDev(z["tables"] // 4 - 1, i32)),
        "int64 lengths": ("cl", FakeDev(z["lens"] // 4, i64)),
        "short lengths": ("cl", FakeDev(1, i32)),
        "strided out": ("out", FakeDev(z["q"] // 2, f16, contiguous=False)),
        "short out": ("out", FakeDev(8, f16)),
    }
    for what, (key, bad) in cases.items():
        a = ok()
        a[key] = bad
        with pytest.raises(coopt.CooptError):
            decode(a)
    # cache write: int32 slots would be read as half as many int64 values
    rows = FakeDev(4 * z["row"] // 2, f16)
    with pytest.raises(coopt.CooptError, match="slot_mapping"):
        coopt.kv_cache_write_fp8(rows, rows, FakeDev(4, i32), FakeDev(z["cache"], u8), FakeDev(z["cache"], u8),
                                 FakeDev(z["scale"] // 4, f32), FakeDev(z["scale"] // 4, f32), sh)
    with pytest.raises(coopt.CooptError, match=": k"):
        coopt.kv_cache_write_fp8(FakeDev(3 * z["row"] // 2, f16), rows, FakeDev(4, i64), FakeDev(z["cache"], u8),
                                 FakeDev(z["cache"], u8), FakeDev(z["scale"] // 4, f32),
                                 FakeDev(z["scale"] // 4, f32), sh)
    # fused step: one new row per sequence, a workspace of the plan's size
    a = ok()
    with pytest.raises(coopt.CooptError, match="slot_mapping has 1"):
        coopt.paged_gqa_decode_step(FakeDev(z["row"] // 2, f16), FakeDev(z["row"] // 2, f16), FakeDev(1, i64),
                                    a["q"], a["kc"], a["vc"], a["ks"], a["vs"], a["bt"], a["cl"], a["out"],
                                    FakeDev(16, u8), sh)
    rows2 = FakeDev(sh.num_seqs * z["row"] // 2, f16)
    with pytest.raises(coopt.CooptError, match="workspace"):
        coopt.paged_gqa_decode_step(rows2, rows2, FakeDev(sh.num_seqs, i64), a["q"], a["kc"], a["vc"],
                                    a["ks"], a["vs"], a["bt"], a["cl"], a["out"],
                                    FakeDev(coopt.decode_workspace_bytes(sh) - 1, u8), sh)
    with pytest.raises(coopt.CooptError, match="query_start"):
        coopt.paged_gqa_prefill_chunk(a["q"], a["kc"], a["vc"], a["ks"], a["vs"], a["bt"], a["cl"],
                                      FakeDev(sh.num_seqs, i32), 2, 1, a["out"], sh)


def test_empty_batches_are_accepted_without_launch(lib):
    """num_seqs = 0 / num_tokens = 0 / no query rows: COOPT_OK before any pointer is looked at."""
    sh = _shape(num_seqs=0)
    z = ctypes.c_size_t(0)
    assert lib.coopt_paged_gqa_decode(None, None, None, None, None, None, None, None, None, z, None, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_decode_step(None, None, None, None, None, None, None, None, None, None, None, None, z, None, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_decode_split(None, None, None, None, None, None, None, None, z, None, ctypes.byref(sh), None) == 0
    assert lib.coopt_decode_schedule_prepare(None, None, None, None, z, None, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_decode_scheduled(None, None, None, None, None, None, None, None, None, None, None, z, None, z, None, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_prefill_chunk(None, None, None, None, None, None, None, None, 0, 0, None, ctypes.byref(sh), None) == 0
    sh1 = _shape()
    assert lib.coopt_kv_cache_write_fp8(None, None, None, 0, None, None, None, None, ctypes.byref(sh1), None) == 0
    assert lib.coopt_kv_cache_write_skipset(None, None, None, None, 0, None, None, None, None, ctypes.byref(sh1), None) == 0
    assert lib.coopt_paged_gqa_prefill_chunk(None, None, None, None, None, None, None, None, 0, 0, None, ctypes.byref(sh1), None) == 0
