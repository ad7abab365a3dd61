"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed);
argument validation returns error codes before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2602_09323_amd as coopt
from paper_2602_09323_amd import binding
from paper_2602_09323_amd.build import build, needs_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "coopt_attn.h")


@pytest.fixture(scope="module")
def lib():
    if needs_build():
        build(force=True)
    return coopt.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(coopt_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), f"{name} declared in the header but not exported"
    assert sorted(binding.EXPORTS) == names


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
                                 dict(num_q_heads=8 * 17), dict(kv_dtype=2), dict(num_blocks=0),
                                 dict(num_kv_heads=0), dict(num_seqs=(1 << 20) + 1),
                                 dict(num_q_heads=8192, num_kv_heads=1024),
                                 dict(max_blocks_per_seq=(1 << 24) + 1),
                                 dict(num_blocks=1 << 29, num_kv_heads=8)])
def test_unsupported_shapes_are_refused_without_launch(lib, bad):
    sh = _shape(**bad)
    one = ctypes.c_void_p(16)          # never dereferenced: validation comes first
    assert lib.coopt_kv_cache_write_fp8(one, one, one, 1, one, one, one, one, ctypes.byref(sh), None) == -2
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, None, ctypes.c_size_t(0), ctypes.byref(sh), None) == -2
    assert lib.coopt_paged_gqa_reduce(one, one, one, one, 16, 1, one, ctypes.byref(sh), None) == -2
    assert lib.coopt_decode_workspace_bytes(ctypes.byref(sh)) == 0
    assert lib.coopt_decode_schedule_bytes(ctypes.byref(sh)) == 0


def test_null_pointers_and_bad_arguments(lib):
    # sizes go in as ctypes.c_size_t: a bare Python int is passed as a 32-bit int, and the upper
    # half of a size_t argument on the stack would be whatever was there
    sh = _shape()
    one = ctypes.c_void_p(16)
    assert lib.coopt_kv_cache_write_fp8(None, one, one, 1, one, one, one, one, ctypes.byref(sh), None) == -1
    assert lib.coopt_kv_cache_write_fp8(one, one, one, 1, one, one, None, one, ctypes.byref(sh), None) == -1
    assert lib.coopt_kv_cache_write_fp8(one, one, one, 0, one, one, one, one, ctypes.byref(sh), None) == 0
    assert lib.coopt_kv_cache_write_fp16(one, one, one, 1, one, one, ctypes.byref(sh), None) == -2  # wrong dtype
    assert lib.coopt_paged_gqa_decode(one, one, one, None, one, one, one, one, None, ctypes.c_size_t(0), ctypes.byref(sh), None) == -1
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, None, None, ctypes.c_size_t(0), ctypes.byref(sh), None) == -1
    # split decode with a workspace that is too small / misaligned
    # (every call below is refused by validation before any launch: pointers are never read)
    sh2 = _shape(max_blocks_per_seq=128)
    need2 = lib.coopt_decode_workspace_bytes(ctypes.byref(sh2))
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, one, ctypes.c_size_t(need2 - 1), ctypes.byref(sh2), None) == -3
    assert lib.coopt_paged_gqa_decode(one, one, one, one, one, one, one, one, ctypes.c_void_p(8), ctypes.c_size_t(need2), ctypes.byref(sh2), None) == -3
    assert lib.coopt_kv_cache_write_skipset(None, one, one, one, 1, one, one, one, one, ctypes.byref(sh), None) == -1
    assert lib.coopt_kv_cache_write_skipset(one, one, one, None, 0, one, one, one, one, ctypes.byref(sh), None) == 0
    assert lib.coopt_kv_cache_write_skipset(one, one, one, one, 1, one, one, one, one, None, None) == -1
    # fused step: the new rows and a workspace are required
    assert lib.coopt_paged_gqa_decode_step(None, one, one, one, one, one, one, one, one, one, one, one, ctypes.c_size_t(need2), ctypes.byref(sh2), None) == -1
    assert lib.coopt_paged_gqa_decode_step(one, one, one, one, one, one, one, one, one, one, one, None, ctypes.c_size_t(need2), ctypes.byref(sh2), None) == -1
    assert lib.coopt_paged_gqa_decode_step(one, one, one, one, one, one, one, one, one, one, one, one, ctypes.c_size_t(need2 - 1), ctypes.byref(sh2), None) == -3
    # prepared schedule: buffers are required, sized and aligned; a fused call needs all three rows
    nsched = lib.coopt_decode_schedule_bytes(ctypes.byref(sh2))
    assert nsched > 0 and nsched % 16 == 0
    cs = ctypes.c_size_t
    assert lib.coopt_decode_schedule_prepare(one, one, None, None, cs(nsched), ctypes.byref(sh2), None) == -1
    assert lib.coopt_decode_schedule_prepare(None, one, None, one, cs(nsched), ctypes.byref(sh2), None) == -1
    assert lib.coopt_decode_schedule_prepare(one, one, None, one, cs(nsched - 1), ctypes.byref(sh2), None) == -3
    assert lib.coopt_decode_schedule_prepare(one, one, None, ctypes.c_void_p(8), cs(nsched), ctypes.byref(sh2), None) == -3
    run = lib.coopt_paged_gqa_decode_scheduled
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), None, cs(nsched), ctypes.byref(sh2), None) == -1
    assert run(one, None, one, one, one, one, one, one, one, one, one, cs(need2), one, cs(nsched), ctypes.byref(sh2), None) == -1
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2 - 1), one, cs(nsched), ctypes.byref(sh2), None) == -3
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), one, cs(nsched - 1), ctypes.byref(sh2), None) == -3
    assert run(None, None, None, one, one, one, one, one, one, one, one, cs(need2), ctypes.c_void_p(8), cs(nsched), ctypes.byref(sh2), None) == -3
    assert run(None, None, None, None, one, one, one, one, one, one, one, cs(need2), one, cs(nsched), ctypes.byref(sh2), None) == -1
    # partitioned: partition size must be a positive multiple of 16; buffers must cover the table
    assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 24, one, one, one, 8, ctypes.byref(sh), None) == -2
    assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 16, one, one, one, 7, ctypes.byref(sh), None) == -3
    assert lib.coopt_paged_gqa_decode_partitioned(one, one, one, one, one, one, one, 16, None, one, one, 8, ctypes.byref(sh), None) == -1
    assert lib.coopt_gather_cached_kv(one, one, one, one, one, 5, 0, 4, one, one, ctypes.byref(sh), None) == -2
    assert lib.coopt_gather_cached_kv(one, one, one, one, one, 0, 0, 999, one, one, ctypes.byref(sh), None) == -2
    # the streaming-read probe: launch shape and alignment are checked before anything else
    assert lib.coopt_stream_read_probe(one, ctypes.c_size_t(1 << 20), 0, one, None) == -2
    assert lib.coopt_stream_read_probe(one, ctypes.c_size_t(1 << 20), (1 << 20) + 1, one, None) == -2
    assert lib.coopt_stream_read_probe(ctypes.c_void_p(24), ctypes.c_size_t(1 << 20), 64, one, None) == -2
    assert lib.coopt_stream_read_probe(None, ctypes.c_size_t(1 << 20), 64, one, None) == -1
    assert lib.coopt_stream_read_probe(one, ctypes.c_size_t(1 << 20), 64, None, None) == -1
    assert lib.coopt_stream_read_probe(None, ctypes.c_size_t(0), 64, None, None) == 0
    good = dict(coopt.get_decode_plan())
    for bad in (dict(tokens_per_group=100), dict(tokens_per_group=0), dict(waves_per_group=3),
                dict(pipeline_depth=4), dict(pipeline_depth=0), dict(grid_waves=0),
                dict(grid_waves=-5), dict(softmax_reduction=2)):
        with pytest.raises(coopt.CooptError):
            coopt.set_decode_plan(**bad)
        assert coopt.get_decode_plan() == good        # a refused plan changes nothing
    coopt.set_decode_plan(**good)
    assert lib.coopt_set_decode_plan(None) == -1


def test_empty_batches_are_accepted_without_launch(lib):
    """num_seqs = 0 / num_tokens = 0 / no query rows: COOPT_OK before any pointer is looked at."""
    sh = _shape(num_seqs=0)
    z = ctypes.c_size_t(0)
    assert lib.coopt_paged_gqa_decode(None, None, None, None, None, None, None, None, None, z, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_decode_step(None, None, None, None, None, None, None, None, None, None, None, None, z, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_decode_split(None, None, None, None, None, None, None, None, z, ctypes.byref(sh), None) == 0
    assert lib.coopt_decode_schedule_prepare(None, None, None, None, z, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_decode_scheduled(None, None, None, None, None, None, None, None, None, None, None, z, None, z, ctypes.byref(sh), None) == 0
    assert lib.coopt_paged_gqa_prefill_chunk(None, None, None, None, None, None, None, None, 0, 0, None, ctypes.byref(sh), None) == 0
    sh1 = _shape()
    assert lib.coopt_kv_cache_write_fp8(None, None, None, 0, None, None, None, None, ctypes.byref(sh1), None) == 0
    assert lib.coopt_kv_cache_write_skipset(None, None, None, None, 0, None, None, None, None, ctypes.byref(sh1), None) == 0
    assert lib.coopt_paged_gqa_prefill_chunk(None, None, None, None, None, None, None, None, 0, 0, None, ctypes.byref(sh1), None) == 0
