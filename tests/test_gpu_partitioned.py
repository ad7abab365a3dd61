"""GPU parity: partitioned decode + cross-partition reduce (the paper's "partitioned parallel"
reduction; each partition is Opt-Pa Alg. 3 on its token range) against the oracle."""
import numpy as np
import pytest
import torch

import paper_2602_09323_amd as coopt
import workloads
from gpu_utils import planned, assert_close, cache_to_dev, dev, shape_of
from helpers import oracle_fill

pytestmark = pytest.mark.gpu


def _hip_partitioned(w, dcache, P, max_parts, lens=None):
    shape = shape_of(w)
    dq, dbt = dev(w.q.view(np.uint16)), dev(w.block_tables)
    dlen = dev(w.context_lens if lens is None else lens)
    tmp = torch.full((w.S, w.H_q, max_parts, w.d), float("nan"), dtype=torch.float32, device="cuda")
    ml = torch.full((w.S, w.H_q, max_parts), float("nan"), dtype=torch.float32, device="cuda")
    es = torch.full((w.S, w.H_q, max_parts), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.full((w.S, w.H_q, w.d), -7.0, dtype=torch.float16, device="cuda")
    planned.paged_gqa_decode_partitioned(dq, *dcache, dbt, dlen, P, tmp, ml, es, max_parts, shape)
    coopt.paged_gqa_reduce(tmp, ml, es, dlen, P, max_parts, out, shape)
    torch.cuda.synchronize()
    return (out.cpu().numpy().astype(np.float64), tmp.cpu().numpy().astype(np.float64),
            ml.cpu().numpy().astype(np.float64), es.cpu().numpy().astype(np.float64))


@pytest.mark.parametrize("P", [16, 64, 512, 2048])
def test_partition_sizes_ragged(oracle_mod, P):
    lens = [300, 17, 512, 1, 1500]
    w = workloads.make_custom("part", seed=41, S=len(lens), H_q=10, H_k=2, d=128, B=16, NB=160,
                              context_lens=lens, k_outlier_frac=0.02, max_blocks=96)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q,
                                      H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    max_parts = (96 * 16 + P - 1) // P
    out, tmp, ml, es = _hip_partitioned(w, cache_to_dev(cache), P, max_parts)
    assert_close(out, ref, f"P={P}")
    # what is unique about the partials: o_p, and l_p*exp(m_p) (any running max is legal)
    otmp, oml, oes = oracle_mod.paged_gqa_decode_partitioned(
        w.q, *cache, w.block_tables, w.context_lens, P, max_parts, H_q=w.H_q, H_k=w.H_k, d=w.d,
        B=w.B, softmax_scale=w.softmax_scale)
    used = ~np.isnan(oml)
    assert np.isnan(ml[~used]).all() and not np.isnan(ml[used]).any()      # untouched beyond nparts
    assert_close(tmp[used], otmp[used], f"partials P={P}")
    lse_gpu = ml[used] + np.log(es[used])
    lse_ref = oml[used] + np.log(oes[used])
    assert np.max(np.abs(lse_gpu - lse_ref)) <= 2e-3


def test_long_context_config_reduced(oracle_mod):
    w = workloads.make(3, shrink=8)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q,
                                      H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    max_parts = (w.max_blocks * 16 + 511) // 512
    out, *_ = _hip_partitioned(w, cache_to_dev(cache), 512, max_parts)
    assert_close(out, ref, "cfg3/8")


def test_long_context_config_full_size(oracle_mod):
    w = workloads.make(3)
    print(f"full cfg3: tokens={w.total_tokens}", flush=True)
    cache = oracle_fill(oracle_mod, w)
    ref = oracle_mod.paged_gqa_decode(w.q, *cache, w.block_tables, w.context_lens, H_q=w.H_q,
                                      H_k=w.H_k, d=w.d, B=w.B, softmax_scale=w.softmax_scale)
    max_parts = (w.max_blocks * 16 + 511) // 512
    out, *_ = _hip_partitioned(w, cache_to_dev(cache), 512, max_parts)
    print("full cfg3 max-abs %.2e" % assert_close(out, ref, "cfg3"), flush=True)


def test_reduce_alone_matches_oracle(oracle_mod):
    rng = np.random.default_rng(42)
    S, H_q, max_parts, d, P = 3, 5, 9, 128, 64
    lens = np.array([0, 70, 576], np.int32)
    tmp = rng.standard_normal((S, H_q, max_parts, d))
    ml = rng.normal(0, 5, (S, H_q, max_parts)); es = rng.uniform(1, 60, (S, H_q, max_parts))
    ref = oracle_mod.paged_gqa_reduce(tmp, ml, es, lens, P)
    shape = coopt.Shape(S, H_q, H_q, d, 16, 64, 36, 1, 0.1)
    out = torch.full((S, H_q, d), -7.0, dtype=torch.float16, device="cuda")
    coopt.paged_gqa_reduce(dev(tmp.astype(np.float32)), dev(ml.astype(np.float32)),
                           dev(es.astype(np.float32)), dev(lens), P, max_parts, out, shape)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(got[0] == 0)
    assert_close(got, ref, "reduce")
