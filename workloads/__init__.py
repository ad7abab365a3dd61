"""Seeded synthetic inputs for paged decode attention.

This module is shared by the tests, the benchmark, the oracle side and the HIP side.  It holds
NONE of the method's arithmetic: no quantisation, no softmax, no cache layout.  It only draws
random fp16 tensors, context lengths and a paging structure (block tables and the slot of each
token).  Filling a cache from these tokens is done by whichever write path is under test.

The five named workloads have the shapes and value distributions of the decode workloads the
method is evaluated on (LLaMa-13B attention shape: 40 query heads of 128 dims; grouped variant
with 8 KV heads).  They stand in for serving traces: lengths are uniform in a range, the pool is
one seeded permutation of the physical blocks dealt to the sequences in order.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

BASE_SEED = 9323


@dataclasses.dataclass
class Workload:
    name: str
    S: int                    # sequences
    H_q: int                  # query heads
    H_k: int                  # KV heads
    d: int                    # head dim
    B: int                    # tokens per block
    NB: int                   # physical blocks in the pool
    kv_dtype: str             # "e4m3" or "fp16"
    softmax_scale: float
    context_lens: np.ndarray  # [S] int32, tokens visible to the step (new tokens included)
    block_tables: np.ndarray  # [S, max_blocks] int32, -1 = unused
    seq_start: np.ndarray     # [S+1] int64 offsets of each sequence in k_ctx / v_ctx / slots
    k_ctx: np.ndarray         # [sum(context_lens), H_k, d] fp16, every token of every sequence
    v_ctx: np.ndarray         # same
    slots: np.ndarray         # [sum(context_lens)] int64, physical slot of every token
    q: np.ndarray             # decode: [S, H_q, d] fp16; prefill: [sum(new), H_q, d]
    new_per_seq: int          # tokens written by the timed step per sequence (1 = decode)
    partition_size: Optional[int] = None
    query_start: Optional[np.ndarray] = None   # [S+1] int32 row offsets of each sequence in q

    @property
    def max_blocks(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def total_tokens(self) -> int:
        return int(self.seq_start[-1])

    def history_index(self) -> np.ndarray:
        """Indices (into k_ctx) of tokens that are in the cache before the timed step."""
        idx = [np.arange(self.seq_start[s], self.seq_start[s + 1] - self.new_per_seq)
               for s in range(self.S)]
        return np.concatenate(idx) if idx else np.zeros(0, dtype=np.int64)

    def new_index(self) -> np.ndarray:
        """Indices (into k_ctx) of the tokens the timed step writes, sequence-major."""
        idx = [np.arange(self.seq_start[s + 1] - self.new_per_seq, self.seq_start[s + 1])
               for s in range(self.S)]
        return np.concatenate(idx) if idx else np.zeros(0, dtype=np.int64)


def _normal_fp16(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32).astype(np.float16)


def make_paging(rng: np.random.Generator, context_lens: np.ndarray, B: int, NB: int,
                max_blocks: Optional[int] = None):
    """One permutation of the pool dealt to the sequences in order, ceil(t/B) blocks each."""
    S = len(context_lens)
    need = [(int(t) + B - 1) // B for t in context_lens]
    if sum(need) > NB:
        raise ValueError("pool too small")
    if max_blocks is None:
        max_blocks = max(need + [1])
    perm = rng.permutation(NB).astype(np.int32)
    block_tables = np.full((S, max_blocks), -1, dtype=np.int32)
    slots = []
    pos = 0
    for s in range(S):
        blocks = perm[pos:pos + need[s]]
        pos += need[s]
        block_tables[s, :need[s]] = blocks
        j = np.arange(int(context_lens[s]), dtype=np.int64)
        slots.append(blocks[j // B].astype(np.int64) * B + (j % B))
    seq_start = np.zeros(S + 1, dtype=np.int64)
    seq_start[1:] = np.cumsum(context_lens)
    slots = np.concatenate(slots) if slots else np.zeros(0, dtype=np.int64)
    return block_tables, slots, seq_start


def make_custom(name: str, *, seed: int, S: int, H_q: int, H_k: int, d: int, B: int, NB: int,
                context_lens, kv_dtype: str = "e4m3", new_per_seq: int = 1,
                k_outlier_frac: float = 0.0, k_outlier_gain: float = 20.0,
                partition_size: Optional[int] = None, max_blocks: Optional[int] = None) -> Workload:
    rng = np.random.default_rng(seed)
    context_lens = np.asarray(context_lens, dtype=np.int32)
    assert context_lens.shape == (S,)
    block_tables, slots, seq_start = make_paging(rng, context_lens, B, NB, max_blocks)
    total = int(seq_start[-1])
    k_ctx = _normal_fp16(rng, (total, H_k, d))
    v_ctx = _normal_fp16(rng, (total, H_k, d))
    if k_outlier_frac > 0.0:
        hit = rng.random(total) < k_outlier_frac          # per (sequence, token), all KV heads
        k32 = k_ctx.astype(np.float32)
        k32[hit] *= np.float32(k_outlier_gain)
        k_ctx = k32.astype(np.float16)
    n_q = S * new_per_seq
    q = _normal_fp16(rng, (n_q, H_q, d))
    query_start = (np.arange(S + 1, dtype=np.int32) * new_per_seq).astype(np.int32)
    return Workload(name=name, S=S, H_q=H_q, H_k=H_k, d=d, B=B, NB=NB, kv_dtype=kv_dtype,
                    softmax_scale=float(np.float32(1.0 / math.sqrt(d))),
                    context_lens=context_lens, block_tables=block_tables, seq_start=seq_start,
                    k_ctx=k_ctx, v_ctx=v_ctx, slots=slots, q=q, new_per_seq=new_per_seq,
                    partition_size=partition_size, query_start=query_start)


NAMES = ["tiny_paged_decode", "llama13b_gqa_fp8_decode", "llama13b_mha_fp16_decode",
         "long_context_partitioned_decode", "chunked_prefill"]


def make(index: int, *, seed: Optional[int] = None, shrink: int = 1) -> Workload:
    """Workload ``index`` (0..4).  ``shrink`` > 1 divides sequence counts / lengths for quick runs
    (the shapes per head stay the same); shrink == 1 is the full named configuration."""
    seed = BASE_SEED + index if seed is None else seed
    lens_rng = np.random.default_rng(seed + 1000)
    if index == 0:
        return make_custom(NAMES[0], seed=seed, S=1, H_q=4, H_k=2, d=64, B=16, NB=64,
                           context_lens=[256])
    if index in (1, 2):
        S = max(1, 32 // shrink)
        lens = lens_rng.integers(512 // shrink, 2048 // shrink + 1, size=S)
        H_k = 8 if index == 1 else 40
        return make_custom(NAMES[index], seed=seed, S=S, H_q=40, H_k=H_k, d=128, B=16,
                           NB=8192 // shrink, context_lens=lens,
                           kv_dtype="e4m3" if index == 1 else "fp16",
                           max_blocks=2048 // shrink // 16)
    if index == 3:
        S = max(1, 4 // min(shrink, 4))
        lens = lens_rng.integers(16384 // shrink, 32768 // shrink + 1, size=S)
        return make_custom(NAMES[3], seed=seed, S=S, H_q=40, H_k=8, d=128, B=16,
                           NB=16384 // shrink, context_lens=lens, k_outlier_frac=0.01,
                           partition_size=512, max_blocks=32768 // shrink // 16)
    if index == 4:
        S = max(1, 8 // shrink)
        ctx, C = 8192 // shrink, 512 // shrink
        return make_custom(NAMES[4], seed=seed, S=S, H_q=40, H_k=8, d=128, B=16,
                           NB=8192 // shrink, context_lens=[ctx + C] * S, new_per_seq=C,
                           max_blocks=(ctx + C + 15) // 16)
    raise IndexError(index)
