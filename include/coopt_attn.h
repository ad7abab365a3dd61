/*
 * coopt_attn.h -- C ABI of the MI355X (gfx950) paged FP8 grouped-query decode-attention library.
 *
 * The library implements the data-parallel hot path that the three LLM-CoOpt strategies act on:
 * Opt-KV (skip-filtered, FP8-compressed KV-cache write and dequantising read), Opt-GQA (query
 * heads grouped onto shared KV heads) and Opt-Pa (attention over the valid blocks of a paged
 * cache only, with a numerically stable block-wise softmax), plus the partitioned form for long
 * contexts that the paper's conclusion names and a chunked-prefill form for query length > 1.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - Every pointer argument is a DEVICE pointer owned by the caller, except `const coopt_shape*`
 *    (host) and `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *  - Unless a comment says otherwise the library allocates nothing, frees nothing, copies nothing
 *    to the host and never synchronises: kernels are enqueued on `hip_stream` and the call returns.
 *  - Return value: COOPT_OK (0) or a negative coopt_status.  Arguments are validated before the
 *    first launch: on COOPT_ERR_NULL, _SHAPE or _WORKSPACE nothing was launched.  COOPT_ERR_LAUNCH
 *    means the HIP runtime refused a launch; for an entry point of two launches the first may
 *    then already be enqueued.
 *  - There is no process-wide state: every call takes what it depends on as arguments.
 *  - Indices: slots are int64, block numbers and lengths int32.  Floating point: q / new k,v /
 *    out are IEEE binary16; scales and partials are binary32.
 *
 * Tensor layouts (NB = physical blocks, H_k = KV heads, B = block_size = 16, d = head_dim)
 * ---------------------------------------------------------------------------------------
 * The cache is a pool of tiles; one tile holds the B tokens x d dims of one (physical block, KV
 * head), as u8 OCP-E4M3 (or E5M2) codes or as fp16, in the order the matrix-core operands consume them, so
 * that every wavefront load is 64 x 16 contiguous bytes.  With E = elements per 16 bytes (16 for
 * E4M3, 8 for fp16), tile index = block * H_k + head, and element indices within a tile:
 *   k_cache  [NB*H_k][d/E][B][E]            (tok, dim) -> ((dim/E)*B + tok)*E + dim%E
 *                                           (16-byte chunks of a token's row, chunk-major)
 *   v_cache  [NB*H_k][d/(4E)][B/4][16][E/4][4]   with c = dim/16, n = dim%16, W = E/4:
 *                                           (tok, dim) -> ((((c/W)*(B/4) + tok/4)*16 + n)*W + c%W)*4 + tok%4
 *                                           (token index innermost in runs of 4, then W dim groups)
 *   k_scale  [NB*H_k][B]   binary32, one-byte caches only: value = code * scale
 *   v_scale  [NB*H_k][B]
 *   block_tables [S][max_blocks_per_seq]   logical block -> physical block; only entries
 *                                          b < ceil(context_len/B) are ever used (Opt-Pa, Eq. 9)
 *   slot = physical_block * B + offset_in_block
 *
 * Device-side preconditions that are NOT checked: non-negative slots are < NB*B and unique within
 * one write call; block table entries that are read lie in [0, NB); 0 <= context_lens[s] <=
 * max_blocks_per_seq*B; inputs are finite.  Cache bytes of tokens >= context_len, and of blocks
 * past the last valid one, may hold anything (NaN codes included): they never reach the result.
 */
#ifndef COOPT_ATTN_H
#define COOPT_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum coopt_status {
    COOPT_OK = 0,
    COOPT_ERR_NULL = -1,        /* a required pointer is NULL */
    COOPT_ERR_SHAPE = -2,       /* unsupported or inconsistent shape / argument value */
    COOPT_ERR_WORKSPACE = -3,   /* workspace or partial buffers too small */
    COOPT_ERR_LAUNCH = -4       /* the HIP runtime refused the launch */
} coopt_status;

/* Cache element type.  E4M3 is the method as this library reads it (Opt-KV says "FP8"); E5M2 and
 * the scale modes below are the alternatives that choice stands against, built so that they can be
 * measured on the same kernels. */
enum { COOPT_KV_FP16 = 0, COOPT_KV_E4M3 = 1, COOPT_KV_E5M2 = 2 };

/* How a written row gets its scale (coopt_kv_cache_write_fp8_scaled). */
enum { COOPT_SCALE_TOKEN = 0, COOPT_SCALE_BLOCK = 1, COOPT_SCALE_STATIC = 2 };

/*
 * Problem shape.  Supported: head_dim 64 or 128; block_size 16; num_q_heads a multiple of
 * num_kv_heads (Opt-GQA, Eq. 7 needs an integer group size H_g = H_q/H_k) with H_g <= 16.
 * Sizes are 32-bit inside the kernels' index arithmetic: num_seqs <= 2^20, num_q_heads <= 2^12,
 * num_seqs * num_q_heads <= 2^27, max_blocks_per_seq <= 2^24 (268 M tokens a sequence),
 * num_blocks * num_kv_heads < 2^31 (and, for the partitioned call, num_seqs * num_kv_heads *
 * max_parts < 2^31);
 * anything beyond is COOPT_ERR_SHAPE.
 */
typedef struct coopt_shape {
    int32_t num_seqs;            /* S */
    int32_t num_q_heads;         /* H_q */
    int32_t num_kv_heads;        /* H_k */
    int32_t head_dim;            /* d */
    int32_t block_size;          /* B */
    int32_t num_blocks;          /* NB */
    int32_t max_blocks_per_seq;  /* row stride of block_tables */
    int32_t kv_dtype;            /* COOPT_KV_FP16, COOPT_KV_E4M3 or COOPT_KV_E5M2 */
    float softmax_scale;         /* multiplies q.k before the softmax; 1/sqrt(d) in Eq. 1 */
} coopt_shape;

/*
 * Launch plan of the decode entry points (tuning knobs).  Every entry point that depends on it
 * takes a `const coopt_decode_plan* plan` (host memory, read during the call only); NULL means the
 * default plan for the current device, which coopt_default_decode_plan writes out.  Calls that
 * share a workspace or a schedule (split and merge; prepare and the scheduled decode; the size
 * queries and the calls they size for) must be given the same plan: a schedule carries a tag of
 * the plan it was prepared for and a workspace one of the plan its partial results were laid out
 * for, and a launch that finds another tag writes nothing (see the entry points).
 *
 * coopt_paged_gqa_decode with a workspace flattens the batch's work and cuts it into shares that
 * differ by at most one two-block group, one share per single-wavefront workgroup: at most
 * `grid_waves` wavefronts in the whole grid (default: one per SIMD of the device, 4 x its
 * compute-unit count = 1024 on MI355X), a share never smaller than `tokens_per_group` tokens (a
 * positive multiple of 32; default 128) unless the whole batch is.
 * coopt_paged_gqa_decode_partitioned runs `waves_per_group` (1, 2, 4 or 8; default 1) wavefronts
 * per partition; the balanced kernel ignores that field.  In both, every wavefront keeps
 * `pipeline_depth` (1, 2 or 3; default 2) two-block groups of the cache in flight.
 * `softmax_reduction` selects how the balanced kernel keeps the softmax statistics: 0 (default) =
 * a running reference max per lane that is raised only when a score exceeds it by a margin, sums
 * reduced once at the end; 1 = the mechanism Opt-Pa states (Alg. 3, Eq. 10): max and sum of every
 * group of blocks reduced through shared memory and the accumulator rescaled each time -- kept to
 * compare the two on this hardware (pipeline_depth is then 2).
 * A plan with a field out of range makes the call return COOPT_ERR_SHAPE (size queries: 0).
 */
typedef struct coopt_decode_plan {
    int32_t tokens_per_group;
    int32_t waves_per_group;
    int32_t pipeline_depth;
    int32_t grid_waves;
    int32_t softmax_reduction;
} coopt_decode_plan;

/* Writes the default plan for the current HIP device into *plan (host memory). */
void coopt_default_decode_plan(coopt_decode_plan* plan);

/*
 * Quantise-on-write of new tokens into the paged cache (Opt-KV: Eq. 5 and Alg. 1 phase 1).
 * For token i: slot_mapping[i] < 0 means "skip, write nothing" (the filter of Eq. 5; any other
 * skip set is expressed by the caller passing a negative slot).  Otherwise, for every KV head and
 * for K and V separately: amax = max|x| over the d elements, scale = amax/448 in binary32
 * (1.0 if amax == 0), code = E4M3(round-to-nearest-even(x/scale)), saturated at +-448, sign kept.
 *   k, v           [num_tokens][H_k][d] fp16, contiguous            (read)
 *   slot_mapping   [num_tokens] int64                               (read)
 *   k_cache, v_cache, k_scale, v_scale                              (written at the named slots only)
 * shape->kv_dtype must be COOPT_KV_E4M3, or COOPT_KV_E5M2 (OCP E5M2: 1-5-2, bias 15, max finite
 * 57344; the same rule with 57344 in place of 448).  num_tokens == 0 is a no-op.
 */
int coopt_kv_cache_write_fp8(const void* k, const void* v, const int64_t* slot_mapping,
                             int32_t num_tokens, uint8_t* k_cache, uint8_t* v_cache,
                             float* k_scale, float* v_scale, const coopt_shape* shape,
                             void* hip_stream);

/*
 * The same write with another scale rule: what Opt-KV's FP8 compression looks like under the
 * scale granularities the paper leaves open (it says only "FP8"), kept to measure the dynamic
 * per-token scale against them on the same cache layout and the same read kernels -- the scale
 * arrays keep one entry per (token, KV head) in every mode, so all read entry points serve all
 * modes unchanged.
 *   scale_mode  COOPT_SCALE_TOKEN   as coopt_kv_cache_write_fp8
 *               COOPT_SCALE_BLOCK   one scale for all rows of THIS CALL that land in the same
 *                                   cache block and KV head: (largest absmax among them) / max
 *                                   code; rows written to the block by other calls keep theirs
 *               COOPT_SCALE_STATIC  k_static[head] / v_static[head] (device, float [H_k], > 0),
 *                                   fixed by the caller in advance; values beyond scale * max
 *                                   code saturate
 *   k_static, v_static  NULL unless COOPT_SCALE_STATIC
 * kv_dtype COOPT_KV_E4M3 or COOPT_KV_E5M2.  COOPT_ERR_SHAPE for another scale_mode.
 */
int coopt_kv_cache_write_fp8_scaled(const void* k, const void* v, const int64_t* slot_mapping,
                                    int32_t num_tokens, uint8_t* k_cache, uint8_t* v_cache,
                                    float* k_scale, float* v_scale, int32_t scale_mode,
                                    const float* k_static, const float* v_static,
                                    const coopt_shape* shape, void* hip_stream);

/*
 * The same scatter without compression: fp16 bit patterns are stored unchanged (the unquantised
 * cache the paper's Background describes, kept as the comparison case).  kv_dtype must be
 * COOPT_KV_FP16; k_cache / v_cache hold fp16 in the layouts above.
 */
int coopt_kv_cache_write_fp16(const void* k, const void* v, const int64_t* slot_mapping,
                              int32_t num_tokens, void* k_cache, void* v_cache,
                              const coopt_shape* shape, void* hip_stream);

/*
 * The same write with the SkipSet of Opt-KV Eq. 5 spelled out: token index i of this call is left
 * out if bit i%32 of skip_set[i/32] is set (device, uint32 [ceil(num_tokens/32)]; NULL = empty
 * set) or its slot is negative.  Dispatches on shape->kv_dtype: E4M3 as coopt_kv_cache_write_fp8,
 * fp16 as coopt_kv_cache_write_fp16 (k_scale and v_scale are then ignored and may be NULL).
 */
int coopt_kv_cache_write_skipset(const void* k, const void* v, const int64_t* slot_mapping,
                                 const uint32_t* skip_set, int32_t num_tokens, void* k_cache,
                                 void* v_cache, float* k_scale, float* v_scale,
                                 const coopt_shape* shape, void* hip_stream);

/*
 * Single-step grouped-query decode attention over the paged cache
 * (Background Eq. 1; Opt-KV Eq. 6 and Alg. 1 phase 2; Opt-GQA Eq. 7-8 and Alg. 2; Opt-Pa Eq. 9-10
 * and Alg. 3).  For sequence s and query head h, with KV head g = floor(h / (H_q/H_k)):
 *   out[s][h] = softmax_j( softmax_scale * q[s][h] . k~[j][g] ) . v~[j][g],  j < context_lens[s],
 * where k~, v~ are the dequantised cache rows reached through block_tables.  All H_g query heads
 * of a group are served by one read of each K/V tile.
 *   q [S][H_q][d] fp16 (read); out [S][H_q][d] fp16 (written; zeros where context_lens[s] == 0)
 *   k_scale, v_scale: NULL iff kv_dtype == COOPT_KV_FP16
 *   context_lens [S] int32: tokens visible, the token written this step included
 *   workspace: scratch for the load-balanced split of the batch's work over the whole chip (two
 *     kernels: split attention into partial results, then their merge).  NULL (then
 *     workspace_bytes is ignored) runs one workgroup per (sequence, KV head) over the whole context
 *     instead, which is only adequate for small batches of short contexts.  Otherwise it must hold
 *     at least coopt_decode_workspace_bytes(shape, plan) bytes and be 16-byte aligned; its contents are
 *     undefined afterwards.  Two calls that share a workspace must be ordered on one stream.
 */
int coopt_paged_gqa_decode(const void* q, const void* k_cache, const void* v_cache,
                           const float* k_scale, const float* v_scale,
                           const int32_t* block_tables, const int32_t* context_lens, void* out,
                           void* workspace, size_t workspace_bytes, const coopt_decode_plan* plan,
                           const coopt_shape* shape, void* hip_stream);

/*
 * coopt_paged_gqa_decode for callers that can neither allocate device memory nor hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and result as coopt_paged_gqa_decode with a workspace (the same two kernels),
 * but the partial results go to a device array built into the library,
 * coopt_decode_builtin_workspace_bytes() = 32 MiB per GPU, held from the library's first use on
 * that GPU until the process ends.  The call allocates and frees nothing (the first call on a
 * device asks the runtime for the array's address, once).
 *   COOPT_ERR_WORKSPACE  coopt_decode_workspace_bytes(shape, plan) exceeds the built-in array
 *                        (e.g. 4 sequences of 32 k tokens with 40 query heads under the default
 *                        plan need 21 MB and fit; 16 such sequences do not): nothing is launched
 * All calls on one GPU share that GPU's array, which keeps the last call's contents; nothing in it
 * has to be cleared between calls.  Calls on one GPU must be ordered (one stream, or events):
 * two that overlap race on the array and both results are undefined.
 */
int coopt_paged_gqa_decode_noalloc(const void* q, const void* k_cache, const void* v_cache,
                                   const float* k_scale, const float* v_scale,
                                   const int32_t* block_tables, const int32_t* context_lens,
                                   void* out, const coopt_decode_plan* plan,
                                   const coopt_shape* shape, void* hip_stream);
size_t coopt_decode_builtin_workspace_bytes(void);

/*
 * The two kernels of coopt_paged_gqa_decode as separate calls, for callers that time or schedule
 * them apart: `split` runs attention over equal shares of the batch's work and leaves one partial
 * (reference max, exponential sum, normalised output) per share segment in the workspace; `merge`
 * combines the partials of each (sequence, query head) into the fp16 output row.  Arguments as in
 * coopt_paged_gqa_decode; the workspace is required, and shape, context_lens and the decode plan
 * must be the same for both calls.  `split` leaves a tag of shape and plan in the workspace's
 * first 16 bytes; a `merge` that expects another tag (its plan or shape differs) writes nothing
 * and `out` keeps its old contents.
 */
int coopt_paged_gqa_decode_split(const void* q, const void* k_cache, const void* v_cache,
                                 const float* k_scale, const float* v_scale,
                                 const int32_t* block_tables, const int32_t* context_lens,
                                 void* workspace, size_t workspace_bytes,
                                 const coopt_decode_plan* plan, const coopt_shape* shape,
                                 void* hip_stream);
int coopt_paged_gqa_decode_merge(const int32_t* context_lens, const void* workspace,
                                 size_t workspace_bytes, void* out, const coopt_decode_plan* plan,
                                 const coopt_shape* shape, void* hip_stream);

/*
 * One decode step in two launches instead of three: Opt-KV's write of each sequence's new token
 * (Eq. 5, Alg. 1 phase 1) fused with the attention of Opt-GQA / Opt-Pa (Eq. 6-10).  The result is
 * that of coopt_kv_cache_write_fp8 / _fp16 with num_tokens = num_seqs followed by
 * coopt_paged_gqa_decode with a workspace: the same bytes end up in the cache, and `out` agrees
 * within the attention tolerance.  In the first launch the wavefront that reads the last cache
 * blocks of a (sequence, KV head) pair quantises the pair's new row and attends over it from
 * registers, in place of whatever the cache holds at that position; that launch has no other
 * wavefronts than the plain decode's, reads the cache only, and nothing in it waits for anything
 * else.  The rows are stored into the cache by extra wavefronts of the second (merge) launch.
 *   k, v          device, fp16 [num_seqs][num_kv_heads][head_dim]: token s is the LAST token of
 *                 sequence s, i.e. position context_lens[s]-1
 *   slot_mapping  device, int64 [num_seqs]: negative = write nothing for this sequence and attend
 *                 to whatever the cache holds at that position, as the two separate calls would.
 *                 Otherwise the row is written where block_tables places position
 *                 context_lens[s]-1; the slot must name that same place (not checked; only its
 *                 sign is used)
 *   k_cache .. v_scale   as in coopt_paged_gqa_decode, but written to (scales NULL iff fp16 cache)
 *   context_lens  INCLUDES the new token; 0 = empty sequence (nothing written, zero output rows)
 *   workspace     required here; coopt_decode_workspace_bytes(shape, plan) bytes, 16-byte aligned
 * Errors as for the two separate calls.
 */
int coopt_paged_gqa_decode_step(const void* k, const void* v, const int64_t* slot_mapping,
                                const void* q, void* k_cache, void* v_cache, float* k_scale,
                                float* v_scale, const int32_t* block_tables,
                                const int32_t* context_lens, void* out, void* workspace,
                                size_t workspace_bytes, const coopt_decode_plan* plan,
                                const coopt_shape* shape, void* hip_stream);
/*
 * The same decode with its schedule prepared ahead.  Block tables, context lengths and the slots of
 * the new tokens are the same for every layer of a model during one decoding step, so the schedule
 * that coopt_paged_gqa_decode derives inside every launch (which workgroup reads which cache tiles
 * of Eq. 9, where each (sequence, KV head) pair's partial results go) can be derived once per step:
 * coopt_decode_schedule_prepare writes it to device memory, and coopt_paged_gqa_decode_scheduled
 * runs any number of layers from it.  A scheduled launch reaches its first cache load one memory
 * round trip after it starts, without the schedule arithmetic and the block-table read.
 *
 *   schedule      device, coopt_decode_schedule_bytes(shape, plan) bytes, 16-byte aligned, owned by the
 *                 caller; opaque.  Valid for the shape, the decode plan and the mode (plain decode
 *                 or fused step) it was prepared with, and for as long as block_tables,
 *                 context_lens and slot_mapping keep their contents.
 *   prepare:  slot_mapping NULL = schedule for plain decode (attention over context_lens tokens);
 *             non-NULL = schedule for the fused step (as coopt_paged_gqa_decode_step: sequences
 *             with a non-negative slot append their last token in the same launch).
 *   scheduled decode:  k, v, slot_mapping all NULL = plain decode, all non-NULL = fused step
 *             (COOPT_ERR_NULL if mixed); the other arguments as in coopt_paged_gqa_decode_step,
 *             without block_tables.  out NULL = the first launch only (a tuning and timing aid):
 *             the workspace then holds the partial results (the pairs' partial counts stay in
 *             the schedule), and in a fused step the new rows are NOT stored, because that is
 *             the second launch's work.
 * prepare only enqueues a kernel on hip_stream: the launches that use the schedule must be ordered
 * after it (same stream, or an event), and two launches that use one schedule may overlap.
 * A schedule prepared for another shape, plan or mode is recognised on the device by a tag: such a
 * launch writes nothing except word 1 of the schedule, which it sets to 1 (prepare
 * resets it to 0), and `out` keeps its old contents.  A schedule whose tables or lengths have
 * changed since it was prepared is NOT recognised: prepare again.  Host-side errors as for
 * coopt_paged_gqa_decode_step, COOPT_ERR_WORKSPACE also for a schedule buffer that is too small or
 * misaligned, COOPT_ERR_SHAPE (bytes: 0) where a share or a pair's partial count would not fit the
 * record fields (more than 65 535 partials per pair).
 */
size_t coopt_decode_schedule_bytes(const coopt_shape* shape, const coopt_decode_plan* plan);
int coopt_decode_schedule_prepare(const int32_t* block_tables, const int32_t* context_lens,
                                  const int64_t* slot_mapping, void* schedule, size_t schedule_bytes,
                                  const coopt_decode_plan* plan, const coopt_shape* shape,
                                  void* hip_stream);
int coopt_paged_gqa_decode_scheduled(const void* k, const void* v, const int64_t* slot_mapping,
                                     const void* q, void* k_cache, void* v_cache, float* k_scale,
                                     float* v_scale, const int32_t* context_lens, void* out,
                                     void* workspace, size_t workspace_bytes, const void* schedule,
                                     size_t schedule_bytes, const coopt_decode_plan* plan,
                                     const coopt_shape* shape, void* hip_stream);


/* Bytes of workspace coopt_paged_gqa_decode needs for `shape` under `plan` (0 if the shape or the
 * plan is unsupported).  tokens_per_group and grid_waves change it. */
size_t coopt_decode_workspace_bytes(const coopt_shape* shape, const coopt_decode_plan* plan);

/*
 * Partitioned decode for long contexts (the "partitioned parallel" reduction of the paper's
 * conclusion; each partition is Opt-Pa Alg. 3 on its own token range).  Partition p of sequence s
 * covers tokens [p*partition_size, min((p+1)*partition_size, context_lens[s])) and emits
 *   max_logits[s][h][p] = m_p = max_j z_j            (natural-log units, z = softmax_scale*q.k~)
 *   exp_sums  [s][h][p] = l_p = sum_j exp(z_j - m_p)
 *   tmp_out   [s][h][p][:] = o_p = sum_j exp(z_j - m_p) v~_j / l_p
 * Any running maximum is a legal m_p: only (l_p*exp(m_p), o_p) is determined, so callers must
 * merge with coopt_paged_gqa_reduce or the same formula.  Partitions at or beyond
 * ceil(context_lens[s]/partition_size) are not written.
 *   partition_size: positive multiple of block_size
 *   tmp_out [S][H_q][max_parts][d] f32, max_logits / exp_sums [S][H_q][max_parts] f32 (written)
 *   max_parts >= ceil(max_blocks_per_seq*B / partition_size), else COOPT_ERR_WORKSPACE
 */
int coopt_paged_gqa_decode_partitioned(const void* q, const void* k_cache, const void* v_cache,
                                       const float* k_scale, const float* v_scale,
                                       const int32_t* block_tables, const int32_t* context_lens,
                                       int32_t partition_size, float* tmp_out, float* max_logits,
                                       float* exp_sums, int32_t max_parts,
                                       const coopt_decode_plan* plan, const coopt_shape* shape,
                                       void* hip_stream);

/*
 * Cross-partition merge: M = max_p m_p, w_p = l_p*exp(m_p - M),
 *   out[s][h] = sum_p w_p o_p / sum_p w_p   over p < ceil(context_lens[s]/partition_size),
 * written as fp16 [S][H_q][d]; zeros where context_lens[s] == 0.  Uses num_seqs, num_q_heads and
 * head_dim of `shape` only.
 */
int coopt_paged_gqa_reduce(const float* tmp_out, const float* max_logits, const float* exp_sums,
                           const int32_t* context_lens, int32_t partition_size, int32_t max_parts,
                           void* out, const coopt_shape* shape, void* hip_stream);

/*
 * Chunked prefill: causal attention of new query rows over a paged cache that already holds the
 * chunk's own K/V (write them first with coopt_kv_cache_write_*).  The paper's abstract describes
 * cutting long sequences into chunks; each row is Eq. 1 over its visible prefix.  Sequence s owns
 * rows query_start[s] .. query_start[s+1]-1 of q and out; with C_s rows and t_s = context_lens[s]
 * (chunk included), local row i attends to tokens j < t_s - C_s + i + 1.
 *   q, out [query_start[S]][H_q][d] fp16;  query_start [S+1] int32 (device), increasing from 0
 *   num_query_rows: query_start[S] as known to the host (sizes the launch); C_s <= t_s
 */
int coopt_paged_gqa_prefill_chunk(const void* q, const void* k_cache, const void* v_cache,
                                  const float* k_scale, const float* v_scale,
                                  const int32_t* block_tables, const int32_t* context_lens,
                                  const int32_t* query_start, int32_t num_query_rows,
                                  int32_t max_chunk_len, void* out, const coopt_shape* shape,
                                  void* hip_stream);

/*
 * The same chunked prefill (Abstract: chunking of long sequences; Eq. 1 per row) with a workspace
 * for the launch's last, partly filled round of workgroups (one workgroup = 256 query rows of one
 * (sequence, KV head) pair; a round = one workgroup per compute unit).  Where the tiles of a chunk
 * do not fill a whole number of rounds, coopt_paged_gqa_prefill_chunk runs the last tiles of
 * every pair in smaller workgroups, or leaves the round partly empty; with a workspace they run
 * in full-size workgroups, 2 to 8 per 256 rows, that each stream one of as many equal runs of the
 * pair's cache, leave (m, l, unnormalised sums) per 16 rows and run in the workspace, and a merge
 * launch combines the runs by the online-softmax rule (Opt-Pa Eq. 10).  A launch of fewer
 * workgroups than compute units is all "last round": this is the call for one or a few
 * sequences.  Results agree with coopt_paged_gqa_prefill_chunk within the rounding of that merge
 * (same tolerance against the definition); rows outside those tiles are the same bits.
 *   workspace        device memory, at least coopt_prefill_workspace_bytes(shape, max_chunk_len)
 *                    bytes (0 when the launch has no such round: then it may be NULL and the call
 *                    is coopt_paged_gqa_prefill_chunk); contents on entry are ignored, on return
 *                    they are scratch.  The caller owns it; calls that share it must not overlap.
 *   workspace_bytes  its size; COOPT_ERR_WORKSPACE if too small, COOPT_ERR_NULL if needed and NULL
 * Allocates nothing, synchronises nothing; three launches at most.
 */
size_t coopt_prefill_workspace_bytes(const coopt_shape* shape, int32_t max_chunk_len);
int coopt_paged_gqa_prefill_chunk_ws(const void* q, const void* k_cache, const void* v_cache,
                                     const float* k_scale, const float* v_scale,
                                     const int32_t* block_tables, const int32_t* context_lens,
                                     const int32_t* query_start, int32_t num_query_rows,
                                     int32_t max_chunk_len, void* out, void* workspace,
                                     size_t workspace_bytes, const coopt_shape* shape,
                                     void* hip_stream);

/*
 * Dequantising gather (the read half of Opt-KV, Eq. 6; the paper's gather_cached_kv): contiguous
 * fp16 K and V of logical tokens [tok_begin, tok_end) of sequence `seq`:
 *   k_out, v_out [tok_end - tok_begin][H_k][d] fp16, value = fp16(code * scale) (round to nearest
 *   even) for E4M3 caches, the stored pattern for fp16 caches.
 * The caller guarantees tok_end <= the sequence's context length.
 */
int coopt_gather_cached_kv(const void* k_cache, const void* v_cache, const float* k_scale,
                           const float* v_scale, const int32_t* block_tables, int32_t seq,
                           int32_t tok_begin, int32_t tok_end, void* k_out, void* v_out,
                           const coopt_shape* shape, void* hip_stream);

/* Static, human-readable text for a coopt_status value. */
const char* coopt_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* COOPT_ATTN_H */
