// Chunked prefill over the paged cache for gfx950: causal attention of a chunk of new query rows
// against history + chunk, both already in the cache (each row is Background Eq. 1 over its
// visible prefix, with the grouping of Opt-GQA Eq. 7 and the valid-block rule of Opt-Pa Eq. 9).
//
// Query length > 1 makes this a dense contraction, so the matrix cores are used at full width:
// a score tile has 16 query rows of ONE query head as its columns (column n = chunk row i0+n), and
// a wavefront carries NR such tiles against every K/V tile it loads, so each cache byte fetched
// and converted once feeds 16*NR query rows.  The per-block arithmetic is in attn_tile.hpp; the
// only difference from decode is that the visible-token limit is per column (causal).
#include "attn_tile.hpp"

namespace coopt {

struct PrefillArgs {
    const half_t* q;
    CacheView cv;
    const int32_t* block_tables;
    const int32_t* context_lens;
    const int32_t* query_start;
    half_t* out;
    int32_t H_q, H_k, G;
    int32_t max_blocks;
    int32_t pool_tiles;
    float scale_log2e;
};

constexpr int kPrefillWaves = 4;

template <int HEAD_DIM, int KV, int NR, int DEPTH, bool BIG>
__global__ void __launch_bounds__(64 * kPrefillWaves)
prefill_chunk_kernel(const PrefillArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform((int)(threadIdx.x >> 6));
    const int n = lane & 15, grp = lane >> 4;
    const int seq = blockIdx.y / a.H_k;
    const int g = blockIdx.y - seq * a.H_k;

    const int qs = a.query_start[seq];
    const int C = a.query_start[seq + 1] - qs;
    const int t = a.context_lens[seq];
    const int t_ctx = t - C;
    if (C <= 0) return;
    const int tiles_per_head = (C + 15) / 16;
    const int total_tiles = a.G * tiles_per_head;
    const int first_tile = (blockIdx.x * kPrefillWaves + wave) * NR;
    if (first_tile >= total_tiles) return;          // no barrier below: a wave may leave alone

    half8_t qop[NR][HEAD_DIM / 32];
    int limit[NR];          // tokens visible to column n of tile r
    int row0[NR], head[NR];
    int max_limit = 0, min_row = 0x7fffffff;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int tile = min(first_tile + r, total_tiles - 1);   // surplus tiles repeat the last
        const int hh = tile / tiles_per_head;
        const int i0 = (tile - hh * tiles_per_head) * 16;
        const int row = min(i0 + n, C - 1);                      // surplus rows repeat row C-1
        head[r] = g * a.G + hh;
        row0[r] = i0;
        limit[r] = t_ctx + row + 1;
        max_limit = max(max_limit, t_ctx + min(i0 + 15, C - 1) + 1);
        min_row = min(min_row, i0);
        load_q_operand<HEAD_DIM, KV>(qop[r], a.q + ((size_t)(qs + row) * a.H_q + head[r]) * HEAD_DIM,
                                     true, grp);
    }
    const int nblk = (max_limit + kBlock - 1) / kBlock;
    const int32_t* bt = a.block_tables + (size_t)seq * a.max_blocks;

    float m[NR], l[NR];
    floatx4 acc[NR][HEAD_DIM / 16];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        m[r] = -INFINITY;
        l[r] = 0.0f;
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c) acc[r][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const TileLoader<HEAD_DIM, KV, BIG> loader(a.cv, lane, a.pool_tiles);
    BlockRegs<HEAD_DIM, KV> regs[DEPTH][2];
    const int full_limit = min(t, t_ctx + min_row + 1);   // tokens visible to every column
    for (int cb = 0; cb < nblk; cb += 64) {          // 64 block numbers per vector load
        const int nc = min(64, nblk - cb);
        const int ng = (nc + 1) >> 1;
        int idv = 0;
        if (lane < nc) idv = bt[cb + lane];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int id = __builtin_amdgcn_readlane(idv, 2 * u + h);
                loader.issue(regs[u][h], id * a.H_k + g, 2 * u + h < nc);
            }
            __builtin_amdgcn_sched_barrier(0);     // keep the stages' loads in program order
        }
        for (int i = 0; i < ng; i += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int gi = i + u;
                if (gi < ng) {
                    const int baseA = (cb + 2 * gi) * kBlock;           // uniform
                    const int tokA = baseA + 4 * grp;
                    const bool hasB = 2 * gi + 1 < nc;
                    const int cacheA = t - tokA, cacheB = hasB ? cacheA - kBlock : 0;
                    const bool tail = !(hasB && baseA + 2 * kBlock <= full_limit);
#pragma unroll
                    for (int r = 0; r < NR; ++r) {
                        const int visA = limit[r] - tokA;
                        group_update<HEAD_DIM, KV>(regs[u][0], regs[u][1], qop[r], m[r], l[r], acc[r],
                                                   tail, visA, hasB ? visA - kBlock : 0, cacheA, cacheB,
                                                   a.scale_log2e);
                    }
                }
                // refill only after the stage's registers are dead, so the loads can land in place
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int nb = 2 * (gi + DEPTH) + h;
                    const int id = __builtin_amdgcn_readlane(idv, min(nb, 63));
                    loader.issue(regs[u][h], id * a.H_k + g, nb < nc);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

#pragma unroll
    for (int r = 0; r < NR; ++r) {
        float L = l[r];
        L += __shfl_xor(L, 16);
        L += __shfl_xor(L, 32);
        const float inv = 1.0f / L;                       // the common power of two of acc and l cancels
        const int row = row0[r] + n;
        if (first_tile + r < total_tiles && row < C) {
            half_t* dst = a.out + ((size_t)(qs + row) * a.H_q + head[r]) * HEAD_DIM + 4 * grp;
#pragma unroll
            for (int c = 0; c < HEAD_DIM / 16; ++c) {
                half4_t h;
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = (half_t)(acc[r][c][i] * inv);
                *reinterpret_cast<half4_t*>(dst + 16 * c) = h;
            }
        }
    }
}

}  // namespace coopt

using namespace coopt;

extern "C" int coopt_paged_gqa_prefill_chunk(const void* q, const void* k_cache, const void* v_cache,
                                             const float* k_scale, const float* v_scale,
                                             const int32_t* block_tables,
                                             const int32_t* context_lens,
                                             const int32_t* query_start, int32_t num_query_rows,
                                             int32_t max_chunk_len, void* out,
                                             const coopt_shape* sh, void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (num_query_rows < 0 || max_chunk_len < 0) return COOPT_ERR_SHAPE;
    if (sh->num_seqs == 0 || num_query_rows == 0 || max_chunk_len == 0) return COOPT_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !context_lens || !query_start || !out)
        return COOPT_ERR_NULL;
    if (sh->kv_dtype == COOPT_KV_E4M3 && (!k_scale || !v_scale)) return COOPT_ERR_NULL;
    if ((long long)sh->num_seqs * sh->num_kv_heads > 65535) return COOPT_ERR_SHAPE;

    PrefillArgs a{};
    a.q = (const half_t*)q;
    a.cv = CacheView{(const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale};
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.query_start = query_start;
    a.out = (half_t*)out;
    a.H_q = sh->num_q_heads;
    a.H_k = sh->num_kv_heads;
    a.G = sh->num_q_heads / sh->num_kv_heads;
    a.max_blocks = sh->max_blocks_per_seq;
    a.pool_tiles = sh->num_blocks * sh->num_kv_heads;
    a.scale_log2e = sh->softmax_scale * kLog2e;

    constexpr int NR = 2, DEPTH = 1;
    const int tiles = a.G * ((max_chunk_len + 15) / 16);
    const dim3 grid((unsigned)((tiles + kPrefillWaves * NR - 1) / (kPrefillWaves * NR)),
                    (unsigned)(sh->num_seqs * sh->num_kv_heads));
    const dim3 block(64 * kPrefillWaves);
    hipStream_t stream = (hipStream_t)hip_stream;
#define COOPT_PREFILL(D, KV, BIG) \
    hipLaunchKernelGGL((prefill_chunk_kernel<D, KV, NR, DEPTH, BIG>), grid, block, 0, stream, a)
    const bool big = !pool_fits_small(sh);
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) { if (big) COOPT_PREFILL(128, COOPT_KV_E4M3, true); else COOPT_PREFILL(128, COOPT_KV_E4M3, false); }
        else { if (big) COOPT_PREFILL(64, COOPT_KV_E4M3, true); else COOPT_PREFILL(64, COOPT_KV_E4M3, false); }
    } else {
        if (sh->head_dim == 128) { if (big) COOPT_PREFILL(128, COOPT_KV_FP16, true); else COOPT_PREFILL(128, COOPT_KV_FP16, false); }
        else { if (big) COOPT_PREFILL(64, COOPT_KV_FP16, true); else COOPT_PREFILL(64, COOPT_KV_FP16, false); }
    }
#undef COOPT_PREFILL
    return launch_status();
}
