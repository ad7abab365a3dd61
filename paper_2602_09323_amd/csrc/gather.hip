// Dequantising gather (the read half of Opt-KV: Eq. 6, Alg. 1 phase 2): paged cache rows of one
// sequence -> contiguous fp16 K and V.  One wavefront per (token, KV head) row, d/64 elements per
// lane; pure data movement, bandwidth-bound, no reuse.
#include "common.hpp"

namespace coopt {

template <int HEAD_DIM, int KV>
__global__ void __launch_bounds__(256)
gather_cached_kv_kernel(const uint8_t* __restrict__ k_cache, const uint8_t* __restrict__ v_cache,
                        const float* __restrict__ k_scale, const float* __restrict__ v_scale,
                        const int32_t* __restrict__ bt_row, int tok_begin, int num_rows, int H_k,
                        half_t* __restrict__ k_out, half_t* __restrict__ v_out)
{
    constexpr int E = HEAD_DIM / 64;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);        // local token * H_k + head
    if (row >= num_rows) return;
    const int lane = threadIdx.x & 63;
    const int jt = row / H_k, head = row - jt * H_k;
    const int j = tok_begin + jt;
    const size_t tile = (size_t)bt_row[j / kBlock] * H_k + head;
    const int off = j % kBlock;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int dim = lane * E + e;
        constexpr int ES = (KV == COOPT_KV_E4M3) ? 1 : 2;
        const size_t ki = tile * (kBlock * HEAD_DIM) + k_tile_index<ES>(off, dim);
        const size_t vi = tile * (kBlock * HEAD_DIM) + v_tile_index<ES>(off, dim);
        half_t kv, vv;
        if constexpr (KV == COOPT_KV_E4M3) {
            const float ks = k_scale[tile * kBlock + off], vs = v_scale[tile * kBlock + off];
            kv = (half_t)((float)e4m3x2_to_half2<false>(k_cache[ki]).x * ks);
            vv = (half_t)((float)e4m3x2_to_half2<false>(v_cache[vi]).x * vs);
        } else {
            kv = reinterpret_cast<const half_t*>(k_cache)[ki];
            vv = reinterpret_cast<const half_t*>(v_cache)[vi];
        }
        k_out[(size_t)row * HEAD_DIM + dim] = kv;
        v_out[(size_t)row * HEAD_DIM + dim] = vv;
    }
}

}  // namespace coopt

using namespace coopt;

extern "C" int coopt_gather_cached_kv(const void* k_cache, const void* v_cache, const float* k_scale,
                                      const float* v_scale, const int32_t* block_tables, int32_t seq,
                                      int32_t tok_begin, int32_t tok_end, void* k_out, void* v_out,
                                      const coopt_shape* sh, void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (seq < 0 || seq >= sh->num_seqs || tok_begin < 0 || tok_end < tok_begin) return COOPT_ERR_SHAPE;
    if ((long long)tok_end > (long long)sh->max_blocks_per_seq * kBlock) return COOPT_ERR_SHAPE;
    if (tok_end == tok_begin) return COOPT_OK;
    if (!k_cache || !v_cache || !block_tables || !k_out || !v_out) return COOPT_ERR_NULL;
    if (sh->kv_dtype == COOPT_KV_E4M3 && (!k_scale || !v_scale)) return COOPT_ERR_NULL;
    const long long rows = (long long)(tok_end - tok_begin) * sh->num_kv_heads;
    if (rows > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    hipStream_t stream = (hipStream_t)hip_stream;
    const int32_t* bt_row = block_tables + (size_t)seq * sh->max_blocks_per_seq;
#define COOPT_GATHER(D, KV)                                                                        \
    hipLaunchKernelGGL((gather_cached_kv_kernel<D, KV>), grid, block, 0, stream,                   \
                       (const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale, bt_row, \
                       tok_begin, (int)rows, sh->num_kv_heads, (half_t*)k_out, (half_t*)v_out)
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) COOPT_GATHER(128, COOPT_KV_E4M3);
        else COOPT_GATHER(64, COOPT_KV_E4M3);
    } else {
        if (sh->head_dim == 128) COOPT_GATHER(128, COOPT_KV_FP16);
        else COOPT_GATHER(64, COOPT_KV_FP16);
    }
#undef COOPT_GATHER
    return launch_status();
}

extern "C" const char* coopt_status_string(int status)
{
    switch (status) {
    case COOPT_OK: return "ok";
    case COOPT_ERR_NULL: return "a required pointer is NULL";
    case COOPT_ERR_SHAPE: return "unsupported or inconsistent shape or argument";
    case COOPT_ERR_WORKSPACE: return "workspace or partial buffers too small or misaligned";
    case COOPT_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    default: return "unknown status";
    }
}
