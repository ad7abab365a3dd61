// Quantise-on-write of new K/V rows into the paged cache (Opt-KV: Eq. 5, Alg. 1 phase 1).
//
// One wavefront owns one (token, KV head) row: the 64 lanes hold the row's d elements (d/64 per
// lane), a butterfly max gives the row's absmax, and each lane encodes and stores its own
// elements.  Both tiles are stored in matrix-core operand order (see attn_tile.hpp), so a row is
// scattered in 16-byte (K) and 1-byte (V) pieces.  Write volume is a few hundred bytes per
// row, against kilobytes per token read by attention, so this kernel is latency-, not
// bandwidth-bound and is kept simple.
#include "kv_quant.hpp"

namespace coopt {

// Eq. 5's SkipSet as a bitmap over the call's token indices (NULL = empty).
__device__ __forceinline__ bool in_skip_set(const uint32_t* skip_set, int tok)
{
    return skip_set != nullptr && ((skip_set[tok >> 5] >> (tok & 31)) & 1u);
}

template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
kv_write_fp8_kernel(const half_t* __restrict__ k, const half_t* __restrict__ v,
                    const int64_t* __restrict__ slot_mapping,
                    const uint32_t* __restrict__ skip_set, int num_rows, int H_k,
                    uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache,
                    float* __restrict__ k_scale, float* __restrict__ v_scale)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);        // token * H_k + head
    if (row >= num_rows) return;
    const int tok = row / H_k, head = row - tok * H_k;
    const int64_t slot = slot_mapping[tok];
    if (slot < 0 || in_skip_set(skip_set, tok)) return;         // Eq. 5: filtered token
    const int64_t blk = slot / kBlock;
    const int off = (int)(slot - blk * kBlock);
    const int lane = threadIdx.x & 63;
    const size_t tile = (size_t)(blk * H_k + head);

    quantise_row_to_cache<HEAD_DIM>(k + (size_t)row * HEAD_DIM, v + (size_t)row * HEAD_DIM, tile, off,
                                    lane, k_cache, v_cache, k_scale, v_scale);
}

template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
kv_write_fp16_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                     const int64_t* __restrict__ slot_mapping,
                     const uint32_t* __restrict__ skip_set, int num_rows, int H_k,
                     uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache)
{
    constexpr int E = HEAD_DIM / 64;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= num_rows) return;
    const int tok = row / H_k, head = row - tok * H_k;
    const int64_t slot = slot_mapping[tok];
    if (slot < 0 || in_skip_set(skip_set, tok)) return;
    const int64_t blk = slot / kBlock;
    const int off = (int)(slot - blk * kBlock);
    const int lane = threadIdx.x & 63;
    const size_t tile = (size_t)(blk * H_k + head);
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int dim = lane * E + e;
        k_cache[tile * (kBlock * HEAD_DIM) + k_tile_index<2>(off, dim)] = k[(size_t)row * HEAD_DIM + dim];
        v_cache[tile * (kBlock * HEAD_DIM) + v_tile_index<2>(off, dim)] = v[(size_t)row * HEAD_DIM + dim];
    }
}

}  // namespace coopt

using namespace coopt;

static int write_fp8(const void* k, const void* v, const int64_t* slot_mapping,
                     const uint32_t* skip_set, int32_t num_tokens, uint8_t* k_cache,
                     uint8_t* v_cache, float* k_scale, float* v_scale, const coopt_shape* shape,
                     void* hip_stream)
{
    int st = check_shape(shape);
    if (st != COOPT_OK) return st;
    if (shape->kv_dtype != COOPT_KV_E4M3 || num_tokens < 0) return COOPT_ERR_SHAPE;
    if (num_tokens == 0) return COOPT_OK;
    if (!k || !v || !slot_mapping || !k_cache || !v_cache || !k_scale || !v_scale)
        return COOPT_ERR_NULL;
    const long long rows = (long long)num_tokens * shape->num_kv_heads;
    if (rows > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    hipStream_t stream = (hipStream_t)hip_stream;
    if (shape->head_dim == 128)
        hipLaunchKernelGGL(kv_write_fp8_kernel<128>, grid, block, 0, stream, (const half_t*)k,
                           (const half_t*)v, slot_mapping, skip_set, (int)rows, shape->num_kv_heads,
                           k_cache, v_cache, k_scale, v_scale);
    else
        hipLaunchKernelGGL(kv_write_fp8_kernel<64>, grid, block, 0, stream, (const half_t*)k,
                           (const half_t*)v, slot_mapping, skip_set, (int)rows, shape->num_kv_heads,
                           k_cache, v_cache, k_scale, v_scale);
    return launch_status();
}

static int write_fp16(const void* k, const void* v, const int64_t* slot_mapping,
                      const uint32_t* skip_set, int32_t num_tokens, void* k_cache, void* v_cache,
                      const coopt_shape* shape, void* hip_stream)
{
    int st = check_shape(shape);
    if (st != COOPT_OK) return st;
    if (shape->kv_dtype != COOPT_KV_FP16 || num_tokens < 0) return COOPT_ERR_SHAPE;
    if (num_tokens == 0) return COOPT_OK;
    if (!k || !v || !slot_mapping || !k_cache || !v_cache) return COOPT_ERR_NULL;
    const long long rows = (long long)num_tokens * shape->num_kv_heads;
    if (rows > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    hipStream_t stream = (hipStream_t)hip_stream;
    if (shape->head_dim == 128)
        hipLaunchKernelGGL(kv_write_fp16_kernel<128>, grid, block, 0, stream, (const uint16_t*)k,
                           (const uint16_t*)v, slot_mapping, skip_set, (int)rows,
                           shape->num_kv_heads, (uint16_t*)k_cache, (uint16_t*)v_cache);
    else
        hipLaunchKernelGGL(kv_write_fp16_kernel<64>, grid, block, 0, stream, (const uint16_t*)k,
                           (const uint16_t*)v, slot_mapping, skip_set, (int)rows,
                           shape->num_kv_heads, (uint16_t*)k_cache, (uint16_t*)v_cache);
    return launch_status();
}

extern "C" int coopt_kv_cache_write_fp8(const void* k, const void* v, const int64_t* slot_mapping,
                                        int32_t num_tokens, uint8_t* k_cache, uint8_t* v_cache,
                                        float* k_scale, float* v_scale, const coopt_shape* shape,
                                        void* hip_stream)
{
    return write_fp8(k, v, slot_mapping, nullptr, num_tokens, k_cache, v_cache, k_scale, v_scale,
                     shape, hip_stream);
}

extern "C" int coopt_kv_cache_write_fp16(const void* k, const void* v, const int64_t* slot_mapping,
                                         int32_t num_tokens, void* k_cache, void* v_cache,
                                         const coopt_shape* shape, void* hip_stream)
{
    return write_fp16(k, v, slot_mapping, nullptr, num_tokens, k_cache, v_cache, shape, hip_stream);
}

extern "C" int coopt_kv_cache_write_skipset(const void* k, const void* v,
                                            const int64_t* slot_mapping, const uint32_t* skip_set,
                                            int32_t num_tokens, void* k_cache, void* v_cache,
                                            float* k_scale, float* v_scale,
                                            const coopt_shape* shape, void* hip_stream)
{
    if (shape && shape->kv_dtype == COOPT_KV_FP16)
        return write_fp16(k, v, slot_mapping, skip_set, num_tokens, k_cache, v_cache, shape, hip_stream);
    return write_fp8(k, v, slot_mapping, skip_set, num_tokens, (uint8_t*)k_cache, (uint8_t*)v_cache,
                     k_scale, v_scale, shape, hip_stream);
}
