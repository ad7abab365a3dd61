// Internal helpers shared by the gfx950 kernels of the paged decode-attention library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "coopt_attn.h"

namespace coopt {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 16;          // tokens per cache block (the only supported block_size)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kE4M3Max = 448.0f;
constexpr float kE5M2Max = 57344.0f;

// One-byte floating-point caches (OCP E4M3 or E5M2 codes with binary32 scales) against fp16 ones.
template <int KV>
inline constexpr bool kIsFp8 = KV != COOPT_KV_FP16;
// Largest finite value of the cache's code: what a row's absmax is mapped to.
template <int KV>
inline constexpr float kFp8Max = KV == COOPT_KV_E5M2 ? kE5M2Max : kE4M3Max;

// Element index of (token, dim) inside one cache tile; ES = bytes per element, E = elements per
// 16 bytes.  K tiles are [d/E chunks][16 tokens][E]; V tiles are [d/(4E)][4][16][E/4][4 tokens].
template <int ES>
__host__ __device__ __forceinline__ int k_tile_index(int tok, int dim)
{
    constexpr int E = 16 / ES;
    return ((dim / E) * kBlock + tok) * E + dim % E;
}
template <int ES>
__host__ __device__ __forceinline__ int v_tile_index(int tok, int dim)
{
    constexpr int W = 4 / ES;                    // 16-dim groups per 16 bytes
    const int c = dim >> 4, n = dim & 15;
    return ((((c / W) * (kBlock / 4) + (tok >> 2)) * 16 + n) * W + c % W) * 4 + (tok & 3);
}

// Host-side validation common to all entry points.  Returns COOPT_OK or the error to hand back.
inline int check_shape(const coopt_shape* sh)
{
    if (!sh) return COOPT_ERR_NULL;
    if (sh->num_seqs < 0 || sh->num_q_heads <= 0 || sh->num_kv_heads <= 0) return COOPT_ERR_SHAPE;
    if (sh->head_dim != 64 && sh->head_dim != 128) return COOPT_ERR_SHAPE;
    if (sh->block_size != kBlock) return COOPT_ERR_SHAPE;
    if (sh->num_q_heads % sh->num_kv_heads != 0) return COOPT_ERR_SHAPE;
    if (sh->num_q_heads / sh->num_kv_heads > 16) return COOPT_ERR_SHAPE;
    if (sh->num_blocks <= 0 || sh->max_blocks_per_seq <= 0) return COOPT_ERR_SHAPE;
    // index arithmetic in the kernels is 32-bit where the products below fit
    if (sh->num_seqs > (1 << 20) || sh->num_q_heads > (1 << 12)) return COOPT_ERR_SHAPE;
    if (sh->max_blocks_per_seq > (1 << 24)) return COOPT_ERR_SHAPE;
    if ((long long)sh->num_seqs * sh->num_q_heads > (1LL << 27)) return COOPT_ERR_SHAPE;
    if ((long long)sh->num_blocks * sh->num_kv_heads > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    if (sh->kv_dtype != COOPT_KV_FP16 && sh->kv_dtype != COOPT_KV_E4M3 && sh->kv_dtype != COOPT_KV_E5M2)
        return COOPT_ERR_SHAPE;
    return COOPT_OK;
}

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? COOPT_OK : COOPT_ERR_LAUNCH;
}

// Two one-byte codes (bytes 0,1 or 2,3 of w) -> two fp16, exact: every E4M3 value is an fp16
// value (the gfx950 convert does it), and an E5M2 code IS the high byte of the fp16 pattern of
// its value (a byte shuffle does it; infinities and NaN codes map to fp16's own).
template <int KV, bool HI>
__device__ __forceinline__ half2_t fp8x2_to_half2(uint32_t w)
{
    if constexpr (KV == COOPT_KV_E5M2)
        return __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(0u, w, HI ? 0x030c020cu : 0x010c000cu));
    else
        return __builtin_amdgcn_cvt_scalef32_pk_f16_fp8((int)w, 1.0f, HI);
}

template <int KV>
__device__ __forceinline__ half4_t fp8x4_to_half4(uint32_t w)
{
    half2_t lo = fp8x2_to_half2<KV, false>(w);
    half2_t hi = fp8x2_to_half2<KV, true>(w);
    return half4_t{lo.x, lo.y, hi.x, hi.y};
}

template <int KV>
__device__ __forceinline__ half8_t fp8x8_to_half8(uint32_t w0, uint32_t w1)
{
    half2_t a = fp8x2_to_half2<KV, false>(w0);
    half2_t b = fp8x2_to_half2<KV, true>(w0);
    half2_t c = fp8x2_to_half2<KV, false>(w1);
    half2_t d = fp8x2_to_half2<KV, true>(w1);
    return half8_t{a.x, a.y, b.x, b.y, c.x, c.y, d.x, d.y};
}

// Matrix-core tiles used throughout (wave64, lane = 16*grp + n):
//   A operand: row n,  k-slots owned by lane group grp (8 per lane for x32, 4 for x16)
//   B operand: column n, the same k-slots
//   C/D:       D[4*grp + r][n] in register r (r = 0..3)
// Any k-slot numbering works as long as A and B agree, because lanes of equal grp own equal slots.
__device__ __forceinline__ floatx4 mfma_16x16x32(half8_t a, half8_t b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ floatx4 mfma_16x16x16(half4_t a, half4_t b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float wave_uniform(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}
__device__ __forceinline__ int wave_uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

}  // namespace coopt
