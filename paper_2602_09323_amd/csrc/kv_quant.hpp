// Quantise-on-write of one (token, KV head) row by one wavefront (Opt-KV: Eq. 5, Alg. 1 phase 1):
// dynamic per-row scale amax/448, OCP E4M3 codes, both tiles stored in matrix-core operand order.
// Shared by the cache-write kernel and the fused decode step.
#pragma once

#include "common.hpp"

namespace coopt {

__device__ __forceinline__ float wave_max(float a)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a = fmaxf(a, __shfl_xor(a, o));
    return a;
}

// Dynamic per-row scale and the scaled, clamped values (binary32, correctly rounded divisions so
// that the stored bytes are defined bit for bit).
template <int E>
__device__ __forceinline__ float scale_row(const float (&x)[E], float (&y)[E])
{
    float amax = 0.0f;
#pragma unroll
    for (int e = 0; e < E; ++e) amax = fmaxf(amax, fabsf(x[e]));
    amax = wave_max(amax);
    const float scale = (amax == 0.0f) ? 1.0f : __fdiv_rn(amax, kE4M3Max);
#pragma unroll
    for (int e = 0; e < E; ++e) {
        float q = __fdiv_rn(x[e], scale);
        y[e] = fminf(fmaxf(q, -kE4M3Max), kE4M3Max);
    }
    return scale;
}

// binary32 -> OCP E4M3 by the gfx950 convert (round to nearest even; inputs are already in
// [-448, 448], so the instruction's overflow behaviour never comes into play).
__device__ __forceinline__ uint32_t encode_pair(float a, float b)
{
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu;
}

// The row's codes and scales.  Lane i holds elements i*E .. i*E+E-1 (E = HEAD_DIM/64).
template <int HEAD_DIM>
struct QuantRow {
    static constexpr int E = HEAD_DIM / 64;
    uint32_t k_codes, v_codes;      // E bytes each, element e in byte e
    float k_scale, v_scale;
};

// Quantises one K row and one V row (HEAD_DIM values each, lane i holding elements i*E .. i*E+E-1
// as binary32) and stores codes and scales into tile `tile` (= physical block * H_k + KV head) at
// token offset `off`.  Returns what it stored.
template <int HEAD_DIM>
__device__ __forceinline__ QuantRow<HEAD_DIM> quantise_values_to_cache(
    const float (&kx)[HEAD_DIM / 64], const float (&vx)[HEAD_DIM / 64], size_t tile, int off, int lane,
    uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache, float* __restrict__ k_scale,
    float* __restrict__ v_scale)
{
    constexpr int E = HEAD_DIM / 64;
    QuantRow<HEAD_DIM> qr;
    float y[E];
    // ---- K tile [d/16][16 tokens][16]: the lane's E dims are neighbours inside one 16-byte chunk
    qr.k_scale = scale_row<E>(kx, y);
    uint8_t* kdst = k_cache + tile * (kBlock * HEAD_DIM) + k_tile_index<1>(off, lane * E);
    if constexpr (E == 2) {
        qr.k_codes = encode_pair(y[0], y[1]);
        *reinterpret_cast<uint16_t*>(kdst) = (uint16_t)qr.k_codes;
    } else {
        qr.k_codes = encode_pair(y[0], 0.0f) & 0xffu;
        *kdst = (uint8_t)qr.k_codes;
    }
    if (lane == 0) k_scale[tile * kBlock + off] = qr.k_scale;

    // ---- V tile: token index innermost, one byte per (dim, token)
    qr.v_scale = scale_row<E>(vx, y);
    uint8_t* vtile = v_cache + tile * (kBlock * HEAD_DIM);
    if constexpr (E == 2) {
        qr.v_codes = encode_pair(y[0], y[1]);
        vtile[v_tile_index<1>(off, lane * E)] = (uint8_t)(qr.v_codes & 0xffu);
        vtile[v_tile_index<1>(off, lane * E + 1)] = (uint8_t)(qr.v_codes >> 8);
    } else {
        qr.v_codes = encode_pair(y[0], 0.0f) & 0xffu;
        vtile[v_tile_index<1>(off, lane)] = (uint8_t)qr.v_codes;
    }
    if (lane == 0) v_scale[tile * kBlock + off] = qr.v_scale;
    return qr;
}

// A lane's E elements of an fp16 row, widened.
template <int HEAD_DIM>
__device__ __forceinline__ void load_row_values(const half_t* __restrict__ row, int lane,
                                                float (&x)[HEAD_DIM / 64])
{
    constexpr int E = HEAD_DIM / 64;
#pragma unroll
    for (int e = 0; e < E; ++e) x[e] = (float)row[lane * E + e];
}

// The same from the rows in memory (HEAD_DIM fp16 values each).
template <int HEAD_DIM>
__device__ __forceinline__ QuantRow<HEAD_DIM> quantise_row_to_cache(
    const half_t* __restrict__ k_row, const half_t* __restrict__ v_row, size_t tile, int off, int lane,
    uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache, float* __restrict__ k_scale,
    float* __restrict__ v_scale)
{
    float kx[HEAD_DIM / 64], vx[HEAD_DIM / 64];
    load_row_values<HEAD_DIM>(k_row, lane, kx);
    load_row_values<HEAD_DIM>(v_row, lane, vx);
    return quantise_values_to_cache<HEAD_DIM>(kx, vx, tile, off, lane, k_cache, v_cache, k_scale, v_scale);
}

}  // namespace coopt
