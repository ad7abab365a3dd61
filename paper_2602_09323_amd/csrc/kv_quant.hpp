// Quantise-on-write of one (token, KV head) row by one wavefront (Opt-KV: Eq. 5, Alg. 1 phase 1):
// a scale (by default the row's own, amax / the code's largest value), OCP E4M3 or E5M2 codes,
// both tiles stored in matrix-core operand order.  Shared by the cache-write kernels and the fused
// decode step.  KV names the code: COOPT_KV_E4M3 (max 448) or COOPT_KV_E5M2 (max 57344).
#pragma once

#include <type_traits>

#include "common.hpp"

namespace coopt {

// Maximum over the 64 lanes, on the vector ALU: row shifts, then the two row broadcasts that carry
// a row's result into the following rows, leave it in lane 63 (no LDS round trips).  Lanes a step
// does not reach keep their own value.
__device__ __forceinline__ float wave_max(float a)
{
    int v = __builtin_bit_cast(int, a);
    auto step = [&](auto ctrl, auto rows) {
        const int o = __builtin_amdgcn_update_dpp(v, v, decltype(ctrl)::value, decltype(rows)::value, 0xf, false);
        v = __builtin_bit_cast(int, fmaxf(__builtin_bit_cast(float, v), __builtin_bit_cast(float, o)));
    };
    step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xf>{});   // row_shr:1
    step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xf>{});   // row_shr:2
    step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xf>{});   // row_shr:4
    step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xf>{});   // row_shr:8
    step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 -> rows 1, 3
    step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast:31 -> rows 2, 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(v, 63));
}

// The row's absmax over the wavefront's lanes.
template <int E>
__device__ __forceinline__ float row_absmax(const float (&x)[E])
{
    float amax = 0.0f;
#pragma unroll
    for (int e = 0; e < E; ++e) amax = fmaxf(amax, fabsf(x[e]));
    return wave_max(amax);
}

// The scale that maps absmax `amax` to the code's largest value (binary32, correctly rounded
// division so that the stored scale is defined bit for bit; an all-zero row gets 1).
template <int KV>
__device__ __forceinline__ float scale_of_absmax(float amax)
{
    return (amax == 0.0f) ? 1.0f : __fdiv_rn(amax, kFp8Max<KV>);
}

// The scaled, clamped values under `scale` (correctly rounded division again).
template <int KV, int E>
__device__ __forceinline__ void scale_values(const float (&x)[E], float scale, float (&y)[E])
{
#pragma unroll
    for (int e = 0; e < E; ++e) {
        float q = __fdiv_rn(x[e], scale);
        y[e] = fminf(fmaxf(q, -kFp8Max<KV>), kFp8Max<KV>);
    }
}

// Dynamic per-row scale and the scaled, clamped values.
template <int KV, int E>
__device__ __forceinline__ float scale_row(const float (&x)[E], float (&y)[E])
{
    const float scale = scale_of_absmax<KV>(row_absmax<E>(x));
    scale_values<KV, E>(x, scale, y);
    return scale;
}

// binary32 -> OCP E4M3 / E5M2 by the gfx950 converts (round to nearest even; inputs are already
// inside the code's finite range, so the instructions' overflow behaviour never comes into play).
template <int KV>
__device__ __forceinline__ uint32_t encode_pair(float a, float b)
{
    if constexpr (KV == COOPT_KV_E5M2)
        return (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, 0, false) & 0xffffu;
    else
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
// as binary32): the rows' scales and codes, nothing stored.
// k_given / v_given > 0: the scales to use (a static or a block's scale) instead of the rows' own.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ QuantRow<HEAD_DIM> quantise_values(const float (&kx)[HEAD_DIM / 64],
                                                              const float (&vx)[HEAD_DIM / 64],
                                                              float k_given = 0.0f,
                                                              float v_given = 0.0f)
{
    constexpr int E = HEAD_DIM / 64;
    QuantRow<HEAD_DIM> qr;
    float y[E];
    qr.k_scale = k_given > 0.0f ? k_given : scale_of_absmax<KV>(row_absmax<E>(kx));
    scale_values<KV, E>(kx, qr.k_scale, y);
    if constexpr (E == 2) qr.k_codes = encode_pair<KV>(y[0], y[1]);
    else qr.k_codes = encode_pair<KV>(y[0], 0.0f) & 0xffu;
    qr.v_scale = v_given > 0.0f ? v_given : scale_of_absmax<KV>(row_absmax<E>(vx));
    scale_values<KV, E>(vx, qr.v_scale, y);
    if constexpr (E == 2) qr.v_codes = encode_pair<KV>(y[0], y[1]);
    else qr.v_codes = encode_pair<KV>(y[0], 0.0f) & 0xffu;
    return qr;
}

// Stores a quantised row into tile `tile` (= physical block * H_k + KV head) at token offset `off`.
template <int HEAD_DIM>
__device__ __forceinline__ void store_quant_row(const QuantRow<HEAD_DIM>& qr, size_t tile, int off,
                                                int lane, uint8_t* __restrict__ k_cache,
                                                uint8_t* __restrict__ v_cache,
                                                float* __restrict__ k_scale,
                                                float* __restrict__ v_scale)
{
    constexpr int E = HEAD_DIM / 64;
    // ---- K tile [d/16][16 tokens][16]: the lane's E dims are neighbours inside one 16-byte chunk
    uint8_t* kdst = k_cache + tile * (kBlock * HEAD_DIM) + k_tile_index<1>(off, lane * E);
    if constexpr (E == 2) *reinterpret_cast<uint16_t*>(kdst) = (uint16_t)qr.k_codes;
    else *kdst = (uint8_t)qr.k_codes;
    if (lane == 0) k_scale[tile * kBlock + off] = qr.k_scale;
    // ---- V tile: token index innermost, one byte per (dim, token)
    uint8_t* vtile = v_cache + tile * (kBlock * HEAD_DIM);
    if constexpr (E == 2) {
        vtile[v_tile_index<1>(off, lane * E)] = (uint8_t)(qr.v_codes & 0xffu);
        vtile[v_tile_index<1>(off, lane * E + 1)] = (uint8_t)(qr.v_codes >> 8);
    } else {
        vtile[v_tile_index<1>(off, lane)] = (uint8_t)qr.v_codes;
    }
    if (lane == 0) v_scale[tile * kBlock + off] = qr.v_scale;
}

// Both: quantises the rows and stores codes and scales.  Returns what it stored.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ QuantRow<HEAD_DIM> quantise_values_to_cache(
    const float (&kx)[HEAD_DIM / 64], const float (&vx)[HEAD_DIM / 64], size_t tile, int off, int lane,
    uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache, float* __restrict__ k_scale,
    float* __restrict__ v_scale, float k_given = 0.0f, float v_given = 0.0f)
{
    const QuantRow<HEAD_DIM> qr = quantise_values<HEAD_DIM, KV>(kx, vx, k_given, v_given);
    store_quant_row<HEAD_DIM>(qr, tile, off, lane, k_cache, v_cache, k_scale, v_scale);
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
template <int HEAD_DIM, int KV>
__device__ __forceinline__ QuantRow<HEAD_DIM> quantise_row_to_cache(
    const half_t* __restrict__ k_row, const half_t* __restrict__ v_row, size_t tile, int off, int lane,
    uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache, float* __restrict__ k_scale,
    float* __restrict__ v_scale)
{
    float kx[HEAD_DIM / 64], vx[HEAD_DIM / 64];
    load_row_values<HEAD_DIM>(k_row, lane, kx);
    load_row_values<HEAD_DIM>(v_row, lane, vx);
    return quantise_values_to_cache<HEAD_DIM, KV>(kx, vx, tile, off, lane, k_cache, v_cache, k_scale, v_scale);
}

}  // namespace coopt
