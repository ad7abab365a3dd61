// Partial attention results and their merge (the cross-partition reduction): every partial is
// (m, l, o) = (reference max, sum of exp(z - m), normalised output) over one token range; any
// reference max is legal.  M = max m_p, w_p = l_p exp(m_p - M), out = sum w_p o_p / sum w_p.
#pragma once

#include "common.hpp"

namespace coopt {

// One wavefront merges the `count` partials of one (sequence, query head) row and writes the fp16
// output row.  ml / es point at the row's first partial, po at its first partial row of HEAD_DIM
// floats.  Lane i owns dims i and i+64.  count == 0 writes zeros.
template <int HEAD_DIM>
__device__ __forceinline__ void merge_row(const float* __restrict__ ml, const float* __restrict__ es,
                                          const float* __restrict__ po, int count,
                                          half_t* __restrict__ out_row, int lane)
{
    constexpr int E = HEAD_DIM / 64;
    float o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.0f;
    if (count > 0) {
        float M = -INFINITY;
        for (int p = lane; p < count; p += 64) M = fmaxf(M, ml[p]);
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) M = fmaxf(M, __shfl_xor(M, s));
        float W = 0.0f;
        for (int base = 0; base < count; base += 64) {
            // lane p holds the weight of partial base+p; the partial rows are then streamed with
            // independent loads and the weight of each is broadcast from its lane
            const int p = base + lane;
            const float wv = p < count ? es[p] * __expf(ml[p] - M) : 0.0f;
            W += wv;
            const int cnt = min(64, count - base);
            for (int j = 0; j < cnt; ++j) {
                const float wj = __builtin_bit_cast(
                    float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), j));
#pragma unroll
                for (int e = 0; e < E; ++e)
                    o[e] += wj * po[(size_t)(base + j) * HEAD_DIM + lane + 64 * e];
            }
        }
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) W += __shfl_xor(W, s);
        const float inv = 1.0f / W;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] *= inv;
    }
#pragma unroll
    for (int e = 0; e < E; ++e) out_row[lane + 64 * e] = (half_t)o[e];
}

}  // namespace coopt
