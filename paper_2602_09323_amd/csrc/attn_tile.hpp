// Register-level building blocks shared by the decode and chunked-prefill kernels: the loads of
// one (physical block, KV head) tile, its conversion to matrix-core operands, and one
// online-softmax update of a 16-column score tile against it.
//
// Per 16-token block, with lane = 16*grp + n:
//   S^T[token][col] = K[token][:] . q[col][:]        A = K tile (row n = token n), B = q^T (col n
//                                                    = query row / head slot n); 16x16x32 MFMAs.
//   lane (n, grp) then holds the scores of column n for tokens 4*grp .. 4*grp+3.  They are scaled
//   by k_scale[token]*softmax_scale, masked beyond the column's visible prefix, exponentiated
//   against the running max of column n, multiplied by v_scale[token] and rounded to fp16:
//   exactly the B operand (column n, k-slots = tokens 4*grp..4*grp+3) of
//   O^T[dim][col] += V^T[dim][token] * P^T[token][col]   A = V tile rows (row n = dim 16c+n),
//                                                    16x16x16 MFMAs, c = 0 .. d/16-1.
//   No cross-lane traffic is needed between the two products; the running max is kept equal in
//   the four lanes (n, 0..3) by a two-step butterfly that only runs when some lane saw a larger
//   score (a wave-uniform branch).
//
// E4M3 codes are exact in fp16, so both products are exact in the fp32 accumulators up to
// accumulation order; the only rounding beyond fp32 is P*v_scale*2^8 -> fp16 (the 2^8 keeps small
// weights out of the fp16 subnormal range; it is divided out at the end).
#pragma once

#include "common.hpp"

namespace coopt {

struct CacheView {
    const uint8_t* k_cache;
    const uint8_t* v_cache;
    const float* k_scale;
    const float* v_scale;
};

// P is carried as P * v_scale * 2^8 in fp16 for E4M3 caches (plain P for fp16 caches).
constexpr float kPScale = 256.0f;

template <int KV>
__device__ __forceinline__ constexpr float out_unscale()
{
    return KV == COOPT_KV_E4M3 ? 1.0f / kPScale : 1.0f;
}

// Raw bytes of one tile as loaded by lane (n, grp).
template <int HEAD_DIM, int KV>
struct BlockRegs {
    static constexpr int NK = (KV == COOPT_KV_E4M3) ? HEAD_DIM / 64 : HEAD_DIM / 32;
    static constexpr int NV = HEAD_DIM / 16;
    static constexpr int VW = (KV == COOPT_KV_E4M3) ? 1 : 2;   // 32-bit words per V operand
    uint4 k[NK];
    uint32_t v[NV][VW];
    floatx4 ks, vs;
};

// Matrix-core operands of one tile.
template <int HEAD_DIM>
struct BlockOps {
    half8_t k[HEAD_DIM / 32];    // A of S^T: token n, 8 dims per MFMA (see q_dim_offset)
    half4_t v[HEAD_DIM / 16];    // A of O^T: dim 16c+n, tokens 4grp..4grp+3
    floatx4 ks, vs;
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Loads of one (physical block, KV head) tile through buffer descriptors.  Each tile gets its own
// descriptor (base = tile start, extent = tile bytes), built on the scalar unit from the
// wave-uniform block number, so a lane's address is a per-lane constant plus an immediate: no
// vector address arithmetic in the loop, no 4 GiB limit on the pool, and hardware bounds checking
// confined to the tile.  An extent of zero turns the loads of a pipeline stage that has no block
// left into no-ops that still count in program order, which keeps the number of loads in flight
// the same on every path through the loop, so the waits the compiler inserts stay exact.
//   K [tile][16 tokens][d]: lane (n, grp) reads 16 bytes of token n per K load;
//   V [tile][d][16 tokens]: the lane's 4 tokens 4grp..4grp+3 of dim 16c+n, for every c;
//   scales [tile][16]: the lane's 4 tokens.
template <int HEAD_DIM, int KV>
struct TileLoader {
    static constexpr int ES = (KV == COOPT_KV_E4M3) ? 1 : 2;
    static constexpr int kTileBytes = kBlock * HEAD_DIM * ES;
    static constexpr int kRsrcFlags = 0x00020000;      // gfx9 raw buffer, 32-bit data format
    CacheView cv;
    int k_off, v_off, s_off;

    __device__ __forceinline__ TileLoader(const CacheView& view, int n, int grp) : cv(view)
    {
        k_off = n * HEAD_DIM * ES + 16 * grp;          // + 64*j per K load
        v_off = (n * kBlock + 4 * grp) * ES;           // + 16*kBlock*ES*c per V load
        s_off = 16 * grp;
    }

    static __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* base, int bytes)
    {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, kRsrcFlags);
    }

    // `tile` must be wave-uniform.  valid == false issues the same loads against an empty extent.
    __device__ __forceinline__ void issue(BlockRegs<HEAD_DIM, KV>& r, size_t tile, bool valid) const
    {
        const __amdgpu_buffer_rsrc_t rk = rsrc(cv.k_cache + tile * kTileBytes, valid ? kTileBytes : 0);
        const __amdgpu_buffer_rsrc_t rv = rsrc(cv.v_cache + tile * kTileBytes, valid ? kTileBytes : 0);
#pragma unroll
        for (int j = 0; j < BlockRegs<HEAD_DIM, KV>::NK; ++j) {
            const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rk, k_off + 64 * j, 0, 0);
            r.k[j] = uint4{w.x, w.y, w.z, w.w};
        }
        if constexpr (KV == COOPT_KV_E4M3) {
#pragma unroll
            for (int c = 0; c < HEAD_DIM / 16; ++c)
                r.v[c][0] = __builtin_amdgcn_raw_buffer_load_b32(rv, v_off + 16 * kBlock * c, 0, 0);
            const __amdgpu_buffer_rsrc_t rks =
                rsrc(cv.k_scale + tile * kBlock, valid ? kBlock * 4 : 0);
            const __amdgpu_buffer_rsrc_t rvs =
                rsrc(cv.v_scale + tile * kBlock, valid ? kBlock * 4 : 0);
            r.ks = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rks, s_off, 0, 0));
            r.vs = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rvs, s_off, 0, 0));
        } else {
#pragma unroll
            for (int c = 0; c < HEAD_DIM / 16; ++c) {
                const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rv, v_off + 32 * kBlock * c, 0, 0);
                r.v[c][0] = w.x;
                r.v[c][1] = w.y;
            }
        }
    }
};

// First of the 8 head dims that lane group grp feeds into S^T MFMA number jj; the q^T operand
// must use the same dims.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ int q_dim_offset(int jj, int grp)
{
    if constexpr (KV == COOPT_KV_E4M3)
        return 64 * (jj >> 1) + 16 * grp + 8 * (jj & 1);   // halves of one 16-byte K load
    else
        return 32 * jj + 8 * grp;
}

// q^T operand of column n from a contiguous fp16 row (zero operand if !present).
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void load_q_operand(half8_t (&qop)[HEAD_DIM / 32], const half_t* qrow,
                                               bool present, int grp)
{
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj) {
        uint4 w = {0u, 0u, 0u, 0u};
        if (present)
            w = *reinterpret_cast<const uint4*>(qrow + q_dim_offset<HEAD_DIM, KV>(jj, grp));
        qop[jj] = __builtin_bit_cast(half8_t, w);
    }
}

// Raw tile -> operands.  cache_valid = how many of this lane's 4 tokens exist in the cache at all
// (>= 4 everywhere except in the last block of a context): V of the others is zeroed so that
// stale NaN codes cannot poison the accumulators through 0 * NaN.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void convert_block(BlockOps<HEAD_DIM>& o, const BlockRegs<HEAD_DIM, KV>& r,
                                              int cache_valid)
{
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj) {
        if constexpr (KV == COOPT_KV_E4M3) {
            const uint4 w = r.k[jj >> 1];
            o.k[jj] = (jj & 1) ? e4m3x8_to_half8(w.z, w.w) : e4m3x8_to_half8(w.x, w.y);
        } else {
            o.k[jj] = __builtin_bit_cast(half8_t, r.k[jj]);
        }
    }
    uint32_t mask0 = 0xffffffffu, mask1 = 0xffffffffu;
    if (cache_valid < 4) {
        if constexpr (KV == COOPT_KV_E4M3) {
            mask0 = cache_valid <= 0 ? 0u : (0xffffffffu >> (8 * (4 - cache_valid)));
        } else {
            mask0 = cache_valid <= 0 ? 0u : (cache_valid == 1 ? 0x0000ffffu : 0xffffffffu);
            mask1 = cache_valid <= 2 ? 0u : 0x0000ffffu;
        }
    }
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) {
        if constexpr (KV == COOPT_KV_E4M3) {
            o.v[c] = e4m3x4_to_half4(r.v[c][0] & mask0);
        } else {
            const uint2 w = {r.v[c][0] & mask0, r.v[c][1] & mask1};
            o.v[c] = __builtin_bit_cast(half4_t, w);
        }
    }
    o.ks = r.ks;
    o.vs = r.vs;
}

// One online-softmax step of a 16-column tile against one block.
//   n_visible: how many of this lane's 4 tokens column n may attend to (<= 0: none, >= 4: all).
//   m: running max of column n in log2 units, identical in the four lanes (n, 0..3).
//   l: this lane's share of the running sum.  acc[c][r] = O^T[16c + 4grp + r][n].
// Requirement: whenever m is still -inf, the block holds a token visible to column n.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void tile_update(const BlockOps<HEAD_DIM>& o,
                                            const half8_t (&qop)[HEAD_DIM / 32], float& m, float& l,
                                            floatx4 (&acc)[HEAD_DIM / 16], int n_visible,
                                            float scale_log2e)
{
    floatx4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj) s = mfma_16x16x32(o.k[jj], qop[jj], s);
    float z[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float zi = s[i] * scale_log2e;
        if constexpr (KV == COOPT_KV_E4M3) zi *= o.ks[i];
        z[i] = (i < n_visible) ? zi : -INFINITY;          // Opt-Pa Eq. 9 / causal limit
    }
    const float bm = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
    if (__builtin_amdgcn_ballot_w64(bm > m) != 0) {        // wave-uniform: someone saw a new max
        float nm = fmaxf(bm, __shfl_xor(bm, 16));
        nm = fmaxf(nm, __shfl_xor(nm, 32));
        nm = fmaxf(nm, m);
        const float alpha = __builtin_amdgcn_exp2f(m - nm);   // m = -inf at the start gives 0
        l *= alpha;
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] *= alpha;
        m = nm;
    }
    half4_t pop;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(z[i] - m);     // masked: exp2(-inf) = 0
        l += p;
        float pv = p;
        if constexpr (KV == COOPT_KV_E4M3) pv = p * kPScale * o.vs[i];
        pop[i] = (half_t)((i < n_visible) ? pv : 0.0f);       // stale scales must not leak NaN
    }
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = mfma_16x16x16(o.v[c], pop, acc[c]);
}

}  // namespace coopt
