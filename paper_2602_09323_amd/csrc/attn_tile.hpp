// Register-level building blocks shared by the decode and chunked-prefill kernels: the loads of
// one (physical block, KV head) tile and one online-softmax update of a 16-column score tile
// against a GROUP of two cache blocks (32 tokens).
//
// Lane numbering: lane = 16*grp + n, n = 0..15, grp = 0..3.
//
// Per group (blocks A and B, 16 tokens each):
//   S^T[token][col] = K[token][:] . q[col][:]      per block: A operand = K tile (row n = token n),
//       B operand = q^T (column n = query row / head slot n), 16x16x32 MFMAs over the head dims.
//       Lane (n, grp) then holds the scores of column n for tokens 4grp..4grp+3 of each block.
//   They are scaled by k_scale[token]*softmax_scale*log2(e), masked beyond the column's visible
//   prefix (tail groups only), exponentiated against the running max of column n, multiplied by
//   v_scale[token] and split into an fp16 pair hi + lo.  The 8 values a lane holds are exactly
//   its share of the B operand of
//   O^T[dim][col] += V^T[dim][token] * P^T[token][col]     16x16x32 MFMAs over the 32 tokens, with
//       k-slots 8grp..8grp+3 = tokens 4grp..4grp+3 of block A and 8grp+4..8grp+7 = the same tokens
//       of block B; A operand = V tile rows (row n = dim 16c+n), c = 0 .. d/16-1.
//   No cross-lane traffic is needed between the two products; the running max is kept equal in
//   the four lanes (n, 0..3) by a two-step butterfly that only runs when some lane saw a larger
//   score (a wave-uniform branch).
//
// Numerics: E4M3 codes are exact in fp16, so both products are exact in the fp32 accumulators up
// to accumulation order, and the weights P*v_scale enter the second product as hi + lo (21
// significant bits, two MFMAs against the same V operand).  The weights are carried times a power
// of two (the reference max is offset in the exponent, which costs nothing) so that P*v_scale
// stays out of the fp16 subnormal range; the factor is common to the accumulator and the running
// sum and cancels in O/L.
//
// Cache tile layouts (one tile = 16 tokens x d dims of one KV head; E = elements per 16 bytes):
//   K tile  [d/E chunks][16 tokens][E]             element (tok, dim) at ((dim/E)*16 + tok)*E + dim%E
//   V tile  [d/(4E)][4 grp][16 n][E/4][4 tokens]   element (tok, dim), c = dim/16, n = dim%16:
//           ((((c/(E/4))*4 + tok/4)*16 + n)*(E/4) + c%(E/4))*4 + tok%4
// Both are the order in which the matrix-core operands consume them: every load instruction of a
// wave reads 64 x 16 contiguous bytes.
#pragma once

#include "common.hpp"

namespace coopt {

struct CacheView {
    const uint8_t* k_cache;
    const uint8_t* v_cache;
    const float* k_scale;
    const float* v_scale;
};

// Weights are carried as P * 2^kPShift, and the reference max m is only raised when a score
// exceeds it by more than kRescaleSlack (log2 units), so weights stay <= 2^(kPShift+kRescaleSlack)
// = 2^8: times a v_scale of at most 65504/448 that is still inside fp16.  Raising m lazily makes
// the rescale branch rare after the first group (a later score must beat the running max by a
// factor of 4), and any reference works: it cancels in O/L and in the merge of partials.
// An E5M2 cache's scales are 2^-7 of an E4M3 cache's (largest code 57344 against 448), so its
// weights are carried 2^7 higher: P * 2^13 * v_scale then lies where the E4M3 weights lie, well
// inside fp16's normal range for value rows of ordinary magnitude, and at most 2^15 * 65504/57344.
constexpr float kPShift = 6.0f;                     // (chunked prefill: it normalises the scales itself)
constexpr float kRescaleSlack = 2.0f;
template <int KV> constexpr float kPShiftOf = KV == COOPT_KV_E5M2 ? 13.0f : 6.0f;
template <int KV> constexpr float kPUnshiftOf = KV == COOPT_KV_E5M2 ? 1.0f / 8192.0f : 1.0f / 64.0f;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Raw bytes of one tile as loaded by lane (n, grp): NL 16-byte pieces of K and of V, 4 + 4 scales.
template <int HEAD_DIM, int KV>
struct BlockRegs {
    static constexpr int ES = kIsFp8<KV> ? 1 : 2;
    static constexpr int NL = HEAD_DIM * ES / 64;     // 16-byte loads per lane for K (and for V)
    u32x4 k[NL];
    u32x4 v[NL];
    floatx4 ks, vs;
};

// Loads of one tile through buffer descriptors, so that a lane's address is the constant 16*lane
// plus an immediate: no vector address arithmetic in the loop.  The wave-uniform tile number
// reaches the address through the scalar unit, in one of two ways:
//   BIG = false (pool < 2 GiB per tensor): one descriptor per tensor over the whole pool and the
//         tile's byte offset in the instruction's scalar offset; per tile only a multiply/shift.
//   BIG = true: one descriptor per tile (base = tile start, extent = tile bytes), 64-bit base
//         arithmetic on the scalar unit; no limit on the pool size.
// In both, an extent of zero turns the loads of a pipeline stage that has no block left into
// no-ops that return zeros and still count in program order, which keeps the number of loads in
// flight the same on every path through the loop, so the waits the compiler inserts stay exact.
// Tile loads carry the non-temporal hint: every byte of the cache is read once per step.
template <int HEAD_DIM, int KV, bool BIG>
struct TileLoader {
    static constexpr int ES = kIsFp8<KV> ? 1 : 2;
    static constexpr int kTileBytes = kBlock * HEAD_DIM * ES;
    static constexpr int kRsrcFlags = 0x00020000;      // gfx9 raw buffer, 32-bit data format
    static constexpr int kAuxStream = 2;               // nt
    CacheView cv;
    int lane_off, s_off;
    int kv_pool_bytes, scale_pool_bytes;               // BIG = false only

    __device__ __forceinline__ TileLoader(const CacheView& view, int lane, int pool_tiles) : cv(view)
    {
        lane_off = 16 * lane;
        s_off = 16 * (lane >> 4);
        kv_pool_bytes = pool_tiles * kTileBytes;
        scale_pool_bytes = pool_tiles * kBlock * 4;
    }

    static __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* base, int bytes)
    {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, kRsrcFlags);
    }

    // Single pieces of a tile, for kernels that split a tile's loads between wavefronts:
    // piece = 0 .. NL-1 of K or of V (16 bytes per lane each), or the lane group's 4 scales.
    // `tile` must be wave-uniform; valid = false returns zeros.
    __device__ __forceinline__ u32x4 load_piece(const uint8_t* pool, int tile, int piece, bool valid) const
    {
        if constexpr (BIG) {
            const __amdgpu_buffer_rsrc_t r =
                rsrc(pool + (size_t)(uint32_t)tile * kTileBytes, valid ? kTileBytes : 0);
            return __builtin_amdgcn_raw_buffer_load_b128(r, lane_off + 1024 * piece, 0, kAuxStream);
        } else {
            const __amdgpu_buffer_rsrc_t r = rsrc(pool, valid ? kv_pool_bytes : 0);
            return __builtin_amdgcn_raw_buffer_load_b128(r, lane_off + 1024 * piece, tile * kTileBytes, kAuxStream);
        }
    }
    __device__ __forceinline__ floatx4 load_scales(const float* pool, int tile, bool valid) const
    {
        if constexpr (BIG) {
            const __amdgpu_buffer_rsrc_t r =
                rsrc(pool + (size_t)(uint32_t)tile * kBlock, valid ? kBlock * 4 : 0);
            return __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, s_off, 0, 0));
        } else {
            const __amdgpu_buffer_rsrc_t r = rsrc(pool, valid ? scale_pool_bytes : 0);
            return __builtin_bit_cast(
                floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, s_off, tile * (kBlock * 4), 0));
        }
    }

    // `tile` (= physical block * H_k + KV head) must be wave-uniform.
    __device__ __forceinline__ void issue(BlockRegs<HEAD_DIM, KV>& r, int tile, bool valid) const
    {
        constexpr int NL = BlockRegs<HEAD_DIM, KV>::NL;
        if constexpr (BIG) {
            const size_t off = (size_t)(uint32_t)tile * kTileBytes;
            const int extent = valid ? kTileBytes : 0;
            const __amdgpu_buffer_rsrc_t rk = rsrc(cv.k_cache + off, extent);
            const __amdgpu_buffer_rsrc_t rv = rsrc(cv.v_cache + off, extent);
#pragma unroll
            for (int j = 0; j < NL; ++j)
                r.k[j] = __builtin_amdgcn_raw_buffer_load_b128(rk, lane_off + 1024 * j, 0, kAuxStream);
#pragma unroll
            for (int j = 0; j < NL; ++j)
                r.v[j] = __builtin_amdgcn_raw_buffer_load_b128(rv, lane_off + 1024 * j, 0, kAuxStream);
            if constexpr (kIsFp8<KV>) {
                const size_t soff = (size_t)(uint32_t)tile * kBlock;
                const int sext = valid ? kBlock * 4 : 0;
                const __amdgpu_buffer_rsrc_t rks = rsrc(cv.k_scale + soff, sext);
                const __amdgpu_buffer_rsrc_t rvs = rsrc(cv.v_scale + soff, sext);
                r.ks = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rks, s_off, 0, 0));
                r.vs = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rvs, s_off, 0, 0));
            }
        } else {
            const int extent = valid ? kv_pool_bytes : 0;
            const __amdgpu_buffer_rsrc_t rk = rsrc(cv.k_cache, extent);
            const __amdgpu_buffer_rsrc_t rv = rsrc(cv.v_cache, extent);
            const int so = tile * kTileBytes;
#pragma unroll
            for (int j = 0; j < NL; ++j)
                r.k[j] = __builtin_amdgcn_raw_buffer_load_b128(rk, lane_off + 1024 * j, so, kAuxStream);
#pragma unroll
            for (int j = 0; j < NL; ++j)
                r.v[j] = __builtin_amdgcn_raw_buffer_load_b128(rv, lane_off + 1024 * j, so, kAuxStream);
            if constexpr (kIsFp8<KV>) {
                const int sext = valid ? scale_pool_bytes : 0;
                const __amdgpu_buffer_rsrc_t rks = rsrc(cv.k_scale, sext);
                const __amdgpu_buffer_rsrc_t rvs = rsrc(cv.v_scale, sext);
                const int sso = tile * (kBlock * 4);
                r.ks = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rks, s_off, sso, 0));
                r.vs = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rvs, s_off, sso, 0));
            }
        }
    }
};

// True when every tensor of the pool can be addressed with a 31-bit byte offset.
inline bool pool_fits_small(const coopt_shape* sh)
{
    const long long es = sh->kv_dtype == COOPT_KV_FP16 ? 2 : 1;
    return (long long)sh->num_blocks * sh->num_kv_heads * kBlock * sh->head_dim * es < (1LL << 31);
}

// First of the 8 head dims that lane group grp feeds into S^T MFMA number jj (K chunk 4j+grp of
// the lane's j-th K load, low or high half); the q^T operand must use the same dims.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ int q_dim_offset(int jj, int grp)
{
    if constexpr (kIsFp8<KV>)
        return 64 * (jj >> 1) + 16 * grp + 8 * (jj & 1);
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

// The same operand through a buffer descriptor over the G query rows of one (sequence, KV head)
// pair: no branch around the loads, lanes of absent heads (n >= G) fall outside the descriptor and
// read zeros, and `valid` = false (wave-uniform) turns the whole load into zeros.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void load_q_operand_rows(half8_t (&qop)[HEAD_DIM / 32],
                                                    const half_t* pair_rows, int G, bool valid,
                                                    int n, int grp)
{
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half_t*>(pair_rows), 0, valid ? G * HEAD_DIM * 2 : 0, 0x00020000);
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj)
        qop[jj] = __builtin_bit_cast(
            half8_t, __builtin_amdgcn_raw_buffer_load_b128(
                         rq, 2 * (n * HEAD_DIM + q_dim_offset<HEAD_DIM, KV>(jj, grp)), 0, 0));
}

// K operand number jj (8 dims of token n) of a loaded tile.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ half8_t k_operand(const BlockRegs<HEAD_DIM, KV>& r, int jj)
{
    if constexpr (kIsFp8<KV>) {
        const u32x4 w = r.k[jj >> 1];
        return (jj & 1) ? fp8x8_to_half8<KV>(w.z, w.w) : fp8x8_to_half8<KV>(w.x, w.y);
    } else {
        return __builtin_bit_cast(half8_t, r.k[jj]);
    }
}

// V operand half of dim group c (dim 16c+n, the lane's 4 tokens).
template <int HEAD_DIM, int KV>
__device__ __forceinline__ half4_t v_operand(const BlockRegs<HEAD_DIM, KV>& r, int c)
{
    if constexpr (kIsFp8<KV>) {
        return fp8x4_to_half4<KV>(r.v[c >> 2][c & 3]);
    } else {
        const u32x4 w = r.v[c >> 1];
        const uint2 h = (c & 1) ? uint2{w.z, w.w} : uint2{w.x, w.y};
        return __builtin_bit_cast(half4_t, h);
    }
}

// Byte masks that zero the V entries of tokens beyond `cache_valid` (of this lane's 4 tokens).
template <int KV>
__device__ __forceinline__ void token_masks(int cache_valid, uint32_t& m0, uint32_t& m1)
{
    m0 = 0xffffffffu;
    m1 = 0xffffffffu;
    if (cache_valid < 4) {
        if constexpr (kIsFp8<KV>) {
            m0 = cache_valid <= 0 ? 0u : (0xffffffffu >> (8 * (4 - cache_valid)));
        } else {
            m0 = cache_valid <= 0 ? 0u : (cache_valid == 1 ? 0x0000ffffu : 0xffffffffu);
            m1 = cache_valid <= 2 ? 0u : (cache_valid == 3 ? 0x0000ffffu : 0xffffffffu);
        }
    }
}

// The group's 2 x 4 scores of this lane in log2 units, z[i] for block A's tokens 4grp+i and
// z[4+i] for block B's (Opt-KV Eq. 6 dequantisation folded into one multiply per token, Opt-GQA
// Eq. 8's scaled dot products on the matrix cores), with the tail fix-ups applied.
//   tail (wave-uniform) = false: every token of both blocks is in the cache and visible to every
//                 column; the vis / cache arguments are ignored.
//   tail = true:  visA / visB = how many of this lane's 4 tokens of block A / B column n may
//                 attend to (<= 0 none, >= 4 all); cacheA / cacheB = how many exist in the cache.
//                 Scores of invisible tokens are capped to -inf (Opt-Pa Eq. 9 / causal limit) with
//                 a min, which also discards NaN scores from stale keys or scales; V bytes and
//                 v_scale of absent tokens are zeroed in place, so stale NaN codes or scales
//                 cannot reach the accumulators.  The fix-ups sit in small branches that touch only
//                 temporaries and the loaded tile, so the accumulators stay in place across the loop.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void group_scores(BlockRegs<HEAD_DIM, KV>& A, BlockRegs<HEAD_DIM, KV>& B,
                                             const half8_t (&qop)[HEAD_DIM / 32], bool tail, int visA,
                                             int visB, int cacheA, int cacheB, float scale_log2e,
                                             float (&z)[8])
{
    floatx4 sA = {0.f, 0.f, 0.f, 0.f}, sB = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj) {
        sA = mfma_16x16x32(k_operand<HEAD_DIM, KV>(A, jj), qop[jj], sA);
        sB = mfma_16x16x32(k_operand<HEAD_DIM, KV>(B, jj), qop[jj], sB);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (kIsFp8<KV>) {
            z[i] = sA[i] * (A.ks[i] * scale_log2e);
            z[4 + i] = sB[i] * (B.ks[i] * scale_log2e);
        } else {
            z[i] = sA[i] * scale_log2e;
            z[4 + i] = sB[i] * scale_log2e;
        }
    }
    if (tail) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            z[i] = fminf(z[i], (i < visA) ? INFINITY : -INFINITY);          // min drops a NaN score
            z[4 + i] = fminf(z[4 + i], (i < visB) ? INFINITY : -INFINITY);
        }
        if constexpr (kIsFp8<KV>) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {                 // a stale scale times a zero weight
                A.vs[i] = (i < cacheA) ? A.vs[i] : 0.0f;
                B.vs[i] = (i < cacheB) ? B.vs[i] : 0.0f;
            }
        }
        uint32_t a0, a1, b0, b1;
        token_masks<KV>(cacheA, a0, a1);
        token_masks<KV>(cacheB, b0, b1);
#pragma unroll
        for (int j = 0; j < BlockRegs<HEAD_DIM, KV>::NL; ++j) {
            if constexpr (kIsFp8<KV>) {
                A.v[j] &= a0;
                B.v[j] &= b0;
            } else {
                A.v[j] &= u32x4{a0, a1, a0, a1};
                B.v[j] &= u32x4{b0, b1, b0, b1};
            }
        }
    }
}

// Eight binary32 weights as an fp16 pair hi + lo (the B operand of the P.V products is fp16):
// hi = w with its significand cut to fp16's 11 bits, which the convert then takes over exactly,
// lo = the remainder, again cut.  hi + lo carries 21 significant bits of w, so the products lose
// nothing that shows in an fp16 result; a single rounded fp16 weight (11 bits) moved outputs near
// |x| = 3 by up to 1.3e-3 when one token carries the softmax.  Weights below fp16's normal range
// (2^-14) keep an absolute error of at most 2^-24 each.
__device__ __forceinline__ void split_weights(const float (&w)[8], half8_t& hi, half8_t& lo)
{
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const float h0 = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, w[i]) & 0xffffe000u);
        const float h1 = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, w[i + 1]) & 0xffffe000u);
        const half2_t ph = __builtin_bit_cast(half2_t, __builtin_amdgcn_cvt_pkrtz(h0, h1));
        const half2_t pl =
            __builtin_bit_cast(half2_t, __builtin_amdgcn_cvt_pkrtz(w[i] - h0, w[i + 1] - h1));
        hi[i] = ph.x;
        hi[i + 1] = ph.y;
        lo[i] = pl.x;
        lo[i + 1] = pl.y;
    }
}

// O^T += V^T . P^T for the group (Opt-Pa Alg. 3 phase 2): p[0..3] / p[4..7] = this lane's weights
// of block A's / B's tokens, multiplied here by the tokens' v_scale (Opt-KV Eq. 6) and fed to the
// matrix cores as an fp16 hi + lo pair against the same V operand.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void group_pv(const BlockRegs<HEAD_DIM, KV>& A,
                                         const BlockRegs<HEAD_DIM, KV>& B, float (&p)[8],
                                         floatx4 (&acc)[HEAD_DIM / 16])
{
    if constexpr (kIsFp8<KV>) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] *= A.vs[i];
            p[4 + i] *= B.vs[i];
        }
    }
    half8_t hi, lo;
    split_weights(p, hi, lo);
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) {
        const half4_t va = v_operand<HEAD_DIM, KV>(A, c);
        const half4_t vb = v_operand<HEAD_DIM, KV>(B, c);
        const half8_t vop = {va[0], va[1], va[2], va[3], vb[0], vb[1], vb[2], vb[3]};
        acc[c] = mfma_16x16x32(vop, hi, acc[c]);
        acc[c] = mfma_16x16x32(vop, lo, acc[c]);
    }
}

// One online-softmax step of a 16-column tile against a group of two blocks (Opt-Pa Eq. 10).
// tail / vis / cache arguments as in group_scores.
//   m: reference max of column n in log2 units (within kRescaleSlack of the true running max),
//      identical in the four lanes (n, 0..3).
//   l: this lane's share of the running sum, acc[c][r] = O^T[16c + 4grp + r][n], both times 2^kPShiftOf<KV>.
// Requirement: whenever m is still -inf, the group holds a token visible to column n.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void group_update(BlockRegs<HEAD_DIM, KV>& A, BlockRegs<HEAD_DIM, KV>& B,
                                             const half8_t (&qop)[HEAD_DIM / 32], float& m, float& l,
                                             floatx4 (&acc)[HEAD_DIM / 16], bool tail, int visA,
                                             int visB, int cacheA, int cacheB, float scale_log2e)
{
    float z[8];
    group_scores<HEAD_DIM, KV>(A, B, qop, tail, visA, visB, cacheA, cacheB, scale_log2e, z);
    const float bm = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])),
                           fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
    if (__builtin_amdgcn_ballot_w64(bm > m + kRescaleSlack) != 0) {   // wave-uniform, rare
        float nm = fmaxf(bm, __shfl_xor(bm, 16));
        nm = fmaxf(nm, __shfl_xor(nm, 32));
        nm = fmaxf(nm, m);
        const float alpha = __builtin_amdgcn_exp2f(m - nm);   // m = -inf at the start gives 0
        l *= alpha;
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] *= alpha;
        m = nm;
    }
    const float mm = m - kPShiftOf<KV>;
    float p[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        p[i] = __builtin_amdgcn_exp2f(z[i] - mm);             // invisible: exp2(-inf) = 0
        l += p[i];
    }
    group_pv<HEAD_DIM, KV>(A, B, p, acc);
}

// The same step with the softmax statistics reduced the way Opt-Pa states it (Alg. 3, Eq. 10): a
// max reduction and a sum reduction ("block_sum") over the group's tokens through shared memory,
// and the accumulator rescaled at every group to the exact running max.  Kept to measure that
// mechanism against group_update on this machine; the results agree up to rounding.  `red` is
// 128 floats of LDS private to the wavefront, which must be the only one of its workgroup (the
// barriers only order this wave's own LDS traffic).  l ends up in the lanes of group 0, so the
// caller's sum over the four lane groups still gives the column's total.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void group_update_block_reduce(
    BlockRegs<HEAD_DIM, KV>& A, BlockRegs<HEAD_DIM, KV>& B, const half8_t (&qop)[HEAD_DIM / 32],
    float& m, float& l, floatx4 (&acc)[HEAD_DIM / 16], bool tail, int visA, int visB, int cacheA,
    int cacheB, float scale_log2e, float* red, int lane)
{
    const int n = lane & 15;
    float z[8];
    group_scores<HEAD_DIM, KV>(A, B, qop, tail, visA, visB, cacheA, cacheB, scale_log2e, z);
    // ---- max over the group's 32 tokens of column n, through shared memory
    red[lane] = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])),
                      fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
    __syncthreads();
    const float nm = fmaxf(m, fmaxf(fmaxf(red[n], red[16 + n]), fmaxf(red[32 + n], red[48 + n])));
    const float alpha = __builtin_amdgcn_exp2f(m - nm);       // m = -inf at the start gives 0
    m = nm;
    const float mm = m - kPShiftOf<KV>;
    float p[8], ps = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        p[i] = __builtin_amdgcn_exp2f(z[i] - mm);
        ps += p[i];
    }
    // ---- block_sum: the group's exponential sum of column n, through shared memory
    red[64 + lane] = ps;
    __syncthreads();
    const float bs = (red[64 + n] + red[80 + n]) + (red[96 + n] + red[112 + n]);
    l = l * alpha + (lane < 16 ? bs : 0.0f);
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] *= alpha;
    group_pv<HEAD_DIM, KV>(A, B, p, acc);
}

}  // namespace coopt
