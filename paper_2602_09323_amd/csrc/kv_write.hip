// Quantise-on-write of new K/V rows into the paged cache (Opt-KV: Eq. 5, Alg. 1 phase 1).
//
// One wavefront owns one (token, KV head) row: the 64 lanes hold the row's d elements (d/64 per
// lane), a butterfly max gives the row's absmax, and each lane encodes and stores its own
// elements.  Both tiles are stored in matrix-core operand order (see attn_tile.hpp), so a row is
// scattered in 16-byte (K) and 1-byte (V) pieces.  Write volume is a few hundred bytes per
// row, against kilobytes per token read by attention, so for a decode step's one token per sequence
// this kernel is latency-, not bandwidth-bound and is kept simple; calls with many tokens take the
// bulk kernel further down.
#include "kv_quant.hpp"

namespace coopt {

// Eq. 5's SkipSet as a bitmap over the call's token indices (NULL = empty).
__device__ __forceinline__ bool in_skip_set(const uint32_t* skip_set, int tok)
{
    return skip_set != nullptr && ((skip_set[tok >> 5] >> (tok & 31)) & 1u);
}

// scale_mode (see coopt_kv_cache_write_fp8_scaled): COOPT_SCALE_TOKEN = every row's own scale;
// COOPT_SCALE_STATIC = k_static[head] / v_static[head]; COOPT_SCALE_BLOCK = one scale for all rows
// of this call that land in the row's cache block (the largest of their absmaxes): the wavefront
// scans the call's slots for the others and takes their rows' absmax itself (every row of a block
// does the same scan -- this is the comparison scheme, not the method's).
template <int HEAD_DIM, int KV>
__global__ void __launch_bounds__(256)
kv_write_fp8_kernel(const half_t* __restrict__ k, const half_t* __restrict__ v,
                    const int64_t* __restrict__ slot_mapping,
                    const uint32_t* __restrict__ skip_set, int num_rows, int H_k,
                    uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache,
                    float* __restrict__ k_scale, float* __restrict__ v_scale, int scale_mode,
                    const float* __restrict__ k_static, const float* __restrict__ v_static)
{
    constexpr int E = HEAD_DIM / 64;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);        // token * H_k + head
    if (row >= num_rows) return;
    const int tok = row / H_k, head = row - tok * H_k;
    const int lane = threadIdx.x & 63;
    // the rows are asked for together with the slot, not after it: one memory round trip
    float kx[E], vx[E];
    load_row_values<HEAD_DIM>(k + (size_t)row * HEAD_DIM, lane, kx);
    load_row_values<HEAD_DIM>(v + (size_t)row * HEAD_DIM, lane, vx);
    const int64_t slot = slot_mapping[tok];
    const bool skip = in_skip_set(skip_set, tok);
    if (slot < 0 || skip) return;                               // Eq. 5: filtered token
    const int64_t blk = slot / kBlock;
    const int off = (int)(slot - blk * kBlock);
    const size_t tile = (size_t)(blk * H_k + head);
    float k_given = 0.0f, v_given = 0.0f;                       // 0: the row's own scale
    if (scale_mode == COOPT_SCALE_STATIC) {
        k_given = k_static[head];
        v_given = v_static[head];
    } else if (scale_mode == COOPT_SCALE_BLOCK) {
        float ka = row_absmax<E>(kx), va = row_absmax<E>(vx);
        const int num_tokens = num_rows / H_k;
        for (int base = 0; base < num_tokens; base += 64) {
            const int t2 = base + lane;
            bool same = false;
            if (t2 < num_tokens && t2 != tok) {
                const int64_t s2 = slot_mapping[t2];
                same = s2 >= 0 && s2 / kBlock == blk && !in_skip_set(skip_set, t2);
            }
            unsigned long long todo = __builtin_amdgcn_ballot_w64(same);
            while (todo) {                                      // wave-uniform
                const int other = base + __builtin_ctzll(todo);
                todo &= todo - 1;
                float k2[E], v2[E];
                load_row_values<HEAD_DIM>(k + ((size_t)other * H_k + head) * HEAD_DIM, lane, k2);
                load_row_values<HEAD_DIM>(v + ((size_t)other * H_k + head) * HEAD_DIM, lane, v2);
                ka = fmaxf(ka, row_absmax<E>(k2));
                va = fmaxf(va, row_absmax<E>(v2));
            }
        }
        k_given = scale_of_absmax<KV>(ka);
        v_given = scale_of_absmax<KV>(va);
    }
    quantise_values_to_cache<HEAD_DIM, KV>(kx, vx, tile, off, lane, k_cache, v_cache, k_scale, v_scale,
                                           k_given, v_given);
}

// ---- bulk form (prefill chunks, cache fills): many tokens per call.
//
// The row-per-wavefront kernel above stores a row's V codes one byte at a time (the V tile keeps
// four tokens of one dim in a dword), which is fine for one token per sequence and slow for
// thousands.  Here 16 dims (one 16-byte K chunk) belong to a lane, d/16 lanes make a row and a
// wavefront takes 64/(d/16) CONSECUTIVE tokens of one KV head: K is one 16-byte store per lane;
// and wherever four consecutive tokens sit in four consecutive slots of one block, starting at a
// multiple of four -- the usual case of a chunk written into fresh blocks -- their V codes are
// exchanged between the four rows' lanes and leave as whole dwords.  Any other slot pattern
// (skipped tokens, scattered slots) falls back to byte stores, row by row.  Same arithmetic as the
// row kernel, hence the same bytes.

// max over the groups of CH neighbouring lanes (CH a power of two)
template <int CH>
__device__ __forceinline__ float group_max(float a)
{
#pragma unroll
    for (int o = CH / 2; o > 0; o >>= 1) a = fmaxf(a, __shfl_xor(a, o));
    return a;
}

typedef unsigned int wu32x4 __attribute__((ext_vector_type(4)));

// 16 fp16 values (two 16-byte words) -> their group's scale and 16 one-byte codes, element e in byte e
template <int CH, int KV>
__device__ __forceinline__ wu32x4 quantise_chunk(wu32x4 lo, wu32x4 hi, float& scale)
{
    float x[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // (through scalars: a bit cast taken straight from a vector element reads element 0)
        const uint32_t wl = lo[i], wh = hi[i];
        const half2_t a = __builtin_bit_cast(half2_t, wl), b = __builtin_bit_cast(half2_t, wh);
        x[2 * i] = (float)a[0];
        x[2 * i + 1] = (float)a[1];
        x[8 + 2 * i] = (float)b[0];
        x[8 + 2 * i + 1] = (float)b[1];
    }
    float amax = 0.0f;
#pragma unroll
    for (int e = 0; e < 16; ++e) amax = fmaxf(amax, fabsf(x[e]));
    amax = group_max<CH>(amax);
    scale = scale_of_absmax<KV>(amax);
    wu32x4 codes;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            y[e] = fminf(fmaxf(__fdiv_rn(x[4 * d + e], scale), -kFp8Max<KV>), kFp8Max<KV>);
        int w;
        if constexpr (KV == COOPT_KV_E5M2) {
            w = __builtin_amdgcn_cvt_pk_bf8_f32(y[0], y[1], 0, false);
            w = __builtin_amdgcn_cvt_pk_bf8_f32(y[2], y[3], w, true);
        } else {
            w = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
            w = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], w, true);
        }
        codes[d] = (uint32_t)w;
    }
    return codes;
}

template <int HEAD_DIM, int KV>
__global__ void __launch_bounds__(256)
kv_write_fp8_bulk_kernel(const half_t* __restrict__ k, const half_t* __restrict__ v,
                         const int64_t* __restrict__ slot_mapping,
                         const uint32_t* __restrict__ skip_set, int num_tokens, int H_k,
                         uint8_t* __restrict__ k_cache, uint8_t* __restrict__ v_cache,
                         float* __restrict__ k_scale, float* __restrict__ v_scale)
{
    constexpr int CH = HEAD_DIM / 16;           // lanes per row
    constexpr int R = 64 / CH;                  // rows (consecutive tokens) per wavefront
    const int lane = threadIdx.x & 63;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);       // token group * H_k + head
    const int tg = unit / H_k, head = unit - tg * H_k;
    if (tg * R >= num_tokens) return;
    const int r = lane / CH, c = lane % CH;
    const int tok = tg * R + r;
    const bool in_range = tok < num_tokens;
    const int64_t slot = in_range ? slot_mapping[tok] : -1;
    const bool valid = slot >= 0 && !in_skip_set(skip_set, in_range ? tok : 0);   // Eq. 5
    const int64_t blk = valid ? slot / kBlock : 0;
    const int off = valid ? (int)(slot - blk * kBlock) : 0;
    const size_t tile = (size_t)(blk * H_k + head);

    // ---- the quad (rows 4q .. 4q+3) stores V as dwords if its four tokens fill slots s, s+1, s+2,
    // s+3 with s a multiple of four (then they share a block and a token quad of the tile)
    const int j = r & 3;                                        // row inside its quad
    const int64_t slot0 = __shfl(slot, (lane & ~(3 * CH)) | 0, 64);   // the quad's first row, same c
    int fits = (valid && slot == slot0 + j && (slot0 & 3) == 0) ? 1 : 0;
    fits &= __shfl_xor(fits, CH);                 // every lane takes part in both exchanges
    fits &= __shfl_xor(fits, 2 * CH);
    const bool quad = fits != 0;

    const size_t row_at = ((size_t)(in_range ? tok : 0) * H_k + head) * HEAD_DIM + 16 * c;
    const wu32x4* kp = reinterpret_cast<const wu32x4*>(k + row_at);
    const wu32x4* vp = reinterpret_cast<const wu32x4*>(v + row_at);
    const wu32x4 k_lo = kp[0], k_hi = kp[1], v_lo = vp[0], v_hi = vp[1];

    float ks, vs;
    const wu32x4 kc = quantise_chunk<CH, KV>(k_lo, k_hi, ks);
    const wu32x4 vc = quantise_chunk<CH, KV>(v_lo, v_hi, vs);

    uint8_t* ktile = k_cache + tile * (kBlock * HEAD_DIM);
    uint8_t* vtile = v_cache + tile * (kBlock * HEAD_DIM);
    if (valid) {
        // K tile [d/16][16 tokens][16]
        *reinterpret_cast<wu32x4*>(ktile + (c * kBlock + off) * 16) = kc;
        if (c == 0) {
            k_scale[tile * kBlock + off] = ks;
            v_scale[tile * kBlock + off] = vs;
        }
    }

    // ---- V: lane j of a quad collects dword j (dims 4j .. 4j+3 of the chunk) of all four rows
    uint32_t got[4];
    got[0] = vc[0];
#pragma unroll
    for (int x = 1; x < 4; ++x) {
        // send the partner (row j ^ x) its dword, receive mine from it
        const int want = j ^ x;
        const uint32_t send = want == 0 ? vc[0] : want == 1 ? vc[1] : want == 2 ? vc[2] : vc[3];
        got[x] = (uint32_t)__shfl_xor((int)send, x * CH);
    }
    got[0] = j == 0 ? vc[0] : j == 1 ? vc[1] : j == 2 ? vc[2] : vc[3];
    // got[x] = dword j of row j ^ x; order them by row
    uint32_t g4[4];
    {
        const bool s1 = (j & 1) != 0, s2 = (j & 2) != 0;
        const uint32_t a0 = s1 ? got[1] : got[0], a1 = s1 ? got[0] : got[1];
        const uint32_t a2 = s1 ? got[3] : got[2], a3 = s1 ? got[2] : got[3];
        g4[0] = s2 ? a2 : a0;
        g4[1] = s2 ? a3 : a1;
        g4[2] = s2 ? a0 : a2;
        g4[3] = s2 ? a1 : a3;
    }
    if (quad) {
        // byte b of g4[t] = code of dim 16c + 4j + b, token t of the quad: transpose to dwords of
        // four tokens
        const uint32_t lo01 = __builtin_amdgcn_perm(g4[1], g4[0], 0x05010400u);
        const uint32_t hi01 = __builtin_amdgcn_perm(g4[1], g4[0], 0x07030602u);
        const uint32_t lo23 = __builtin_amdgcn_perm(g4[3], g4[2], 0x05010400u);
        const uint32_t hi23 = __builtin_amdgcn_perm(g4[3], g4[2], 0x07030602u);
        const uint32_t out[4] = {__builtin_amdgcn_perm(lo23, lo01, 0x05040100u),
                                 __builtin_amdgcn_perm(lo23, lo01, 0x07060302u),
                                 __builtin_amdgcn_perm(hi23, hi01, 0x05040100u),
                                 __builtin_amdgcn_perm(hi23, hi01, 0x07060302u)};
        const int off0 = off - j;                                // the quad's first token
#pragma unroll
        for (int b = 0; b < 4; ++b)
            *reinterpret_cast<uint32_t*>(vtile + v_tile_index<1>(off0, 16 * c + 4 * j + b)) = out[b];
    } else if (valid) {
#pragma unroll
        for (int n = 0; n < 16; ++n)
            vtile[v_tile_index<1>(off, 16 * c + n)] = (uint8_t)(vc[n >> 2] >> (8 * (n & 3)));
    }
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

// The bulk form for fp16 caches: a pure scatter.  8 dims (one 16-byte K chunk) per lane, d/8 lanes
// per row, 64/(d/8) consecutive tokens of one KV head per wavefront.  K is one 16-byte store per
// lane.  The V tile keeps four tokens of one dim in 8 bytes: the lanes of an aligned run of four
// tokens exchange their halves and store 8 bytes per dim, else 2 bytes each.
template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
kv_write_fp16_bulk_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                          const int64_t* __restrict__ slot_mapping,
                          const uint32_t* __restrict__ skip_set, int num_tokens, int H_k,
                          uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache)
{
    constexpr int CH = HEAD_DIM / 8;            // lanes per row
    constexpr int R = 64 / CH;                  // rows (consecutive tokens) per wavefront: 4 or 8
    const int lane = threadIdx.x & 63;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);       // token group * H_k + head
    const int tg = unit / H_k, head = unit - tg * H_k;
    if (tg * R >= num_tokens) return;
    const int r = lane / CH, c = lane % CH;
    const int tok = tg * R + r;
    const bool in_range = tok < num_tokens;
    const int64_t slot = in_range ? slot_mapping[tok] : -1;
    const bool valid = slot >= 0 && !in_skip_set(skip_set, in_range ? tok : 0);   // Eq. 5
    const int64_t blk = valid ? slot / kBlock : 0;
    const int off = valid ? (int)(slot - blk * kBlock) : 0;
    const size_t tile = (size_t)(blk * H_k + head);

    const int j = r & 3;                                        // row inside its quad
    const int64_t slot0 = __shfl(slot, lane & ~(3 * CH), 64);   // the quad's first row, same c
    int fits = (valid && slot == slot0 + j && (slot0 & 3) == 0) ? 1 : 0;
    fits &= __shfl_xor(fits, CH);                 // every lane takes part in both exchanges
    fits &= __shfl_xor(fits, 2 * CH);
    const bool quad = fits != 0;

    const size_t row_at = ((size_t)(in_range ? tok : 0) * H_k + head) * HEAD_DIM + 8 * c;
    const wu32x4 kc = *reinterpret_cast<const wu32x4*>(k + row_at);   // dims 8c .. 8c+7
    const wu32x4 vc = *reinterpret_cast<const wu32x4*>(v + row_at);
    uint16_t* ktile = k_cache + tile * (kBlock * HEAD_DIM);
    uint16_t* vtile = v_cache + tile * (kBlock * HEAD_DIM);
    // K tile [d/8][16 tokens][8]
    if (valid) *reinterpret_cast<wu32x4*>(ktile + (c * kBlock + off) * 8) = kc;

    // ---- V: lane j of a quad collects dword j (dims 8c + 2j, 8c + 2j + 1) of all four rows
    uint32_t got[4];
#pragma unroll
    for (int x = 1; x < 4; ++x) {
        const int want = j ^ x;
        const uint32_t send = want == 0 ? vc[0] : want == 1 ? vc[1] : want == 2 ? vc[2] : vc[3];
        got[x] = (uint32_t)__shfl_xor((int)send, x * CH);
    }
    got[0] = j == 0 ? vc[0] : j == 1 ? vc[1] : j == 2 ? vc[2] : vc[3];
    uint32_t g4[4];                                              // g4[t] = dword j of row t
    {
        const bool s1 = (j & 1) != 0, s2 = (j & 2) != 0;
        const uint32_t a0 = s1 ? got[1] : got[0], a1 = s1 ? got[0] : got[1];
        const uint32_t a2 = s1 ? got[3] : got[2], a3 = s1 ? got[2] : got[3];
        g4[0] = s2 ? a2 : a0;
        g4[1] = s2 ? a3 : a1;
        g4[2] = s2 ? a0 : a2;
        g4[3] = s2 ? a1 : a3;
    }
    if (quad) {
        const int off0 = off - j;
#pragma unroll
        for (int h = 0; h < 2; ++h) {           // dim 8c + 2j + h: the four tokens' halves
            const uint32_t sel = h == 0 ? 0x05040100u : 0x07060302u;
            const uint32_t t01 = __builtin_amdgcn_perm(g4[1], g4[0], sel);
            const uint32_t t23 = __builtin_amdgcn_perm(g4[3], g4[2], sel);
            typedef unsigned int wu32x2 __attribute__((ext_vector_type(2)));
            *reinterpret_cast<wu32x2*>(vtile + v_tile_index<2>(off0, 8 * c + 2 * j + h)) = wu32x2{t01, t23};
        }
    } else if (valid) {
#pragma unroll
        for (int n = 0; n < 8; ++n)
            vtile[v_tile_index<2>(off, 8 * c + n)] = (uint16_t)(vc[n >> 1] >> (16 * (n & 1)));
    }
}

}  // namespace coopt

using namespace coopt;

// From this many tokens per call on, the bulk kernel (a call of a decode step has one per sequence).
constexpr int kBulkWriteTokens = 64;

template <int HEAD_DIM, int KV>
static void launch_write_fp8(const void* k, const void* v, const int64_t* slot_mapping,
                             const uint32_t* skip_set, int32_t num_tokens, uint8_t* k_cache,
                             uint8_t* v_cache, float* k_scale, float* v_scale, int scale_mode,
                             const float* k_static, const float* v_static, int H_k,
                             hipStream_t stream)
{
    const dim3 block(256);
    if (num_tokens >= kBulkWriteTokens && scale_mode == COOPT_SCALE_TOKEN) {
        // 64 / (d/16) consecutive tokens of one head per wavefront
        constexpr int per_wave = 64 / (HEAD_DIM / 16);
        const long long units = (long long)((num_tokens + per_wave - 1) / per_wave) * H_k;
        const dim3 grid((unsigned)((units + 3) / 4));
        hipLaunchKernelGGL((kv_write_fp8_bulk_kernel<HEAD_DIM, KV>), grid, block, 0, stream,
                           (const half_t*)k, (const half_t*)v, slot_mapping, skip_set, num_tokens, H_k,
                           k_cache, v_cache, k_scale, v_scale);
        return;
    }
    const long long rows = (long long)num_tokens * H_k;
    const dim3 grid((unsigned)((rows + 3) / 4));
    hipLaunchKernelGGL((kv_write_fp8_kernel<HEAD_DIM, KV>), grid, block, 0, stream, (const half_t*)k,
                       (const half_t*)v, slot_mapping, skip_set, (int)rows, H_k, k_cache, v_cache,
                       k_scale, v_scale, scale_mode, k_static, v_static);
}

static int write_fp8(const void* k, const void* v, const int64_t* slot_mapping,
                     const uint32_t* skip_set, int32_t num_tokens, uint8_t* k_cache,
                     uint8_t* v_cache, float* k_scale, float* v_scale, int scale_mode,
                     const float* k_static, const float* v_static, const coopt_shape* shape,
                     void* hip_stream)
{
    int st = check_shape(shape);
    if (st != COOPT_OK) return st;
    if ((shape->kv_dtype != COOPT_KV_E4M3 && shape->kv_dtype != COOPT_KV_E5M2) || num_tokens < 0)
        return COOPT_ERR_SHAPE;
    if (scale_mode != COOPT_SCALE_TOKEN && scale_mode != COOPT_SCALE_BLOCK &&
        scale_mode != COOPT_SCALE_STATIC)
        return COOPT_ERR_SHAPE;
    if (num_tokens == 0) return COOPT_OK;
    if (!k || !v || !slot_mapping || !k_cache || !v_cache || !k_scale || !v_scale)
        return COOPT_ERR_NULL;
    if (scale_mode == COOPT_SCALE_STATIC && (!k_static || !v_static)) return COOPT_ERR_NULL;
    const long long rows = (long long)num_tokens * shape->num_kv_heads;
    if (rows > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int H_k = shape->num_kv_heads;
#define COOPT_WRITE(D, KV)                                                                          \
    launch_write_fp8<D, KV>(k, v, slot_mapping, skip_set, num_tokens, k_cache, v_cache, k_scale,    \
                            v_scale, scale_mode, k_static, v_static, H_k, stream)
    if (shape->kv_dtype == COOPT_KV_E5M2) {
        if (shape->head_dim == 128) COOPT_WRITE(128, COOPT_KV_E5M2);
        else COOPT_WRITE(64, COOPT_KV_E5M2);
    } else {
        if (shape->head_dim == 128) COOPT_WRITE(128, COOPT_KV_E4M3);
        else COOPT_WRITE(64, COOPT_KV_E4M3);
    }
#undef COOPT_WRITE
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
    hipStream_t stream = (hipStream_t)hip_stream;
    const dim3 block(256);
    if (num_tokens >= kBulkWriteTokens) {
        const int per_wave = shape->head_dim == 128 ? 4 : 8;     // 64 / (d/8) tokens per wavefront
        const long long units = (long long)((num_tokens + per_wave - 1) / per_wave) * shape->num_kv_heads;
        const dim3 grid((unsigned)((units + 3) / 4));
        if (shape->head_dim == 128)
            hipLaunchKernelGGL(kv_write_fp16_bulk_kernel<128>, grid, block, 0, stream, (const uint16_t*)k,
                               (const uint16_t*)v, slot_mapping, skip_set, num_tokens,
                               shape->num_kv_heads, (uint16_t*)k_cache, (uint16_t*)v_cache);
        else
            hipLaunchKernelGGL(kv_write_fp16_bulk_kernel<64>, grid, block, 0, stream, (const uint16_t*)k,
                               (const uint16_t*)v, slot_mapping, skip_set, num_tokens,
                               shape->num_kv_heads, (uint16_t*)k_cache, (uint16_t*)v_cache);
        return launch_status();
    }
    const dim3 grid((unsigned)((rows + 3) / 4));
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
                     COOPT_SCALE_TOKEN, nullptr, nullptr, shape, hip_stream);
}

extern "C" int coopt_kv_cache_write_fp8_scaled(const void* k, const void* v,
                                               const int64_t* slot_mapping, int32_t num_tokens,
                                               uint8_t* k_cache, uint8_t* v_cache, float* k_scale,
                                               float* v_scale, int32_t scale_mode,
                                               const float* k_static, const float* v_static,
                                               const coopt_shape* shape, void* hip_stream)
{
    return write_fp8(k, v, slot_mapping, nullptr, num_tokens, k_cache, v_cache, k_scale, v_scale,
                     scale_mode, k_static, v_static, shape, hip_stream);
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
                     k_scale, v_scale, COOPT_SCALE_TOKEN, nullptr, nullptr, shape, hip_stream);
}
