// Dequantising gather (the read half of Opt-KV: Eq. 6, Alg. 1 phase 2): paged cache rows of one
// sequence -> contiguous fp16 K and V.  Pure data movement: 264 bytes read and 512 written per
// (token, KV head) at d = 128 with an E4M3 cache, no reuse, bound by HBM.
//
// One wavefront per (block, KV head) tile.  The unit of output is 16 bytes (8 fp16 dims of one
// token); unit u of a tile is token u / (d/8), dims 8 (u % (d/8)) .. +7, so the 64 lanes of one
// store instruction cover whole output rows.  K tiles hold a token's dims contiguously, so a K unit
// is one 8-byte (E4M3) or 16-byte (fp16) load.  V tiles are laid out for the attention kernels'
// matrix operands (4 tokens x 4/ES dims per 16 bytes): they are loaded as stored, transposed
// through a [16][d] LDS tile of the wave's own, and then follow the K path.
#include "common.hpp"

namespace coopt {

typedef unsigned int gu32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int gu32x2 __attribute__((ext_vector_type(2)));

// fp16(code * scale) with a single rounding.  The binary32 product is inexact (4 x 24 significant
// bits), and rounding it again to fp16 would be wrong whenever it lands on an fp16 tie; so the
// product is taken to binary32 by round-to-odd (truncate, then set the last bit if anything was
// lost), after which the conversion's round-to-nearest-even sees where the exact value lies.
__device__ __forceinline__ float mul_round_to_odd(float c, float s)
{
    const float p = c * s;
    const float e = __builtin_fmaf(c, s, -p);                  // exact: code*scale - p
    uint32_t u = __builtin_bit_cast(uint32_t, p);
    const uint32_t away = (__builtin_bit_cast(uint32_t, e) ^ u) >> 31;   // p overshot in magnitude
    u = (e != 0.0f) ? ((u - away) | 1u) : u;
    return __builtin_bit_cast(float, u);
}

// 8 one-byte codes (two dwords; E4M3 or E5M2) times one scale -> 8 fp16
template <int KV>
__device__ __forceinline__ half8_t dequant8(uint32_t w0, uint32_t w1, float scale)
{
    floatx2 c[4];
    if constexpr (KV == COOPT_KV_E5M2) {
        c[0] = __builtin_amdgcn_cvt_pk_f32_bf8((int)w0, false);
        c[1] = __builtin_amdgcn_cvt_pk_f32_bf8((int)w0, true);
        c[2] = __builtin_amdgcn_cvt_pk_f32_bf8((int)w1, false);
        c[3] = __builtin_amdgcn_cvt_pk_f32_bf8((int)w1, true);
    } else {
        c[0] = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false);
        c[1] = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
        c[2] = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false);
        c[3] = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
    }
    half8_t r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r[2 * i] = (half_t)mul_round_to_odd(c[i].x, scale);
        r[2 * i + 1] = (half_t)mul_round_to_odd(c[i].y, scale);
    }
    return r;
}

constexpr int kGatherWaves = 4;

template <int HEAD_DIM, int KV>
__global__ void __launch_bounds__(64 * kGatherWaves)
gather_cached_kv_kernel(const uint8_t* __restrict__ k_cache, const uint8_t* __restrict__ v_cache,
                        const float* __restrict__ k_scale, const float* __restrict__ v_scale,
                        const int32_t* __restrict__ bt_row, int tok_begin, int tok_end,
                        int first_block, int num_tiles, int H_k,
                        half_t* __restrict__ k_out, half_t* __restrict__ v_out)
{
    constexpr bool FP8 = kIsFp8<KV>;
    constexpr int ES = FP8 ? 1 : 2;                    // bytes per cache element
    constexpr int UPR = HEAD_DIM / 8;                  // 16-byte output units per row
    constexpr int NU = kBlock * UPR / 64;              // units per lane and tile
    constexpr int NP = kBlock * HEAD_DIM * ES / 1024;  // 16-byte cache pieces per lane and tile
    constexpr int W = 4 / ES;                          // dims per 16-byte V piece (x 4 tokens)
    constexpr int RS = HEAD_DIM * ES + 16;             // LDS row stride: [token][dim] + skew
    __shared__ __attribute__((aligned(16))) unsigned char lds[kGatherWaves][kBlock * RS];

    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform((int)(threadIdx.x >> 6));
    const int tile_id = blockIdx.x * kGatherWaves + wave;
    if (tile_id >= num_tiles) return;
    const int b = first_block + tile_id / H_k;         // logical block
    const int head = tile_id % H_k;
    const size_t tile = (size_t)bt_row[b] * H_k + head;
    const unsigned char* kt = k_cache + tile * (kBlock * HEAD_DIM * ES);
    const unsigned char* vt = v_cache + tile * (kBlock * HEAD_DIM * ES);
    unsigned char* my = lds[wave];

    // ---- all loads of the tile up front: V pieces as stored, K by output unit, scales by token
    gu32x4 vp[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j)
        vp[j] = __builtin_nontemporal_load(reinterpret_cast<const gu32x4*>(vt) + j * 64 + lane);
    gu32x4 ku[NU];                                      // E4M3: .x/.y only
    float ks[NU], vs[NU];
#pragma unroll
    for (int i = 0; i < NU; ++i) {
        const int u = i * 64 + lane, tok = u / UPR, piece = u % UPR;
        if constexpr (FP8) {
            // K tile [d/16][16 tokens][16]: the unit is half of a 16-byte chunk
            const gu32x2 w = __builtin_nontemporal_load(
                reinterpret_cast<const gu32x2*>(kt + ((piece >> 1) * kBlock + tok) * 16 + (piece & 1) * 8));
            ku[i] = gu32x4{w.x, w.y, 0u, 0u};
            ks[i] = k_scale[tile * kBlock + tok];
            vs[i] = v_scale[tile * kBlock + tok];
        } else {
            // K tile [d/8][16 tokens][8]: the unit is one chunk
            ku[i] = __builtin_nontemporal_load(reinterpret_cast<const gu32x4*>(kt) + piece * kBlock + tok);
        }
    }

    // ---- V: element (token, dim) of the tile to my[token * RS + dim * ES]
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        // piece index j*64 + lane = ((dim16 / W) * 4 + token / 4) * 16 + n
        const int pi = j * 64 + lane, n = pi & 15, tq = (pi >> 4) & 3, cq = pi >> 6;
#pragma unroll
        for (int cc = 0; cc < W; ++cc) {
            const int dim = 16 * (cq * W + cc) + n;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                unsigned char* dst = my + (4 * tq + t4) * RS + dim * ES;
                if constexpr (FP8) {
                    *dst = (unsigned char)(vp[j][cc] >> (8 * t4));
                } else {
                    const uint32_t w = vp[j][2 * cc + (t4 >> 1)];
                    *reinterpret_cast<unsigned short*>(dst) = (unsigned short)(w >> (16 * (t4 & 1)));
                }
            }
        }
    }
    // the wave reads what its own lanes wrote: order the LDS traffic, no workgroup barrier needed
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- convert and store, whole rows per instruction
#pragma unroll
    for (int i = 0; i < NU; ++i) {
        const int u = i * 64 + lane, tok = u / UPR, piece = u % UPR;
        const int j = b * kBlock + tok;                // logical token
        half8_t kh, vh;
        if constexpr (FP8) {
            const gu32x2 w = *reinterpret_cast<const gu32x2*>(my + tok * RS + piece * 8);
            kh = dequant8<KV>(ku[i].x, ku[i].y, ks[i]);
            vh = dequant8<KV>(w.x, w.y, vs[i]);
        } else {
            kh = __builtin_bit_cast(half8_t, ku[i]);
            vh = *reinterpret_cast<const half8_t*>(my + tok * RS + piece * 16);
        }
        if (j >= tok_begin && j < tok_end) {
            const size_t row = (size_t)(j - tok_begin) * H_k + head;
            __builtin_nontemporal_store(kh, reinterpret_cast<half8_t*>(k_out + row * HEAD_DIM) + piece);
            __builtin_nontemporal_store(vh, reinterpret_cast<half8_t*>(v_out + row * HEAD_DIM) + piece);
        }
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
    if (sh->kv_dtype != COOPT_KV_FP16 && (!k_scale || !v_scale)) return COOPT_ERR_NULL;
    const int first_block = tok_begin / kBlock;
    const long long tiles = (long long)((tok_end + kBlock - 1) / kBlock - first_block) * sh->num_kv_heads;
    if (tiles > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 grid((unsigned)((tiles + kGatherWaves - 1) / kGatherWaves)), block(64 * kGatherWaves);
    hipStream_t stream = (hipStream_t)hip_stream;
    const int32_t* bt_row = block_tables + (size_t)seq * sh->max_blocks_per_seq;
#define COOPT_GATHER(D, KV)                                                                        \
    hipLaunchKernelGGL((gather_cached_kv_kernel<D, KV>), grid, block, 0, stream,                   \
                       (const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale, bt_row, \
                       tok_begin, tok_end, first_block, (int)tiles, sh->num_kv_heads,              \
                       (half_t*)k_out, (half_t*)v_out)
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) COOPT_GATHER(128, COOPT_KV_E4M3);
        else COOPT_GATHER(64, COOPT_KV_E4M3);
    } else if (sh->kv_dtype == COOPT_KV_E5M2) {
        if (sh->head_dim == 128) COOPT_GATHER(128, COOPT_KV_E5M2);
        else COOPT_GATHER(64, COOPT_KV_E5M2);
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
