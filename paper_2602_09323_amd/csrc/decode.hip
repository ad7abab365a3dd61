// Paged grouped-query decode attention for gfx950 (Opt-KV Eq. 6, Opt-GQA Eq. 7-8, Opt-Pa Eq. 9-10).
//
// Work item = (sequence, KV head, token range).  A workgroup of W wavefronts owns one item; its
// waves take the item's 16-token cache blocks round-robin, each keeps a private online softmax
// (running max m, sum l, accumulator O) over its own blocks for ALL query heads of the group, and
// the waves are merged through LDS at the end.  The result is either the final fp16 output row or
// one partition's (m, l, O/l) triple for the cross-partition reduce kernel.
//
// Why matrix cores in a bandwidth-bound kernel: at group size 5 the plain-VALU form needs about
// 3-5 lane-instructions per cache byte (convert + one multiply-add per query head), which on
// 256 CUs x 64 lanes x 2.4 GHz is the same ~10 us as the HBM time of the whole step, so the loads
// cannot hide it.  The 16x16 MFMA tile does the per-byte work of all heads at once and leaves the
// VALU with one convert per two bytes plus the softmax of 4 scores per lane per block.
//
// The per-block arithmetic (two MFMA products around an in-register softmax) is in attn_tile.hpp.
#include "attn_tile.hpp"

namespace coopt {

struct DecodeArgs {
    const half_t* q;
    CacheView cv;
    const int32_t* block_tables;
    const int32_t* context_lens;
    half_t* out;          // final rows (direct mode)
    float* tmp_out;       // partition mode: [S][H_q][max_parts][d]
    float* max_logits;    //                 [S][H_q][max_parts]
    float* exp_sums;
    int32_t H_q, H_k, G;
    int32_t max_blocks;
    int32_t tokens_per_part;   // multiple of 16
    int32_t max_parts;         // parts per (seq, kv head) in the grid
    int32_t direct;            // 1: the single part writes `out`
    float scale_log2e;         // softmax_scale * log2(e)
};

template <int HEAD_DIM, int KV, int DEPTH>
__global__ void __launch_bounds__(512)
paged_decode_kernel(const DecodeArgs a)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform((int)(threadIdx.x >> 6));
    const int nwaves = blockDim.x >> 6;
    const int n = lane & 15, grp = lane >> 4;

    const int part = blockIdx.x % a.max_parts;
    const int sg = blockIdx.x / a.max_parts;
    const int g = sg % a.H_k;
    const int seq = sg / a.H_k;
    const int t = a.context_lens[seq];
    const int tok0 = part * a.tokens_per_part;
    if (tok0 >= t) {
        if (a.direct && part == 0) {                       // empty context: zero rows
            for (int i = threadIdx.x; i < a.G * HEAD_DIM; i += blockDim.x)
                a.out[((size_t)seq * a.H_q + g * a.G) * HEAD_DIM + i] = (half_t)0.0f;
        }
        return;
    }
    const int tok1 = min(t, tok0 + a.tokens_per_part);
    const int blk0 = tok0 / kBlock;
    const int nblk = (tok1 + kBlock - 1) / kBlock - blk0;
    const int nmine = wave < nblk ? (nblk - wave + nwaves - 1) / nwaves : 0;
    // this wave's blocks are blk0 + wave + i * nwaves, i < nmine
    const int32_t* bt = a.block_tables + (size_t)seq * a.max_blocks + blk0 + wave;

    // q^T operand: head slot n of this group, zero for slots beyond the group size
    half8_t qop[HEAD_DIM / 32];
    load_q_operand<HEAD_DIM, KV>(qop, a.q + ((size_t)seq * a.H_q + g * a.G + n) * HEAD_DIM,
                                 n < a.G, grp);

    float m = -INFINITY, l = 0.0f;
    floatx4 acc[HEAD_DIM / 16];
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    const TileLoader<HEAD_DIM, KV> loader(a.cv, n, grp);
    BlockRegs<HEAD_DIM, KV> regs[DEPTH];

    // Up to 64 physical block numbers are fetched with one vector load (lane i holds the i-th) and
    // handed to the scalar unit with readlane; inside a chunk the loop is a software pipeline with
    // DEPTH tiles in flight and no data-dependent branch around any load.
    for (int cb = 0; cb < nmine; cb += 64) {
        const int nc = min(64, nmine - cb);
        int idv = 0;
        if (lane < nc) idv = bt[(cb + lane) * nwaves];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const int id = __builtin_amdgcn_readlane(idv, u);
            loader.issue(regs[u], (size_t)id * a.H_k + g, u < nc);
            __builtin_amdgcn_sched_barrier(0);     // keep the stages' loads in program order
        }
        for (int i = 0; i < nc; i += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int ii = i + u;
                const int nx = ii + DEPTH;
                const int id = __builtin_amdgcn_readlane(idv, min(nx, 63));
                if (ii < nc) {
                    const int visible = t - ((blk0 + wave + (cb + ii) * nwaves) * kBlock + 4 * grp);
                    BlockOps<HEAD_DIM> ops;
                    convert_block<HEAD_DIM, KV>(ops, regs[u], visible);
                    tile_update<HEAD_DIM, KV>(ops, qop, m, l, acc, visible, a.scale_log2e);
                }
                // refill only after the stage's registers are dead, so the load can land in place
                __builtin_amdgcn_sched_barrier(0);
                loader.issue(regs[u], (size_t)id * a.H_k + g, nx < nc);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- merge the waves of the workgroup through LDS
    // smem: acc [nwaves][G][HEAD_DIM], then m [nwaves][16], then l [nwaves][16]
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    float* sm_acc = smem;
    float* sm_m = smem + nwaves * a.G * HEAD_DIM;
    float* sm_l = sm_m + nwaves * 16;
    if (n < a.G) {
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c)
            *reinterpret_cast<floatx4*>(sm_acc + ((wave * a.G + n) * HEAD_DIM + 16 * c + 4 * grp)) =
                acc[c];
    }
    if (grp == 0) {
        sm_m[wave * 16 + n] = m;
        sm_l[wave * 16 + n] = l;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < a.G * HEAD_DIM; idx += blockDim.x) {
        const int hh = idx / HEAD_DIM, dim = idx - hh * HEAD_DIM;
        float M = -INFINITY;
        for (int w = 0; w < nwaves; ++w) M = fmaxf(M, sm_m[w * 16 + hh]);
        float L = 0.0f, O = 0.0f;
        for (int w = 0; w < nwaves; ++w) {
            const float f = __builtin_amdgcn_exp2f(sm_m[w * 16 + hh] - M);  // idle waves: exp2(-inf) = 0
            L += sm_l[w * 16 + hh] * f;
            O += sm_acc[(w * a.G + hh) * HEAD_DIM + dim] * f;
        }
        const float o = O / L * out_unscale<KV>();
        const size_t row = (size_t)seq * a.H_q + g * a.G + hh;
        if (a.direct) {
            a.out[row * HEAD_DIM + dim] = (half_t)o;
        } else {
            a.tmp_out[(row * a.max_parts + part) * HEAD_DIM + dim] = o;
            if (dim == 0) {
                a.max_logits[row * a.max_parts + part] = M * kLn2;
                a.exp_sums[row * a.max_parts + part] = L;
            }
        }
    }
}

// One wavefront per (sequence, query head): M = max_p m_p, w_p = l_p exp(m_p - M),
// out = sum_p w_p o_p / sum_p w_p.  Lane i owns dims i and i+64.
template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
partition_reduce_kernel(const float* __restrict__ tmp_out, const float* __restrict__ max_logits,
                        const float* __restrict__ exp_sums, const int32_t* __restrict__ context_lens,
                        int partition_size, int max_parts, half_t* __restrict__ out, int H_q,
                        int num_rows)
{
    constexpr int E = HEAD_DIM / 64;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);        // seq * H_q + head
    if (row >= num_rows) return;
    const int lane = threadIdx.x & 63;
    const int seq = row / H_q;
    const int t = context_lens[seq];
    const int nparts = min((t + partition_size - 1) / partition_size, max_parts);
    float o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.0f;
    if (nparts > 0) {
        const float* ml = max_logits + (size_t)row * max_parts;
        const float* es = exp_sums + (size_t)row * max_parts;
        float M = -INFINITY;
        for (int p = lane; p < nparts; p += 64) M = fmaxf(M, ml[p]);
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) M = fmaxf(M, __shfl_xor(M, s));
        float W = 0.0f;
        for (int p = 0; p < nparts; ++p) {
            const float w = es[p] * __expf(ml[p] - M);
            W += w;
#pragma unroll
            for (int e = 0; e < E; ++e)
                o[e] += w * tmp_out[((size_t)row * max_parts + p) * HEAD_DIM + lane + 64 * e];
        }
        const float inv = 1.0f / W;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] *= inv;
    }
#pragma unroll
    for (int e = 0; e < E; ++e) out[(size_t)row * HEAD_DIM + lane + 64 * e] = (half_t)o[e];
}

// ------------------------------------------------------------------ host side

struct DecodePlan {
    int tokens_per_group = 256;
    int waves = 4;
    int depth = 4;
};
static DecodePlan g_plan;

template <int HEAD_DIM, int KV>
static void launch_decode_depth(const DecodeArgs& a, int depth, dim3 grid, dim3 block, size_t lds,
                                hipStream_t stream)
{
    switch (depth) {
    case 1: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 1>), grid, block, lds, stream, a); break;
    case 2: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 2>), grid, block, lds, stream, a); break;
    case 3: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 3>), grid, block, lds, stream, a); break;
    case 6: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 6>), grid, block, lds, stream, a); break;
    default: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 4>), grid, block, lds, stream, a); break;
    }
}

static size_t decode_lds_bytes(int waves, int G, int head_dim)
{
    return ((size_t)waves * G * head_dim + 2 * waves * 16) * sizeof(float);
}

static void launch_decode(const DecodeArgs& a, const coopt_shape* sh, int waves, int depth,
                          hipStream_t stream)
{
    while (waves > 1 && decode_lds_bytes(waves, a.G, sh->head_dim) > 48 * 1024) waves /= 2;
    const dim3 grid((unsigned)((long long)sh->num_seqs * sh->num_kv_heads * a.max_parts));
    const dim3 block(64 * waves);
    const size_t lds = decode_lds_bytes(waves, a.G, sh->head_dim);
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) launch_decode_depth<128, COOPT_KV_E4M3>(a, depth, grid, block, lds, stream);
        else launch_decode_depth<64, COOPT_KV_E4M3>(a, depth, grid, block, lds, stream);
    } else {
        if (sh->head_dim == 128) launch_decode_depth<128, COOPT_KV_FP16>(a, depth, grid, block, lds, stream);
        else launch_decode_depth<64, COOPT_KV_FP16>(a, depth, grid, block, lds, stream);
    }
}

static void launch_reduce(const float* tmp_out, const float* max_logits, const float* exp_sums,
                          const int32_t* context_lens, int partition_size, int max_parts,
                          void* out, const coopt_shape* sh, hipStream_t stream)
{
    const int rows = sh->num_seqs * sh->num_q_heads;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (sh->head_dim == 128)
        hipLaunchKernelGGL(partition_reduce_kernel<128>, grid, block, 0, stream, tmp_out, max_logits,
                           exp_sums, context_lens, partition_size, max_parts, (half_t*)out,
                           sh->num_q_heads, rows);
    else
        hipLaunchKernelGGL(partition_reduce_kernel<64>, grid, block, 0, stream, tmp_out, max_logits,
                           exp_sums, context_lens, partition_size, max_parts, (half_t*)out,
                           sh->num_q_heads, rows);
}

static DecodeArgs make_args(const void* q, const void* k_cache, const void* v_cache,
                            const float* k_scale, const float* v_scale,
                            const int32_t* block_tables, const int32_t* context_lens,
                            const coopt_shape* sh)
{
    DecodeArgs a{};
    a.q = (const half_t*)q;
    a.cv = CacheView{(const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale};
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.H_q = sh->num_q_heads;
    a.H_k = sh->num_kv_heads;
    a.G = sh->num_q_heads / sh->num_kv_heads;
    a.max_blocks = sh->max_blocks_per_seq;
    a.scale_log2e = sh->softmax_scale * kLog2e;
    return a;
}

static int check_decode_ptrs(const void* q, const void* k_cache, const void* v_cache,
                             const float* k_scale, const float* v_scale, const int32_t* bt,
                             const int32_t* cl, const coopt_shape* sh)
{
    if (!q || !k_cache || !v_cache || !bt || !cl) return COOPT_ERR_NULL;
    if (sh->kv_dtype == COOPT_KV_E4M3 && (!k_scale || !v_scale)) return COOPT_ERR_NULL;
    return COOPT_OK;
}

static int parts_for(const coopt_shape* sh, int tokens_per_part)
{
    const long long max_tokens = (long long)sh->max_blocks_per_seq * kBlock;
    return (int)((max_tokens + tokens_per_part - 1) / tokens_per_part);
}

}  // namespace coopt

using namespace coopt;

extern "C" int coopt_set_decode_plan(int32_t tokens_per_group, int32_t waves, int32_t depth)
{
    if (tokens_per_group < 0 || tokens_per_group % kBlock != 0) return COOPT_ERR_SHAPE;
    if (waves != 0 && waves != 1 && waves != 2 && waves != 4 && waves != 8) return COOPT_ERR_SHAPE;
    if (depth != 0 && depth != 1 && depth != 2 && depth != 3 && depth != 4 && depth != 6)
        return COOPT_ERR_SHAPE;
    if (tokens_per_group) g_plan.tokens_per_group = tokens_per_group;
    if (waves) g_plan.waves = waves;
    if (depth) g_plan.depth = depth;
    return COOPT_OK;
}

extern "C" void coopt_get_decode_plan(int32_t* tokens_per_group, int32_t* waves, int32_t* depth)
{
    if (tokens_per_group) *tokens_per_group = g_plan.tokens_per_group;
    if (waves) *waves = g_plan.waves;
    if (depth) *depth = g_plan.depth;
}

extern "C" size_t coopt_decode_workspace_bytes(const coopt_shape* sh)
{
    if (check_shape(sh) != COOPT_OK) return 0;
    const size_t parts = (size_t)parts_for(sh, g_plan.tokens_per_group);
    return (size_t)sh->num_seqs * sh->num_q_heads * parts * (sh->head_dim + 2) * sizeof(float);
}

extern "C" int coopt_paged_gqa_decode(const void* q, const void* k_cache, const void* v_cache,
                                      const float* k_scale, const float* v_scale,
                                      const int32_t* block_tables, const int32_t* context_lens,
                                      void* out, void* workspace, size_t workspace_bytes,
                                      const coopt_shape* sh, void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    if (st != COOPT_OK) return st;
    if (!out) return COOPT_ERR_NULL;
    hipStream_t stream = (hipStream_t)hip_stream;
    DecodeArgs a = make_args(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    a.out = (half_t*)out;
    const int parts = workspace ? parts_for(sh, g_plan.tokens_per_group) : 1;
    if (parts == 1) {
        // one workgroup per (sequence, KV head) covers the whole context and writes `out`
        a.tokens_per_part = sh->max_blocks_per_seq * kBlock;
        a.max_parts = 1;
        a.direct = 1;
        launch_decode(a, sh, workspace ? g_plan.waves : 8, g_plan.depth, stream);
        return launch_status();
    }
    if (workspace_bytes < coopt_decode_workspace_bytes(sh)) return COOPT_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 15u) != 0) return COOPT_ERR_WORKSPACE;
    const size_t rows = (size_t)sh->num_seqs * sh->num_q_heads;
    a.tmp_out = (float*)workspace;
    a.max_logits = a.tmp_out + rows * parts * sh->head_dim;
    a.exp_sums = a.max_logits + rows * parts;
    a.tokens_per_part = g_plan.tokens_per_group;
    a.max_parts = parts;
    a.direct = 0;
    launch_decode(a, sh, g_plan.waves, g_plan.depth, stream);
    st = launch_status();
    if (st != COOPT_OK) return st;
    launch_reduce(a.tmp_out, a.max_logits, a.exp_sums, context_lens, a.tokens_per_part, parts, out,
                  sh, stream);
    return launch_status();
}

extern "C" int coopt_paged_gqa_decode_partitioned(
    const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
    const float* v_scale, const int32_t* block_tables, const int32_t* context_lens,
    int32_t partition_size, float* tmp_out, float* max_logits, float* exp_sums, int32_t max_parts,
    const coopt_shape* sh, void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (partition_size <= 0 || partition_size % kBlock != 0 || max_parts <= 0)
        return COOPT_ERR_SHAPE;
    if (sh->num_seqs == 0) return COOPT_OK;
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    if (st != COOPT_OK) return st;
    if (!tmp_out || !max_logits || !exp_sums) return COOPT_ERR_NULL;
    if (max_parts < parts_for(sh, partition_size)) return COOPT_ERR_WORKSPACE;
    DecodeArgs a = make_args(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    a.tmp_out = tmp_out;
    a.max_logits = max_logits;
    a.exp_sums = exp_sums;
    a.tokens_per_part = partition_size;
    a.max_parts = max_parts;
    a.direct = 0;
    launch_decode(a, sh, g_plan.waves, g_plan.depth, (hipStream_t)hip_stream);
    return launch_status();
}

extern "C" int coopt_paged_gqa_reduce(const float* tmp_out, const float* max_logits,
                                      const float* exp_sums, const int32_t* context_lens,
                                      int32_t partition_size, int32_t max_parts, void* out,
                                      const coopt_shape* sh, void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (partition_size <= 0 || max_parts <= 0) return COOPT_ERR_SHAPE;
    if (sh->num_seqs == 0) return COOPT_OK;
    if (!tmp_out || !max_logits || !exp_sums || !context_lens || !out) return COOPT_ERR_NULL;
    launch_reduce(tmp_out, max_logits, exp_sums, context_lens, partition_size, max_parts, out, sh,
                  (hipStream_t)hip_stream);
    return launch_status();
}
