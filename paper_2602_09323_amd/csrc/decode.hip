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
#include <atomic>

#include "attn_tile.hpp"
#include "decode_internal.hpp"

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
    int32_t num_seqs, H_q, H_k, G;
    int32_t max_blocks;
    int32_t tokens_per_part;   // multiple of 16
    int32_t max_parts;         // parts per (seq, kv head) in the grid
    int32_t direct;            // 1: the single part writes `out`
    int32_t pool_tiles;        // num_blocks * H_k
    float scale_log2e;         // softmax_scale * log2(e)
};

template <int HEAD_DIM, int KV, int DEPTH, bool BIG>
__global__ void __launch_bounds__(512)
paged_decode_kernel(const DecodeArgs a)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform((int)(threadIdx.x >> 6));
    const int nwaves = blockDim.x >> 6;
    const int n = lane & 15, grp = lane >> 4;

    // Work item order: token range slowest, then sequence, then KV head.  Consecutive workgroup
    // ids land on different XCDs, so each XCD gets every 8th (sequence, head) pair of every token
    // range instead of one token range of all of them, and the ranges that can be empty (beyond
    // the shorter contexts) sit at the end of the grid.  (Dealing the items to the XCDs two at a
    // time, so that neighbouring KV heads -- whose scale rows share 128-byte lines -- meet in one
    // L2, did not change this kernel's time.)
    const int g = blockIdx.x % a.H_k;
    const int sp = blockIdx.x / a.H_k;
    const int seq = sp % a.num_seqs;
    const int part = sp / a.num_seqs;
    const int tok0 = part * a.tokens_per_part;
    const int blk0 = tok0 / kBlock;

    // The first 64 block numbers of this wave are fetched before the context length is known
    // (bounded by the table row), so that the two loads overlap.  This wave's blocks are
    // blk0 + wave + i * nwaves.
    const int32_t* bt = a.block_tables + (size_t)seq * a.max_blocks;
    int idv = 0;
    {
        const int b = blk0 + wave + lane * nwaves;
        if (b < a.max_blocks) idv = bt[b];
    }
    const int t = a.context_lens[seq];
    if (tok0 >= t) {
        if (a.direct && part == 0) {                       // empty context: zero rows
            for (int i = threadIdx.x; i < a.G * HEAD_DIM; i += blockDim.x)
                a.out[((size_t)seq * a.H_q + g * a.G) * HEAD_DIM + i] = (half_t)0.0f;
        }
        return;
    }
    const int tok1 = min(t, tok0 + a.tokens_per_part);
    const int nblk = (tok1 + kBlock - 1) / kBlock - blk0;
    const int nmine = wave < nblk ? (nblk - wave + nwaves - 1) / nwaves : 0;

    // q^T operand: head slot n of this group, zero for slots beyond the group size
    half8_t qop[HEAD_DIM / 32];
    load_q_operand<HEAD_DIM, KV>(qop, a.q + ((size_t)seq * a.H_q + g * a.G + n) * HEAD_DIM,
                                 n < a.G, grp);

    float m = -INFINITY, l = 0.0f;
    floatx4 acc[HEAD_DIM / 16];
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    const TileLoader<HEAD_DIM, KV, BIG> loader(a.cv, lane, a.pool_tiles);
    BlockRegs<HEAD_DIM, KV> regs[DEPTH][2];

    // Blocks are consumed in groups of two.  Inside a chunk of 64 blocks (32 groups) the loop is a
    // software pipeline with DEPTH groups in flight and no data-dependent branch around any load;
    // block numbers reach the scalar unit by readlane from the vector fetched above.
    for (int cb = 0; cb < nmine; cb += 64) {
        if (cb > 0) {
            idv = 0;
            if (cb + lane < nmine) idv = bt[blk0 + wave + (cb + lane) * nwaves];
        }
        const int nc = min(64, nmine - cb);          // blocks in this chunk
        const int ng = (nc + 1) >> 1;                // groups in this chunk
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int id = __builtin_amdgcn_readlane(idv, 2 * u + h);
                loader.issue(regs[u][h], id * a.H_k + g, 2 * u + h < nc);
            }
            __builtin_amdgcn_sched_barrier(0);     // keep the stages' loads in program order
        }
        for (int i = 0; i < ng; i += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int gi = i + u;                // group index within the chunk
                if (gi < ng) {
                    // tokens of this lane in blocks A and B of the group, relative to the context end
                    const int baseA = (blk0 + wave + (cb + 2 * gi) * nwaves) * kBlock;   // uniform
                    const int visA = t - baseA - 4 * grp;
                    const int visB = (2 * gi + 1 < nc) ? visA - nwaves * kBlock : 0;
                    const bool tail = (2 * gi + 1 >= nc) || (baseA + (nwaves + 1) * kBlock > t);
                    group_update<HEAD_DIM, KV>(regs[u][0], regs[u][1], qop, m, l, acc, tail, visA,
                                               visB, visA, visB, a.scale_log2e);
                }
                // refill only after the stage's registers are dead, so the loads can land in place
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int nb = 2 * (gi + DEPTH) + h;
                    const int id = __builtin_amdgcn_readlane(idv, min(nb, 63));
                    loader.issue(regs[u][h], id * a.H_k + g, nb < nc);
                }
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
            const float f = __builtin_amdgcn_exp2f(sm_m[w * 16 + hh] - M);  // idle waves: 0
            L += sm_l[w * 16 + hh] * f;
            O += sm_acc[(w * a.G + hh) * HEAD_DIM + dim] * f;
        }
        const float o = O / L;                           // the common power of two of O and L cancels
        const size_t row = (size_t)seq * a.H_q + g * a.G + hh;
        if (a.direct) {
            a.out[row * HEAD_DIM + dim] = (half_t)o;
        } else {
            a.tmp_out[(row * a.max_parts + part) * HEAD_DIM + dim] = o;
            if (dim == 0) {
                a.max_logits[row * a.max_parts + part] = M * kLn2;
                a.exp_sums[row * a.max_parts + part] = L * kPUnshiftOf<KV>;
            }
        }
    }
}

// One workgroup of 4 wavefronts per (sequence, query head) row: M = max_p m_p,
// w_p = l_p exp(m_p - M), out = sum_p w_p o_p / sum_p w_p.  Every wave derives M and the weights
// (a row has few partials); the partial rows are dealt to the waves, read with independent
// 16-byte loads (HEAD_DIM/4 lanes per row, so one wave-wide load covers 2 or 4 partials), and the
// four waves' sums meet in LDS.  A slot beyond the row's partial count is replaced by partial 0
// with weight 0, so memory nobody wrote is never read.
template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
partition_reduce_kernel(const float* __restrict__ tmp_out, const float* __restrict__ max_logits,
                        const float* __restrict__ exp_sums, const int32_t* __restrict__ context_lens,
                        int partition_size, int max_parts, half_t* __restrict__ out, int H_q)
{
    constexpr int LPR = HEAD_DIM / 4;          // lanes per partial row
    constexpr int PPW = 64 / LPR;              // partial rows per wave-wide load
    __shared__ float sm[4][HEAD_DIM];
    const int row = blockIdx.x;                // seq * H_q + head
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sub = lane / LPR, piece = lane % LPR;
    const int seq = row / H_q;
    half_t* out_row = out + (size_t)row * HEAD_DIM;
    const float* ml = max_logits + (size_t)row * max_parts;
    const float* es = exp_sums + (size_t)row * max_parts;
    const float* po = tmp_out + (size_t)row * max_parts * HEAD_DIM + 4 * piece;
    // Everything whose address does not depend on the length is asked for before the length is
    // back: the first 64 (max, sum) pairs and this lane's rows of the first 64 partials (slots
    // beyond the sequence's partitions hold whatever the caller left there: selected away below).
    constexpr int kRows = 64 / (4 * PPW);       // rows per lane and 64 partials
    const int t = context_lens[seq];
    const float ml0 = lane < max_parts ? ml[lane] : -INFINITY;
    const float es0 = lane < max_parts ? es[lane] : 0.0f;
    floatx4 x0[kRows];
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        const int j = (i * 4 + wave) * PPW + sub;
        x0[i] = *reinterpret_cast<const floatx4*>(po + (size_t)min(j, max_parts - 1) * HEAD_DIM);
    }
    const int nparts = min((t + partition_size - 1) / partition_size, max_parts);
    if (nparts <= 0) {                         // the whole workgroup takes this branch together
        if (threadIdx.x < HEAD_DIM) out_row[threadIdx.x] = (half_t)0.0f;
        return;
    }

    float M = lane < nparts ? ml0 : -INFINITY;
    for (int p = 64 + lane; p < nparts; p += 64) M = fmaxf(M, ml[p]);
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) M = fmaxf(M, __shfl_xor(M, s));
    floatx4 o = {0.f, 0.f, 0.f, 0.f};
    float W = 0.0f;
    for (int base = 0; base < nparts; base += 64) {
        const int p = base + lane;
        float wv = 0.0f;                                                   // weight of partial base+lane
        if (p < nparts) wv = base == 0 ? es0 * __expf(ml0 - M) : es[p] * __expf(ml[p] - M);
        W += wv;
        const int cnt = min(64, nparts - base);
#pragma unroll
        for (int i = 0; i < kRows; ++i) {
            const int j = (i * 4 + wave) * PPW + sub;                      // < 64
            const float wj = __shfl(wv, j);
            const bool ok = j < cnt;
            floatx4 x;
            if (base == 0) {
                x = x0[i];
            } else {
                x = *reinterpret_cast<const floatx4*>(po + (size_t)(base + (ok ? j : 0)) * HEAD_DIM);
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] += ok ? x[c] * wj : 0.0f;     // (an unused slot may hold NaN)
        }
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) W += __shfl_xor(W, s);
#pragma unroll
    for (int s = LPR; s < 64; s <<= 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] += __shfl_xor(o[i], s);
    }
    if (sub == 0) *reinterpret_cast<floatx4*>(&sm[wave][4 * piece]) = o;
    __syncthreads();
    if (threadIdx.x < HEAD_DIM) {
        const int dim = threadIdx.x;
        const float v = sm[0][dim] + sm[1][dim] + sm[2][dim] + sm[3][dim];
        out_row[dim] = (half_t)(v / W);
    }
}

// ------------------------------------------------------------------ host side

template <int HEAD_DIM, int KV, bool BIG>
static void launch_decode_depth(const DecodeArgs& a, int depth, dim3 grid, dim3 block, size_t lds,
                                hipStream_t stream)
{
    switch (depth) {
    case 1: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 1, BIG>), grid, block, lds, stream, a); break;
    case 3: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 3, BIG>), grid, block, lds, stream, a); break;
    default: hipLaunchKernelGGL((paged_decode_kernel<HEAD_DIM, KV, 2, BIG>), grid, block, lds, stream, a); break;
    }
}

template <int HEAD_DIM, int KV>
static void launch_decode_pool(const DecodeArgs& a, bool big, int depth, dim3 grid, dim3 block,
                               size_t lds, hipStream_t stream)
{
    if (big) launch_decode_depth<HEAD_DIM, KV, true>(a, depth, grid, block, lds, stream);
    else launch_decode_depth<HEAD_DIM, KV, false>(a, depth, grid, block, lds, stream);
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
    const bool big = !pool_fits_small(sh);
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) launch_decode_pool<128, COOPT_KV_E4M3>(a, big, depth, grid, block, lds, stream);
        else launch_decode_pool<64, COOPT_KV_E4M3>(a, big, depth, grid, block, lds, stream);
    } else if (sh->kv_dtype == COOPT_KV_E5M2) {
        if (sh->head_dim == 128) launch_decode_pool<128, COOPT_KV_E5M2>(a, big, depth, grid, block, lds, stream);
        else launch_decode_pool<64, COOPT_KV_E5M2>(a, big, depth, grid, block, lds, stream);
    } else {
        if (sh->head_dim == 128) launch_decode_pool<128, COOPT_KV_FP16>(a, big, depth, grid, block, lds, stream);
        else launch_decode_pool<64, COOPT_KV_FP16>(a, big, depth, grid, block, lds, stream);
    }
}

static void launch_reduce(const float* tmp_out, const float* max_logits, const float* exp_sums,
                          const int32_t* context_lens, int partition_size, int max_parts,
                          void* out, const coopt_shape* sh, hipStream_t stream)
{
    const int rows = sh->num_seqs * sh->num_q_heads;
    const dim3 grid((unsigned)rows), block(256);
    if (sh->head_dim == 128)
        hipLaunchKernelGGL(partition_reduce_kernel<128>, grid, block, 0, stream, tmp_out, max_logits,
                           exp_sums, context_lens, partition_size, max_parts, (half_t*)out,
                           sh->num_q_heads);
    else
        hipLaunchKernelGGL(partition_reduce_kernel<64>, grid, block, 0, stream, tmp_out, max_logits,
                           exp_sums, context_lens, partition_size, max_parts, (half_t*)out,
                           sh->num_q_heads);
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
    a.num_seqs = sh->num_seqs;
    a.H_q = sh->num_q_heads;
    a.H_k = sh->num_kv_heads;
    a.G = sh->num_q_heads / sh->num_kv_heads;
    a.max_blocks = sh->max_blocks_per_seq;
    a.pool_tiles = sh->num_blocks * sh->num_kv_heads;
    a.scale_log2e = sh->softmax_scale * kLog2e;
    return a;
}

static int check_decode_ptrs(const void* q, const void* k_cache, const void* v_cache,
                             const float* k_scale, const float* v_scale, const int32_t* bt,
                             const int32_t* cl, const coopt_shape* sh)
{
    if (!q || !k_cache || !v_cache || !bt || !cl) return COOPT_ERR_NULL;
    if (sh->kv_dtype != COOPT_KV_FP16 && (!k_scale || !v_scale)) return COOPT_ERR_NULL;
    return COOPT_OK;
}

static int parts_for(const coopt_shape* sh, int tokens_per_part)
{
    const long long max_tokens = (long long)sh->max_blocks_per_seq * kBlock;
    return (int)((max_tokens + tokens_per_part - 1) / tokens_per_part);
}

}  // namespace coopt

using namespace coopt;

// Wavefronts that fill the current device once: one per SIMD, four SIMDs per compute unit.  The
// compute-unit count is asked of the runtime once per device and kept (256 on MI355X; also the
// answer where no device can be asked, e.g. size queries on a machine without a GPU).
static int device_simd_count()
{
    static std::atomic<int> known[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 4 * 256;
    }
    const int slot = dev >= 0 && dev < 64 ? dev : 63;
    int v = known[slot].load(std::memory_order_relaxed);
    if (v == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        }
        v = 4 * cus;
        known[slot].store(v, std::memory_order_relaxed);
    }
    return v;
}

static int check_plan(const coopt_decode_plan* p)
{
    if (p->tokens_per_group <= 0 || p->tokens_per_group % (2 * kBlock) != 0) return COOPT_ERR_SHAPE;
    const int w = p->waves_per_group;
    if (w != 1 && w != 2 && w != 4 && w != 8) return COOPT_ERR_SHAPE;
    if (p->pipeline_depth < 1 || p->pipeline_depth > 3) return COOPT_ERR_SHAPE;
    if (p->grid_waves <= 0 || p->grid_waves > (1 << 20)) return COOPT_ERR_SHAPE;
    if (p->softmax_reduction != 0 && p->softmax_reduction != 1) return COOPT_ERR_SHAPE;
    return COOPT_OK;
}

extern "C" void coopt_default_decode_plan(coopt_decode_plan* p)
{
    if (!p) return;
    p->tokens_per_group = 128;
    p->waves_per_group = 1;
    p->pipeline_depth = 2;
    p->grid_waves = device_simd_count();
    p->softmax_reduction = 0;
}

// The plan a call runs under: the caller's (validated), or the default for the current device.
static int resolve_plan(const coopt_decode_plan* given, coopt_decode_plan* plan)
{
    if (given) {
        *plan = *given;
        return check_plan(plan);
    }
    coopt_default_decode_plan(plan);
    return COOPT_OK;
}

static FlatPlan flat_plan(const coopt_decode_plan& p)
{
    return FlatPlan{p.tokens_per_group, p.pipeline_depth, p.grid_waves, p.softmax_reduction};
}

// Shape, plan and the workspace's size and alignment, for the entry points of the balanced path.
static int check_balanced(const coopt_shape* sh, const coopt_decode_plan* given,
                          coopt_decode_plan* plan, const void* workspace, size_t workspace_bytes)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    st = resolve_plan(given, plan);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    if (!workspace) return COOPT_ERR_NULL;
    if (workspace_bytes < flat_workspace_bytes(sh, flat_plan(*plan))) return COOPT_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 15u) != 0) return COOPT_ERR_WORKSPACE;
    return COOPT_OK;
}

extern "C" size_t coopt_decode_workspace_bytes(const coopt_shape* sh, const coopt_decode_plan* given)
{
    coopt_decode_plan plan;
    if (check_shape(sh) != COOPT_OK || resolve_plan(given, &plan) != COOPT_OK) return 0;
    return flat_workspace_bytes(sh, flat_plan(plan));
}

extern "C" int coopt_paged_gqa_decode(const void* q, const void* k_cache, const void* v_cache,
                                      const float* k_scale, const float* v_scale,
                                      const int32_t* block_tables, const int32_t* context_lens,
                                      void* out, void* workspace, size_t workspace_bytes,
                                      const coopt_decode_plan* given, const coopt_shape* sh,
                                      void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    st = resolve_plan(given, &plan);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    if (st != COOPT_OK) return st;
    if (!out) return COOPT_ERR_NULL;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (!workspace) {
        // one workgroup per (sequence, KV head) covers the whole context and writes `out`
        DecodeArgs a = make_args(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
        a.out = (half_t*)out;
        a.tokens_per_part = sh->max_blocks_per_seq * kBlock;
        a.max_parts = 1;
        a.direct = 1;
        launch_decode(a, sh, 8, plan.pipeline_depth, stream);
        return launch_status();
    }
    st = check_balanced(sh, given, &plan, workspace, workspace_bytes);
    if (st != COOPT_OK) return st;
    st = launch_flat_split(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                           workspace, sh, flat_plan(plan), stream);
    if (st != COOPT_OK) return st;
    return launch_flat_merge(context_lens, workspace, out, sh, flat_plan(plan), stream);
}

// ---- a decode entry point that allocates nothing and takes no workspace
//
// The partial results of the balanced split live in a file-scope device array.  In host code the
// array's name is only a stand-in: its device address is asked of the runtime once per device
// (each GPU holds its own copy at its own address) and that pointer is what the kernels get.
constexpr size_t kBuiltinWorkspaceBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kBuiltinWorkspaceBytes];

static int builtin_workspace(void** workspace)
{
    static std::atomic<void*> known[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return COOPT_ERR_LAUNCH;
    }
    if (dev < 0 || dev >= 64) return COOPT_ERR_SHAPE;
    void* p = known[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return COOPT_ERR_LAUNCH;
        }
        known[dev].store(p, std::memory_order_release);
    }
    *workspace = p;
    return COOPT_OK;
}

extern "C" size_t coopt_decode_builtin_workspace_bytes(void) { return kBuiltinWorkspaceBytes; }

extern "C" int coopt_paged_gqa_decode_noalloc(const void* q, const void* k_cache, const void* v_cache,
                                              const float* k_scale, const float* v_scale,
                                              const int32_t* block_tables,
                                              const int32_t* context_lens, void* out,
                                              const coopt_decode_plan* given, const coopt_shape* sh,
                                              void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    st = resolve_plan(given, &plan);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    if (st != COOPT_OK) return st;
    if (!out) return COOPT_ERR_NULL;
    // the partials of this shape and plan must fit the array
    if (flat_workspace_bytes(sh, flat_plan(plan)) > kBuiltinWorkspaceBytes) return COOPT_ERR_WORKSPACE;
    void* workspace = nullptr;
    st = builtin_workspace(&workspace);
    if (st != COOPT_OK) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    // nothing in the workspace has to start at zero: the split kernel writes the tag, every count
    // and every partial that the merge kernel reads
    st = launch_flat_split(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                           workspace, sh, flat_plan(plan), stream);
    if (st != COOPT_OK) return st;
    return launch_flat_merge(context_lens, workspace, out, sh, flat_plan(plan), stream);
}

extern "C" int coopt_paged_gqa_decode_step(const void* k, const void* v,
                                           const int64_t* slot_mapping, const void* q,
                                           void* k_cache, void* v_cache, float* k_scale,
                                           float* v_scale, const int32_t* block_tables,
                                           const int32_t* context_lens, void* out, void* workspace,
                                           size_t workspace_bytes, const coopt_decode_plan* given,
                                           const coopt_shape* sh, void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_balanced(sh, given, &plan, workspace, workspace_bytes);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    if (!k || !v || !slot_mapping) return COOPT_ERR_NULL;
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    if (st != COOPT_OK) return st;
    if (!out) return COOPT_ERR_NULL;
    hipStream_t stream = (hipStream_t)hip_stream;
    const FlatAppend append{k, v, slot_mapping};
    const FlatCacheW cache{k_cache, v_cache, k_scale, v_scale};
    st = launch_flat_split(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                           workspace, sh, flat_plan(plan), stream, &append);
    if (st != COOPT_OK) return st;
    return launch_flat_merge(context_lens, workspace, out, sh, flat_plan(plan), stream, nullptr, false,
                             &append, &cache);
}

extern "C" size_t coopt_decode_schedule_bytes(const coopt_shape* sh, const coopt_decode_plan* given)
{
    coopt_decode_plan plan;
    if (check_shape(sh) != COOPT_OK || resolve_plan(given, &plan) != COOPT_OK) return 0;
    return flat_schedule_bytes(sh, flat_plan(plan));
}

extern "C" int coopt_decode_schedule_prepare(const int32_t* block_tables,
                                             const int32_t* context_lens,
                                             const int64_t* slot_mapping, void* schedule,
                                             size_t schedule_bytes, const coopt_decode_plan* given,
                                             const coopt_shape* sh, void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    st = resolve_plan(given, &plan);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    if (!block_tables || !context_lens || !schedule) return COOPT_ERR_NULL;
    const size_t need = flat_schedule_bytes(sh, flat_plan(plan));
    if (need == 0) return COOPT_ERR_SHAPE;
    if (schedule_bytes < need || ((uintptr_t)schedule & 15u) != 0) return COOPT_ERR_WORKSPACE;
    return launch_flat_prepare(block_tables, context_lens, slot_mapping, schedule, sh, flat_plan(plan),
                               (hipStream_t)hip_stream);
}

extern "C" int coopt_paged_gqa_decode_scheduled(const void* k, const void* v,
                                                const int64_t* slot_mapping, const void* q,
                                                void* k_cache, void* v_cache, float* k_scale,
                                                float* v_scale, const int32_t* context_lens,
                                                void* out, void* workspace, size_t workspace_bytes,
                                                const void* schedule, size_t schedule_bytes,
                                                const coopt_decode_plan* given,
                                                const coopt_shape* sh, void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_balanced(sh, given, &plan, workspace, workspace_bytes);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    const bool fused = k || v || slot_mapping;
    if (fused && (!k || !v || !slot_mapping)) return COOPT_ERR_NULL;
    // no block table here: the schedule's records name the tiles
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, context_lens, context_lens, sh);
    if (st != COOPT_OK) return st;
    if (!schedule) return COOPT_ERR_NULL;
    const size_t need = flat_schedule_bytes(sh, flat_plan(plan));
    if (need == 0) return COOPT_ERR_SHAPE;
    if (schedule_bytes < need || ((uintptr_t)schedule & 15u) != 0) return COOPT_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    const FlatAppend append{k, v, slot_mapping};
    st = launch_flat_split(q, k_cache, v_cache, k_scale, v_scale, nullptr, context_lens, workspace,
                           sh, flat_plan(plan), stream, fused ? &append : nullptr, schedule);
    if (st != COOPT_OK || !out) return st;
    const FlatCacheW cache{k_cache, v_cache, k_scale, v_scale};
    return launch_flat_merge(context_lens, workspace, out, sh, flat_plan(plan), stream, schedule, fused,
                             fused ? &append : nullptr, &cache);
}

extern "C" int coopt_paged_gqa_decode_split(const void* q, const void* k_cache, const void* v_cache,
                                            const float* k_scale, const float* v_scale,
                                            const int32_t* block_tables,
                                            const int32_t* context_lens, void* workspace,
                                            size_t workspace_bytes, const coopt_decode_plan* given,
                                            const coopt_shape* sh, void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_balanced(sh, given, &plan, workspace, workspace_bytes);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    st = check_decode_ptrs(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, sh);
    if (st != COOPT_OK) return st;
    return launch_flat_split(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens,
                             workspace, sh, flat_plan(plan), (hipStream_t)hip_stream);
}

extern "C" int coopt_paged_gqa_decode_merge(const int32_t* context_lens, const void* workspace,
                                            size_t workspace_bytes, void* out,
                                            const coopt_decode_plan* given, const coopt_shape* sh,
                                            void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_balanced(sh, given, &plan, workspace, workspace_bytes);
    if (st != COOPT_OK) return st;
    if (sh->num_seqs == 0) return COOPT_OK;
    if (!context_lens || !out) return COOPT_ERR_NULL;
    return launch_flat_merge(context_lens, const_cast<void*>(workspace), out, sh, flat_plan(plan),
                             (hipStream_t)hip_stream);
}

extern "C" int coopt_paged_gqa_decode_partitioned(
    const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
    const float* v_scale, const int32_t* block_tables, const int32_t* context_lens,
    int32_t partition_size, float* tmp_out, float* max_logits, float* exp_sums, int32_t max_parts,
    const coopt_decode_plan* given, const coopt_shape* sh, void* hip_stream)
{
    coopt_decode_plan plan;
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    st = resolve_plan(given, &plan);
    if (st != COOPT_OK) return st;
    if (partition_size <= 0 || partition_size % kBlock != 0 || max_parts <= 0)
        return COOPT_ERR_SHAPE;
    if ((long long)sh->num_seqs * sh->num_kv_heads * max_parts > 0x7fffffffLL - 16) return COOPT_ERR_SHAPE;
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
    launch_decode(a, sh, plan.waves_per_group, plan.pipeline_depth, (hipStream_t)hip_stream);
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
