// Load-balanced paged grouped-query decode attention for gfx950: the kernel behind
// coopt_paged_gqa_decode when a workspace is given (Opt-KV Eq. 6, Opt-GQA Eq. 7-8, Opt-Pa Eq. 9-10).
//
// Decode is a stream of ~2 KB tiles read once, so the kernel is organised around keeping as many
// tile loads in flight as early as possible and ending all workgroups at the same time:
//
//   * The work of the whole batch is flattened into one sequence of two-block groups, ordered
//     [sequence][KV head][group], and cut into equal contiguous shares, one per workgroup
//     (share = max(min_share, ceil(total / workgroups))).  Context lengths live on the device, so
//     every workgroup derives the schedule itself: one vector load of the lengths and a wave scan.
//     There are no empty or short workgroups, and consecutive workgroup ids (which land on
//     different XCDs) carry equal work.
//   * A share may straddle the boundary between two (sequence, KV head) pairs.  It is processed as
//     segments, one per pair; a segment's groups go round-robin to the waves of the workgroup,
//     each wave runs the software-pipelined group loop over its own, and the waves are merged
//     through LDS into ONE partial (m, l, o) per segment.
//   * Partial j of a pair is written by workgroup first_wg(pair) + j, and the pair's first
//     workgroup also records how many partials the pair gets; the merge kernel combines them into
//     the fp16 output rows.
//
// The per-group arithmetic is in attn_tile.hpp.
#include "attn_tile.hpp"
#include "decode_internal.hpp"
#include "partials.hpp"

namespace coopt {

__device__ __forceinline__ int groups_of(int context_len)
{
    const int nb = (context_len + kBlock - 1) / kBlock;
    return (nb + 1) >> 1;
}

// Inclusive prefix sum over the 64 lanes on the vector ALU (DPP row shifts, then the two row
// broadcasts that carry a row's total into the following rows); no LDS round trips.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

// The flattened schedule, derived identically by every wavefront that needs it.
struct FlatSchedule {
    const int32_t* lens;
    int S, H_k, lane;
    // cache of the first 64 sequences (the whole batch when S <= 64)
    int t0, incl0, total0;

    __device__ __forceinline__ FlatSchedule(const int32_t* context_lens, int num_seqs, int kv_heads,
                                            int lane_id)
        : lens(context_lens), S(num_seqs), H_k(kv_heads), lane(lane_id)
    {
        t0 = lane < S ? lens[lane] : 0;
        incl0 = wave_inclusive_scan(H_k * groups_of(t0));
        total0 = __builtin_amdgcn_readlane(incl0, 63);
    }

    // Groups (times KV heads) of the whole batch.
    __device__ __forceinline__ int total() const
    {
        int sum = total0;
        for (int base = 64; base < S; base += 64) {
            const int t = base + lane < S ? lens[base + lane] : 0;
            int v = H_k * groups_of(t);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
            sum += wave_uniform(v);      // equal in all lanes; tell the compiler so
        }
        return sum;
    }

    // Sequence that owns flattened group x (x < total): its index, the flattened index of its
    // first group, and its context length.  All results are wave-uniform.
    __device__ __forceinline__ void locate(int x, int& seq, int& first, int& t) const
    {
        int carry = 0, tl = t0, incl = incl0, tile_total = total0;
        for (int base = 0;; base += 64) {
            if (base > 0) {
                tl = base + lane < S ? lens[base + lane] : 0;
                incl = wave_inclusive_scan(H_k * groups_of(tl));
                tile_total = __builtin_amdgcn_readlane(incl, 63);
            }
            if (x < carry + tile_total || base + 64 >= S) {
                const unsigned long long before = __builtin_amdgcn_ballot_w64(carry + incl <= x);
                const int idx = min(__builtin_popcountll(before), 63);
                seq = min(base + idx, S - 1);
                t = __builtin_amdgcn_readlane(tl, idx);
                first = carry + __builtin_amdgcn_readlane(incl - H_k * groups_of(tl), idx);
                return;
            }
            carry += tile_total;
        }
    }
};

struct FlatArgs {
    const half_t* q;
    CacheView cv;
    const int32_t* block_tables;
    const int32_t* context_lens;
    float* tmp_out;       // [S*H_q][max_slots][d]
    float* max_logits;    // [S*H_q][max_slots]
    float* exp_sums;
    int32_t* counts;      // [S*H_k] partials per (sequence, KV head), written by the split kernel
    half_t* out;
    int32_t num_seqs, H_q, H_k, G;
    int32_t max_blocks;
    int32_t max_slots;
    int32_t min_share;    // groups per workgroup, lower bound
    int32_t pool_tiles;   // num_blocks * H_k
    float scale_log2e;
};

__device__ __forceinline__ int flat_share(int total, int num_groups, int min_share)
{
    return max(min_share, (total + num_groups - 1) / num_groups);
}

template <int HEAD_DIM, int KV, int DEPTH, bool BIG>
__global__ void __launch_bounds__(512)
flat_decode_kernel(const FlatArgs a)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform((int)(threadIdx.x >> 6));
    const int nwaves = blockDim.x >> 6;
    const int n = lane & 15, grp = lane >> 4;

    const FlatSchedule sched(a.context_lens, a.num_seqs, a.H_k, lane);
    const int total = sched.total();
    const int share = flat_share(total, gridDim.x, a.min_share);
    const int x_begin = blockIdx.x * share;
    if (x_begin >= total) return;
    const int x_end = min(total, x_begin + share);

    const TileLoader<HEAD_DIM, KV, BIG> loader(a.cv, lane, a.pool_tiles);
    BlockRegs<HEAD_DIM, KV> regs[DEPTH][2];

    for (int x = x_begin; x < x_end;) {
        // ---- segment: the part of this workgroup's share that lies in one (sequence, KV head)
        int seq, seq_first, t;
        sched.locate(x, seq, seq_first, t);
        const int nb = (t + kBlock - 1) / kBlock;
        const int ng = (nb + 1) >> 1;
        const int g = (x - seq_first) / ng;
        const int gi0 = x - seq_first - g * ng;            // first group of the segment in the pair
        const int seg = min(x_end - x, ng - gi0);          // groups in the segment
        const int pair_first = seq_first + g * ng;
        const int slot = blockIdx.x - pair_first / share;
        if (slot == 0 && threadIdx.x == 0)              // the pair's first workgroup counts its partials
            a.counts[seq * a.H_k + g] = (pair_first + ng - 1) / share - pair_first / share + 1;
        x += seg;

        // this wave's groups: gi0 + wave + i * nwaves, i < nmine
        const int nmine = wave < seg ? (seg - wave + nwaves - 1) / nwaves : 0;
        const int32_t* bt = a.block_tables + (size_t)seq * a.max_blocks;

        half8_t qop[HEAD_DIM / 32];
        load_q_operand<HEAD_DIM, KV>(qop, a.q + ((size_t)seq * a.H_q + g * a.G + n) * HEAD_DIM,
                                     n < a.G, grp);
        float m = -INFINITY, l = 0.0f;
        floatx4 acc[HEAD_DIM / 16];
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

        // 32 groups (64 block numbers, lane 2i+h = block h of the wave's i-th group) per vector
        // load; inside such a chunk the loop is a software pipeline with DEPTH groups in flight and
        // no data-dependent branch around any load.
        for (int cg = 0; cg < nmine; cg += 32) {
            const int ncg = min(32, nmine - cg);                    // groups in this chunk
            int idv = 0;
            {
                const int b = 2 * (gi0 + wave + (cg + (lane >> 1)) * nwaves) + (lane & 1);
                if ((lane >> 1) < ncg && b < nb) idv = bt[b];
            }
            auto block_of = [&](int gi, int h) {                     // logical block, gi within chunk
                return 2 * (gi0 + wave + (cg + gi) * nwaves) + h;
            };
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int id = __builtin_amdgcn_readlane(idv, 2 * u + h);
                    loader.issue(regs[u][h], id * a.H_k + g, u < ncg && block_of(u, h) < nb);
                }
                __builtin_amdgcn_sched_barrier(0);     // keep the stages' loads in program order
            }
            for (int i = 0; i < ncg; i += DEPTH) {
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) {
                    const int gi = i + u;
                    if (gi < ncg) {
                        const int baseA = block_of(gi, 0) * kBlock;          // wave-uniform
                        const int visA = t - baseA - 4 * grp;
                        group_update<HEAD_DIM, KV>(regs[u][0], regs[u][1], qop, m, l, acc,
                                                   baseA + 2 * kBlock > t, visA, visA - kBlock, visA,
                                                   visA - kBlock, a.scale_log2e);
                    }
                    // refill only after the stage's registers are dead, so the loads land in place
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int gn = gi + DEPTH;
                        const int id = __builtin_amdgcn_readlane(idv, min(2 * gn + h, 63));
                        loader.issue(regs[u][h], id * a.H_k + g, gn < ncg && block_of(gn, h) < nb);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }

        // ---- one partial per segment
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const size_t row0 = (size_t)seq * a.H_q + g * a.G;
        if (nwaves == 1) {
            // straight from the accumulator registers: lane (n, grp) owns dims 16c+4grp..+3 of head n
            if (n < a.G) {
                const float inv = 1.0f / l;
                float* dst = a.tmp_out + ((row0 + n) * a.max_slots + slot) * HEAD_DIM + 4 * grp;
#pragma unroll
                for (int c = 0; c < HEAD_DIM / 16; ++c)
                    *reinterpret_cast<floatx4*>(dst + 16 * c) = acc[c] * inv;
                if (grp == 0) {
                    a.max_logits[(row0 + n) * a.max_slots + slot] = m * kLn2;
                    a.exp_sums[(row0 + n) * a.max_slots + slot] = l * kPUnshift;
                }
            }
        } else {
            // smem: acc [nwaves][G][HEAD_DIM], then m [nwaves][16], then l [nwaves][16]
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
                    const float f = __builtin_amdgcn_exp2f(sm_m[w * 16 + hh] - M);   // idle waves: 0
                    L += sm_l[w * 16 + hh] * f;
                    O += sm_acc[(w * a.G + hh) * HEAD_DIM + dim] * f;
                }
                a.tmp_out[((row0 + hh) * a.max_slots + slot) * HEAD_DIM + dim] = O / L;
                if (dim == 0) {
                    a.max_logits[(row0 + hh) * a.max_slots + slot] = M * kLn2;
                    a.exp_sums[(row0 + hh) * a.max_slots + slot] = L * kPUnshift;
                }
            }
            __syncthreads();       // LDS is reused by the next segment
        }
    }
}

// One wavefront per (sequence, query head) row merges the row's partials.  The number of partials
// of the row's (sequence, KV head) pair was left by the split kernel; pairs with no token at all
// have no writer, so the context length decides whether the count is meaningful.  All loads of the
// first kSpec partials are issued before the count is known (they lie inside the workspace whatever
// the count is), so the kernel is one memory round trip deep.
template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
flat_merge_kernel(const FlatArgs a)
{
    constexpr int E = HEAD_DIM / 64;
    constexpr int kSpec = 8;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);        // seq * H_q + head
    if (row >= a.num_seqs * a.H_q) return;
    const int lane = threadIdx.x & 63;
    const int seq = row / a.H_q;
    const int g = (row - seq * a.H_q) / a.G;
    const size_t base = (size_t)row * a.max_slots;
    const float* ml = a.max_logits + base;
    const float* es = a.exp_sums + base;
    const float* po = a.tmp_out + base * HEAD_DIM + lane;

    const int nspec = min(kSpec, a.max_slots);
    float o_spec[kSpec][E];
#pragma unroll
    for (int j = 0; j < kSpec; ++j)
#pragma unroll
        for (int e = 0; e < E; ++e) o_spec[j][e] = j < nspec ? po[(size_t)j * HEAD_DIM + 64 * e] : 0.0f;
    const float ml_l = lane < a.max_slots ? ml[lane] : 0.0f;
    const float es_l = lane < a.max_slots ? es[lane] : 0.0f;
    const int t = a.context_lens[seq];
    int count = a.counts[seq * a.H_k + g];
    if (t <= 0) count = 0;
    count = wave_uniform(min(count, a.max_slots));

    float o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.0f;
    if (count > 0) {
        float M = lane < count ? ml_l : -INFINITY;
        for (int p = 64 + lane; p < count; p += 64) M = fmaxf(M, ml[p]);
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) M = fmaxf(M, __shfl_xor(M, s));
        const float wv = lane < count ? es_l * __expf(ml_l - M) : 0.0f;   // weights of partials 0..63
        float W = wv;
#pragma unroll
        for (int j = 0; j < kSpec; ++j) {
            const float wj = __builtin_bit_cast(
                float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), j));
            if (j < count) {
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] += wj * o_spec[j][e];
            }
        }
        for (int j = kSpec; j < min(count, 64); ++j) {
            const float wj = __builtin_bit_cast(
                float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), j));
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] += wj * po[(size_t)j * HEAD_DIM + 64 * e];
        }
        for (int b0 = 64; b0 < count; b0 += 64) {                          // very long contexts
            const int p = b0 + lane;
            const float w2 = p < count ? es[p] * __expf(ml[p] - M) : 0.0f;
            W += w2;
            const int cnt = min(64, count - b0);
            for (int j = 0; j < cnt; ++j) {
                const float wj = __builtin_bit_cast(
                    float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w2), j));
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] += wj * po[(size_t)(b0 + j) * HEAD_DIM + 64 * e];
            }
        }
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) W += __shfl_xor(W, s);
        const float inv = 1.0f / W;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] *= inv;
    }
#pragma unroll
    for (int e = 0; e < E; ++e) a.out[(size_t)row * HEAD_DIM + lane + 64 * e] = (half_t)o[e];
}

template <int HEAD_DIM, int KV, bool BIG>
static void launch_flat_depth(const FlatArgs& a, int depth, dim3 grid, dim3 block, size_t lds,
                              hipStream_t stream)
{
    switch (depth) {
    case 1: hipLaunchKernelGGL((flat_decode_kernel<HEAD_DIM, KV, 1, BIG>), grid, block, lds, stream, a); break;
    case 3: hipLaunchKernelGGL((flat_decode_kernel<HEAD_DIM, KV, 3, BIG>), grid, block, lds, stream, a); break;
    default: hipLaunchKernelGGL((flat_decode_kernel<HEAD_DIM, KV, 2, BIG>), grid, block, lds, stream, a); break;
    }
}

template <int HEAD_DIM, int KV>
static void launch_flat_pool(const FlatArgs& a, bool big, int depth, dim3 grid, dim3 block,
                             size_t lds, hipStream_t stream)
{
    if (big) launch_flat_depth<HEAD_DIM, KV, true>(a, depth, grid, block, lds, stream);
    else launch_flat_depth<HEAD_DIM, KV, false>(a, depth, grid, block, lds, stream);
}

int flat_max_slots(const coopt_shape* sh, const FlatPlan& plan)
{
    const int max_groups = (sh->max_blocks_per_seq + 1) / 2;
    const int min_share = plan.min_share_groups();
    return (max_groups + min_share - 1) / min_share + 1;
}

size_t flat_workspace_bytes(const coopt_shape* sh, const FlatPlan& plan)
{
    return (size_t)sh->num_seqs * sh->num_q_heads * flat_max_slots(sh, plan) *
               (sh->head_dim + 2) * sizeof(float) +
           (size_t)sh->num_seqs * sh->num_kv_heads * sizeof(int32_t);
}

static int flat_grid_groups(const coopt_shape* sh, const FlatPlan& plan, int& waves)
{
    const int G = sh->num_q_heads / sh->num_kv_heads;
    waves = plan.waves;
    while (waves > 1 && ((size_t)waves * G * sh->head_dim + 2 * waves * 16) * sizeof(float) > 48 * 1024)
        waves /= 2;
    // enough workgroups to give every wave slot of the chip one wave, but never more than the
    // work's upper bound at the minimum share
    const int min_share = plan.min_share_groups();
    const long long max_total =
        (long long)sh->num_seqs * sh->num_kv_heads * ((sh->max_blocks_per_seq + 1) / 2);
    long long groups = plan.grid_waves / waves;
    groups = std::min(groups, (max_total + min_share - 1) / min_share);
    return (int)std::max(groups, 1LL);
}

static FlatArgs flat_args(const coopt_shape* sh, const FlatPlan& plan, void* workspace)
{
    FlatArgs a{};
    a.num_seqs = sh->num_seqs;
    a.H_q = sh->num_q_heads;
    a.H_k = sh->num_kv_heads;
    a.G = sh->num_q_heads / sh->num_kv_heads;
    a.max_blocks = sh->max_blocks_per_seq;
    a.max_slots = flat_max_slots(sh, plan);
    a.min_share = plan.min_share_groups();
    a.pool_tiles = sh->num_blocks * sh->num_kv_heads;
    a.scale_log2e = sh->softmax_scale * kLog2e;
    const size_t rows = (size_t)sh->num_seqs * sh->num_q_heads;
    a.tmp_out = (float*)workspace;
    a.max_logits = a.tmp_out + rows * a.max_slots * sh->head_dim;
    a.exp_sums = a.max_logits + rows * a.max_slots;
    a.counts = reinterpret_cast<int32_t*>(a.exp_sums + rows * a.max_slots);
    return a;
}

int launch_flat_split(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                      const float* v_scale, const int32_t* block_tables,
                      const int32_t* context_lens, void* workspace, const coopt_shape* sh,
                      const FlatPlan& plan, hipStream_t stream)
{
    FlatArgs a = flat_args(sh, plan, workspace);
    a.q = (const half_t*)q;
    a.cv = CacheView{(const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale};
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    int waves;
    const int groups = flat_grid_groups(sh, plan, waves);
    const dim3 grid((unsigned)groups), block(64 * waves);
    const size_t lds = waves > 1 ? ((size_t)waves * a.G * sh->head_dim + 2 * waves * 16) * sizeof(float) : 0;
    const bool big = !pool_fits_small(sh);
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_E4M3>(a, big, plan.depth, grid, block, lds, stream);
        else launch_flat_pool<64, COOPT_KV_E4M3>(a, big, plan.depth, grid, block, lds, stream);
    } else {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_FP16>(a, big, plan.depth, grid, block, lds, stream);
        else launch_flat_pool<64, COOPT_KV_FP16>(a, big, plan.depth, grid, block, lds, stream);
    }
    return launch_status();
}

int launch_flat_merge(const int32_t* context_lens, void* workspace, void* out, const coopt_shape* sh,
                      const FlatPlan& plan, hipStream_t stream)
{
    FlatArgs a = flat_args(sh, plan, workspace);
    a.context_lens = context_lens;
    a.out = (half_t*)out;
    const size_t rows = (size_t)sh->num_seqs * sh->num_q_heads;
    const dim3 rgrid((unsigned)((rows + 3) / 4)), rblock(256);
    if (sh->head_dim == 128)
        hipLaunchKernelGGL(flat_merge_kernel<128>, rgrid, rblock, 0, stream, a);
    else
        hipLaunchKernelGGL(flat_merge_kernel<64>, rgrid, rblock, 0, stream, a);
    return launch_status();
}

}  // namespace coopt
