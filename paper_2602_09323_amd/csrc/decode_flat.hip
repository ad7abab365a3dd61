// Load-balanced paged grouped-query decode attention for gfx950: the kernel behind
// coopt_paged_gqa_decode when a workspace is given (Opt-KV Eq. 6, Opt-GQA Eq. 7-8, Opt-Pa Eq. 9-10).
//
// Decode is a stream of ~2 KB tiles read once, so the kernel is organised around keeping as many
// tile loads in flight as early as possible and ending all wavefronts at the same time:
//
//   * The work of the whole batch is flattened into one sequence of two-block groups, ordered
//     [sequence][KV head][group], and cut into contiguous shares that differ by at most one group,
//     one share per single-wave workgroup.  Context lengths live on the device, so every workgroup
//     derives the schedule itself: one vector load of the lengths and a wave scan.  There are no
//     empty or short workgroups, and consecutive workgroup ids (which land on different XCDs)
//     carry equal work.
//   * A share may straddle the boundary between (sequence, KV head) pairs; the part in one pair is
//     a segment.  The software pipeline runs across segment boundaries: tiles of the next pair are
//     in flight while the current pair's last groups are consumed, and a segment ends with ONE
//     partial (m, l, o) stored straight from the accumulator registers.
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

// How the flattened groups are cut into contiguous shares: `nwg` workgroups, the first `r` with
// q + 1 groups and the rest with q, so no two shares differ by more than one group.  q is at least
// the plan's minimum share unless the whole batch is smaller than that.
struct FlatCut {
    int nwg, q, r;
    __host__ __device__ FlatCut(int total, int grid, int min_share)
    {
        nwg = max(1, min(grid, total / max(min_share, 1)));
        q = total / nwg;
        r = total - q * nwg;
    }
    __host__ __device__ int begin(int wg) const { return wg * q + min(wg, r); }
    __host__ __device__ int wg_of(int x) const
    {
        const int xr = r * (q + 1);
        return x < xr ? x / (q + 1) : r + (x - xr) / max(q, 1);
    }
};

// One wave per workgroup; the wave's share is ONE stream of groups that runs across the
// boundaries between (sequence, KV head) pairs.  The loads of the next pair's first groups are in
// flight while the last groups of the current pair are being consumed, and the pair's partial is
// stored from the accumulator registers in between.  The block numbers of up to 32 groups come from
// one gathered vector load (lane 2j+h = block h of the j-th group), whatever pairs they belong to.
template <int HEAD_DIM, int KV, int DEPTH, bool BIG>
__global__ void __launch_bounds__(64)
flat_stream_kernel(const FlatArgs a)
{
    const int lane = threadIdx.x;
    const int n = lane & 15, grp = lane >> 4;

    const FlatSchedule sched(a.context_lens, a.num_seqs, a.H_k, lane);
    const int total = sched.total();
    if (total == 0) return;
    const FlatCut cut(total, gridDim.x, a.min_share);
    if ((int)blockIdx.x >= cut.nwg) return;
    const int x_begin = cut.begin(blockIdx.x), x_end = cut.begin(blockIdx.x + 1);

    const TileLoader<HEAD_DIM, KV, BIG> loader(a.cv, lane, a.pool_tiles);
    BlockRegs<HEAD_DIM, KV> regs[DEPTH][2];
    half8_t q_cur[HEAD_DIM / 32], q_nxt[HEAD_DIM / 32];
    float m = -INFINITY, l = 0.0f;
    floatx4 acc[HEAD_DIM / 16];
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int xc = x_begin; xc < x_end; xc += 32) {
        const int nc = min(32, x_end - xc);                 // groups in this chunk
        // ---- per-lane description of entry j = lane / 2, block h = lane & 1
        const int xl = xc + (lane >> 1);
        int seq_l = 0, first_l = 0, t_l = 0;
        for (int xs = xc; xs < xc + nc;) {
            int s, first, t;
            sched.locate(xs, s, first, t);
            const int span_end = first + a.H_k * groups_of(t);     // > xs: the owner has groups
            if (xl >= xs && xl < span_end) { seq_l = s; first_l = first; t_l = t; }
            xs = span_end;
        }
        const int nb_l = (t_l + kBlock - 1) / kBlock;
        const int ng_l = max((nb_l + 1) >> 1, 1);
        const int g_l = (xl - first_l) / ng_l;
        const int gi_l = xl - first_l - g_l * ng_l;
        const int b_l = 2 * gi_l + (lane & 1);
        const bool in_chunk = (lane >> 1) < nc;
        int tile_l = -1;
        if (in_chunk && b_l < nb_l) tile_l = a.block_tables[(size_t)seq_l * a.max_blocks + b_l] * a.H_k + g_l;
        // entries that end a segment: last group of their pair, or last group of the share
        const unsigned long long last_mask = __builtin_amdgcn_ballot_w64(
            in_chunk && (lane & 1) == 0 && (gi_l == ng_l - 1 || xl == x_end - 1));

        auto q_rows = [&](int e) {         // q rows of the pair that entry e belongs to
            const int s = __builtin_amdgcn_readlane(seq_l, 2 * e), g = __builtin_amdgcn_readlane(g_l, 2 * e);
            return a.q + ((size_t)s * a.H_q + g * a.G) * HEAD_DIM;
        };
        // first entry of the segment after the one that contains entry e (nc if there is none)
        auto next_segment = [&](int e) {
            const unsigned long long rest = e < 32 ? last_mask >> (2 * e) : 0ull;
            return rest ? e + (__builtin_ctzll(rest) >> 1) + 1 : nc;
        };
        load_q_operand_rows<HEAD_DIM, KV>(q_cur, q_rows(0), a.G, true, n, grp);
        {
            const int e1 = next_segment(0);
            load_q_operand_rows<HEAD_DIM, KV>(q_nxt, q_rows(min(e1, nc - 1)), a.G, e1 < nc, n, grp);
        }

        auto issue_entry = [&](BlockRegs<HEAD_DIM, KV> (&r)[2], int e) {
            const int ec = min(e, 31);
            const int tA = __builtin_amdgcn_readlane(tile_l, 2 * ec);
            const int tB = __builtin_amdgcn_readlane(tile_l, 2 * ec + 1);
            loader.issue(r[0], max(tA, 0), e < nc && tA >= 0);
            loader.issue(r[1], max(tB, 0), e < nc && tB >= 0);
        };
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            issue_entry(regs[u], u);
            __builtin_amdgcn_sched_barrier(0);     // keep the stages' loads in program order
        }
        for (int j = 0; j < nc; j += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int e = j + u;
                if (e < nc) {
                    const int t = __builtin_amdgcn_readlane(t_l, 2 * e);
                    const int gi = __builtin_amdgcn_readlane(gi_l, 2 * e);
                    const int baseA = 2 * gi * kBlock;
                    const int visA = t - baseA - 4 * grp;
                    group_update<HEAD_DIM, KV>(regs[u][0], regs[u][1], q_cur, m, l, acc,
                                               baseA + 2 * kBlock > t, visA, visA - kBlock, visA,
                                               visA - kBlock, a.scale_log2e);
                    if ((last_mask >> (2 * e)) & 1) {
                        // ---- the segment's partial, straight from the accumulator registers:
                        // lane (n, grp) owns dims 16c+4grp..+3 of head n
                        const int seq = __builtin_amdgcn_readlane(seq_l, 2 * e);
                        const int g = __builtin_amdgcn_readlane(g_l, 2 * e);
                        const int ng = (((t + kBlock - 1) / kBlock) + 1) >> 1;
                        const int pair_first = xc + e - gi;
                        const int slot = blockIdx.x - cut.wg_of(pair_first);
                        if (slot == 0 && lane == 0)      // the pair's first workgroup counts its partials
                            a.counts[seq * a.H_k + g] = cut.wg_of(pair_first + ng - 1) - cut.wg_of(pair_first) + 1;
                        l += __shfl_xor(l, 16);
                        l += __shfl_xor(l, 32);
                        if (n < a.G) {
                            const size_t row = (size_t)seq * a.H_q + g * a.G + n;
                            const float inv = 1.0f / l;
                            float* dst = a.tmp_out + (row * a.max_slots + slot) * HEAD_DIM + 4 * grp;
#pragma unroll
                            for (int c = 0; c < HEAD_DIM / 16; ++c)
                                *reinterpret_cast<floatx4*>(dst + 16 * c) = acc[c] * inv;
                            if (grp == 0) {
                                a.max_logits[row * a.max_slots + slot] = m * kLn2;
                                a.exp_sums[row * a.max_slots + slot] = l * kPUnshift;
                            }
                        }
                        m = -INFINITY;
                        l = 0.0f;
#pragma unroll
                        for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
                        // the next segment's q is already here; fetch the one after it
#pragma unroll
                        for (int jj = 0; jj < HEAD_DIM / 32; ++jj) q_cur[jj] = q_nxt[jj];
                        const int e2 = next_segment(e + 1);
                        load_q_operand_rows<HEAD_DIM, KV>(q_nxt, q_rows(min(e2, nc - 1)), a.G, e2 < nc, n, grp);
                    }
                }
                // refill only after the stage's registers are dead, so the loads land in place
                __builtin_amdgcn_sched_barrier(0);
                issue_entry(regs[u], e + DEPTH);
                __builtin_amdgcn_sched_barrier(0);
            }
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
static void launch_flat_depth(const FlatArgs& a, int depth, dim3 grid, hipStream_t stream)
{
    const dim3 block(64);
    switch (depth) {
    case 1: hipLaunchKernelGGL((flat_stream_kernel<HEAD_DIM, KV, 1, BIG>), grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL((flat_stream_kernel<HEAD_DIM, KV, 3, BIG>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((flat_stream_kernel<HEAD_DIM, KV, 2, BIG>), grid, block, 0, stream, a); break;
    }
}

template <int HEAD_DIM, int KV>
static void launch_flat_pool(const FlatArgs& a, bool big, int depth, dim3 grid, hipStream_t stream)
{
    if (big) launch_flat_depth<HEAD_DIM, KV, true>(a, depth, grid, stream);
    else launch_flat_depth<HEAD_DIM, KV, false>(a, depth, grid, stream);
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

// Workgroups (= wavefronts) to launch: the plan's grid, but never more than the work's upper bound
// at the minimum share.
static int flat_grid_groups(const coopt_shape* sh, const FlatPlan& plan)
{
    const int min_share = plan.min_share_groups();
    const long long max_total =
        (long long)sh->num_seqs * sh->num_kv_heads * ((sh->max_blocks_per_seq + 1) / 2);
    const long long groups = std::min((long long)plan.grid_waves, (max_total + min_share - 1) / min_share);
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
    const dim3 grid((unsigned)flat_grid_groups(sh, plan));
    const bool big = !pool_fits_small(sh);
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_E4M3>(a, big, plan.depth, grid, stream);
        else launch_flat_pool<64, COOPT_KV_E4M3>(a, big, plan.depth, grid, stream);
    } else {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_FP16>(a, big, plan.depth, grid, stream);
        else launch_flat_pool<64, COOPT_KV_FP16>(a, big, plan.depth, grid, stream);
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
