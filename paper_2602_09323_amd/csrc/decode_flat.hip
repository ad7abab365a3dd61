// Load-balanced paged grouped-query decode attention for gfx950: the kernel behind
// coopt_paged_gqa_decode when a workspace is given (Opt-KV Eq. 6, Opt-GQA Eq. 7-8, Opt-Pa Eq. 9-10).
//
// Decode is a stream of ~2 KB tiles read once, so the kernel is organised around keeping as many
// tile loads in flight as early as possible and ending all wavefronts at the same time:
//
//   * The work of the whole batch is flattened into one sequence of two-block groups, ordered
//     [sequence][KV head][group], and cut into contiguous shares, one per single-wave workgroup.
//     The cut is made on a cost axis that charges a few group times for every (sequence, KV head)
//     pair that ends inside a share; shares differ by at most one cost unit.  Context lengths live
//     on the device, so every workgroup derives the schedule itself: one vector load of the
//     lengths and wave scans.  There are no empty or short workgroups; all shares carry equal
//     work, and each XCD's workgroups take a contiguous eighth of them (share_of_workgroup).
//   * A share may straddle the boundary between (sequence, KV head) pairs; the part in one pair is
//     a segment.  The software pipeline runs across segment boundaries: tiles of the next pair are
//     in flight while the current pair's last groups are consumed, the next pair's q operand waits
//     in LDS, and a segment that ends mid-share parks its partial (m, l, o) in LDS so that no store
//     sits between the tile loads; partials go to memory when the share is done.
//   * Partial j of a pair is written by workgroup first_wg(pair) + j, and the pair's first
//     workgroup also records how many partials the pair gets; the merge kernel combines them into
//     the fp16 output rows.
//
// The per-group arithmetic is in attn_tile.hpp.
#include "attn_tile.hpp"
#include "decode_internal.hpp"
#include "kv_quant.hpp"

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

// The flattened schedule, derived identically by every wavefront that needs it.  Two axes run
// side by side over [sequence][KV head][group]: the REAL one counts groups; the COST one also gives
// every (sequence, KV head) pair `extra` units in front of its groups, the price (in group times)
// of ending a pair inside a share: the masked last group and the hand-over to the next pair.
// Shares are cut on the cost axis, so a wave that crosses a pair boundary gets fewer groups.
struct FlatSchedule {
    const int32_t* lens;
    const int64_t* new_slots;   // fused step only: slot of the token each sequence appends, or NULL
    int S, H_k, extra, lane;
    // cache of the first 64 sequences (the whole batch when S <= 64)
    int t0, incl0, total0, cincl0, ctotal0;

    __device__ __forceinline__ int real_weight(int t) const { return H_k * groups_of(t); }
    __device__ __forceinline__ int cost_weight(int t) const
    {
        return t > 0 ? H_k * (groups_of(t) + extra) : 0;
    }

    // Tokens of sequence s that this launch attends to.  In the fused step that includes the token
    // the launch itself appends: the wavefront that streams the pair's last group takes it from
    // the new rows (see take_new_token), not from the cache.
    __device__ __forceinline__ int cached_len(int s) const { return lens[s]; }

    // Fused step: does sequence s append a token in this launch (Opt-KV Eq. 5: a negative slot
    // filters the token out; an empty sequence has none)?
    __device__ __forceinline__ bool appends(int s, int t) const
    {
        return new_slots != nullptr && t > 0 && new_slots[s] >= 0;
    }

    __device__ __forceinline__ FlatSchedule(const int32_t* context_lens, const int64_t* appended,
                                            int num_seqs, int kv_heads, int pair_extra, int lane_id)
        : lens(context_lens), new_slots(appended), S(num_seqs), H_k(kv_heads), extra(pair_extra),
          lane(lane_id)
    {
        t0 = lane < S ? cached_len(lane) : 0;
        incl0 = wave_inclusive_scan(real_weight(t0));
        total0 = __builtin_amdgcn_readlane(incl0, 63);
        cincl0 = wave_inclusive_scan(cost_weight(t0));
        ctotal0 = __builtin_amdgcn_readlane(cincl0, 63);
    }

    // Length of the cost axis for the whole batch.
    __device__ __forceinline__ int cost_total() const
    {
        int sum = ctotal0;
        for (int base = 64; base < S; base += 64) {
            int v = cost_weight(base + lane < S ? cached_len(base + lane) : 0);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
            sum += wave_uniform(v);      // equal in all lanes; tell the compiler so
        }
        return sum;
    }

    // Sequence that owns position x of the real axis (COST = false) or of the cost axis (COST =
    // true), x below that axis' total: its index, the positions of its first unit on both axes, and
    // its context length.  All results are wave-uniform.
    template <bool COST>
    __device__ __forceinline__ void locate(int x, int& seq, int& first, int& cfirst, int& t) const
    {
        int carry = 0, ccarry = 0, tl = t0, incl = incl0, cincl = cincl0;
        int tile_total = total0, ctile_total = ctotal0;
        for (int base = 0;; base += 64) {
            if (base > 0) {
                tl = base + lane < S ? cached_len(base + lane) : 0;
                incl = wave_inclusive_scan(real_weight(tl));
                tile_total = __builtin_amdgcn_readlane(incl, 63);
                cincl = wave_inclusive_scan(cost_weight(tl));
                ctile_total = __builtin_amdgcn_readlane(cincl, 63);
            }
            const bool here = COST ? x < ccarry + ctile_total : x < carry + tile_total;
            if (here || base + 64 >= S) {
                const unsigned long long before =
                    __builtin_amdgcn_ballot_w64(COST ? ccarry + cincl <= x : carry + incl <= x);
                const int idx = min(__builtin_popcountll(before), 63);
                seq = min(base + idx, S - 1);
                t = __builtin_amdgcn_readlane(tl, idx);
                first = carry + __builtin_amdgcn_readlane(incl - real_weight(tl), idx);
                cfirst = ccarry + __builtin_amdgcn_readlane(cincl - cost_weight(tl), idx);
                return;
            }
            carry += tile_total;
            ccarry += ctile_total;
        }
    }

    // Cost-axis position of sequence seq's first unit.
    __device__ __forceinline__ int cost_first_of(int seq) const
    {
        int ccarry = 0;
        for (int base = 0;; base += 64) {
            const int tl = base == 0 ? t0 : (base + lane < S ? cached_len(base + lane) : 0);
            const int cincl = base == 0 ? cincl0 : wave_inclusive_scan(cost_weight(tl));
            if (seq < base + 64)
                return ccarry + __builtin_amdgcn_readlane(cincl - cost_weight(tl), seq - base);
            ccarry += __builtin_amdgcn_readlane(cincl, 63);
        }
    }

    // Number of groups whose cost-axis position is below v (0 <= v <= cost_total): the real-axis
    // position at which a share that begins at v begins.
    __device__ __forceinline__ int real_before(int v, int ctotal) const
    {
        int seq, first, cfirst, t;
        locate<true>(min(v, ctotal - 1), seq, first, cfirst, t);
        const int ng = groups_of(t);
        const int r = v - cfirst;                     // v = ctotal lands past the last pair
        const int g = min(r / (ng + extra), H_k);
        const int gi = min(max(r - g * (ng + extra) - extra, 0), ng);
        return first + min(g * ng + gi, H_k * ng);
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
    uint32_t* ws_header;  // first 16 bytes of the workspace: [0] ws_tag, left by the split kernel
    half_t* out;
    int32_t num_seqs, H_q, H_k, G;
    int32_t max_blocks;
    int32_t max_slots;
    int32_t min_share;    // cost units (groups plus pair extras) per workgroup, lower bound
    int32_t pair_extra;   // cost units charged to a share for every pair that ends inside it
    int32_t pool_tiles;   // num_blocks * H_k
    int32_t decode_wgs;   // workgroups (= wavefronts) of the attention launch
    int32_t append_wgs;   // fused step: workgroups at the head of the merge launch's grid whose
                          // wavefronts store one new row each (0 otherwise)
    int32_t kv_dtype;     // cache type, for the merge launch's row stores
    uint32_t ws_tag;      // names the plan the workspace's partials were laid out for (see ws_tag_of)
    float scale_log2e;
    // fused step only (new_slots != NULL): the token every sequence appends, and the cache as
    // written to
    const int64_t* new_slots;
    const half_t* k_new;
    const half_t* v_new;
    uint8_t* k_cache_w;
    uint8_t* v_cache_w;
    float* k_scale_w;
    float* v_scale_w;
    // prepared schedule (see PreparedSource): read by the prepared kernels, written by the
    // prepare kernel; offsets and the region stride in 32-bit words
    const uint32_t* sched;
    uint32_t* sched_w;
    uint32_t sched_tag;
    int32_t sched_regions;
    int32_t sched_stride;
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

// Where one partial goes: first output row of its (sequence, KV head) pair, slot among the pair's
// partials, and -- for the pair's first workgroup only (count_at >= 0) -- where to leave the
// number of partials of the pair.  All wave-uniform.
struct PartialSlot {
    int row0, slot, count_at, count;
};

// Lane (n, grp) owns dims 16c + 4grp .. +3 of head n: o[c].  m in natural-log units.
template <int HEAD_DIM>
__device__ __forceinline__ void store_partial(const FlatArgs& a, const PartialSlot& ps,
                                              const floatx4 (&o)[HEAD_DIM / 16], float m_ln, float l,
                                              int lane)
{
    const int n = lane & 15, grp = lane >> 4;
    if (ps.count_at >= 0 && lane == 0) a.counts[ps.count_at] = ps.count;
    if (n < a.G) {
        const size_t at = (size_t)(ps.row0 + n) * a.max_slots + ps.slot;
        float* dst = a.tmp_out + at * HEAD_DIM + 4 * grp;
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c) *reinterpret_cast<floatx4*>(dst + 16 * c) = o[c];
        if (grp == 0) {
            a.max_logits[at] = m_ln;
            a.exp_sums[at] = l;
        }
    }
}

// The same for a partial parked in LDS (each lane reads back what it wrote itself).
template <int HEAD_DIM>
__device__ __forceinline__ void store_parked(const FlatArgs& a, const PartialSlot& ps,
                                             const unsigned char* park, int lane)
{
    floatx4 o[HEAD_DIM / 16];
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c)
        o[c] = *reinterpret_cast<const floatx4*>(park + 16 * (64 * c + lane));
    const float m_ln = *reinterpret_cast<const float*>(park + HEAD_DIM / 16 * 1024 + 4 * lane);
    const float l = *reinterpret_cast<const float*>(park + HEAD_DIM / 16 * 1024 + 256 + 4 * lane);
    store_partial<HEAD_DIM>(a, ps, o, m_ln, l, lane);
}

// Stage the q^T operand of one (sequence, KV head) pair in LDS with loads that write LDS directly:
// operand jj of lane i lands at stage + 1024 * jj + 16 * i.  Lanes of absent heads (n >= G) repeat
// the last head; their columns are never stored.  The compiler does not track these loads, so the
// reader waits on the vector-memory counter itself.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void stage_q_operand(unsigned char* stage, const half_t* pair_rows, int G,
                                                int n, int grp)
{
#if defined(__HIP_DEVICE_COMPILE__)      // the host pass rejects the cast to the LDS address space
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half_t*>(pair_rows), 0, G * HEAD_DIM * 2, 0x00020000);
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rq, (__attribute__((address_space(3))) void*)(stage + 1024 * jj), 16,
            2 * (min(n, G - 1) * HEAD_DIM + q_dim_offset<HEAD_DIM, KV>(jj, grp)), 0, 0, 0);
#endif
}

// Partials the attention workgroups write for (sequence, KV head) pair `pair`, from the schedule.
__device__ __forceinline__ int attention_partials_of(const FlatArgs& a, const FlatSchedule& sched,
                                                     const FlatCut& cut, int ctotal, int pair)
{
    const int seq = pair / a.H_k;
    const int g = pair - seq * a.H_k;
    const int ng = groups_of(sched.cached_len(seq));
    if (ng <= 0 || ctotal <= 0) return 0;
    const int pair_first = sched.cost_first_of(seq) + g * (ng + a.pair_extra) + a.pair_extra;
    return cut.wg_of(pair_first + ng - 1) - cut.wg_of(pair_first) + 1;
}

// Where a wavefront's share comes from.  A source describes the share as entries 0 .. size()-1
// (one two-block group each), 32 at a time: load_chunk(c0) makes entries c0 .. c0+nc-1 current, and
// the accessors below answer for entry e of the current chunk.  Everything they return is
// wave-uniform.
//
// LiveSource derives the schedule in the kernel from the context lengths (and reads the block
// table); PreparedSource reads records that coopt_decode_schedule_prepare left in memory.

// Lane 2j + h of the current chunk describes block h of entry j.
struct LiveSource {
    const FlatArgs& a;
    const FlatSchedule& sched;
    const FlatCut& cut;
    int lane, share, x_begin, x_end;
    int nc = 0;
    int seq_l = 0, cfirst_l = 0, t_l = 0, g_l = 0, gi_l = 0, tile_l = -1;
    unsigned long long last_mask = 0, append_mask = 0;

    __device__ __forceinline__ LiveSource(const FlatArgs& args, const FlatSchedule& s, const FlatCut& c,
                                          int lane_id, int share_id, int xb, int xe)
        : a(args), sched(s), cut(c), lane(lane_id), share(share_id), x_begin(xb), x_end(xe) {}
    __device__ __forceinline__ int size() const { return x_end - x_begin; }

    __device__ __forceinline__ void load_chunk(int c0)
    {
        const int xc = x_begin + c0;
        nc = min(32, x_end - xc);
        const int xl = xc + (lane >> 1);
        int first_l = 0;
        seq_l = 0; cfirst_l = 0; t_l = 0;
        for (int xs = xc; xs < xc + nc;) {
            int s, first, cfirst, t;
            sched.template locate<false>(xs, s, first, cfirst, t);
            const int span_end = first + a.H_k * groups_of(t);     // > xs: the owner has groups
            if (xl >= xs && xl < span_end) { seq_l = s; first_l = first; cfirst_l = cfirst; t_l = t; }
            xs = span_end;
        }
        const int nb_l = (t_l + kBlock - 1) / kBlock;
        const int ng_l = max((nb_l + 1) >> 1, 1);
        g_l = (xl - first_l) / ng_l;
        gi_l = xl - first_l - g_l * ng_l;
        const int b_l = 2 * gi_l + (lane & 1);
        const bool in_chunk = (lane >> 1) < nc;
        tile_l = -1;
        if (in_chunk && b_l < nb_l) tile_l = a.block_tables[(size_t)seq_l * a.max_blocks + b_l] * a.H_k + g_l;
        // entries that end a segment: last group of their pair, or last group of the share
        last_mask = __builtin_amdgcn_ballot_w64(
            in_chunk && (lane & 1) == 0 && (gi_l == ng_l - 1 || xl == x_end - 1));
        // entries that hold the token their sequence appends in this launch (the pair's last group)
        append_mask = 0;
        if (a.new_slots)
            append_mask = __builtin_amdgcn_ballot_w64(in_chunk && (lane & 1) == 0 && gi_l == ng_l - 1 &&
                                                      sched.appends(seq_l, t_l));
    }
    __device__ __forceinline__ void tiles(int e, int& tA, int& tB) const
    {
        tA = __builtin_amdgcn_readlane(tile_l, 2 * e);
        tB = __builtin_amdgcn_readlane(tile_l, 2 * e + 1);
    }
    // tokens of the pair from the entry's first token on (the entry sees min(rem, 32) of them)
    __device__ __forceinline__ int rem(int e) const
    {
        return __builtin_amdgcn_readlane(t_l, 2 * e) - 2 * kBlock * __builtin_amdgcn_readlane(gi_l, 2 * e);
    }
    __device__ __forceinline__ bool last(int e) const { return (last_mask >> (2 * e)) & 1; }
    __device__ __forceinline__ bool appends(int e) const { return (append_mask >> (2 * e)) & 1; }
    __device__ __forceinline__ int pair(int e) const
    {
        return __builtin_amdgcn_readlane(seq_l, 2 * e) * a.H_k + __builtin_amdgcn_readlane(g_l, 2 * e);
    }
    // first entry of the segment after the one that contains entry e (nc if there is none)
    __device__ __forceinline__ int next_segment(int e) const
    {
        const unsigned long long rest = e < 32 ? last_mask >> (2 * e) : 0ull;
        return rest ? e + (__builtin_ctzll(rest) >> 1) + 1 : nc;
    }
    __device__ __forceinline__ const half_t* q_rows(int e, int head_dim) const
    {
        const int s = __builtin_amdgcn_readlane(seq_l, 2 * e), g = __builtin_amdgcn_readlane(g_l, 2 * e);
        return a.q + ((size_t)s * a.H_q + g * a.G) * head_dim;
    }
    __device__ __forceinline__ PartialSlot slot(int e) const
    {
        const int seq = __builtin_amdgcn_readlane(seq_l, 2 * e);
        const int g = __builtin_amdgcn_readlane(g_l, 2 * e);
        const int t = __builtin_amdgcn_readlane(t_l, 2 * e);
        const int ng = (((t + kBlock - 1) / kBlock) + 1) >> 1;
        // cost-axis position of the pair's first group
        const int pair_first = __builtin_amdgcn_readlane(cfirst_l, 2 * e) +
                               g * (ng + a.pair_extra) + a.pair_extra;
        PartialSlot ps;
        ps.row0 = seq * a.H_q + g * a.G;
        ps.slot = share - cut.wg_of(pair_first);
        // the pair's first workgroup also counts the pair's partials
        ps.count_at = ps.slot == 0 ? seq * a.H_k + g : -1;
        ps.count = cut.wg_of(pair_first + ng - 1) - cut.wg_of(pair_first) + 1;
        return ps;
    }
};

// A prepared schedule in memory (32-bit words):
//   [0] layout tag  [1] status (0, or 1 once a launch found the wrong tag)  [2..15] unused
//   counts[num_seqs * H_k]: partials per (sequence, KV head)       (rounded up to 4 words)
//   one region per attention workgroup, `stride` words each:
//     [0] entries in the share  [1..3] unused  then one 4-word record per entry:
//     tile of block A, tile of block B (-1: absent), pair | appends << 30 | last << 31,
//     rem | slot << 16
//   pair = sequence * H_k + KV head (< 2^27); appends = the entry is the pair's last group and its
//   sequence appends a token in the launch (fused step); rem as LiveSource::rem, capped at 0x7fff;
//   slot = index of the partial this workgroup writes for the pair.
constexpr int kSchedHeaderWords = 16;
constexpr int kSchedRemCap = 0x7fff;
constexpr int kSchedPairMask = 0x3fffffff;

typedef unsigned int sched_rec_t __attribute__((ext_vector_type(4)));

// Lane j of the current chunk holds the record of entry j.  The records of the first chunk are
// loaded by the kernel before it knows the share's size (a region always has room for 32).
struct PreparedSource {
    const FlatArgs& a;
    const uint32_t* region;
    int lane, count;
    sched_rec_t first;
    int nc = 0;
    uint32_t tA_l = ~0u, tB_l = ~0u, pair_l = 0, rs_l = 0;
    unsigned long long last_mask = 0, append_mask = 0;

    __device__ __forceinline__ PreparedSource(const FlatArgs& args, const uint32_t* reg, int lane_id, int n,
                                              sched_rec_t first_chunk)
        : a(args), region(reg), lane(lane_id), count(n), first(first_chunk) {}
    __device__ __forceinline__ int size() const { return count; }

    __device__ __forceinline__ void load_chunk(int c0)
    {
        nc = min(32, count - c0);
        sched_rec_t r = first;
        if (c0 > 0 && lane < nc) r = *reinterpret_cast<const sched_rec_t*>(region + 4 + 4 * (c0 + lane));
        const bool have = lane < nc;
        tA_l = have ? r.x : ~0u;
        tB_l = have ? r.y : ~0u;
        pair_l = have ? r.z : 0u;
        rs_l = have ? r.w : 0u;
        last_mask = __builtin_amdgcn_ballot_w64(have && (pair_l >> 31) != 0);
        append_mask = __builtin_amdgcn_ballot_w64(have && ((pair_l >> 30) & 1u) != 0);
    }
    __device__ __forceinline__ void tiles(int e, int& tA, int& tB) const
    {
        tA = __builtin_amdgcn_readlane((int)tA_l, e);
        tB = __builtin_amdgcn_readlane((int)tB_l, e);
    }
    __device__ __forceinline__ int rem(int e) const
    {
        return __builtin_amdgcn_readlane((int)rs_l, e) & 0xffff;
    }
    __device__ __forceinline__ bool last(int e) const { return (last_mask >> e) & 1; }
    __device__ __forceinline__ bool appends(int e) const { return (append_mask >> e) & 1; }
    __device__ __forceinline__ int pair(int e) const
    {
        return __builtin_amdgcn_readlane((int)pair_l, e) & kSchedPairMask;
    }
    __device__ __forceinline__ int next_segment(int e) const
    {
        const unsigned long long rest = e < 32 ? last_mask >> e : 0ull;
        return rest ? e + __builtin_ctzll(rest) + 1 : nc;
    }
    __device__ __forceinline__ const half_t* q_rows(int e, int head_dim) const
    {
        return a.q + (size_t)pair(e) * a.G * head_dim;
    }
    __device__ __forceinline__ PartialSlot slot(int e) const
    {
        PartialSlot ps;
        ps.row0 = pair(e) * a.G;
        ps.slot = (int)((uint32_t)__builtin_amdgcn_readlane((int)rs_l, e) >> 16);
        ps.count_at = -1;                  // the counts were written with the schedule
        ps.count = 0;
        return ps;
    }
};

// ---- fused step: the token a sequence appends in this step (Opt-KV Eq. 5, Alg. 1 phase 1)
//
// The wavefront that streams a pair's last group also takes the pair's new token: it quantises the
// row exactly as the cache-write kernel does (kv_quant.hpp) and puts the row's cache elements into
// the K and V operand registers of that group in place of whatever the cache holds at that slot,
// so that the attention launch sees the token without anything in it waiting for a store.  The
// row itself is stored into the cache by extra wavefronts of the MERGE launch that follows (same
// quantiser, same bytes): stores into the cache pool from the attention launch cost it 0.8 us
// at the LLaMa-13B decode shape wherever they were issued (at once, at the end of a share, as
// whole tiles), while the merge launch has the time.

// Replaces token `pos` (wave-uniform, 0..31: block A holds 0..15, block B the rest) of a loaded
// group by the row staged in LDS at `row` (K row, then V row, cache elements in dim order).
// K: the four lanes (off, grp), off = pos % 16, take the 16-byte chunks 4j+grp of the row.  V: the
// sixteen lanes (n, off/4) insert the row's element of dim 16*(W*j+cc)+n at element 4*cc + off%4 of
// their 16 bytes.  Both blocks get whole-register selects with constant element indices (the block
// is chosen by the masks, not by a branch: a branch over two tiles would make the compiler address
// them through a pointer and move the whole pipeline's registers to scratch memory).
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void patch_token(BlockRegs<HEAD_DIM, KV>& A, BlockRegs<HEAD_DIM, KV>& B,
                                            int pos, const unsigned char* row, int lane, float ks,
                                            float vs)
{
    constexpr int ES = BlockRegs<HEAD_DIM, KV>::ES;
    constexpr int NL = BlockRegs<HEAD_DIM, KV>::NL;
    constexpr int W = 4 / ES;                           // 16-dim groups per 16 bytes of a V tile
    const int n = lane & 15, grp = lane >> 4;
    const int off = pos & (kBlock - 1);
    const bool in_a = pos < kBlock;
    const bool k_lane = n == off;
    const bool v_lane = grp == (off >> 2);
    const unsigned char* vrow = row + HEAD_DIM * ES;
    const uint32_t ka = (k_lane && in_a) ? 0xffffffffu : 0u;
    const uint32_t kb = (k_lane && !in_a) ? 0xffffffffu : 0u;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const u32x4 kk = *reinterpret_cast<const u32x4*>(row + 16 * (4 * j + grp));
        A.k[j] = (A.k[j] & ~ka) | (kk & ka);
        B.k[j] = (B.k[j] & ~kb) | (kk & kb);
    }
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        u32x4 val, mask;
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
            if constexpr (ES == 1) {          // dword dw = dim group cc = dw, byte off%4 of it
                const uint32_t b = vrow[16 * (W * j + dw) + n];
                const int sh = 8 * (off & 3);
                val[dw] = b << sh;
                mask[dw] = v_lane ? (0xffu << sh) : 0u;
            } else {                          // dword dw = dim group cc = dw/2, tokens 2(dw%2), +1
                const uint32_t h = *reinterpret_cast<const uint16_t*>(vrow + 2 * (16 * (W * j + (dw >> 1)) + n));
                const int sh = 16 * (off & 1);
                val[dw] = h << sh;
                mask[dw] = (v_lane && ((off & 3) >> 1) == (dw & 1)) ? (0xffffu << sh) : 0u;
            }
        }
        const u32x4 ma = in_a ? mask : u32x4{0u, 0u, 0u, 0u};
        const u32x4 mb = in_a ? u32x4{0u, 0u, 0u, 0u} : mask;
        A.v[j] = (A.v[j] & ~ma) | (val & ma);
        B.v[j] = (B.v[j] & ~mb) | (val & mb);
    }
    if constexpr (kIsFp8<KV>) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool mine = v_lane && i == (off & 3);
            A.ks[i] = (mine && in_a) ? ks : A.ks[i];
            A.vs[i] = (mine && in_a) ? vs : A.vs[i];
            B.ks[i] = (mine && !in_a) ? ks : B.ks[i];
            B.vs[i] = (mine && !in_a) ? vs : B.vs[i];
        }
    }
}

// row_k / row_v: the lane's E fp16 values of the new K / V row as loaded (low bits first).  pos =
// the token's position inside the group (0..31).  `stage` is 2 * HEAD_DIM cache elements of LDS
// private to the wavefront.
template <int HEAD_DIM, int KV>
__device__ __forceinline__ void take_new_token(BlockRegs<HEAD_DIM, KV>& A, BlockRegs<HEAD_DIM, KV>& B,
                                               uint32_t row_k, uint32_t row_v, int pos,
                                               unsigned char* stage, int lane)
{
    constexpr int E = HEAD_DIM / 64;
    constexpr int ES = BlockRegs<HEAD_DIM, KV>::ES;
    uint32_t ck = row_k, cv = row_v;                    // the row's cache elements of this lane
    float ks = 1.0f, vs = 1.0f;
    if constexpr (kIsFp8<KV>) {
        float kx[E], vx[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            kx[e] = (float)__builtin_bit_cast(half_t, (uint16_t)(row_k >> (16 * e)));
            vx[e] = (float)__builtin_bit_cast(half_t, (uint16_t)(row_v >> (16 * e)));
        }
        const QuantRow<HEAD_DIM> qr = quantise_values<HEAD_DIM, KV>(kx, vx);
        ck = qr.k_codes;
        cv = qr.v_codes;
        ks = qr.k_scale;
        vs = qr.v_scale;
    }
    constexpr int LB = E * ES;                          // bytes per lane and row
    unsigned char* kd = stage + LB * lane;
    unsigned char* vd = stage + HEAD_DIM * ES + LB * lane;
    if constexpr (LB == 1) {
        *kd = (unsigned char)ck;
        *vd = (unsigned char)cv;
    } else if constexpr (LB == 2) {
        *reinterpret_cast<uint16_t*>(kd) = (uint16_t)ck;
        *reinterpret_cast<uint16_t*>(vd) = (uint16_t)cv;
    } else {
        *reinterpret_cast<uint32_t*>(kd) = ck;
        *reinterpret_cast<uint32_t*>(vd) = cv;
    }
    patch_token<HEAD_DIM, KV>(A, B, pos, stage, lane, ks, vs);
}

// APPEND (fused step): entries flagged by the source also take their pair's new token.
template <int HEAD_DIM, int KV, int DEPTH, bool BIG, bool BLOCK_REDUCE, bool APPEND, typename Source>
__device__ __forceinline__ void stream_share(const FlatArgs& a, Source& src, unsigned char* q_stage,
                                             int lane)
{
    // vector-memory loads per group: two blocks of K and V chunks plus, for FP8, their scales;
    // in the fused step also the two new rows (requested with every group, empty where the group
    // appends nothing, so that the count is the same on every path)
    constexpr int kGroupLoads = 2 * (2 * BlockRegs<HEAD_DIM, KV>::NL + (kIsFp8<KV> ? 2 : 0)) +
                                (APPEND ? 2 : 0);
    // s_waitcnt immediates (gfx9 layout: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
    constexpr int kWaitStaged = (kGroupLoads & 15) | (7 << 4) | (15 << 8) | ((kGroupLoads >> 4) << 14);
    constexpr int kWaitLds = 15 | (7 << 4) | (0 << 8) | (3 << 14);
    static_assert(kGroupLoads < 64, "vmcnt is a 6-bit counter");
    const int n = lane & 15, grp = lane >> 4;

    const TileLoader<HEAD_DIM, KV, BIG> loader(a.cv, lane, a.pool_tiles);
    BlockRegs<HEAD_DIM, KV> regs[DEPTH][2];
    // q operand of the pair in progress; the next pair's is staged in LDS by loads that write LDS
    // directly, so taking it over is an LDS read and never waits on a register in flight.
    constexpr int kParkAcc = HEAD_DIM / 16 * 1024;               // parked o, then m and l per lane
    unsigned char* park = q_stage + HEAD_DIM / 32 * 1024;
    float* red = reinterpret_cast<float*>(park + kParkAcc + 512);  // BLOCK_REDUCE: 128 floats
    unsigned char* row_stage = park + kParkAcc + 1024;             // APPEND: one new K row, one V row
    uint32_t row_k[DEPTH], row_v[DEPTH];                           // APPEND: the rows in flight
    PartialSlot parked;
    parked.row0 = -1;
    half8_t q_cur[HEAD_DIM / 32];
    float m = -INFINITY, l = 0.0f;
    floatx4 acc[HEAD_DIM / 16];
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int total = src.size();
    for (int c0 = 0; c0 < total; c0 += 32) {
        src.load_chunk(c0);
        const int nc = src.nc;
        load_q_operand_rows<HEAD_DIM, KV>(q_cur, src.q_rows(0, HEAD_DIM), a.G, true, n, grp);
        stage_q_operand<HEAD_DIM, KV>(q_stage, src.q_rows(min(src.next_segment(0), nc - 1), HEAD_DIM),
                                      a.G, n, grp);

        auto issue_entry = [&](BlockRegs<HEAD_DIM, KV> (&r)[2], int e) {
            int tA, tB;
            src.tiles(min(e, 31), tA, tB);
            loader.issue(r[0], max(tA, 0), e < nc && tA >= 0);
            loader.issue(r[1], max(tB, 0), e < nc && tB >= 0);
        };
        // the lane's E fp16 values of the new K and V rows of entry e's pair (zeros unless flagged)
        auto issue_rows = [&](uint32_t& rk, uint32_t& rv, int e) {
            constexpr int E = HEAD_DIM / 64;
            const int ee = min(e, 31);
            const int extent = (e < nc && src.appends(ee)) ? HEAD_DIM * 2 : 0;
            const size_t at = (size_t)src.pair(ee) * HEAD_DIM;
            const __amdgpu_buffer_rsrc_t bk = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<half_t*>(a.k_new + at), 0, extent, 0x00020000);
            const __amdgpu_buffer_rsrc_t bv = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<half_t*>(a.v_new + at), 0, extent, 0x00020000);
            if constexpr (E == 2) {
                rk = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(bk, 4 * lane, 0, 0);
                rv = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(bv, 4 * lane, 0, 0);
            } else {
                rk = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(bk, 2 * lane, 0, 0);
                rv = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(bv, 2 * lane, 0, 0);
            }
        };
#pragma unroll
        // (the new rows are requested ahead of their entry's tiles: loads return in order, so the
        // rows are there -- and get quantised -- while the wave would only wait for the tiles)
        for (int u = 0; u < DEPTH; ++u) {
            if constexpr (APPEND) issue_rows(row_k[u], row_v[u], u);
            issue_entry(regs[u], u);
            __builtin_amdgcn_sched_barrier(0);     // keep the stages' loads in program order
        }
        for (int j = 0; j < nc; j += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int e = j + u;
                if (e < nc) {
                    const int rem = src.rem(e);
                    const int visA = rem - 4 * grp;
                    if constexpr (APPEND) {
                        if (src.appends(e)) {        // the pair's new token is the group's last
                            take_new_token<HEAD_DIM, KV>(regs[u][0], regs[u][1], row_k[u], row_v[u],
                                                         rem - 1, row_stage, lane);
                        }
                    }
                    if constexpr (BLOCK_REDUCE)
                        group_update_block_reduce<HEAD_DIM, KV>(
                            regs[u][0], regs[u][1], q_cur, m, l, acc, rem < 2 * kBlock, visA,
                            visA - kBlock, visA, visA - kBlock, a.scale_log2e, red, lane);
                    else
                        group_update<HEAD_DIM, KV>(regs[u][0], regs[u][1], q_cur, m, l, acc,
                                                   rem < 2 * kBlock, visA, visA - kBlock, visA,
                                                   visA - kBlock, a.scale_log2e);
                }
                // refill only after the stage's registers are dead, so the loads land in place --
                // and before the work at a segment's end, so that this does not delay them
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (APPEND) issue_rows(row_k[u], row_v[u], e + DEPTH);
                issue_entry(regs[u], e + DEPTH);
                __builtin_amdgcn_sched_barrier(0);
                if (e < nc) {
                    if (src.last(e)) {
                        // ---- the segment ends: its partial is (m, l, acc / l)
                        const PartialSlot ps = src.slot(e);
                        l += __shfl_xor(l, 16);
                        l += __shfl_xor(l, 32);
                        const float inv = 1.0f / l;
                        if (c0 + e == total - 1) {
                            // end of the share: nothing runs behind these stores
#pragma unroll
                            for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] *= inv;
                            store_partial<HEAD_DIM>(a, ps, acc, m * kLn2, l * kPUnshiftOf<KV>, lane);
                            if (parked.row0 >= 0) store_parked<HEAD_DIM>(a, parked, park, lane);
                        } else {
                            // Mid-stream: vector-memory stores here would sit between the tile
                            // loads in the in-order counter and stall the next group on their
                            // completion, so the partial is parked in LDS and stored at the end.
                            if (parked.row0 >= 0) store_parked<HEAD_DIM>(a, parked, park, lane);
#pragma unroll
                            for (int c = 0; c < HEAD_DIM / 16; ++c)
                                *reinterpret_cast<floatx4*>(park + 16 * (64 * c + lane)) = acc[c] * inv;
                            *reinterpret_cast<float*>(park + kParkAcc + 4 * lane) = m * kLn2;
                            *reinterpret_cast<float*>(park + kParkAcc + 256 + 4 * lane) = l * kPUnshiftOf<KV>;
                            parked = ps;
                            m = -INFINITY;
                            l = 0.0f;
#pragma unroll
                            for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
                            // The next segment's q was staged at least one refill (kGroupLoads
                            // tile loads, which complete in issue order behind it) ago.  The
                            // compiler does not track loads that write LDS, hence the explicit waits.
                            __builtin_amdgcn_s_waitcnt(kWaitStaged);
#pragma unroll
                            for (int jj = 0; jj < HEAD_DIM / 32; ++jj)
                                q_cur[jj] = *reinterpret_cast<const half8_t*>(q_stage + 1024 * jj + 16 * lane);
                            __builtin_amdgcn_s_waitcnt(kWaitLds);      // read before it is restaged
                            const int e2 = src.next_segment(e + 1);
                            if (e2 < nc)
                                stage_q_operand<HEAD_DIM, KV>(q_stage, src.q_rows(e2, HEAD_DIM), a.G, n, grp);
                        }
                    }
                }
            }
        }
    }
}

// Which share a workgroup takes.  Workgroup ids are dealt to the 8 XCDs round-robin; this gives the
// workgroups of XCD x the x-th contiguous eighth of the shares, so that neighbouring shares -- which
// read neighbouring KV heads' scale rows (two to a 128-byte line), the same q rows and the same
// block-table rows -- meet in one L2 instead of fetching those lines from HBM once per XCD.  Any
// dealing of workgroups to XCDs gives correct results: this is a bijection on [0, n).
__device__ __forceinline__ int share_of_workgroup(int wg, int n)
{
    const int x = wg & 7, k = wg >> 3, q = n >> 3, r = n & 7;
    return x * q + min(x, r) + k;
}

// One wave per workgroup.  The block numbers of up to 32 groups come from one gathered vector load
// (lane 2j+h = block h of the j-th group), whatever pairs they belong to.
template <int HEAD_DIM, int KV, int DEPTH, bool BIG, bool BLOCK_REDUCE, bool APPEND>
__global__ void __launch_bounds__(64)
flat_stream_kernel(const FlatArgs a)
{
    const int lane = threadIdx.x;
    const FlatSchedule sched(a.context_lens, a.new_slots, a.num_seqs, a.H_k, a.pair_extra, lane);
    const int ctotal = sched.cost_total();
    const FlatCut cut(max(ctotal, 1), a.decode_wgs, a.min_share);   // shares of the cost axis
    if (blockIdx.x == 0 && lane == 0) a.ws_header[0] = a.ws_tag;
    if (ctotal == 0) return;
    const int share = share_of_workgroup(blockIdx.x, a.decode_wgs);
    if (share >= cut.nwg) return;
    const int x_begin = sched.real_before(cut.begin(share), ctotal);
    const int x_end = sched.real_before(cut.begin(share + 1), ctotal);
    if (x_begin >= x_end) return;           // a share that lies inside one pair's extra units

    extern __shared__ __attribute__((aligned(16))) unsigned char q_stage[];    // see launch_flat_kernel
    LiveSource src(a, sched, cut, lane, share, x_begin, x_end);
    stream_share<HEAD_DIM, KV, DEPTH, BIG, BLOCK_REDUCE, APPEND>(a, src, q_stage, lane);
}

// The same stream from a prepared schedule: no schedule arithmetic and no block-table read stand
// between the launch and the first tile load, only the load of the workgroup's records.
template <int HEAD_DIM, int KV, int DEPTH, bool BIG, bool BLOCK_REDUCE, bool APPEND>
__global__ void __launch_bounds__(64)
flat_stream_prepared_kernel(const FlatArgs a)
{
    const int lane = threadIdx.x;
    // the tag, the share's size and its first 32 records are loaded together: one round trip
    const int share = share_of_workgroup(blockIdx.x, a.decode_wgs);
    const uint32_t* region = a.sched + a.sched_regions + (size_t)share * a.sched_stride;
    sched_rec_t first = {~0u, ~0u, 0u, 0u};
    if (lane < 32) first = *reinterpret_cast<const sched_rec_t*>(region + 4 + 4 * lane);
    const int count = wave_uniform((int)region[0]);
    if (wave_uniform((int)a.sched[0]) != (int)a.sched_tag) {
        // not the schedule this launch was told to expect: do nothing, leave a mark
        if (blockIdx.x == 0 && lane == 0) a.sched_w[1] = 1u;
        return;
    }
    if (count <= 0) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char q_stage[];
    PreparedSource src(a, region, lane, min(count, (a.sched_stride - 4) / 4), first);
    stream_share<HEAD_DIM, KV, DEPTH, BIG, BLOCK_REDUCE, APPEND>(a, src, q_stage, lane);
}

// Writes the schedule that flat_stream_prepared_kernel reads: the same grid as the attention launch
// it prepares (one wavefront per share) followed by one wavefront per (sequence, KV head) pair for
// the pairs' partial counts, each wavefront deriving its share exactly as flat_stream_kernel does
// and leaving one record per entry.
__global__ void __launch_bounds__(64)
flat_prepare_kernel(const FlatArgs a)
{
    const int lane = threadIdx.x;
    const FlatSchedule sched(a.context_lens, a.new_slots, a.num_seqs, a.H_k, a.pair_extra, lane);
    const int ctotal = sched.cost_total();
    const FlatCut cut(max(ctotal, 1), a.decode_wgs, a.min_share);
    uint32_t* out = a.sched_w;
    if ((int)blockIdx.x >= a.decode_wgs) {
        const int pair = blockIdx.x - a.decode_wgs;
        if (pair < a.num_seqs * a.H_k) {
            const int count = attention_partials_of(a, sched, cut, ctotal, pair);
            if (lane == 0) out[kSchedHeaderWords + pair] = (uint32_t)count;
        }
        if (pair == 0 && lane == 0) {
            out[1] = 0u;
            out[0] = a.sched_tag;
        }
        return;
    }
    uint32_t* region = out + a.sched_regions + (size_t)blockIdx.x * a.sched_stride;
    int x_begin = 0, x_end = 0;
    if (ctotal > 0 && (int)blockIdx.x < cut.nwg) {
        x_begin = sched.real_before(cut.begin(blockIdx.x), ctotal);
        x_end = sched.real_before(cut.begin(blockIdx.x + 1), ctotal);
    }
    // the region holds every share the cut can produce; the clamp only keeps the stores inside
    const int count = min(max(x_end - x_begin, 0), (a.sched_stride - 4) / 4);
    if (lane == 0) region[0] = (uint32_t)count;
    if (count == 0) return;
    LiveSource src(a, sched, cut, lane, (int)blockIdx.x, x_begin, x_begin + count);   // region = share
    for (int c0 = 0; c0 < count; c0 += 32) {
        src.load_chunk(c0);
        const int tile_b = __shfl_down(src.tile_l, 1);
        const int nb = (src.t_l + kBlock - 1) / kBlock;
        const int ng = max((nb + 1) >> 1, 1);
        const int pair_first = src.cfirst_l + src.g_l * (ng + a.pair_extra) + a.pair_extra;
        const int slot = min(max((int)blockIdx.x - cut.wg_of(pair_first), 0), a.max_slots - 1);
        const int rem = min(src.t_l - 2 * kBlock * src.gi_l, kSchedRemCap);
        const uint32_t last = (uint32_t)((src.last_mask >> lane) & 1);
        const uint32_t app = (uint32_t)((src.append_mask >> lane) & 1);
        const uint32_t pair = (uint32_t)(src.seq_l * a.H_k + src.g_l);
        if ((lane & 1) == 0 && (lane >> 1) < src.nc) {
            *reinterpret_cast<sched_rec_t*>(region + 4 + 4 * (c0 + (lane >> 1))) =
                sched_rec_t{(uint32_t)src.tile_l, (uint32_t)tile_b, pair | (app << 30) | (last << 31),
                      (uint32_t)rem | ((uint32_t)slot << 16)};
        }
    }
}

// Merges the partials of each (sequence, query head) row.  The number of partials of the row's
// (sequence, KV head) pair was left by the split kernel; pairs with no token at all have no writer,
// so the context length decides whether the count is meaningful.  All loads of the first kSpec
// partials are issued before the count is known (they lie inside the workspace whatever the count
// is), so the kernel is one memory round trip deep for rows of up to kSpec partials.
//   WIDE = false: one wavefront per row, four rows per workgroup.
//   WIDE = true (long contexts, tens of partials per row): one workgroup per row; wavefront w takes
//   partials w, w + 4, ... -- 4 * kSpec in the first round trip -- and the four sums meet in LDS.
// Fused step: the merge launch begins with one wavefront per (sequence, KV head) pair (four to a
// workgroup, ahead of the row workgroups: their stores take the longest, so they start first)
// that stores the pair's new row into the cache --
// Opt-KV Eq. 5 and Alg. 1 phase 1, the arithmetic and the bytes of the cache-write kernels.  The
// attention launch before it has already attended over the row from registers.
template <int HEAD_DIM>
__device__ __forceinline__ void append_new_row(const FlatArgs& a, int pair, int lane,
                                               const uint16_t (&kb)[HEAD_DIM / 64],
                                               const uint16_t (&vb)[HEAD_DIM / 64], int64_t slot, int t)
{
    constexpr int E = HEAD_DIM / 64;
    if (pair >= a.num_seqs * a.H_k) return;
    const int seq = pair / a.H_k;
    const int g = pair - seq * a.H_k;
    if (slot < 0 || t <= 0) return;                             // Eq. 5: filtered token
    // where the block table places position t - 1 (the slot names the same place)
    const int64_t blk = slot / kBlock;
    const int off = (int)(slot - blk * kBlock);
    const size_t tile = (size_t)(blk * a.H_k + g);
    if (a.kv_dtype != COOPT_KV_FP16) {
        float kx[E], vx[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            kx[e] = (float)__builtin_bit_cast(half_t, kb[e]);
            vx[e] = (float)__builtin_bit_cast(half_t, vb[e]);
        }
        if (a.kv_dtype == COOPT_KV_E5M2)
            quantise_values_to_cache<HEAD_DIM, COOPT_KV_E5M2>(kx, vx, tile, off, lane, a.k_cache_w,
                                                              a.v_cache_w, a.k_scale_w, a.v_scale_w);
        else
            quantise_values_to_cache<HEAD_DIM, COOPT_KV_E4M3>(kx, vx, tile, off, lane, a.k_cache_w,
                                                              a.v_cache_w, a.k_scale_w, a.v_scale_w);
    } else {
        uint16_t* kc = reinterpret_cast<uint16_t*>(a.k_cache_w) + tile * (kBlock * HEAD_DIM);
        uint16_t* vc = reinterpret_cast<uint16_t*>(a.v_cache_w) + tile * (kBlock * HEAD_DIM);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int dim = lane * E + e;
            kc[k_tile_index<2>(off, dim)] = kb[e];
            vc[v_tile_index<2>(off, dim)] = vb[e];
        }
    }
}

template <int HEAD_DIM, bool WIDE>
__global__ void __launch_bounds__(256)
flat_merge_kernel(const FlatArgs a)
{
    constexpr int E = HEAD_DIM / 64;
    constexpr int kSpec = 8;

    constexpr int kStep = WIDE ? 4 : 1;                 // distance between a wavefront's partials
    // Every load whose address does not depend on loaded data is issued before the first branch --
    // the schedule's tag, the pair's count, the length, the first 64 (max, sum) pairs and the first
    // kSpec partial rows -- so that the kernel is two memory round trips long, not one per check.
    const int wave = wave_uniform((int)(threadIdx.x >> 6));
    const int rows = a.num_seqs * a.H_q;
    // (fused step: the first append_wgs workgroups store the new rows, see below)
    const int wg = (int)blockIdx.x - a.append_wgs;
    const int row_id = WIDE ? wg : wg * 4 + wave;                              // seq * H_q + head
    const int row = min(max(row_id, 0), rows - 1);      // (a surplus wavefront reads the last row,
                                                        // an appending one the first)
    const int first = WIDE ? wave : 0;                  // this wavefront's first partial
    const int lane = threadIdx.x & 63;
    const int seq = row / a.H_q;
    const int g = (row - seq * a.H_q) / a.G;
    // an appending wavefront's row, slot and length are asked for here, with everything else and
    // ahead of it in program order (loads return in order: its wait then covers nothing more)
    const int app_pair = (int)blockIdx.x * 4 + wave;
    const int app_seq = min(app_pair, a.num_seqs * a.H_k - 1) / a.H_k;
    uint16_t app_k[E] = {}, app_v[E] = {};
    int64_t app_slot = -1;
    if (wg < 0) {
        const size_t at = (size_t)min(app_pair, a.num_seqs * a.H_k - 1) * HEAD_DIM + lane * E;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            app_k[e] = reinterpret_cast<const uint16_t*>(a.k_new)[at + e];
            app_v[e] = reinterpret_cast<const uint16_t*>(a.v_new)[at + e];
        }
        app_slot = a.new_slots[app_seq];
    }
    const size_t base = (size_t)row * a.max_slots;
    const float* ml = a.max_logits + base;
    const float* es = a.exp_sums + base;
    const float* po = a.tmp_out + base * HEAD_DIM + lane;

    // what the partials were laid out for: the schedule's tag, or the one the split kernel left
    const uint32_t* tag_at = a.sched ? a.sched : a.ws_header;
    const uint32_t tag = *tag_at;
    const int t = a.context_lens[wg < 0 ? app_seq : seq];
    int count = a.counts[seq * a.H_k + g];
    float o_spec[kSpec][E];
#pragma unroll
    for (int j = 0; j < kSpec; ++j) {
        const int p = first + kStep * j;
#pragma unroll
        for (int e = 0; e < E; ++e) o_spec[j][e] = p < a.max_slots ? po[(size_t)p * HEAD_DIM + 64 * e] : 0.0f;
    }
    const float ml_l = lane < a.max_slots ? ml[lane] : 0.0f;
    const float es_l = lane < a.max_slots ? es[lane] : 0.0f;
    // (the three scalar loads are taken here, together: left to the compiler, each moves down to
    // its first use, behind a branch that waits for the one before)
    asm volatile("" : "+s"(count) : "s"(tag), "s"(t));
    // a prepared schedule that is not the expected one (the split kernel wrote nothing), or partials
    // that a split call with another plan or shape left: nothing is written
    if (tag != (a.sched ? a.sched_tag : a.ws_tag)) return;
    if (wg < 0) {                                        // fused step only: the grid's head
        append_new_row<HEAD_DIM>(a, app_pair, lane, app_k, app_v, app_slot, t);
        return;
    }
    if (row_id >= rows) return;                         // (WIDE: never, the grid is the row count)
    if (t <= 0) count = 0;
    count = wave_uniform(min(count, a.max_slots));

    float o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.0f;
    float W = 1.0f;
    if (count > 0) {
        float M = lane < count ? ml_l : -INFINITY;
        for (int p = 64 + lane; p < count; p += 64) M = fmaxf(M, ml[p]);
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) M = fmaxf(M, __shfl_xor(M, s));
        const float wv = lane < count ? es_l * __expf(ml_l - M) : 0.0f;   // weights of partials 0..63
        W = wv;
#pragma unroll
        for (int j = 0; j < kSpec; ++j) {
            const int p = first + kStep * j;                               // < 64
            const float wj = __builtin_bit_cast(
                float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), p));
            if (p < count) {
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] += wj * o_spec[j][e];
            }
        }
        // further partials kSpec at a time, all loads of a batch in flight together (long contexts
        // have tens of partials per row: one dependent load per partial would cost a round trip each).
        // w holds the weights of partials b0 .. b0+63; the batch is partials p0, p0 + kStep, ...
        auto add_batch = [&](float w, int b0, int p0, int end) {
            float x[kSpec][E];
#pragma unroll
            for (int jj = 0; jj < kSpec; ++jj) {
                const int p = min(p0 + kStep * jj, end - 1);
#pragma unroll
                for (int e = 0; e < E; ++e) x[jj][e] = po[(size_t)p * HEAD_DIM + 64 * e];
            }
#pragma unroll
            for (int jj = 0; jj < kSpec; ++jj) {
                const int p = p0 + kStep * jj;
                const float wj = __builtin_bit_cast(
                    float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), (p - b0) & 63));
                if (p < end) {
#pragma unroll
                    for (int e = 0; e < E; ++e) o[e] += wj * x[jj][e];
                }
            }
        };
        const int end0 = min(count, 64);
        for (int p0 = first + kStep * kSpec; p0 < end0; p0 += kStep * kSpec) add_batch(wv, 0, p0, end0);
        for (int b0 = 64; b0 < count; b0 += 64) {                          // very long contexts
            const int p = b0 + lane;
            const float w2 = p < count ? es[p] * __expf(ml[p] - M) : 0.0f;
            W += w2;
            const int end = min(b0 + 64, count);
            for (int p0 = b0 + first; p0 < end; p0 += kStep * kSpec) add_batch(w2, b0, p0, end);
        }
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) W += __shfl_xor(W, s);
    }
    if constexpr (WIDE) {
        __shared__ float sm[4][HEAD_DIM];
#pragma unroll
        for (int e = 0; e < E; ++e) sm[wave][lane + 64 * e] = o[e];
        __syncthreads();
        if (wave == 0) {
            const float inv = count > 0 ? 1.0f / W : 0.0f;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int d = lane + 64 * e;
                a.out[(size_t)row * HEAD_DIM + d] = (half_t)((sm[0][d] + sm[1][d] + sm[2][d] + sm[3][d]) * inv);
            }
        }
    } else {
        const float inv = count > 0 ? 1.0f / W : 0.0f;
#pragma unroll
        for (int e = 0; e < E; ++e) a.out[(size_t)row * HEAD_DIM + lane + 64 * e] = (half_t)(o[e] * inv);
    }
}

template <int HEAD_DIM, int KV, bool BIG, int DEPTH, bool BLOCK_REDUCE, bool APPEND>
static void launch_flat_kernel(const FlatArgs& a, dim3 grid, hipStream_t stream)
{
    const dim3 block(64);
    // staging area of one q operand + one parked partial (o, m, l per lane) + reduction scratch +
    // the fused step's new K and V row
    const size_t lds = HEAD_DIM / 32 * 1024 + HEAD_DIM / 16 * 1024 + 512 + 512 + 4 * HEAD_DIM;
    if (a.sched)
        hipLaunchKernelGGL((flat_stream_prepared_kernel<HEAD_DIM, KV, DEPTH, BIG, BLOCK_REDUCE, APPEND>),
                           grid, block, lds, stream, a);
    else
        hipLaunchKernelGGL((flat_stream_kernel<HEAD_DIM, KV, DEPTH, BIG, BLOCK_REDUCE, APPEND>), grid,
                           block, lds, stream, a);
}

template <int HEAD_DIM, int KV, bool BIG, bool APPEND>
static void launch_flat_depth(const FlatArgs& a, const FlatPlan& plan, dim3 grid, hipStream_t stream)
{
    if (plan.block_reduce) {             // comparison variant: depth 2 only
        launch_flat_kernel<HEAD_DIM, KV, BIG, 2, true, APPEND>(a, grid, stream);
        return;
    }
    switch (plan.depth) {
    case 1: launch_flat_kernel<HEAD_DIM, KV, BIG, 1, false, APPEND>(a, grid, stream); break;
    case 3: launch_flat_kernel<HEAD_DIM, KV, BIG, 3, false, APPEND>(a, grid, stream); break;
    default: launch_flat_kernel<HEAD_DIM, KV, BIG, 2, false, APPEND>(a, grid, stream); break;
    }
}

template <int HEAD_DIM, int KV>
static void launch_flat_pool(const FlatArgs& a, bool big, const FlatPlan& plan, dim3 grid,
                             hipStream_t stream)
{
    const bool append = a.k_new != nullptr;
    if (big) {
        if (append) launch_flat_depth<HEAD_DIM, KV, true, true>(a, plan, grid, stream);
        else launch_flat_depth<HEAD_DIM, KV, true, false>(a, plan, grid, stream);
    } else {
        if (append) launch_flat_depth<HEAD_DIM, KV, false, true>(a, plan, grid, stream);
        else launch_flat_depth<HEAD_DIM, KV, false, false>(a, plan, grid, stream);
    }
}

int flat_max_slots(const coopt_shape* sh, const FlatPlan& plan)
{
    const int max_groups = (sh->max_blocks_per_seq + 1) / 2;
    const int min_share = plan.min_share_groups();
    // a pair's groups span at most this many shares (of at least min_share cost units each)
    return (max_groups + min_share - 1) / min_share + 1;
}

constexpr size_t kWsHeaderBytes = 16;

size_t flat_workspace_bytes(const coopt_shape* sh, const FlatPlan& plan)
{
    return kWsHeaderBytes +
           (size_t)sh->num_seqs * sh->num_q_heads * flat_max_slots(sh, plan) *
               (sh->head_dim + 2) * sizeof(float) +
           (size_t)sh->num_seqs * sh->num_kv_heads * sizeof(int32_t);
}

// Cost units charged per (sequence, KV head) pair that ends inside a share, in group times: on
// MI355X the masked last group of a pair and the hand-over to the next pair together take about
// as long as two ordinary groups.
constexpr int kPairExtra = 2;

// Upper bound of the cost axis' length (the kernels index it with 32-bit integers).
static long long flat_max_cost(const coopt_shape* sh)
{
    return (long long)sh->num_seqs * sh->num_kv_heads *
           ((sh->max_blocks_per_seq + 1) / 2 + kPairExtra);
}

// Workgroups (= wavefronts) to launch: the plan's grid, but never more than the work's upper bound
// at the minimum share.
static int flat_grid_groups(const coopt_shape* sh, const FlatPlan& plan)
{
    const int min_share = plan.min_share_groups();
    const long long max_total = flat_max_cost(sh);
    const long long groups = std::min((long long)plan.grid_waves, (max_total + min_share - 1) / min_share);
    return (int)std::max(groups, 1LL);
}

// Names what the layout of the partials in a workspace depends on, so that a merge call can tell
// partials that a split call with another shape or plan left.
static uint32_t ws_tag_of(const coopt_shape* sh, const FlatPlan& plan)
{
    uint32_t h = 2166136261u;
    const int fields[] = {0x57535031, sh->num_seqs, sh->num_q_heads, sh->num_kv_heads, sh->head_dim,
                          sh->max_blocks_per_seq, flat_grid_groups(sh, plan), plan.min_share_groups(),
                          kPairExtra, flat_max_slots(sh, plan)};
    for (int f : fields)
        for (int b = 0; b < 4; ++b) h = (h ^ ((uint32_t)f >> (8 * b) & 0xffu)) * 16777619u;
    return h | 1u;
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
    a.pair_extra = kPairExtra;
    a.pool_tiles = sh->num_blocks * sh->num_kv_heads;
    a.scale_log2e = sh->softmax_scale * kLog2e;
    const size_t rows = (size_t)sh->num_seqs * sh->num_q_heads;
    a.ws_header = (uint32_t*)workspace;
    a.ws_tag = ws_tag_of(sh, plan);
    a.tmp_out = (float*)((unsigned char*)workspace + kWsHeaderBytes);
    a.max_logits = a.tmp_out + rows * a.max_slots * sh->head_dim;
    a.exp_sums = a.max_logits + rows * a.max_slots;
    a.counts = reinterpret_cast<int32_t*>(a.exp_sums + rows * a.max_slots);
    return a;
}

// Where the parts of a prepared schedule lie (32-bit words) and the tag that names the layout and
// everything the records depend on besides the block tables and the lengths themselves.
struct SchedLayout {
    uint32_t tag;
    int regions, stride;
    size_t words;
};

static SchedLayout sched_layout(const coopt_shape* sh, const FlatPlan& plan, bool fused)
{
    SchedLayout L;
    const int wgs = flat_grid_groups(sh, plan);
    const int min_share = plan.min_share_groups();
    // a share never exceeds this many cost units, hence groups (see FlatCut): + 2 of slack
    // (and a region always holds 32 records, so the first chunk can be read unconditionally)
    const long long cap = std::max(std::max(flat_max_cost(sh) / wgs, 2LL * min_share) + 3, 32LL);
    L.stride = (int)(4 + 4 * cap);
    const int pairs = sh->num_seqs * sh->num_kv_heads;
    L.regions = kSchedHeaderWords + ((pairs + 3) & ~3);
    L.words = (size_t)L.regions + (size_t)wgs * L.stride;
    uint32_t h = 2166136261u;
    const int fields[] = {0x53434831, sh->num_seqs, sh->num_q_heads, sh->num_kv_heads, sh->head_dim,
                          sh->num_blocks, sh->max_blocks_per_seq, wgs, L.stride, min_share,
                          kPairExtra, flat_max_slots(sh, plan), fused ? 1 : 0};
    for (int f : fields)
        for (int b = 0; b < 4; ++b) h = (h ^ ((uint32_t)f >> (8 * b) & 0xffu)) * 16777619u;
    L.tag = h | 1u;                      // never the zero of fresh memory
    return L;
}

size_t flat_schedule_bytes(const coopt_shape* sh, const FlatPlan& plan)
{
    if (flat_max_cost(sh) > 0x7fffffffLL) return 0;
    const SchedLayout L = sched_layout(sh, plan, false);
    // record fields: 16 bits of slot, a region stride that stays a small int
    if (flat_max_slots(sh, plan) > 0xffff) return 0;
    if (flat_max_cost(sh) / flat_grid_groups(sh, plan) > (1 << 24)) return 0;
    return L.words * sizeof(uint32_t);
}

int launch_flat_prepare(const int32_t* block_tables, const int32_t* context_lens,
                        const int64_t* slot_mapping, void* schedule, const coopt_shape* sh,
                        const FlatPlan& plan, hipStream_t stream)
{
    if (flat_schedule_bytes(sh, plan) == 0) return COOPT_ERR_SHAPE;
    FlatArgs a = flat_args(sh, plan, nullptr);
    const SchedLayout L = sched_layout(sh, plan, slot_mapping != nullptr);
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.new_slots = slot_mapping;
    a.decode_wgs = flat_grid_groups(sh, plan);
    a.sched_w = (uint32_t*)schedule;
    a.sched_tag = L.tag;
    a.sched_regions = L.regions;
    a.sched_stride = L.stride;
    const long long wgs = (long long)a.decode_wgs + (long long)sh->num_seqs * sh->num_kv_heads;
    if (wgs > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    hipLaunchKernelGGL(flat_prepare_kernel, dim3((unsigned)wgs), dim3(64), 0, stream, a);
    return launch_status();
}

int launch_flat_split(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                      const float* v_scale, const int32_t* block_tables,
                      const int32_t* context_lens, void* workspace, const coopt_shape* sh,
                      const FlatPlan& plan, hipStream_t stream, const FlatAppend* append,
                      const void* schedule)
{
    if (flat_max_cost(sh) > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    FlatArgs a = flat_args(sh, plan, workspace);
    a.q = (const half_t*)q;
    a.cv = CacheView{(const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale};
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.decode_wgs = flat_grid_groups(sh, plan);
    long long wgs = a.decode_wgs;
    if (append) {
        a.new_slots = append->slot_mapping;
        a.k_new = (const half_t*)append->k;
        a.v_new = (const half_t*)append->v;
    }
    if (schedule) {
        if (flat_schedule_bytes(sh, plan) == 0) return COOPT_ERR_SHAPE;
        const SchedLayout L = sched_layout(sh, plan, append != nullptr);
        a.sched = (const uint32_t*)schedule;
        a.sched_w = (uint32_t*)const_cast<void*>(schedule);
        a.sched_tag = L.tag;
        a.sched_regions = L.regions;
        a.sched_stride = L.stride;
    }
    if (wgs > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 grid((unsigned)wgs);
    const bool big = !pool_fits_small(sh);
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_E4M3>(a, big, plan, grid, stream);
        else launch_flat_pool<64, COOPT_KV_E4M3>(a, big, plan, grid, stream);
    } else if (sh->kv_dtype == COOPT_KV_E5M2) {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_E5M2>(a, big, plan, grid, stream);
        else launch_flat_pool<64, COOPT_KV_E5M2>(a, big, plan, grid, stream);
    } else {
        if (sh->head_dim == 128) launch_flat_pool<128, COOPT_KV_FP16>(a, big, plan, grid, stream);
        else launch_flat_pool<64, COOPT_KV_FP16>(a, big, plan, grid, stream);
    }
    return launch_status();
}

int launch_flat_merge(const int32_t* context_lens, void* workspace, void* out, const coopt_shape* sh,
                      const FlatPlan& plan, hipStream_t stream, const void* schedule, bool fused,
                      const FlatAppend* append, const FlatCacheW* cache)
{
    FlatArgs a = flat_args(sh, plan, workspace);
    a.context_lens = context_lens;
    a.out = (half_t*)out;
    if (schedule) {    // the prepared counts instead of the ones a live split kernel leaves
        a.counts = reinterpret_cast<int32_t*>(const_cast<void*>(schedule)) + kSchedHeaderWords;
        a.sched = (const uint32_t*)schedule;
        a.sched_tag = sched_layout(sh, plan, fused).tag;
    }
    const size_t rows = (size_t)sh->num_seqs * sh->num_q_heads;
    const bool wide = a.max_slots > 32;      // rows may have tens of partials: a workgroup per row
    long long wgs = wide ? (long long)rows : (long long)((rows + 3) / 4);
    if (append) {
        a.new_slots = append->slot_mapping;
        a.k_new = (const half_t*)append->k;
        a.v_new = (const half_t*)append->v;
        a.k_cache_w = (uint8_t*)cache->k_cache;
        a.v_cache_w = (uint8_t*)cache->v_cache;
        a.k_scale_w = cache->k_scale;
        a.v_scale_w = cache->v_scale;
        a.kv_dtype = sh->kv_dtype;
        a.append_wgs = (int32_t)(((long long)sh->num_seqs * sh->num_kv_heads + 3) / 4);
        wgs += a.append_wgs;
    }
    if (wgs > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 rblock(256), rgrid((unsigned)wgs);
    if (wide) {
        if (sh->head_dim == 128)
            hipLaunchKernelGGL((flat_merge_kernel<128, true>), rgrid, rblock, 0, stream, a);
        else
            hipLaunchKernelGGL((flat_merge_kernel<64, true>), rgrid, rblock, 0, stream, a);
    } else {
        if (sh->head_dim == 128)
            hipLaunchKernelGGL((flat_merge_kernel<128, false>), rgrid, rblock, 0, stream, a);
        else
            hipLaunchKernelGGL((flat_merge_kernel<64, false>), rgrid, rblock, 0, stream, a);
    }
    return launch_status();
}

}  // namespace coopt
