// Chunked prefill over the paged cache for gfx950: causal attention of a chunk of new query rows
// against history + chunk, both already in the cache (each row is Background Eq. 1 over its
// visible prefix, with the grouping of Opt-GQA Eq. 7 and the valid-block rule of Opt-Pa Eq. 9).
//
// Query length > 1 makes this a dense contraction, so the matrix cores are used at full width and
// every cache byte is fetched and converted once per WORKGROUP:
//   * A score tile has 16 query rows of ONE query head as its columns (column n = chunk row
//     i0+n).  A wavefront carries NR such tiles, a workgroup of 8 wavefronts 8*NR of them (256 rows
//     at NR = 2), all of the same (sequence, KV head) pair.
//   * The pair's K/V stream, two 16-token blocks (a group) at a time, through a double-buffered
//     LDS stage in matrix-core operand order, already converted to fp16.  The waves form two
//     producer teams that share a stage's groups three to one (the first team's waves are the
//     older ones on their SIMDs and get through a stage sooner); in a team wave 0 brings block
//     A's K, wave 1 block B's K, waves 2 and 3 the V pieces of both blocks (and zero the V entries
//     and scales of tokens that are not in the cache, so stale bytes cannot reach an accumulator).
//     All eight then read their operands back with 16-byte LDS loads, conflict-free, and run the
//     online-softmax update of attn_tile.hpp's arithmetic on each of their tiles.  One barrier
//     per stage of four groups; the global loads of the stage after next are in flight while a
//     stage is consumed.
//   * Workgroup ids are dealt to the 8 XCDs round-robin, so the mapping puts all workgroups of a
//     pair on ONE XCD: the pair's 2 MB of cache are fetched from HBM once and re-read from that
//     XCD's L2 by the pair's other workgroups.
//   * A launch runs in rounds of one workgroup per CU.  The tiles of a last round that would be
//     mostly empty go to a second launch: of half-size workgroups, or -- when the caller brings a
//     workspace -- of full-size workgroups, 2 to 8 per 16 tiles, that each stream one of as many
//     equal runs of the pair's stages and leave (m, l, unnormalised sums) per tile, which a merge
//     launch combines (Opt-Pa Eq. 10 over the parts).
// The only difference from decode in the arithmetic is that the visible-token limit is per column
// (causal).
#include "attn_tile.hpp"

namespace coopt {

struct PrefillArgs {
    const half_t* q;
    CacheView cv;
    const int32_t* block_tables;
    const int32_t* context_lens;
    const int32_t* query_start;
    half_t* out;
    int32_t H_q, H_k, G;
    int32_t max_blocks;
    int32_t pool_tiles;
    int32_t num_pairs;        // num_seqs * H_k
    int32_t wgs_per_pair;
    int32_t tile_base;        // this launch covers tiles [tile_base, tile_limit) of every pair
    int32_t tile_limit;
    float scale_log2e;
    // split launch (the last tiles of every pair, `split` workgroups per 16 tiles: workgroup p of
    // them streams the p-th of `split` equal runs of the pair's stages and leaves per tile 16 x
    // (m, l) and the 16 x HEAD_DIM unnormalised sums in `part`, which a merge launch combines)
    float* part;
    int32_t split;            // 0: whole streams, rows written to out;  >= 2: that many parts, partials
    int32_t tail_cap;         // tiles per pair the split launch covers (sizes `part`)
};

constexpr int kPrefillWaves = 8;                // two teams of four producer roles
constexpr int kPrefillGroupsPerStage = 4;      // two-block groups between two barriers
// Groups of a stage produced by the first team (waves 0-3); the second team takes the rest.
constexpr int kPrefillFirstTeamGroups = 3;
constexpr float kNoReference = -1.0e30f;        // a running reference below every score
constexpr int kPrefillCUs = 256;               // MI355X: the launch shape is planned for its CU count

// Byte offsets inside one LDS stage (one group = blocks A and B of one KV head).
template <int HEAD_DIM>
struct PrefillStage {
    static constexpr int kKOps = HEAD_DIM / 32;        // S^T MFMAs per block
    static constexpr int kVOps = HEAD_DIM / 16;        // O^T MFMAs per group
    static constexpr int kK = 0;                        // [2 blocks][kKOps][64 lanes] 8 halves
    static constexpr int kV = 2 * kKOps * 1024;         // [kVOps][64 lanes] 4 halves of A, 4 of B
    static constexpr int kS = kV + kVOps * 1024;        // 16 floats each: k_scale*c A, B; log2 v_scale A, B
    static constexpr int kR = kS + 256;                 // [64 lanes] 8 halves: 1/v_scale rows (below)
    static constexpr int kBytes = kR + 1024;
};

// One online-softmax step of a 16-column tile against a group whose operands are ready, in two
// parts so that the caller can issue the score products of all its tiles before the first
// softmax (the matrix pipe then works on the next tile's scores and on this tile's P.V while the
// vector ALU does the exponentials).
//   kA/kB = K operands of blocks A/B, vop = V operands of the group, ksc = k_scale * softmax_scale
//   * log2(e) and lv = log2(v_scale) of this lane's 4 tokens per block.  tail / visA / visB as in
//   group_update (attn_tile.hpp); absent tokens are already zero in vop and have lv = -inf.
template <int HEAD_DIM>
__device__ __forceinline__ void tile_scores(const half8_t (&kA)[HEAD_DIM / 32],
                                            const half8_t (&kB)[HEAD_DIM / 32],
                                            const half8_t (&qop)[HEAD_DIM / 32], floatx4& sA,
                                            floatx4& sB)
{
    sA = floatx4{0.f, 0.f, 0.f, 0.f};
    sB = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < HEAD_DIM / 32; ++jj) {
        sA = mfma_16x16x32(kA[jj], qop[jj], sA);
        sB = mfma_16x16x32(kB[jj], qop[jj], sB);
    }
}

// The weights enter the second product rounded to fp16, w~ = fp16(P * v_scale): one token's weight
// is then off by up to 2^-10 relative, which shows in the output when that token carries the row
// (an fp16 output near |x| = 3 moves by 1.5e-3).  So the row sum is taken from the SAME rounded
// weights, l = sum_j w~_j / v_scale_j: numerator and denominator then describe one softmax with
// weights perturbed by at most 2^-10 relative, whose result differs from the exact one by at most
// that times the weighted mean deviation of the value rows from the result -- nothing for one
// token or a dominant one.  (For the same reason the convert may truncate: a common bias of the
// weights cancels.)  The sum runs on the matrix cores: `rop` is a 16-row operand whose row 0
// holds 2^-8 / v_scale of the group's 32 tokens cut to fp16 and row 1 the remainder (the producers
// write it), so one more 16x16x32 product per tile accumulates it in rows 0 and 1 of `lacc`,
// which replaces eight vector additions.
//
// v_scale reaches the weight through the exponent: the producers leave lv = log2(v_scale) beside
// k_scale (both already normalised, see the kernel), the score of a token is z' = s * ksc + lv in
// one fused multiply-add, and the running reference m follows the maximum of z'.  The weight
// exp2(z' - m) = P * v_scale * 2^(...) then needs no multiplication of its own and is at most
// 2^(kPShift + kRescaleSlack) whatever the scales are.  A token that is not in the cache has
// lv = -inf and so the weight 0.
// The step in four parts, so that the caller can run the parts of its tiles side by side: the
// scores of a token (one fused multiply-add each) and their maximum; the rare raise of the running
// reference; the weights; the two matrix products.  TAIL: some of the group's tokens are not
// visible to every column.
template <bool TAIL>
__device__ __forceinline__ float tile_logits(floatx4 sA, floatx4 sB, floatx4 kscA, floatx4 kscB,
                                             floatx4 lvA, floatx4 lvB, int visA, int visB,
                                             float (&z)[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        z[i] = __builtin_fmaf(sA[i], kscA[i], lvA[i]);
        z[4 + i] = __builtin_fmaf(sB[i], kscB[i], lvB[i]);
    }
    if constexpr (TAIL) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {                   // (a select also drops a NaN score)
            z[i] = (i < visA) ? z[i] : -INFINITY;
            z[4 + i] = (i < visB) ? z[4 + i] : -INFINITY;
        }
    }
    return fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
}

template <int HEAD_DIM>
__device__ __forceinline__ void tile_raise(float bm, float& m, floatx4& lacc, floatx4 (&acc)[HEAD_DIM / 16])
{
    float nm = fmaxf(bm, __shfl_xor(bm, 16));
    nm = fmaxf(nm, __shfl_xor(nm, 32));
    nm = fmaxf(nm, m);
    const float alpha = __builtin_amdgcn_exp2f(m - nm);   // m = kNoReference at the start gives 0
    lacc *= alpha;
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] *= alpha;
    m = nm;
}

__device__ __forceinline__ half8_t tile_weights(const float (&z)[8], float m)
{
    const float mm = m - kPShift;
    half8_t pop;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const half2_t h = __builtin_bit_cast(
            half2_t, __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(z[i] - mm),      // invisible: exp2(-inf) = 0
                                                __builtin_amdgcn_exp2f(z[i + 1] - mm)));
        pop[i] = h.x;
        pop[i + 1] = h.y;
    }
    return pop;
}

template <int HEAD_DIM>
__device__ __forceinline__ void tile_pv(const half8_t (&vop)[HEAD_DIM / 16], half8_t rop, half8_t pop,
                                        floatx4& lacc, floatx4 (&acc)[HEAD_DIM / 16])
{
    lacc = mfma_16x16x32(rop, pop, lacc);
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) acc[c] = mfma_16x16x32(vop[c], pop, acc[c]);
}

template <int HEAD_DIM, int KV, int NR, bool BIG>
__global__ void __launch_bounds__(64 * kPrefillWaves, 2)
prefill_chunk_kernel(const PrefillArgs a)
{
    using St = PrefillStage<HEAD_DIM>;
    constexpr bool FP8 = kIsFp8<KV>;
    constexpr int NL = BlockRegs<HEAD_DIM, KV>::NL;   // 16-byte pieces per lane of a K (or V) tile
    constexpr int NLH = (NL + 1) / 2;                 // V pieces per V wave
    constexpr int NP = NL > 2 * NLH ? NL : 2 * NLH;   // producer registers per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];     // two stages of GPS groups

    const int lane = threadIdx.x & 63;
    const int wave_id = wave_uniform((int)(threadIdx.x >> 6));
    const int wave = wave_id & 3;                      // producer role inside its team
    const int team = wave_id >> 2;                     // which groups of a stage it produces: below
    const int n = lane & 15, grp = lane >> 4;
    // all workgroups of a (sequence, KV head) pair on one XCD (ids go round-robin over 8 XCDs)
    const int k8 = blockIdx.x >> 3;
    const int pair = (k8 / a.wgs_per_pair) * 8 + (blockIdx.x & 7);
    if (pair >= a.num_pairs) return;
    const int seq = pair / a.H_k;
    const int g = pair - seq * a.H_k;

    const int qs = a.query_start[seq];
    const int C = a.query_start[seq + 1] - qs;
    const int t = a.context_lens[seq];
    const int t_ctx = t - C;
    if (C <= 0) return;
    const int tiles_per_head = (C + 15) / 16;
    const int total_tiles = a.G * tiles_per_head;
    const int end_tile = min(total_tiles, a.tile_limit);
    const int in_pair = k8 % a.wgs_per_pair;
    const int parts = max(a.split, 1);
    const int part = in_pair % parts;                  // which run of the pair's stages is mine
    const int wg_first_tile = a.tile_base + (in_pair / parts) * (kPrefillWaves * NR);
    if (wg_first_tile >= end_tile) return;             // the whole workgroup leaves together
    const int first_tile = wg_first_tile + wave_id * NR;
    const bool active = first_tile < end_tile;         // a wave without tiles still produces

    half8_t qop[NR][HEAD_DIM / 32];
    int limit[NR];          // tokens visible to column n of tile r
    int row0[NR], head[NR];
    int my_max = 0, min_row = 0x7fffffff;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int tile = min(first_tile + r, end_tile - 1);      // surplus tiles repeat the last
        const int hh = tile / tiles_per_head;
        const int i0 = (tile - hh * tiles_per_head) * 16;
        const int row = min(i0 + n, C - 1);                      // surplus rows repeat row C-1
        head[r] = g * a.G + hh;
        row0[r] = i0;
        limit[r] = t_ctx + row + 1;
        my_max = max(my_max, t_ctx + min(i0 + 15, C - 1) + 1);
        min_row = min(min_row, i0);
        load_q_operand<HEAD_DIM, KV>(qop[r], a.q + ((size_t)(qs + row) * a.H_q + head[r]) * HEAD_DIM,
                                     true, grp);
    }
    if (!active) my_max = 0;
    // the workgroup streams as far as its longest column needs
    int wg_max = 0;
    for (int i = 0; i < kPrefillWaves * NR; ++i) {
        const int tile = min(wg_first_tile + i, end_tile - 1);
        const int i0 = (tile % tiles_per_head) * 16;
        wg_max = max(wg_max, t_ctx + min(i0 + 15, C - 1) + 1);
    }
    const int nblk = (wg_max + kBlock - 1) / kBlock;
    const int num_groups = (nblk + 1) >> 1;
    const int32_t* bt = a.block_tables + (size_t)seq * a.max_blocks;

    // ---- the pair's largest v_scale as a power of two.  The weights P * v_scale enter the second
    // product as fp16 (5 exponent bits); value rows can be of any magnitude (an E5M2 cache's scales
    // are 2^-7 of an E4M3 cache's, small value rows' smaller still), so every v_scale is divided by
    // the power of two just above the largest one among the tokens this workgroup reads: the
    // weights of the rows that matter then sit at fp16's upper end whatever the rows' magnitude.
    // The row sum divides each weight by the same normalised scale, so the factor stays in the
    // numerator alone and is taken out, exactly, in the final division.  One pass over the pair's
    // scales (64 bytes per block) before the stream starts.
    float vnorm = 1.0f, vdenorm = 1.0f;
    if constexpr (FP8) {
        __shared__ float vmax_of_wave[kPrefillWaves];
        float mx = 0.0f;
        constexpr int kBatch = 8;                          // loads in flight per lane
        for (int b0 = 0; b0 < nblk; b0 += 4 * kPrefillWaves * kBatch) {
            int id[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {             // lane group grp takes block b, all 16 tokens
                const int b = b0 + (u * kPrefillWaves + wave_id) * 4 + grp;
                id[u] = b < nblk ? bt[b] : -1;
            }
            float sc[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int b = b0 + (u * kPrefillWaves + wave_id) * 4 + grp;
                const bool in = id[u] >= 0 && b * kBlock + n < min(wg_max, t);
                sc[u] = in ? a.cv.v_scale[((size_t)id[u] * a.H_k + g) * kBlock + n] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) mx = fmaxf(mx, sc[u]);      // (fmaxf drops a NaN)
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        if (lane == 0) vmax_of_wave[wave_id] = mx;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPrefillWaves; ++i) mx = fmaxf(mx, vmax_of_wave[i]);
        // mx = f * 2^e with f in [1, 2): vnorm = 2^-(e+1), exact; nothing to normalise if no scale is positive
        const uint32_t ebits = (__builtin_bit_cast(uint32_t, mx) >> 23) & 0xffu;
        if (mx > 0.0f && ebits > 0u && ebits < 253u) {
            vnorm = __builtin_bit_cast(float, (253u - ebits) << 23);
            vdenorm = __builtin_bit_cast(float, (ebits + 1u) << 23);
        }
    }


    float m[NR];
    floatx4 lacc[NR];       // rows 0 and 1 (lanes of group 0, registers 0 and 1): the row sums / 2^8
    floatx4 acc[NR][HEAD_DIM / 16];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        // (finite, not -inf: a workgroup that streams a later run of a pair's stages meets
        // columns that see none of a group's tokens before any they do see, and the weights
        // exp2(z - m) of such a column must come out as exp2(-inf) = 0, not exp2(-inf + inf))
        m[r] = kNoReference;
        lacc[r] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < HEAD_DIM / 16; ++c) acc[r][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- which team produces which group of a stage.  The two waves of a SIMD do not get equal
    // shares of it: the older one (a wave of the first team) is through with a stage's groups well
    // before the younger one, so the first team produces more of the next stage.
    constexpr int GPS = kPrefillGroupsPerStage;
    constexpr int kFirst = kPrefillFirstTeamGroups;           // sub-groups 0 .. kFirst-1: team 0
    constexpr int kOwn = kFirst > GPS - kFirst ? kFirst : GPS - kFirst;   // most groups a wave holds
    static_assert(kFirst >= 1 && kFirst <= GPS, "the first team produces at least one group");
    auto owner = [](int sub) { return sub < kFirst ? 0 : 1; };
    auto own_index = [](int sub) { return sub < kFirst ? sub : sub - kFirst; };
    // ---- block numbers: lane 2i + b fetches the number of block b of the team's i-th group, in ONE
    // vector load per stage that is issued a whole stage before the tile loads it serves and ahead
    // of the tile loads of the stage before (the vector-memory counter is in order: by the time
    // those tiles have been waited for, the numbers are back).  Fetched where they are needed --
    // through the scalar unit or not -- their latency sat between two tile loads and again in
    // front of the barrier, every stage.
    const __amdgpu_buffer_rsrc_t bt_rsrc = TileLoader<HEAD_DIM, KV, BIG>::rsrc(bt, a.max_blocks * 4);
    auto load_ids = [&](int stage) {
        const int p = stage * GPS + (team == 0 ? 0 : kFirst) + (lane >> 1);
        const int b = min(2 * p + (lane & 1), nblk - 1);
        return __builtin_amdgcn_raw_buffer_load_b32(bt_rsrc, lane < 2 * kOwn ? 4 * b : 0, 0, 0);
    };
    auto id_of = [&](uint32_t ids, int i, int b) { return __builtin_amdgcn_readlane((int)ids, 2 * i + b); };

    // ---- producer side: this wave's pieces of group p
    const TileLoader<HEAD_DIM, KV, BIG> loader(a.cv, lane, a.pool_tiles);
    u32x4 prs[kOwn][NP];
    floatx4 pscs[kOwn];
    // The four producer roles of a team -- 0: K of block A, 1: K of block B, 2 and 3: the two halves
    // of the V pieces of both blocks (and the v_scale work of block A, B).  A V role costs twice a
    // K role (890 against 440 cycles per group).  The two teams take the roles crosswise: waves w
    // and w + 4 share a SIMD, so with the second team's roles shifted by two every SIMD carries
    // one K role and one V role (1 % faster than the same roles in both teams; shifts of one or
    // three, and rotating the roles from group to group inside a team, were slower).
    auto role_of = [&](int) { return (wave + 2 * team) & 3; };
    auto produce_issue = [&](int p, int blockA, int blockB, u32x4 (&pr)[NP], floatx4& psc) {
        const int role = role_of(p);
        const int vj0 = role == 2 ? 0 : NLH;               // first V piece of a V role
        const int vcnt = role == 2 ? NLH : NL - NLH;       // and how many it brings
        const bool okA = 2 * p < nblk, okB = 2 * p + 1 < nblk;
        const int tA = blockA * a.H_k + g;
        const int tB = blockB * a.H_k + g;
        // (one comparison for "is my block there": a choice between the two flags okA and okB
        // would be made in vector registers, the very ones the loads issued a moment ago will
        // fill, and cost a wait for those loads)
        const int mine = role & 1;                         // roles 0, 2: block A; roles 1, 3: block B
        const bool ok_mine = 2 * p + mine < nblk;
        const int t_mine = mine ? tB : tA;
        if (role < 2) {
#pragma unroll
            for (int j = 0; j < NL; ++j) pr[j] = loader.load_piece(a.cv.k_cache, t_mine, j, ok_mine);
            if constexpr (FP8) psc = loader.load_scales(a.cv.k_scale, t_mine, ok_mine);
        } else {
#pragma unroll
            for (int jj = 0; jj < NLH; ++jj) {
                if (jj < vcnt) {
                    pr[2 * jj] = loader.load_piece(a.cv.v_cache, tA, vj0 + jj, okA);
                    pr[2 * jj + 1] = loader.load_piece(a.cv.v_cache, tB, vj0 + jj, okB);
                }
            }
            if constexpr (FP8) psc = loader.load_scales(a.cv.v_scale, t_mine, ok_mine);
        }
    };
    auto produce_store = [&](int p, unsigned char* st, const u32x4 (&pr)[NP], const floatx4& psc) {
        const int role = role_of(p);
        const int vj0 = role == 2 ? 0 : NLH;
        const int vcnt = role == 2 ? NLH : NL - NLH;
        if (role < 2) {
            unsigned char* kdst = st + St::kK + role * (St::kKOps * 1024) + 16 * lane;
#pragma unroll
            for (int j = 0; j < NL; ++j) {
                if constexpr (FP8) {
                    *reinterpret_cast<half8_t*>(kdst + (2 * j) * 1024) = fp8x8_to_half8<KV>(pr[j].x, pr[j].y);
                    *reinterpret_cast<half8_t*>(kdst + (2 * j + 1) * 1024) = fp8x8_to_half8<KV>(pr[j].z, pr[j].w);
                } else {
                    *reinterpret_cast<u32x4*>(kdst + j * 1024) = pr[j];
                }
            }
            if constexpr (FP8) {
                if (n == 0)
                    *reinterpret_cast<floatx4*>(st + St::kS + 64 * role + 16 * grp) = psc * a.scale_log2e;
            }
        } else {
            // this lane's 4 tokens of block A start at 32p + 4grp, of block B 16 later
            const int cacheA = t - (32 * p + 4 * grp), cacheB = cacheA - kBlock;
            uint32_t a0 = 0xffffffffu, a1 = 0xffffffffu, b0 = 0xffffffffu, b1 = 0xffffffffu;
            if (32 * p + 2 * kBlock > t) {          // wave-uniform: only the cache's last group
                token_masks<KV>(cacheA, a0, a1);
                token_masks<KV>(cacheB, b0, b1);
            }
#pragma unroll
            for (int jj = 0; jj < NLH; ++jj) {
                if (jj < vcnt) {
                    if constexpr (FP8) {
                        const u32x4 wa = pr[2 * jj] & a0, wb = pr[2 * jj + 1] & b0;
#pragma unroll
                        for (int cc = 0; cc < 4; ++cc) {
                            const half4_t va = fp8x4_to_half4<KV>(wa[cc]), vb = fp8x4_to_half4<KV>(wb[cc]);
                            *reinterpret_cast<half8_t*>(st + St::kV + (4 * (vj0 + jj) + cc) * 1024 + 16 * lane) =
                                half8_t{va[0], va[1], va[2], va[3], vb[0], vb[1], vb[2], vb[3]};
                        }
                    } else {
                        const u32x4 wa = pr[2 * jj] & u32x4{a0, a1, a0, a1};
                        const u32x4 wb = pr[2 * jj + 1] & u32x4{b0, b1, b0, b1};
                        *reinterpret_cast<u32x4*>(st + St::kV + (2 * (vj0 + jj)) * 1024 + 16 * lane) =
                            u32x4{wa.x, wa.y, wb.x, wb.y};
                        *reinterpret_cast<u32x4*>(st + St::kV + (2 * (vj0 + jj) + 1) * 1024 + 16 * lane) =
                            u32x4{wa.z, wa.w, wb.z, wb.w};
                    }
                }
            }
            // v_scale of this role's block (role 2: A, role 3: B) times the pair's normaliser (an
            // exact power of two, the same for every token), zero for tokens not in the cache
            // (a stale scale), and the operand of the row-sum product: row 0 = 2^-8 / v_scale cut
            // to fp16, row 1 = the remainder, rows 2..15 zero; block A's tokens are the lane's
            // first four halves, block B's the other four
            const int cache = role == 2 ? cacheA : cacheB;
            floatx4 lv;
            half4_t rr;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float vs = FP8 ? ((i < cache) ? psc[i] * vnorm : 0.0f) : 1.0f;
                lv[i] = __builtin_amdgcn_logf(vs);                   // log2; -inf for an absent token
                // (the hardware reciprocal, 1 ulp: far inside what the fp16 pair keeps)
                const float r = fminf(vs > 0.0f ? 0.00390625f * __builtin_amdgcn_rcpf(vs) : 0.0f, 65504.0f);
                const float hi = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, r) & 0xffffe000u);
                rr[i] = n == 0 ? (half_t)hi : (n == 1 ? (half_t)(r - hi) : (half_t)0.0f);
            }
            if constexpr (FP8) {
                if (n == 0) *reinterpret_cast<floatx4*>(st + St::kS + 64 * role + 16 * grp) = lv;
            }
            *reinterpret_cast<half4_t*>(st + St::kR + 16 * lane + 8 * (role - 2)) = rr;
        }
    };

    // ---- consumer side
    const int full_limit = min(t, t_ctx + min_row + 1);   // tokens visible to every column of mine
    auto consume = [&](const unsigned char* st, int gi) {
        half8_t kA[St::kKOps], kB[St::kKOps], vop[St::kVOps];
#pragma unroll
        for (int jj = 0; jj < St::kKOps; ++jj) {
            kA[jj] = *reinterpret_cast<const half8_t*>(st + St::kK + jj * 1024 + 16 * lane);
            kB[jj] = *reinterpret_cast<const half8_t*>(st + St::kK + (St::kKOps + jj) * 1024 + 16 * lane);
        }
#pragma unroll
        for (int c = 0; c < St::kVOps; ++c)
            vop[c] = *reinterpret_cast<const half8_t*>(st + St::kV + c * 1024 + 16 * lane);
        const half8_t rop = *reinterpret_cast<const half8_t*>(st + St::kR + 16 * lane);
        floatx4 kscA, kscB, lvA, lvB;
        if constexpr (FP8) {
            kscA = *reinterpret_cast<const floatx4*>(st + St::kS + 16 * grp);
            kscB = *reinterpret_cast<const floatx4*>(st + St::kS + 64 + 16 * grp);
            lvA = *reinterpret_cast<const floatx4*>(st + St::kS + 128 + 16 * grp);
            lvB = *reinterpret_cast<const floatx4*>(st + St::kS + 192 + 16 * grp);
        } else {
            kscA = kscB = floatx4{a.scale_log2e, a.scale_log2e, a.scale_log2e, a.scale_log2e};
            lvA = lvB = floatx4{0.f, 0.f, 0.f, 0.f};              // log2 of a unit scale
        }
        const int baseA = 2 * gi * kBlock;
        const int tokA = baseA + 4 * grp;
        const bool hasB = 2 * gi + 1 < nblk;
        const bool tail = !(hasB && baseA + 2 * kBlock <= full_limit);
        floatx4 sA[NR], sB[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) tile_scores<HEAD_DIM>(kA, kB, qop[r], sA[r], sB[r]);
        // every tile's scores and maxima first, ONE (rare) branch for all of them, and then a
        // single stretch of straight-line code in which the weights of one tile (vector ALU,
        // exponentials) and the matrix products of the tile before it can run side by side
        float z[NR][8], bm[NR];
        if (tail) {
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int visA = limit[r] - tokA;
                bm[r] = tile_logits<true>(sA[r], sB[r], kscA, kscB, lvA, lvB, visA, hasB ? visA - kBlock : 0, z[r]);
            }
        } else {
#pragma unroll
            for (int r = 0; r < NR; ++r)
                bm[r] = tile_logits<false>(sA[r], sB[r], kscA, kscB, lvA, lvB, 0, 0, z[r]);
        }
        bool raise = false;
#pragma unroll
        for (int r = 0; r < NR; ++r) raise = raise || bm[r] > m[r] + kRescaleSlack;
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {            // wave-uniform, rare
#pragma unroll
            for (int r = 0; r < NR; ++r)
                if (__builtin_amdgcn_ballot_w64(bm[r] > m[r] + kRescaleSlack) != 0)
                    tile_raise<HEAD_DIM>(bm[r], m[r], lacc[r], acc[r]);
        }
        if constexpr (NR == 2) {
            // tile 0's weights; then tile 0's products with tile 1's weights between them, a pair
            // of exponentials to every two products (the matrix pipe and the vector ALU then work
            // side by side: each order is pinned by a scheduling fence); then tile 1's products
            const half8_t pop0 = tile_weights(z[0], m[0]);
            __builtin_amdgcn_sched_barrier(0);
            const float mm1 = m[1] - kPShift;
            half8_t pop1;
            lacc[0] = mfma_16x16x32(rop, pop0, lacc[0]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int c = 2 * i; c < 2 * i + 2; ++c)
                    if (c < HEAD_DIM / 16) acc[0][c] = mfma_16x16x32(vop[c], pop0, acc[0][c]);
                const half2_t h = __builtin_bit_cast(
                    half2_t, __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(z[1][2 * i] - mm1),
                                                        __builtin_amdgcn_exp2f(z[1][2 * i + 1] - mm1)));
                pop1[2 * i] = h.x;
                pop1[2 * i + 1] = h.y;
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int c = 8; c < HEAD_DIM / 16; ++c) acc[0][c] = mfma_16x16x32(vop[c], pop0, acc[0][c]);
            tile_pv<HEAD_DIM>(vop, rop, pop1, lacc[1], acc[1]);
        } else {
            half8_t pop[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) pop[r] = tile_weights(z[r], m[r]);
#pragma unroll
            for (int r = 0; r < NR; ++r) tile_pv<HEAD_DIM>(vop, rop, pop[r], lacc[r], acc[r]);
        }
    };

    // A stage holds GPS consecutive groups; one barrier per stage.  The workgroup streams stages
    // s_lo .. s_hi-1: all of them, or one of `parts` equal runs in a split launch (an empty run
    // leaves the neutral partial m = kNoReference, l = 0).
    const int num_stages = (num_groups + GPS - 1) / GPS;
    const int s_lo = (int)((long long)num_stages * part / parts);
    const int s_hi = (int)((long long)num_stages * (part + 1) / parts);
    const int g_end = min(num_groups, s_hi * GPS);            // groups below this one are mine
    auto slot = [&](int si, int sub) { return lds + ((si & 1) * GPS + sub) * St::kBytes; };
    // (a wave keeps registers for the sub-groups of its own team)
    uint32_t ids = load_ids(s_lo);
#pragma unroll
    for (int sub = 0; sub < GPS; ++sub)
        if (owner(sub) == team && s_lo * GPS + sub < g_end)
            produce_issue(s_lo * GPS + sub, id_of(ids, own_index(sub), 0), id_of(ids, own_index(sub), 1),
                          prs[own_index(sub)], pscs[own_index(sub)]);
    ids = load_ids(s_lo + 1);
    uint32_t ids_next = load_ids(s_lo + 2);
#pragma unroll
    for (int sub = 0; sub < GPS; ++sub)
        if (owner(sub) == team && s_lo * GPS + sub < g_end)
            produce_store(s_lo * GPS + sub, slot(s_lo, sub), prs[own_index(sub)], pscs[own_index(sub)]);
#pragma unroll
    for (int sub = 0; sub < GPS; ++sub)
        if (owner(sub) == team && (s_lo + 1) * GPS + sub < g_end)
            produce_issue((s_lo + 1) * GPS + sub, id_of(ids, own_index(sub), 0), id_of(ids, own_index(sub), 1),
                          prs[own_index(sub)], pscs[own_index(sub)]);
    __syncthreads();
    for (int si = s_lo; si < s_hi; ++si) {
#pragma unroll
        for (int sub = 0; sub < GPS; ++sub) {
            const int gi = si * GPS + sub;
            if (gi < g_end && 2 * gi * kBlock < my_max) consume(slot(si, sub), gi);
        }
#pragma unroll
        for (int sub = 0; sub < GPS; ++sub) {
            const int gn = (si + 1) * GPS + sub;
            if (owner(sub) == team && gn < g_end)
                produce_store(gn, slot(si + 1, sub), prs[own_index(sub)], pscs[own_index(sub)]);
        }
        // the numbers fetched a stage ago go to scalar registers before anything new is issued,
        // so that taking them waits for nothing younger than the tiles just stored
        int blk[kOwn][2];
#pragma unroll
        for (int i = 0; i < kOwn; ++i) {
            blk[i][0] = id_of(ids_next, i, 0);
            blk[i][1] = id_of(ids_next, i, 1);
            // (pinned here: moved down to their uses, each would wait for the loads issued before it)
            asm volatile("" : "+s"(blk[i][0]), "+s"(blk[i][1]));
        }
        ids_next = load_ids(si + 3);
#pragma unroll
        for (int sub = 0; sub < GPS; ++sub) {
            const int g2 = (si + 2) * GPS + sub;
            if (owner(sub) == team && g2 < g_end)
                produce_issue(g2, blk[own_index(sub)][0], blk[own_index(sub)][1], prs[own_index(sub)],
                              pscs[own_index(sub)]);
        }
        // stage si+1 is complete, and nobody still reads stage si
        __syncthreads();
    }

    if (!active) return;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        // column n's sum sits in rows 0 and 1 of lacc: lane (n, 0), registers 0 and 1
        const float L = __shfl(lacc[r][0] + lacc[r][1], n) * 256.0f;
        // (the 2^kPShift common to acc and l cancels; the normaliser of the v_scales is in acc alone)
        if (a.split) {
            // this run's share of the tile: reference, row sum and unnormalised sums per column
            if (first_tile + r < end_tile) {
                float* dst = a.part + (((size_t)pair * a.tail_cap + (first_tile + r - a.tile_base)) * parts + part) *
                                          (16 * (HEAD_DIM + 2));
                if (grp == 0) {
                    dst[n] = m[r];
                    dst[16 + n] = L;
                }
#pragma unroll
                for (int c = 0; c < HEAD_DIM / 16; ++c)
                    *reinterpret_cast<floatx4*>(dst + 32 + n * HEAD_DIM + 16 * c + 4 * grp) = acc[r][c] * vdenorm;
            }
            continue;
        }
        const float inv = (1.0f / L) * vdenorm;
        const int row = row0[r] + n;
        if (first_tile + r < end_tile && row < C) {
            half_t* dst = a.out + ((size_t)(qs + row) * a.H_q + head[r]) * HEAD_DIM + 4 * grp;
#pragma unroll
            for (int c = 0; c < HEAD_DIM / 16; ++c) {
                half4_t h;
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = (half_t)(acc[r][c][i] * inv);
                *reinterpret_cast<half4_t*>(dst + 16 * c) = h;
            }
        }
    }
}

// Combines the parts a split launch left for every tile: with M = max_p m_p and e_p = 2^(m_p - M),
// row = sum_p A_p e_p / sum_p l_p e_p (the merge rule of the online softmax, Opt-Pa Eq. 10).  One
// wavefront per tile, lane (n, grp) as in the kernel.
template <int HEAD_DIM>
__global__ void __launch_bounds__(256)
prefill_split_merge_kernel(const PrefillArgs a)
{
    constexpr int kPart = 16 * (HEAD_DIM + 2);          // floats per tile and part
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, grp = lane >> 4;
    const long long id = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);      // pair * tail_cap + tile
    if (id >= (long long)a.num_pairs * a.tail_cap) return;
    const int pair = (int)(id / a.tail_cap);
    const int tile = a.tile_base + (int)(id - (long long)pair * a.tail_cap);
    const int seq = pair / a.H_k;
    const int g = pair - seq * a.H_k;
    const int qs = a.query_start[seq];
    const int C = a.query_start[seq + 1] - qs;
    if (C <= 0) return;
    const int tiles_per_head = (C + 15) / 16;
    if (tile >= a.G * tiles_per_head) return;
    const int hh = tile / tiles_per_head;
    const int row = (tile - hh * tiles_per_head) * 16 + n;
    if (row >= C) return;
    const int parts = a.split;
    const float* p0 = a.part + (size_t)id * parts * kPart;
    float M = kNoReference;                 // (a row sees at least one token: some part has a real m)
    for (int p = 0; p < parts; ++p) M = fmaxf(M, p0[p * kPart + n]);
    float den = 0.0f;
    for (int p = 0; p < parts; ++p)
        den += p0[p * kPart + 16 + n] * __builtin_amdgcn_exp2f(p0[p * kPart + n] - M);
    const float inv = 1.0f / den;
    half_t* dst = a.out + ((size_t)(qs + row) * a.H_q + g * a.G + hh) * HEAD_DIM + 4 * grp;
#pragma unroll
    for (int c = 0; c < HEAD_DIM / 16; ++c) {
        floatx4 x = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < parts; ++p)
            x += *reinterpret_cast<const floatx4*>(p0 + p * kPart + 32 + n * HEAD_DIM + 16 * c + 4 * grp) *
                 __builtin_amdgcn_exp2f(p0[p * kPart + n] - M);
        half4_t h;
#pragma unroll
        for (int i = 0; i < 4; ++i) h[i] = (half_t)(x[i] * inv);
        *reinterpret_cast<half4_t*>(dst + 16 * c) = h;
    }
}

// How the tiles of every pair are dealt to launches.  One workgroup (8 waves, 2 tiles each) fills
// a CU, so a launch runs in rounds of one workgroup per CU, and a last round that is mostly empty
// costs a full one.  Where that happens the last tiles of every pair go to a second launch: of
// half-size workgroups (one tile per wave), which takes about 0.65-0.8 of a round -- or, when the
// caller brings a workspace, of full-size workgroups, `parts` per 16 tiles, that each stream one
// of `parts` equal runs of the pair's stages, with `parts` (2 to 8) chosen so that the round is as
// short as it gets (a launch of fewer workgroups than CUs is all "last round": a single
// sequence's chunk is spread over the chip this way); the parts are combined by
// prefill_split_merge_kernel.
constexpr int kPrefillMaxParts = 8;
struct PrefillLaunchPlan {
    int tiles, pairs8, a_per_pair, b_per_pair, rest, parts;
    int nr;          // tiles per wave of the full-size workgroups: 2, or 1 where a pair has at most 8 tiles
    int wg_tiles;    // = 8 nr
    PrefillLaunchPlan(const coopt_shape* sh, int max_chunk_len, bool with_workspace)
    {
        const int G = sh->num_q_heads / sh->num_kv_heads;
        tiles = G * ((max_chunk_len + 15) / 16);
        pairs8 = (sh->num_seqs * sh->num_kv_heads + 7) / 8 * 8;
        // (a short chunk -- 16 rows of a five-head group, say -- gives every wave one tile at
        // most: the one-tile kernel then does the same work with fewer registers and 0.78 of the
        // round time)
        nr = tiles <= kPrefillWaves ? 1 : 2;
        wg_tiles = nr * kPrefillWaves;
        const int full_per_pair = (tiles + wg_tiles - 1) / wg_tiles;
        a_per_pair = full_per_pair;
        b_per_pair = 0;
        rest = 0;
        parts = 0;
        auto rounds = [](long long wgs) { return (double)((wgs + kPrefillCUs - 1) / kPrefillCUs); };
        const long long W = (long long)pairs8 * full_per_pair;
        const int cand = (int)((W / kPrefillCUs) * kPrefillCUs / pairs8);   // full rounds only
        if (cand >= full_per_pair) return;                                   // whole rounds
        const int r = tiles - cand * wg_tiles;                               // tiles of the last round, per pair
        if (with_workspace) {
            // p parts make p times the workgroups, each 1/p as long; a part costs about 2 % of a
            // round on top (its start, its partial rows, its share of the merge)
            const long long last = (long long)pairs8 * ((r + wg_tiles - 1) / wg_tiles);
            int best = 1;
            double best_cost = rounds(last);
            for (int p = 2; p <= kPrefillMaxParts; ++p) {
                const double cost = rounds(last * p) / p + 0.02 * (p - 1);
                if (cost < best_cost) {
                    best_cost = cost;
                    best = p;
                }
            }
            if (best >= 2) {
                a_per_pair = cand;
                rest = r;
                parts = best;
                return;
            }
        }
        if (cand >= 1 && nr == 2) {
            const int small = (r + kPrefillWaves - 1) / kPrefillWaves;
            const double split = rounds((long long)pairs8 * cand) + 0.65 * rounds((long long)pairs8 * small);
            if (split < rounds(W)) {
                a_per_pair = cand;
                b_per_pair = small;
                rest = r;
            }
        }
    }
    // workgroups per pair of the split form of the second launch
    int split_per_pair() const { return parts * ((rest + wg_tiles - 1) / wg_tiles); }
    size_t workspace_bytes(const coopt_shape* sh) const
    {
        if (parts < 2) return 0;
        return (size_t)sh->num_seqs * sh->num_kv_heads * rest * parts * 16 * (sh->head_dim + 2) * sizeof(float);
    }
};

}  // namespace coopt

using namespace coopt;

extern "C" size_t coopt_prefill_workspace_bytes(const coopt_shape* sh, int32_t max_chunk_len)
{
    if (check_shape(sh) != COOPT_OK || max_chunk_len <= 0 || sh->num_seqs == 0) return 0;
    return PrefillLaunchPlan(sh, max_chunk_len, true).workspace_bytes(sh);
}

static int prefill_chunk(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                         const float* v_scale, const int32_t* block_tables, const int32_t* context_lens,
                         const int32_t* query_start, int32_t num_query_rows, int32_t max_chunk_len,
                         void* out, void* workspace, const coopt_shape* sh, void* hip_stream);

extern "C" int coopt_paged_gqa_prefill_chunk(const void* q, const void* k_cache, const void* v_cache,
                                             const float* k_scale, const float* v_scale,
                                             const int32_t* block_tables,
                                             const int32_t* context_lens,
                                             const int32_t* query_start, int32_t num_query_rows,
                                             int32_t max_chunk_len, void* out,
                                             const coopt_shape* sh, void* hip_stream)
{
    return prefill_chunk(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, query_start,
                         num_query_rows, max_chunk_len, out, nullptr, sh, hip_stream);
}

extern "C" int coopt_paged_gqa_prefill_chunk_ws(const void* q, const void* k_cache, const void* v_cache,
                                                const float* k_scale, const float* v_scale,
                                                const int32_t* block_tables,
                                                const int32_t* context_lens,
                                                const int32_t* query_start, int32_t num_query_rows,
                                                int32_t max_chunk_len, void* out, void* workspace,
                                                size_t workspace_bytes, const coopt_shape* sh,
                                                void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (max_chunk_len > 0 && sh->num_seqs > 0) {
        const size_t need = PrefillLaunchPlan(sh, max_chunk_len, true).workspace_bytes(sh);
        if (need > 0 && !workspace) return COOPT_ERR_NULL;
        if (workspace_bytes < need) return COOPT_ERR_WORKSPACE;
        if (need == 0) workspace = nullptr;
    }
    return prefill_chunk(q, k_cache, v_cache, k_scale, v_scale, block_tables, context_lens, query_start,
                         num_query_rows, max_chunk_len, out, workspace, sh, hip_stream);
}

static int prefill_chunk(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                         const float* v_scale, const int32_t* block_tables, const int32_t* context_lens,
                         const int32_t* query_start, int32_t num_query_rows, int32_t max_chunk_len,
                         void* out, void* workspace, const coopt_shape* sh, void* hip_stream)
{
    int st = check_shape(sh);
    if (st != COOPT_OK) return st;
    if (num_query_rows < 0 || max_chunk_len < 0) return COOPT_ERR_SHAPE;
    if (sh->num_seqs == 0 || num_query_rows == 0 || max_chunk_len == 0) return COOPT_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !context_lens || !query_start || !out)
        return COOPT_ERR_NULL;
    if (sh->kv_dtype != COOPT_KV_FP16 && (!k_scale || !v_scale)) return COOPT_ERR_NULL;

    PrefillArgs a{};
    a.q = (const half_t*)q;
    a.cv = CacheView{(const uint8_t*)k_cache, (const uint8_t*)v_cache, k_scale, v_scale};
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.query_start = query_start;
    a.out = (half_t*)out;
    a.H_q = sh->num_q_heads;
    a.H_k = sh->num_kv_heads;
    a.G = sh->num_q_heads / sh->num_kv_heads;
    a.max_blocks = sh->max_blocks_per_seq;
    a.pool_tiles = sh->num_blocks * sh->num_kv_heads;
    a.scale_log2e = sh->softmax_scale * kLog2e;
    a.num_pairs = sh->num_seqs * sh->num_kv_heads;

    const PrefillLaunchPlan lp(sh, max_chunk_len, workspace != nullptr);
    const int pairs8 = lp.pairs8, a_per_pair = lp.a_per_pair, b_per_pair = lp.b_per_pair;
    const bool split = lp.parts >= 2;
    const int split_per_pair = lp.split_per_pair();
    if ((long long)pairs8 * (a_per_pair + b_per_pair + split_per_pair) > 0x7fffffffLL) return COOPT_ERR_SHAPE;
    const dim3 block(64 * kPrefillWaves);
    const size_t lds = 2 * kPrefillGroupsPerStage *
                       (size_t)(sh->head_dim == 128 ? PrefillStage<128>::kBytes : PrefillStage<64>::kBytes);
    hipStream_t stream = (hipStream_t)hip_stream;
    const bool big = !pool_fits_small(sh);
#define COOPT_PREFILL_FULL(D, KV, BIG, NR)                                                          \
    do {                                                                                            \
        a.tile_base = 0;                                                                            \
        a.tile_limit = (b_per_pair || split) ? a_per_pair * lp.wg_tiles : 0x7fffffff;               \
        a.wgs_per_pair = a_per_pair;                                                                \
        if (a_per_pair > 0)                                                                         \
            hipLaunchKernelGGL((prefill_chunk_kernel<D, KV, NR, BIG>),                              \
                               dim3((unsigned)((long long)pairs8 * a_per_pair)), block, lds, stream, a); \
        a.tile_base = a.tile_limit;                                                                 \
        a.tile_limit = 0x7fffffff;                                                                  \
        if (split) {                                                                                \
            a.wgs_per_pair = split_per_pair;                                                        \
            a.part = (float*)workspace;                                                             \
            a.split = lp.parts;                                                                     \
            a.tail_cap = lp.rest;                                                                   \
            hipLaunchKernelGGL((prefill_chunk_kernel<D, KV, NR, BIG>),                              \
                               dim3((unsigned)((long long)pairs8 * split_per_pair)), block, lds, stream, a); \
            const long long waves = (long long)a.num_pairs * lp.rest;                               \
            hipLaunchKernelGGL((prefill_split_merge_kernel<D>), dim3((unsigned)((waves + 3) / 4)),   \
                               dim3(256), 0, stream, a);                                            \
        }                                                                                           \
    } while (0)
#define COOPT_PREFILL(D, KV, BIG)                                                                   \
    do {                                                                                            \
        if (lp.nr == 1) {                                                                           \
            COOPT_PREFILL_FULL(D, KV, BIG, 1);                                                      \
        } else {                                                                                    \
            COOPT_PREFILL_FULL(D, KV, BIG, 2);                                                      \
            if (!split && b_per_pair) {                                                             \
                a.wgs_per_pair = b_per_pair;                                                        \
                hipLaunchKernelGGL((prefill_chunk_kernel<D, KV, 1, BIG>),                           \
                                   dim3((unsigned)((long long)pairs8 * b_per_pair)), block, lds, stream, a); \
            }                                                                                       \
        }                                                                                           \
    } while (0)
    if (sh->kv_dtype == COOPT_KV_E4M3) {
        if (sh->head_dim == 128) { if (big) COOPT_PREFILL(128, COOPT_KV_E4M3, true); else COOPT_PREFILL(128, COOPT_KV_E4M3, false); }
        else { if (big) COOPT_PREFILL(64, COOPT_KV_E4M3, true); else COOPT_PREFILL(64, COOPT_KV_E4M3, false); }
    } else if (sh->kv_dtype == COOPT_KV_E5M2) {
        if (sh->head_dim == 128) { if (big) COOPT_PREFILL(128, COOPT_KV_E5M2, true); else COOPT_PREFILL(128, COOPT_KV_E5M2, false); }
        else { if (big) COOPT_PREFILL(64, COOPT_KV_E5M2, true); else COOPT_PREFILL(64, COOPT_KV_E5M2, false); }
    } else {
        if (sh->head_dim == 128) { if (big) COOPT_PREFILL(128, COOPT_KV_FP16, true); else COOPT_PREFILL(128, COOPT_KV_FP16, false); }
        else { if (big) COOPT_PREFILL(64, COOPT_KV_FP16, true); else COOPT_PREFILL(64, COOPT_KV_FP16, false); }
    }
#undef COOPT_PREFILL
#undef COOPT_PREFILL_FULL
    return launch_status();
}
