// Host-side glue between the decode entry points (decode.hip) and the load-balanced kernel
// (decode_flat.hip).
#pragma once

#include <algorithm>

#include "common.hpp"

namespace coopt {

struct FlatPlan {
    int tokens_per_group;   // minimum share of a workgroup, in tokens (32 per two-block group)
    int depth;              // two-block groups in flight per wavefront
    int grid_waves;         // wavefronts (= single-wave workgroups) in the whole grid
    int block_reduce;       // 1: softmax statistics reduced through LDS at every group (comparison)
    int min_share_groups() const { return std::max(1, tokens_per_group / (2 * kBlock)); }
};

size_t flat_workspace_bytes(const coopt_shape* sh, const FlatPlan& plan);

// The token every sequence appends in a fused step: fp16 rows [num_seqs][H_k][d] and the slot of
// each (negative: that sequence appends nothing).
struct FlatAppend {
    const void* k;
    const void* v;
    const int64_t* slot_mapping;
};

// The cache as the fused step writes to it (scales NULL for fp16 caches).
struct FlatCacheW {
    void* k_cache;
    void* v_cache;
    float* k_scale;
    float* v_scale;
};

// Enqueue the balanced split kernel (attention -> partial results in the workspace; with `append`
// also the cache write of one new token per sequence and that token's partial) and the merge
// kernel (partials -> fp16 output rows; with `append` and `cache` it also stores the new rows,
// which the split kernel only attended over).  Both derive the same schedule from the context lengths
// and the plan, so the plan must not change between them.  With `schedule` (written by
// launch_flat_prepare for the same shape, plan and mode) the split kernel reads its shares from
// there instead of deriving them (block_tables is then unused), and the merge kernel the counts
// (`fused` = the mode the schedule was prepared for).
// Each returns a coopt_status.
int launch_flat_split(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                      const float* v_scale, const int32_t* block_tables,
                      const int32_t* context_lens, void* workspace, const coopt_shape* sh,
                      const FlatPlan& plan, hipStream_t stream, const FlatAppend* append = nullptr,
                      const void* schedule = nullptr);
int launch_flat_merge(const int32_t* context_lens, void* workspace, void* out, const coopt_shape* sh,
                      const FlatPlan& plan, hipStream_t stream, const void* schedule = nullptr,
                      bool fused = false, const FlatAppend* append = nullptr,
                      const FlatCacheW* cache = nullptr);

// Bytes of a prepared schedule for this shape and plan (0: the shape is out of range), and the
// launch that writes one: slot_mapping NULL for plain decode, else the fused step's new tokens.
size_t flat_schedule_bytes(const coopt_shape* sh, const FlatPlan& plan);
int launch_flat_prepare(const int32_t* block_tables, const int32_t* context_lens,
                        const int64_t* slot_mapping, void* schedule, const coopt_shape* sh,
                        const FlatPlan& plan, hipStream_t stream);

}  // namespace coopt
