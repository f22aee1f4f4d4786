// What the fused decode step needs from the allocator (host side, not part of the ABI).
#pragma once

#include "common.h"

namespace roll {

// Page-table deltas that travel to the fused kernel as kernel arguments.
constexpr int kMaxFusedDeltas = 128;

// The changes since the last commit, if they are exactly one decode step: every live slot grew
// by one token, empty slots stayed empty, and each pending page-table delta gives a slot the page
// that holds nothing but its newest token.  The kernel then derives the new lengths from the ones
// on the device and needs only the deltas.
struct FusedPlan {
    int32_t fusable = 0;   // 0: publish with roll_kv_commit_append and run the plain attention
    int32_t n_delta = 0;
    int32_t slot[kMaxFusedDeltas];
    int32_t page[kMaxFusedDeltas];
    int32_t num_slots = 0, max_pages = 0, num_pages = 0, page_size = 0;
    int32_t* page_table_dev = nullptr;
    int32_t* seq_lens_dev = nullptr;
};

int plan_fused_step(roll_kv_pool* pool, hipStream_t stream, FusedPlan* plan);
// After the kernel that applies a fusable plan has been enqueued: the pool's record of what the
// device holds moves on to the host state.
void finish_fused_step(roll_kv_pool* pool);

}  // namespace roll
