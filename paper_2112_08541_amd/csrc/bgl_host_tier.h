// Second cache level in host memory (BGL paper, Sec. 3.2.3: a CPU cache with the
// same FIFO policy sits behind the GPU cache, in front of the feature store).
// Internal interface between the tier (host threads) and the GPU cache's tiered
// lookup, which launches the kernels that read the tier's page-locked rows.
#pragma once

#include <cstdint>

struct bgl_host_tier;

namespace bgl {

struct TierPlan {
    // Misses of the GPU cache are numbered by rank r (their order in miss_pos).
    // Ranks found in the tier and ranks fetched from the store, each in rank
    // order, with the row of the page-locked region (tier buffer rows first,
    // staging rows behind them) that holds each one's features.
    const int32_t *hit_rank;   // device-visible, n_hit entries
    const int64_t *hit_src;
    int64_t n_hit;
    const int32_t *miss_rank;  // device-visible, n_miss entries
    const int64_t *miss_src;
    int64_t n_miss;
};

// Page-locked list the GPU writes the missed node ids to (device-visible
// address) and its host view; capacity max_batch_rows ids.
int32_t *tier_ids_device(bgl_host_tier *t);
// Page-locked word for the GPU cache's hit count (device-visible address, host view).
int64_t *tier_count_device(bgl_host_tier *t);
const volatile int64_t *tier_count_host(bgl_host_tier *t);
const char *tier_rows_device(bgl_host_tier *t);
int64_t tier_max_batch(const bgl_host_tier *t);
int32_t tier_row_bytes(const bgl_host_tier *t);
int64_t tier_num_nodes(const bgl_host_tier *t);

// Step 1 (reads only): look the m ids up, list hits and misses, and move every
// hit row that step 2 is about to overwrite into the staging rows.  After it the
// rows of plan->hit_* may be read by the GPU.  Returns a BGL status.
int tier_lookup(bgl_host_tier *t, int64_t m, TierPlan *plan);
// Step 2: bring the missed rows in from the store and enter them first-in
// first-out.  After it the rows of plan->miss_* may be read.
int tier_insert(bgl_host_tier *t);

}  // namespace bgl
