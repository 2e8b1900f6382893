// Second cache level in host memory (BGL paper, Sec. 3.2.3: a CPU cache with the
// same FIFO policy sits behind the GPU cache, in front of the feature store).
// Internal interface between the tier and the GPU cache's tiered lookup, which
// owns the stream order and launches the kernels that read the tier's rows.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

struct bgl_host_tier;

namespace bgl {

struct TierPlan {
    // Misses of the GPU cache are numbered by rank r (their order in miss_pos).
    int64_t n_hit_gpu;         // hits in the GPU cache (read back with the tier's counts)
    const int32_t *hit_rank;   // device: ranks the tier holds, ascending; the h-th one's row is
    const char *stage;         // copied to row h of these page-locked staging rows (device-visible address)
    int64_t n_hit;
    const int32_t *miss_rank;  // device: ranks it does not hold, ascending (null: all of them); the j-th one's row
    int64_t n_miss;            // goes to ring position (ptail + j) mod ring
    uint64_t ptail;
    int64_t ring;
};

// Page-locked words the device writes counts to: [0] hits in the GPU cache
// (the cache's lookup writes it), [1] tier hits, [2] tier misses, [3] bad-id flag.
int64_t *tier_count_device(bgl_host_tier *t);
const char *tier_rows_device(bgl_host_tier *t);
int64_t tier_max_batch(const bgl_host_tier *t);
int64_t tier_capacity(const bgl_host_tier *t);
// A tier of capacity 0 has no map to look anything up in: the cache's own list kernel writes the ids
// of its misses, in order, to this page-locked list (device-visible address) and the counts
// [1] = 0, [2] = number of misses, [3] |= bad id.  Null for a real tier.
int32_t *tier_ids_device_if_passthrough(bgl_host_tier *t);
// Before the lookup kernels of a batch are enqueued: clear the words they only ever set.
void tier_prepare(bgl_host_tier *t);
int32_t tier_row_bytes(const bgl_host_tier *t);
int64_t tier_num_nodes(const bgl_host_tier *t);

// Enqueue on st: look ids[miss_pos[r]], r < *n_ranks_dev <= n_upper, up in the
// tier's map, build the lists, send the missing ids and the counts to the host.
// gen (0/1, alternating between calls) selects the copy of the lists this batch owns.
int tier_enqueue_lookup(bgl_host_tier *t, const int32_t *ids, const int32_t *miss_pos,
                        const long long *n_ranks_dev, int64_t n_upper, int gen, hipStream_t st);
// Once st has passed that point: read the counts (n = size of the GPU cache's
// lookup), check the ids.  Nothing has changed yet if this fails.
int tier_begin(bgl_host_tier *t, int64_t n, TierPlan *plan);
// Host threads start copying: first the rows the tier holds, in list order, into the
// staging rows, then the rows of the tier misses, in list order, from the store to their
// ring positions.  tier_copy_progress tells how many leading rows of that sequence are in
// place (monotone, reaches n_hit + n_miss); tier_copy_wait ends the job.
int tier_copy_start(bgl_host_tier *t);
int64_t tier_copy_progress(bgl_host_tier *t);
// The calling thread packs a few rows itself (one task of the copy job); false when none is left.
bool tier_copy_help(bgl_host_tier *t);
void tier_copy_wait(bgl_host_tier *t);
// Copy-engine transport (bgl_host_tier_set_copy_engine): the packed rows of the batch whose lists
// have parity gen are copied into tier_landing(t, gen) (device memory, max_batch rows) on
// tier_copy_stream(t) before kernels scatter them; null when the transport is off.
char *tier_landing(bgl_host_tier *t, int gen);
// Mode 2 of the transport: the cache may write its whole output in one pass once the rows have landed.
bool tier_assemble(const bgl_host_tier *t);
hipStream_t tier_copy_stream(bgl_host_tier *t);
hipEvent_t tier_copy_event(bgl_host_tier *t);
// whether that event has ever been recorded (the caller records it behind every copy it enqueues)
bool tier_copy_event_recorded(const bgl_host_tier *t);
void tier_set_copy_event_recorded(bgl_host_tier *t);
// Enqueue the first-in first-out update of the map on st and close the batch.
int tier_enqueue_update(bgl_host_tier *t, const int32_t *ids, const int32_t *miss_pos, hipStream_t st);
// Give up on the batch (after a failed tier_begin or launch).
void tier_abort(bgl_host_tier *t);

}  // namespace bgl
