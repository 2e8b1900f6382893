// The overlapped minibatch loop as one native call (BGL paper, Sec. 3.3: the stages of
// minibatch preparation run as an asynchronous pipeline).  On one GPU the stage that sets
// the pace is the miss fetch over the host link, so the loop keeps the link busy:
//
//   chain stream     lookup(i) -> hit gather(i) -> miss rows(i) -> lookup(i+1) ... in one queue
//   work stream      FIFO map update(i), and in write-through mode with batches of many
//                    thousand ids the map lookup and lists of batch i+1 right behind it
//   sampling stream  sample(i+2) (the work stream itself unless a host tier packs the miss
//                    rows: then the next lookup must not queue behind the sampling)
//
// The cache runs in write-through mode (every lookup is followed by the insert of all its
// misses), so the FIFO update needs no fetched row; cache state still advances strictly batch
// by batch.  Sampling runs two batches ahead, hence three workspaces; the host waits only for
// each sampling call's sizes and, with a host tier, for each batch's lists.
//
// This file is a client of the library's own C ABI (include/bgl.h) and nothing else: it
// enqueues exactly what a caller of those functions would.
#include <algorithm>
#include <new>

#include "bgl_internal.h"

struct bgl_pipeline {
    const bgl_graph *g = nullptr;
    bgl_cache_t *c = nullptr;
    bgl_host_tier_t *tier = nullptr;
    int32_t batch = 0;
    int K = 0;
    int32_t fanouts[BGL_MAX_HOPS] = {};
    bgl_pipeline_buffers_t buf = {};
    int64_t cap = 0;       // upper bound on the input nodes of a batch
    bool early_ok = false;
    hipStream_t chain = nullptr, work = nullptr, samp_own = nullptr;
    hipEvent_t sampled[3] = {nullptr, nullptr, nullptr};
    hipEvent_t fence = nullptr;
    bgl_subgraph_t sg[3] = {};
    const int32_t *last_ids = nullptr;
    int64_t last_n = 0;
};

extern "C" int bgl_pipeline_create(const bgl_graph_t *g, bgl_cache_t *c, bgl_host_tier_t *tier, int32_t batch,
                                   const int32_t *fanouts, int32_t num_hops, const bgl_pipeline_buffers_t *buffers,
                                   int spare_rows, void *work_stream, bgl_pipeline_t **out)
try {
    if (!out) BGL_FAIL(BGL_EINVAL, "out is null");
    *out = nullptr;
    if (!g || !c) BGL_FAIL(BGL_EINVAL, "graph or cache handle is null");
    if (!fanouts || !buffers) BGL_FAIL(BGL_EINVAL, "fanouts or buffers is null");
    if (batch < 1) BGL_FAIL(BGL_EINVAL, "batch must be >= 1");
    if (num_hops < 1 || num_hops > BGL_MAX_HOPS) BGL_FAIL(BGL_EINVAL, "num_hops must be in [1, %d]", BGL_MAX_HOPS);
    size_t need = 0;
    int rc = bgl_sample_workspace_bytes(batch, fanouts, num_hops, g->num_nodes, &need);
    if (rc != BGL_OK) return rc;
    int64_t cap = batch;
    for (int h = 0; h < num_hops; ++h) cap = std::min<int64_t>(g->num_nodes, cap * (1 + (int64_t)fanouts[h]));
    cap = std::min<int64_t>(cap, g->num_nodes);
    for (int k = 0; k < 3; ++k)
        if (!buffers->workspace[k] || !buffers->counts_host[k])
            BGL_FAIL(BGL_EINVAL, "three sampling workspaces and three page-locked counts blocks are needed");
    if (buffers->workspace_bytes < need)
        BGL_FAIL(BGL_ECAPACITY, "a sampling workspace has %zu bytes, %zu needed", buffers->workspace_bytes, need);
    if (!buffers->out_rows || !buffers->out_slot || !buffers->miss_pos)
        BGL_FAIL(BGL_EINVAL, "out_rows, out_slot and miss_pos must not be null");
    if (buffers->cap_rows < cap)
        BGL_FAIL(BGL_ECAPACITY, "the output arrays hold %lld rows, a batch may have %lld input nodes",
                 (long long)buffers->cap_rows, (long long)cap);
    bgl_pipeline *p = new (std::nothrow) bgl_pipeline();
    if (!p) BGL_FAIL(BGL_ENOMEM, "out of host memory");
    auto fail = [&](int code) { bgl_pipeline_destroy(p); return code; };
    p->g = g;
    p->c = c;
    p->tier = tier;
    p->batch = batch;
    p->K = num_hops;
    std::copy(fanouts, fanouts + num_hops, p->fanouts);
    p->buf = *buffers;
    p->cap = cap;
    // an early lookup adds two hand-overs between streams: it pays for batches of many thousand ids
    p->early_ok = cap >= 65536;
    p->work = static_cast<hipStream_t>(work_stream);
    if (hipStreamCreateWithFlags(&p->chain, hipStreamNonBlocking) != hipSuccess) {
        p->chain = nullptr;
        bgl::set_error("could not create a stream");
        return fail(BGL_EHIP);
    }
    for (int k = 0; k < 3; ++k)
        if (hipEventCreateWithFlags(&p->sampled[k], hipEventDisableTiming) != hipSuccess) {
            p->sampled[k] = nullptr;
            bgl::set_error("could not create an event");
            return fail(BGL_EHIP);
        }
    if (hipEventCreateWithFlags(&p->fence, hipEventDisableTiming) != hipSuccess) {
        p->fence = nullptr;
        bgl::set_error("could not create an event");
        return fail(BGL_EHIP);
    }
    // One spare row position in the cache buffer per id of the largest batch: a batch's new rows then never
    // land on a row the same batch still has to read (the cache must be new: no insertion yet).
    if (spare_rows && (rc = bgl_cache_set_spare_rows(c, cap)) != BGL_OK) return fail(rc);
    if ((rc = bgl_cache_set_write_through(c, 1)) != BGL_OK) return fail(rc);
    *out = p;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_pipeline_destroy(bgl_pipeline_t *p)
try {
    if (!p) return BGL_OK;
    (void)hipDeviceSynchronize();
    if (p->chain) (void)hipStreamDestroy(p->chain);
    if (p->samp_own) (void)hipStreamDestroy(p->samp_own);
    for (int k = 0; k < 3; ++k)
        if (p->sampled[k]) (void)hipEventDestroy(p->sampled[k]);
    if (p->fence) (void)hipEventDestroy(p->fence);
    delete p;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_pipeline_set_cache(bgl_pipeline_t *p, bgl_cache_t *c, int spare_rows)
try {
    if (!p) BGL_FAIL(BGL_EINVAL, "pipeline handle is null");
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    int rc;
    if (spare_rows && (rc = bgl_cache_set_spare_rows(c, p->cap)) != BGL_OK) return rc;
    if ((rc = bgl_cache_set_write_through(c, 1)) != BGL_OK) return rc;
    p->c = c;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_pipeline_set_tier(bgl_pipeline_t *p, bgl_host_tier_t *tier)
try {
    if (!p) BGL_FAIL(BGL_EINVAL, "pipeline handle is null");
    p->tier = tier;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_pipeline_streams(bgl_pipeline_t *p, void **chain_stream, void **work_stream)
try {
    if (!p) BGL_FAIL(BGL_EINVAL, "pipeline handle is null");
    if (chain_stream) *chain_stream = p->chain;
    if (work_stream) *work_stream = p->work;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_pipeline_last_batch(bgl_pipeline_t *p, const int32_t **input_nodes, int64_t *n_input)
try {
    if (!p) BGL_FAIL(BGL_EINVAL, "pipeline handle is null");
    if (input_nodes) *input_nodes = p->last_ids;
    if (n_input) *n_input = p->last_n;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_pipeline_run(bgl_pipeline_t *p, const int32_t *seeds, int64_t seed_batches,
                                const uint64_t *rng_seeds, int64_t steps, int64_t first_step, int64_t *n_input,
                                int64_t *n_hit, int64_t *n_hit_tier, bgl_batch_fn on_batch, void *user)
try {
    if (!p) BGL_FAIL(BGL_EINVAL, "pipeline handle is null");
    if (!seeds || !rng_seeds || seed_batches < 1) BGL_FAIL(BGL_EINVAL, "seeds or rng_seeds is null, or there is no seed batch");
    if (steps < 0 || first_step < 0) BGL_FAIL(BGL_EINVAL, "steps and first_step must be >= 0");
    if (steps > 0 && (!n_input || !n_hit)) BGL_FAIL(BGL_EINVAL, "n_input and n_hit must not be null");
    bgl_cache_t *c = p->c;
    hipStream_t chain = p->chain, work = p->work, samp = work;
    const bool tiered = p->tier != nullptr;
    const bool early = p->early_ok;
    if (tiered && early) {
        // With early lookups and host threads that pack the miss rows, sampling gets a stream of its own
        // (created when first needed: a process has few hardware queues).
        if (!p->samp_own) BGL_HIP(hipStreamCreateWithFlags(&p->samp_own, hipStreamNonBlocking));
        samp = p->samp_own;
    }
    // whatever the caller enqueued on the work stream before (the seeds) comes first on the others
    BGL_HIP(hipEventRecord(p->fence, work));
    BGL_HIP(hipStreamWaitEvent(chain, p->fence, 0));
    if (samp != work) BGL_HIP(hipStreamWaitEvent(samp, p->fence, 0));

    auto sample = [&](int64_t i) -> int {
        const int k = (int)(i % 3);
        const int64_t at = first_step + i, b = at % seed_batches;
        const uint64_t seed = rng_seeds[b] ^ (uint64_t)(at / seed_batches);  // a later pass over the seeds samples differently
        const int rc = bgl_sample_khop(p->g, seeds + b * p->batch, p->batch, p->fanouts, p->K, seed, p->buf.workspace[k],
                                       p->buf.workspace_bytes, &p->sg[k], p->buf.counts_host[k], samp);
        if (rc != BGL_OK) return rc;
        BGL_HIP(hipEventRecord(p->sampled[k], samp));
        return BGL_OK;
    };
    int rc;
    if (steps > 0 && (rc = sample(0)) != BGL_OK) return rc;
    if (steps > 1 && (rc = sample(1)) != BGL_OK) return rc;
    for (int64_t i = 0; i < steps; ++i) {
        const int k = (int)(i % 3);
        BGL_HIP(hipEventSynchronize(p->sampled[k]));  // the sizes of batch i
        const volatile int32_t *counts = p->buf.counts_host[k];
        if (counts[BGL_COUNTS_LEN - 1] != 0) BGL_FAIL(counts[BGL_COUNTS_LEN - 1], "sampling reported an error on the device");
        const int64_t n = counts[p->K];
        const int32_t *ids = p->sg[k].input_nodes;
        BGL_HIP(hipStreamWaitEvent(chain, p->sampled[k], 0));
        if (samp != work) BGL_HIP(hipStreamWaitEvent(work, p->sampled[k], 0));
        if (!tiered) {
            // the map lookup and the lists run early, on the work stream, behind the previous batch's map update
            rc = early ? bgl_cache_lookup_gather_early(c, ids, n, p->buf.out_rows, p->buf.out_slot, p->buf.miss_pos,
                                                       n_hit + i, chain, chain, work)
                       : bgl_cache_lookup_gather(c, ids, n, p->buf.out_rows, p->buf.out_slot, p->buf.miss_pos, n_hit + i,
                                                 chain, chain);
            if (rc != BGL_OK) return rc;
        } else {
            // First half of the tiered call: blocks until the lists are on the host, then the host threads pack
            // the rows while this thread enqueues the map update (the next lookup waits for it) and the sampling
            // of batch i+2; the second half sends the packed rows on their way.
            int64_t hits[2] = {0, 0};
            rc = bgl_cache_lookup_tiered_begin(c, p->tier, ids, n, p->buf.out_rows, p->buf.out_slot, p->buf.miss_pos, hits,
                                               chain, chain, early ? work : nullptr, early ? 1 : 0);
            if (rc != BGL_OK) return rc;
            n_hit[i] = hits[0];
            if (n_hit_tier) n_hit_tier[i] = hits[1];
            if ((rc = bgl_cache_insert_fifo(c, ids, p->buf.miss_pos, -1, p->buf.out_rows, work)) != BGL_OK) return rc;
        }
        if (i + 2 < steps) {
            // workspace (i+2) % 3 was batch i-1's; its rows were complete before hit gather(i)
            if ((rc = bgl_cache_wait_lists(c, samp)) != BGL_OK) return rc;
            if ((rc = sample(i + 2)) != BGL_OK) return rc;
        }
        if (tiered) {
            if ((rc = bgl_cache_lookup_tiered_finish(c)) != BGL_OK) return rc;
        } else {
            if ((rc = bgl_cache_insert_fifo(c, ids, p->buf.miss_pos, -1, p->buf.out_rows, work)) != BGL_OK) return rc;
        }
        n_input[i] = n;
        p->last_ids = ids;
        p->last_n = n;
        if (on_batch) on_batch(user, i, k, &p->sg[k], n);
    }
    BGL_HIP(hipDeviceSynchronize());
    return BGL_OK;
} BGL_NOTHROW_END
