/*
 * bgl.h - C ABI of the MI355X minibatch-preparation library.
 *
 * The library implements, as HIP kernels for gfx950, the data path that the
 * BGL paper (arXiv 2112.08541) is about: for every training iteration, sample a
 * k-hop subgraph around a batch of training nodes (Sec. 2.1 stage 1, Sec. 5.1
 * "Mini-batch Sampling Algorithms") and retrieve the features of its nodes
 * through a GPU-resident FIFO feature cache (Sec. 3.2 and the "Feature Cache
 * Engine" paragraphs of Sec. 4).
 *
 * Conventions
 *  - Every call returns a status: BGL_OK or a negative BGL_E* code.  Nothing
 *    throws or aborts; bgl_last_error() returns a thread-local message for the
 *    last failing call on this thread.
 *  - "host" pointers are dereferenced by the CPU inside the call; "device"
 *    pointers are only handed to kernels.  The library never takes ownership of
 *    caller memory.  Handles are opaque, created by *_load_* / *_create and
 *    released by *_destroy.
 *  - Streams are hipStream_t values passed as void* (NULL = the default
 *    stream).  Calls that take a stream only enqueue work; results are valid
 *    once the stream has been synchronised.  Calls on one handle must be
 *    serialised by the caller (the paper serialises all operations on one GPU
 *    cache through one queue, Sec. 3.2.3).
 *  - All ids are int32 node ids in [0, num_nodes).
 */
#ifndef BGL_H
#define BGL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BGL_OK 0
#define BGL_EINVAL (-1)       /* bad argument */
#define BGL_ENOMEM (-2)       /* host or device allocation failed */
#define BGL_EHIP (-3)         /* a HIP runtime call failed */
#define BGL_ECAPACITY (-4)    /* a caller-provided buffer is too small */
#define BGL_EUNSUPPORTED (-5) /* valid request outside the implemented range */

#define BGL_MAX_HOPS 8
#define BGL_MAX_FANOUT 64

/* Where bgl_graph_load_csr keeps the CSR arrays. */
#define BGL_DEVICE 0      /* copy both arrays into HBM */
#define BGL_HOST_PINNED 1 /* caller's arrays are page-locked; kernels read them in place */
#define BGL_HOST_PINNED_COL 2 /* col_idx as BGL_HOST_PINNED; row_ptr is copied into HBM */

typedef struct bgl_graph bgl_graph_t;
typedef struct bgl_cache bgl_cache_t;
typedef struct bgl_host_tier bgl_host_tier_t;

const char *bgl_last_error(void);

/* ------------------------------------------------------------------ graph */

/*
 * Register a graph in CSR form (the graph structure the samplers of Sec. 3.1
 * work on).  Row v holds the neighbors that sampling may pick for v.
 *   row_ptr      host, num_nodes+1 offsets, int32 (row_ptr_bits = 32) or int64 (64)
 *   col_idx      host, num_edges int32 node ids
 *   placement    BGL_DEVICE: arrays are copied to HBM, the caller may free its
 *                copies on return.  BGL_HOST_PINNED: arrays must be page-locked
 *                (hipHostMalloc or equivalent) and stay alive and unchanged
 *                until bgl_graph_destroy.  BGL_HOST_PINNED_COL: the same for
 *                col_idx only; row_ptr (4 or 8 bytes per node) is copied to
 *                HBM, which takes the offset reads of sampling off the host
 *                link, and the caller may free its row_ptr on return.
 * Validated on the host: row_ptr[0] == 0, non-decreasing, row_ptr[N] ==
 * num_edges, every degree < 2^31, every column id in [0, num_nodes).
 * Errors: BGL_EINVAL (null pointers, bad sizes, failed validation, memory not
 * page-locked), BGL_ENOMEM, BGL_EHIP.
 */
int bgl_graph_load_csr(const void *row_ptr, int row_ptr_bits, const int32_t *col_idx,
                       int64_t num_nodes, int64_t num_edges, int placement,
                       bgl_graph_t **out);
int bgl_graph_destroy(bgl_graph_t *g);

/* --------------------------------------------------------------- sampling */

/*
 * Result of bgl_sample_khop.  All pointers are device pointers into the
 * workspace given to that call and stay valid until the workspace is reused.
 * Hop h connects destination nodes input_nodes[0 .. n_frontier[h]) to source
 * nodes input_nodes[0 .. n_frontier[h+1]) in CSR form with local ids:
 * row_ptr[h] has n_frontier[h]+1 entries, col_local[h] has nnz[h] entries.
 * Sizes live in `counts` (device) in this layout:
 *   counts[0 .. num_hops]                          n_frontier[h]
 *   counts[BGL_MAX_HOPS+1 .. BGL_MAX_HOPS+num_hops] nnz[h]
 *   counts[BGL_COUNTS_LEN-1]                       status (0 = ok, else a BGL_E* code)
 * n_input = n_frontier[num_hops].
 */
#define BGL_COUNTS_LEN (2 * BGL_MAX_HOPS + 2)
typedef struct {
    int32_t num_hops;
    int32_t *input_nodes;              /* frontier_K: global ids, unique, seeds first */
    int32_t *row_ptr[BGL_MAX_HOPS];
    int32_t *col_local[BGL_MAX_HOPS];
    int64_t cap_nodes[BGL_MAX_HOPS + 1]; /* upper bounds on n_frontier[h] */
    int64_t cap_edges[BGL_MAX_HOPS];     /* upper bounds on nnz[h] */
    const int32_t *counts;               /* device, BGL_COUNTS_LEN ints */
} bgl_subgraph_t;

/* Bytes of device workspace bgl_sample_khop needs for these arguments. */
int bgl_sample_workspace_bytes(int32_t num_seeds, const int32_t *fanouts, int32_t num_hops,
                               int64_t num_nodes, size_t *bytes);

/*
 * k-hop fanout neighbor sampling with per-hop deduplication (Sec. 3.1:
 * iterative next-hop sampling from the training nodes; Sec. 5.1: one fanout per
 * hop, e.g. {15,10,5}).
 *
 * frontier_0 = seeds with repeats removed (first occurrence kept).  For hop h
 * every node v of frontier_h draws c = min(fanouts[h], degree(v)) distinct
 * edge positions of its CSR row, uniformly (all of them, in row order, when
 * degree <= fanout; otherwise Floyd's subset algorithm on a counter-based
 * generator keyed on (rng_seed, h, v, slot)).  frontier_{h+1} is frontier_h
 * followed by the not-yet-seen sampled neighbors in (frontier index, slot)
 * order, so local ids are stable across hops.
 *
 *   seeds            device, num_seeds ids (any order, repeats allowed)
 *   fanouts          host, num_hops values in [1, BGL_MAX_FANOUT]; fanouts[0] applies at the seeds
 *   rng_seed         per-call seed; the same seed reproduces the same sample
 *   workspace        device, 256-byte aligned, >= bgl_sample_workspace_bytes(...)
 *   out              host struct filled before return (pointers into workspace)
 *   counts_host      optional page-locked host array of BGL_COUNTS_LEN ints that
 *                    receives a copy of out->counts on `stream`
 * Asynchronous on `stream`.  A seed id outside [0, num_nodes) is dropped and
 * sets status BGL_EINVAL in counts.
 * Errors: BGL_EINVAL (null/misaligned pointers, num_seeds < 1, num_hops outside
 * [1, BGL_MAX_HOPS], fanout < 1), BGL_EUNSUPPORTED (fanout > BGL_MAX_FANOUT),
 * BGL_ECAPACITY (workspace too small), BGL_EHIP.
 */
int bgl_sample_khop(const bgl_graph_t *g, const int32_t *seeds, int32_t num_seeds,
                    const int32_t *fanouts, int32_t num_hops, uint64_t rng_seed,
                    void *workspace, size_t workspace_bytes, bgl_subgraph_t *out,
                    int32_t *counts_host, void *stream);

/* ------------------------------------------------------------------ cache */

/*
 * Create a FIFO feature cache in HBM (Sec. 3.2.3: one cache map and one cache
 * buffer per GPU).  The cache buffer holds capacity_rows rows of row_bytes
 * bytes; the map from node id to buffer slot is an open-addressing hash table.
 * Rows are opaque bytes (fp32, bf16, ...).
 *   host_features  the backing store for misses: num_nodes rows of row_bytes
 *                  bytes, 16-byte aligned, in page-locked host memory (read in
 *                  place by kernels over the host link) or in device memory.
 *                  Must stay alive and unchanged until bgl_cache_destroy
 *                  (features do not change during training, Sec. 4).
 *                  May be null for a cache whose misses are only ever served
 *                  through a host tier (bgl_cache_lookup_gather_tiered).
 * Errors: BGL_EINVAL (capacity_rows < 1, row_bytes < 16 or not a multiple of
 * 16, misaligned/pageable features, num_nodes < 1), BGL_ENOMEM, BGL_EHIP.
 */
int bgl_cache_create(int64_t capacity_rows, int32_t row_bytes, const void *host_features,
                     int64_t num_nodes, bgl_cache_t **out);
int bgl_cache_destroy(bgl_cache_t *c);

/*
 * Cache workflow steps 4-6 of Sec. 3.2.3: look the ids up in the cache map,
 * gather the rows of the hits from the cache buffer, fetch the rows of the
 * misses from the backing store.  The lookup sees the cache as it was when the
 * call's work starts on main_stream; nothing in the cache changes (FIFO: a hit
 * does not renew a row).
 *   ids             device, n ids, no repeats (the input_nodes of bgl_sample_khop)
 *   out_rows        device, n * row_bytes bytes, 16-byte aligned; row i = features of ids[i]
 *   out_slot        device, n ints: buffer slot of ids[i], or -1 for a miss
 *   miss_pos        device, room for n ints: the positions i of the misses, ascending
 *   n_hit_host      optional page-locked host int64 that receives the number of hits
 *   main_stream     probe, miss list and hit gather run here; in main_stream
 *                   order out_slot, miss_pos, the hit count and the rows of the
 *                   hits are complete when the call's work is done
 *   side_stream     the miss fetch runs here (NULL: a stream owned by the
 *                   cache), after the hit gather, so that work enqueued on
 *                   main_stream afterwards (the next batch's sampling) overlaps
 *                   the host-link transfer.  The rows of the misses are complete
 *                   for a stream once it has passed bgl_cache_wait_rows or the
 *                   following bgl_cache_insert_fifo.  If side_stream equals
 *                   main_stream everything is in main_stream order.
 * ids, out_rows and miss_pos must stay untouched until the miss fetch is done.
 * An id outside [0, num_nodes) is reported as a miss whose row is left
 * untouched, and sets the cache's status (bgl_cache_stats) to BGL_EINVAL.
 * Errors: BGL_EINVAL (null/misaligned pointers, n < 0 or n >= 2^31), BGL_ENOMEM, BGL_EHIP.
 */
int bgl_cache_lookup_gather(bgl_cache_t *c, const int32_t *ids, int64_t n, void *out_rows,
                            int32_t *out_slot, int32_t *miss_pos, int64_t *n_hit_host,
                            void *main_stream, void *side_stream);

/*
 * bgl_cache_lookup_gather for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same results,
 * same arguments and stream contract, except:
 *  - the call's own lists (per-tile miss counts, the hit list) do not live in
 *    memory the cache allocates and grows on demand but in a fixed array of
 *    device memory inside the library, about 10.5 MB per GPU, held by every GPU
 *    the library runs on until the process ends; hence n <= BGL_NOALLOC_MAX_IDS;
 *  - side_stream NULL means main_stream (no stream is created);
 *  - its kernels are never timed (bgl_cache_set_profiling does not apply to it);
 *  - the current device must be the one the cache was created on.
 * The call makes no hipMalloc / hipFree, creates no stream and no event.  All
 * such calls on one GPU share the one array, whatever cache they are for: the
 * array keeps the last call's contents (every part of it that a call reads is
 * written by that call first, nothing needs clearing), and two such calls whose
 * work overlaps on one GPU (different streams, different caches) race.  A call's
 * lists are read until its hit gather has finished on main_stream.
 * Errors: as bgl_cache_lookup_gather, plus BGL_ECAPACITY (n > BGL_NOALLOC_MAX_IDS),
 * BGL_EINVAL (wrong current device), BGL_EUNSUPPORTED (device ordinal >= 64).
 */
#define BGL_NOALLOC_MAX_IDS 1310720 /* 1.25 x 2^20: above the largest batch bound of the paper's settings */
int bgl_cache_lookup_gather_noalloc(bgl_cache_t *c, const int32_t *ids, int64_t n, void *out_rows,
                                    int32_t *out_slot, int32_t *miss_pos, int64_t *n_hit_host,
                                    void *main_stream, void *side_stream);

/*
 * bgl_cache_lookup_gather with the map lookup and the lists on lookup_stream
 * instead of main_stream (write-through mode only).  When main_stream is the
 * stream that also carries the miss fetches, a plain lookup starts only when the
 * previous call's fetch has left the link; this one does not wait for it: only
 * the hit gather and the fetch stay in main_stream / side_stream order (the
 * gather may need rows the previous fetch is still writing).  The fetch reads
 * the library's own copy of the miss list, so the previous call's fetch is not
 * disturbed by this call's lists.  Conditions: ids ready in lookup_stream order
 * and untouched until this call's fetch is done; the previous call's
 * bgl_cache_insert_fifo already enqueued (this call waits for it on the
 * device); out_slot and miss_pos are rewritten as soon as lookup_stream gets
 * there, so readers of the previous call's lists must be done in lookup_stream
 * order.  With lookup_stream == main_stream it is bgl_cache_lookup_gather.
 * Errors: as bgl_cache_lookup_gather, plus BGL_EINVAL (write-through mode is off).
 */
int bgl_cache_lookup_gather_early(bgl_cache_t *c, const int32_t *ids, int64_t n, void *out_rows,
                                  int32_t *out_slot, int32_t *miss_pos, int64_t *n_hit_host,
                                  void *main_stream, void *side_stream, void *lookup_stream);

/*
 * Cache update of Sec. 3.2.3 (last step) with the FIFO rule of Sec. 4: the
 * buffer is a circular queue with a running `tail`; miss number r of this call
 * (in miss_pos order) takes slot (tail + r) mod capacity, the node that held
 * that slot is removed from the map, the new node is entered and its row
 * copied from out_rows; then tail += n_miss.  The first insertion ever goes to
 * slot 0.  With n_miss > capacity the result equals inserting one by one (only
 * the last `capacity` misses stay).
 *   ids, miss_pos, out_rows   device; as produced by bgl_cache_lookup_gather
 *   n_miss          number of entries of miss_pos to insert, or -1 to use the
 *                   miss count the last bgl_cache_lookup_gather left on the
 *                   device (no host round trip)
 * Called after the lookup_gather that produced its inputs.  On that call's
 * main_stream it is in stream order; on any other stream it first waits (on
 * the device) for that call's lists and hit gather, and the next lookup waits
 * for it.  The map update is enqueued first and does not wait for the miss
 * fetch; the row copy waits for it on the device.
 * Errors: BGL_EINVAL, BGL_EHIP.
 */
int bgl_cache_insert_fifo(bgl_cache_t *c, const int32_t *ids, const int32_t *miss_pos,
                          int64_t n_miss, const void *out_rows, void *stream);

/*
 * Spare row positions in the cache buffer (0 by default).  The FIFO rule of
 * Sec. 4 overwrites the row of the evicted node with the new one, so a row that
 * a lookup has found and that the same call's insertions evict must be read
 * before it is overwritten.  With spare_rows extra positions in the buffer the
 * new rows of a call go to positions that hold no live row as long as the call
 * has at most spare_rows misses (insertion number k sits at position
 * k mod (capacity_rows + spare_rows); its slot stays k mod capacity_rows, and
 * out_slot, bgl_cache_export_state and the eviction order are unchanged).  The
 * one-pass output of bgl_host_tier_set_copy_engine mode 2 then needs no first
 * pass.  Give it the largest number of ids a lookup will be called with.  Costs
 * spare_rows * row_bytes of device memory.
 * Only before the first insertion into the cache (the buffer is allocated
 * anew); synchronises the device.
 * Errors: BGL_EINVAL (null handle, spare_rows < 0 or capacity_rows + spare_rows
 * >= 2^31, insertions have happened), BGL_ENOMEM, BGL_EHIP.
 */
int bgl_cache_set_spare_rows(bgl_cache_t *c, int64_t spare_rows);

/*
 * Write-through mode (off by default).  When on, the caller promises that every
 * bgl_cache_lookup_gather is followed, before any other call on the cache, by
 * bgl_cache_insert_fifo with the same ids and miss_pos and n_miss = -1 (the
 * paper's workflow: every miss is inserted, Sec. 3.2.3).  The miss fetch then
 * stores each row it reads both into out_rows and into the buffer slot the FIFO
 * rule will give it, so the update has no row copy and does not wait for the
 * fetch: the time between two fetches on the host link shrinks to lookup, lists
 * and hit gather.  Results are identical to the default mode.  A call sequence
 * that breaks the promise is rejected with BGL_EINVAL; a stream that reads
 * out_rows must still pass bgl_cache_wait_rows.
 */
int bgl_cache_set_write_through(bgl_cache_t *c, int enable);

/*
 * Make `stream` wait (on the device, not the host) until the miss rows of the
 * most recent bgl_cache_lookup_gather are in out_rows.  A no-op when that call
 * ran on a single stream.  Consumers of out_rows other than
 * bgl_cache_insert_fifo (the model's first layer) call this first.
 */
int bgl_cache_wait_rows(bgl_cache_t *c, void *stream);

/*
 * Make `stream` wait (on the device) until the lists (out_slot, miss_pos, hit
 * count) and the hit rows of the most recent bgl_cache_lookup_gather are
 * complete (the lists only after a tiered lookup whose output is written in one
 * pass, bgl_host_tier_set_copy_engine mode 2: its hit rows come with its miss
 * rows, bgl_cache_wait_rows).  A no-op for that call's main_stream.  bgl_cache_insert_fifo does
 * this itself when it is given another stream than the lookup's main_stream, and
 * the next lookup then waits for that update; so the lookups of one cache may run
 * on one stream (with side_stream = main_stream the whole chain lookup, lists,
 * hit gather, miss fetch stays in one queue) and the FIFO updates on another.
 */
int bgl_cache_wait_lists(bgl_cache_t *c, void *stream);

/*
 * Copy the logical cache state to the host (synchronises the device):
 * slot_to_node[capacity] (-1 = empty slot), tail (insertions so far) and,
 * if buffer is non-NULL, capacity * row_bytes bytes of cached rows.
 */
int bgl_cache_export_state(bgl_cache_t *c, int32_t *slot_to_node, uint64_t *tail, void *buffer);

/*
 * Counters since creation (synchronises the device): ids looked up, hits, rows
 * inserted, rows evicted, and the sticky status word (BGL_OK, or BGL_EINVAL if
 * an out-of-range id was ever seen, BGL_ECAPACITY if the map overflowed).
 * Any output pointer may be NULL.
 */
int bgl_cache_stats(bgl_cache_t *c, uint64_t *lookups, uint64_t *hits, uint64_t *inserts,
                    uint64_t *evictions, int32_t *status);

/*
 * Cost of the cache map's lookups (synchronises the device).  The paper's cache
 * engine serves a whole training job (Sec. 3.2.1, Sec. 4: every insertion evicts
 * the occupant of the next position from the map), so what a lookup costs must
 * not depend on how many insertions and evictions the map has seen.  The map is
 * a hash table of 128-byte buckets; a lookup reads its id's home bucket and goes
 * on to the next one only while the bucket says that some live entry was pushed
 * past it by an insertion that found it full.
 *   ids_looked_up      ids of all lookups since creation
 *   bucket_lines_read  bucket lines (128 bytes each) those lookups read; the
 *                      ratio of the two is the mean length of a lookup
 *   num_buckets        buckets of the map (15 entries each)
 *   buckets_passed     buckets that some live entry is pushed past right now
 *   passes             (live entry, bucket it is pushed past) pairs right now
 * Any output pointer may be NULL.  Errors: BGL_EINVAL (null handle), BGL_EHIP.
 */
int bgl_cache_map_stats(bgl_cache_t *c, uint64_t *ids_looked_up, uint64_t *bucket_lines_read,
                        uint64_t *num_buckets, uint64_t *buckets_passed, uint64_t *passes);

/*
 * Per-kernel timing for measurements.  `stage_mask` has bit (1 << stage) set for
 * every stage the cache shall time (0 = off, BGL_ALL_STAGES = all).  A stage that
 * is one kernel per launch (all but BGL_STAGE_MISS_LIST and BGL_STAGE_LINK_COPY) is timed by the kernel
 * dispatch itself, which records the kernel's begin and end on the device into a
 * pair of events: the figure is the kernel's own duration, the one a kernel
 * trace shows.  BGL_STAGE_MISS_LIST (several small kernels) is bracketed by two
 * event records on its stream, which also times the launch gaps around them.
 * bgl_cache_profile synchronises the device and returns the summed milliseconds
 * and the number of launches of one stage since profiling was (re-)enabled.
 */
#define BGL_STAGE_PROBE 0       /* map lookup */
#define BGL_STAGE_MISS_LIST 1   /* ordered list of miss positions + counters */
#define BGL_STAGE_GATHER_HIT 2  /* cache buffer -> out_rows */
#define BGL_STAGE_FETCH_MISS 3  /* backing store -> out_rows */
#define BGL_STAGE_INSERT_MAP 4  /* evict + enter ids in the map */
#define BGL_STAGE_INSERT_ROWS 5 /* out_rows -> cache buffer */
#define BGL_STAGE_LINK_COPY 6   /* tiered lookup with the copy-engine transport: the copies over the host
                                   link, each bracketed by two event records on the copy stream */
#define BGL_STAGE_ASSEMBLE_PRE 7 /* assembled output: the hits whose slots the call's own misses take */
#define BGL_STAGE_ASSEMBLE 8    /* assembled output: every other row -> out_rows, miss rows -> cache buffer */
#define BGL_NUM_STAGES 9
/* pseudo stage: what two event records read around a kernel that does nothing
 * (measured when profiling is enabled; the share of BGL_STAGE_MISS_LIST that is
 * not kernel time); total_ms is that single figure */
#define BGL_STAGE_EVENT_OVERHEAD 100
#define BGL_ALL_STAGES ((1 << BGL_NUM_STAGES) - 1)
int bgl_cache_set_profiling(bgl_cache_t *c, int stage_mask);
int bgl_cache_profile(bgl_cache_t *c, int stage, double *total_ms, int64_t *launches);
/*
 * Time `stage` only in every `every`-th call (lookups and FIFO updates are counted
 * separately, from the cache's creation, starting at 1): a timed launch holds its
 * stream up for a few microseconds, which a stage of many launches per call would
 * feel.  Default 1.  Errors: BGL_EINVAL.
 */
int bgl_cache_set_profiling_every(bgl_cache_t *c, int stage, int every);

/* ------------------------------------------------------------- host tier */

/*
 * Second cache level in host memory (Sec. 3.2.3: a CPU cache with the same
 * policy as the GPU cache sits between it and the feature store).  The tier is
 * a FIFO cache of capacity_rows rows in page-locked memory.  Its map (node ->
 * row, 4 bytes per node) and slot tables live in device memory of the current
 * device and are looked up and updated by kernels; host threads only move
 * rows: the rows the tier holds into page-locked staging rows, the others from
 * `store` into the tier, both packed in miss order, and the GPU reads them from
 * there as a stream.
 *   store           the feature store: num_nodes rows of row_bytes bytes in
 *                   host memory of any kind (pageable, a mapped file,
 *                   page-locked); stays alive and unchanged until
 *                   bgl_host_tier_destroy
 *   capacity_rows   0 is allowed: nothing is kept, every miss row just passes
 *                   through the page-locked ring.  That alone pays when
 *                   row_bytes is not a multiple of 128: rows read in place move
 *                   whole 128-byte lines over the link, packed rows do not
 *   max_batch_rows  the largest n a tiered lookup will be called with; the
 *                   page-locked ring holds capacity_rows + 2 * max_batch_rows
 *                   rows, the staging rows (capacity_rows > 0) another
 *                   2 * max_batch_rows
 *   num_threads     host threads that copy rows (the calling thread drives the
 *                   GPU meanwhile, and packs too when it has nothing to send);
 *                   0 = three quarters of min(cores, 16): more threads than that
 *                   take host memory bandwidth from the transfers they feed
 * Errors: BGL_EINVAL (null store, sizes out of range, row_bytes not a multiple
 * of 16), BGL_ENOMEM (page-locked, host or device allocation failed), BGL_EHIP.
 */
int bgl_host_tier_create(const void *store, int64_t num_nodes, int32_t row_bytes,
                         int64_t capacity_rows, int64_t max_batch_rows, int32_t num_threads,
                         bgl_host_tier_t **out);
/* Waits for the device to go idle first: kernels may still be reading the rows. */
int bgl_host_tier_destroy(bgl_host_tier_t *t);

/*
 * Transport of the packed rows (0, off, by default).  0: kernels on side_stream
 * read the page-locked rows over the host link and write them to their places,
 * so the link is idle while those kernels wait for the lookup's hit gather.
 * 1: plain copies on a stream of the tier's own move the packed rows into
 * device memory (2 * max_batch_rows rows of it, allocated by this call) as soon
 * as they are packed, independent of the cache's kernels; kernels on
 * side_stream then scatter them from there.  With early lookups the link then
 * carries one batch after the other without a pause.
 * 2: as 1, and where the tier keeps nothing (capacity_rows = 0) and the cache is
 * in write-through mode, the lookup has no hit gather of its own: once the rows
 * have landed one pass writes the whole of out_rows in its own order (a hit's
 * row from the cache buffer, a miss's row from the landed rows, which also go
 * into the cache buffer), after a short pass that saves the hits whose slots
 * this call's misses take.  Every output line is then written whole and the
 * launch is large enough to fill the memory system.  The rows of the hits are
 * then complete when the rows of the misses are (bgl_cache_wait_rows), not
 * earlier.  Elsewhere mode 2 behaves as mode 1.
 * Results are identical in all modes.  Waits for the device to go idle.
 * BGL_STAGE_FETCH_MISS then times the scatter kernels, BGL_STAGE_LINK_COPY the
 * copies, BGL_STAGE_ASSEMBLE_PRE and BGL_STAGE_ASSEMBLE the two passes of mode 2.
 * Errors: BGL_EINVAL (null handle, a batch is being served, mode not 0..2),
 * BGL_ENOMEM, BGL_EHIP.
 */
int bgl_host_tier_set_copy_engine(bgl_host_tier_t *t, int mode);

/*
 * bgl_cache_lookup_gather with the host tier behind the GPU cache (workflow of
 * Sec. 3.2.3: GPU cache map, then the CPU cache for the GPU's misses, then the
 * feature store; both levels updated first-in first-out).  Arguments as for
 * bgl_cache_lookup_gather, except:
 *   n_hit   ordinary host array of 2, set before return: hits in the GPU cache,
 *           hits in the host tier (of the GPU cache's n - n_hit[0] misses)
 * The tier handles the GPU cache's misses, in miss_pos order, as one FIFO batch:
 * looked up against the tier's state at entry, then its own misses inserted in
 * that order (the rule of bgl_cache_insert_fifo, tail advancing by their
 * number).  The call blocks the host until the lists are known and the rows
 * are packed; what moves them starts while the host threads are still copying
 * (kernels on side_stream chunk by chunk, or with the copy-engine transport
 * copies on the tier's own stream followed by kernels on side_stream).  On
 * return the fetch of all miss rows is enqueued on side_stream
 * (bgl_cache_wait_rows as usual) and the tier's update on main_stream (on
 * lookup_stream with early_lookup); the GPU
 * cache still needs its bgl_cache_insert_fifo.  ids, out_slot and miss_pos must
 * stay untouched until main_stream has passed this call.  ids must be distinct.
 * One tier serves one cache's calls in order; it is not thread-safe.
 *   early_lookup    0: lookup_stream is ignored.  1 (needs write-through mode):
 *           the map lookups of both levels and the lists run on
 *           lookup_stream instead of main_stream, i.e. without waiting for the
 *           previous call's miss fetch when that is what main_stream is busy
 *           with, so the host has the missing ids and packs rows while that
 *           fetch is still on the link; the hit gather and everything after it
 *           stay on main_stream and side_stream.  ids must be ready in
 *           lookup_stream order; the previous call's bgl_cache_insert_fifo must
 *           have been enqueued (on lookup_stream, or it is waited for); out_slot
 *           and miss_pos are overwritten as soon as lookup_stream gets there, so
 *           whoever reads the previous call's out_slot / miss_pos must be done
 *           in lookup_stream order too.
 * Errors: as bgl_cache_lookup_gather, plus BGL_EINVAL (cache and tier differ in
 * row_bytes or num_nodes; an id outside [0, num_nodes): no level is changed),
 * BGL_ECAPACITY (n > max_batch_rows).
 */
int bgl_cache_lookup_gather_tiered(bgl_cache_t *c, bgl_host_tier_t *t, const int32_t *ids, int64_t n,
                                   void *out_rows, int32_t *out_slot, int32_t *miss_pos,
                                   int64_t *n_hit, void *main_stream, void *side_stream,
                                   void *lookup_stream, int early_lookup);

/*
 * bgl_cache_lookup_gather_tiered in two halves, for a caller that has other work
 * to enqueue while the host threads pack the batch's rows (Sec. 3.3: the stages
 * of minibatch preparation overlap; here the calling thread's own launches, e.g.
 * the sampling of a later batch, overlap the packing).
 *   bgl_cache_lookup_tiered_begin: same arguments and errors as
 *     bgl_cache_lookup_gather_tiered.  Enqueues the lookups, blocks until their
 *     lists have reached the host, starts the host threads and returns; n_hit
 *     (host, two words, may be null) holds the two hit counts on return.
 *   bgl_cache_lookup_tiered_finish: sends the packed rows on their way as they
 *     get ready and enqueues the kernels that take them to their places; blocks
 *     until the last row is packed.  BGL_EINVAL without a begun call.
 * Between the two the caller may enqueue this batch's bgl_cache_insert_fifo (in
 * write-through mode only: the update then touches the map alone) and work that
 * does not involve this cache or tier; any other lookup, and a change of the
 * cache's modes, fails with BGL_EINVAL.  The arrays handed to begin stay the
 * caller's to keep alive and unchanged until the work finish enqueues is done.
 * begin followed at once by finish is bgl_cache_lookup_gather_tiered.
 */
int bgl_cache_lookup_tiered_begin(bgl_cache_t *c, bgl_host_tier_t *t, const int32_t *ids, int64_t n,
                                  void *out_rows, int32_t *out_slot, int32_t *miss_pos,
                                  int64_t *n_hit, void *main_stream, void *side_stream,
                                  void *lookup_stream, int early_lookup);
int bgl_cache_lookup_tiered_finish(bgl_cache_t *c);

/*
 * Tier state for tests: slot_to_node (capacity_rows ints, -1 = empty), the
 * running tail, the tier's rows by slot (capacity_rows * row_bytes bytes, zeros
 * for empty slots).  Any pointer may be null.  Host memory; waits for the device.
 */
int bgl_host_tier_export_state(bgl_host_tier_t *t, int32_t *slot_to_node, uint64_t *tail,
                               void *buffer_rows);
/*
 * Lifetime counters: ids looked up, ids found, host wall time spent packing rows
 * (milliseconds, per batch from the start of its copies to the moment the
 * calling thread sees the last row in place) over `batches` served batches; and
 * the thread count in use.  Pointers may be null.
 */
int bgl_host_tier_stats(bgl_host_tier_t *t, uint64_t *lookups, uint64_t *hits, double *copy_ms,
                        uint64_t *batches, int32_t *threads);

/* --------------------------------------------------------------- ordering */

/*
 * One BFS sequence of the training nodes (Sec. 3.2.2: training-node sequences
 * generated in BFS order).  The traversal runs on the GPU over the registered
 * graph.  Canonical order: the first-in first-out queue traversal from `root`,
 * the not yet visited out-neighbors of a node entering the queue in the order of
 * its CSR row; when the queue runs empty the traversal restarts at the smallest
 * node id not visited yet, so small components end up at the end of the
 * sequence.  Only the training nodes are recorded.
 *   train_nodes   host, num_train distinct node ids
 *   seq           host, receives num_train ids
 * Synchronous (returns when seq is filled).
 * Errors: BGL_EINVAL (null pointers, root or a training id outside
 * [0, num_nodes), repeated training id, num_train outside [1, num_nodes]),
 * BGL_ENOMEM, BGL_EHIP.
 */
int bgl_order_bfs_sequence(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                           int64_t root, int32_t *seq, void *stream);

/*
 * Proximity-aware order of the training nodes (Sec. 3.2.2): num_sequences BFS
 * sequences from the given roots; sequence j is read cyclically starting at
 * offset shifts[j] (the paper's random shift); the output takes nodes from the
 * sequences in turn (turn t: the next node of sequence t mod num_sequences that
 * no earlier turn has taken), so consecutive batches draw from every sequence.
 * The random roots and shifts are the caller's draws.
 *   roots, shifts host, num_sequences values; 0 <= shifts[j] < num_train
 *   order         host, receives the first num_out <= num_train nodes of the order
 * Synchronous.  Errors as above.
 */
int bgl_order_proximity(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                        int32_t num_sequences, const int64_t *roots, const int64_t *shifts,
                        int64_t num_out, int32_t *order, void *stream);

/*
 * Number of BFS sequences (Sec. 3.2.2: "gradually increases the number of
 * sequences from one until the shuffling error is smaller than the requirement").
 * Computes max_sequences BFS sequences once, then for s = 1, 2, ... merges the
 * first s of them and measures the mean shuffling error of the merged order over
 * batches of `batch`; stops at the first s whose error is <= threshold (the
 * caller's bound, e.g. sqrt(b*M)/n), or at max_sequences.
 *   chosen               host, receives s
 *   mean_tv_per_count    optional host array of max_sequences doubles: the error
 *                        for every count that was tried (entries after `chosen`
 *                        are left untouched)
 *   order                host, num_train ids: the merged order for `chosen`
 * Synchronous.  Errors as bgl_order_proximity and bgl_order_shuffling_error.
 */
int bgl_order_choose_sequences(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                               int32_t max_sequences, const int64_t *roots, const int64_t *shifts,
                               int32_t batch, const int32_t *labels, int32_t num_classes,
                               double threshold, int32_t *chosen, double *mean_tv_per_count,
                               int32_t *order, void *stream);

/*
 * Shuffling error of an order (Sec. 3.2.2, the quantity compared with
 * sqrt(b*M)/n to choose the number of sequences): total variation distance
 * between the label distribution of a batch and the label distribution of all
 * n ordered nodes, as the mean and the maximum over the batches of `batch`
 * consecutive nodes.  Host only.
 *   labels        host, num_nodes labels in [0, num_classes)
 * Errors: BGL_EINVAL.
 */
int bgl_order_shuffling_error(const int32_t *order, int64_t n, int32_t batch, const int32_t *labels,
                              int64_t num_nodes, int32_t num_classes, double *mean_tv, double *max_tv);

/* ------------------------------------------------------ the overlapped loop */

/*
 * Minibatch preparation as one loop over the calls above (Sec. 3.3: the stages
 * of minibatch preparation run as an asynchronous pipeline; on one GPU: batch
 * i+2 is sampled and batch i+1 looked up while batch i's miss rows cross the
 * host link).  Per batch: bgl_sample_khop two batches ahead, the host reads the
 * number of input nodes, bgl_cache_lookup_gather (early form for batches of
 * 65,536 input nodes or more; with a host tier the two halves of
 * bgl_cache_lookup_gather_tiered) and bgl_cache_insert_fifo of all misses.  The
 * loop enqueues what a caller of those functions would, on a stream of its own
 * for lookups, gathers and miss rows, on work_stream for the map updates and
 * early lookups, and (with a host tier and early lookups) on a third for the
 * sampling; results equal those of the calls made one after the other.
 *
 * The buffers stay the caller's (device memory unless stated), alive until
 * bgl_pipeline_destroy:
 *   workspace[3]     sampling workspaces, 256-byte aligned, workspace_bytes >=
 *                    bgl_sample_workspace_bytes(batch, fanouts, ...) each
 *   counts_host[3]   page-locked host memory, BGL_COUNTS_LEN ints each
 *   out_rows         cap_rows * row_bytes bytes, 16-byte aligned: the feature
 *                    rows of the current batch's input nodes
 *   out_slot, miss_pos  cap_rows ints each (as in bgl_cache_lookup_gather)
 *   cap_rows         >= min(num_nodes, batch * prod(1 + fanouts[h])), the bound
 *                    on a batch's input nodes
 */
typedef struct bgl_pipeline bgl_pipeline_t;
typedef struct {
    void *workspace[3];
    size_t workspace_bytes;
    int32_t *counts_host[3];
    void *out_rows;
    int32_t *out_slot;
    int32_t *miss_pos;
    int64_t cap_rows;
} bgl_pipeline_buffers_t;

/*
 * Called on the calling thread once batch `step`'s lookup and FIFO update have
 * been enqueued: sg is the batch's sampled subgraph (in workspace[sampler]),
 * n_input its number of input nodes.  Work the callback enqueues on the chain
 * stream (bgl_pipeline_streams) behind bgl_cache_wait_rows sees the batch's
 * complete out_rows; out_slot and miss_pos are rewritten by the next batch's
 * lookup, which may run on work_stream, so their readers enqueue there.
 */
typedef void (*bgl_batch_fn)(void *user, int64_t step, int32_t sampler, const bgl_subgraph_t *sg,
                             int64_t n_input);

/*
 * The cache is put in write-through mode; spare_rows != 0 also gives it one
 * spare row position per id of the largest batch (bgl_cache_set_spare_rows:
 * the cache must be new).  tier may be null (misses are read from the cache's
 * backing store in place).  work_stream: see above (NULL = the default stream).
 * Errors: BGL_EINVAL, BGL_ECAPACITY (a buffer is too small), BGL_ENOMEM,
 * BGL_EHIP, and those of the calls named.
 */
int bgl_pipeline_create(const bgl_graph_t *g, bgl_cache_t *c, bgl_host_tier_t *tier, int32_t batch,
                        const int32_t *fanouts, int32_t num_hops,
                        const bgl_pipeline_buffers_t *buffers, int spare_rows, void *work_stream,
                        bgl_pipeline_t **out);
int bgl_pipeline_destroy(bgl_pipeline_t *p);
/* Another cache from the next run on: put in write-through mode and (spare_rows != 0; the cache must
 * be new) given its spare row positions, as by bgl_pipeline_create. */
int bgl_pipeline_set_cache(bgl_pipeline_t *p, bgl_cache_t *c, int spare_rows);
/* Another host tier (or none) from the next run on. */
int bgl_pipeline_set_tier(bgl_pipeline_t *p, bgl_host_tier_t *tier);
/* The loop's streams (hipStream_t as void*); either pointer may be null. */
int bgl_pipeline_streams(bgl_pipeline_t *p, void **chain_stream, void **work_stream);
/* The most recent batch: its input nodes (device, inside one of the workspaces; null before the
 * first batch) and their number; out_rows holds their rows.  Either pointer may be null. */
int bgl_pipeline_last_batch(bgl_pipeline_t *p, const int32_t **input_nodes, int64_t *n_input);
/*
 * Prepare `steps` minibatches.  Batch i uses the seeds of seed batch
 * b = (first_step + i) mod seed_batches and the call seed
 * rng_seeds[b] xor ((first_step + i) / seed_batches), so that a later pass over
 * the same seeds samples differently.
 *   seeds        device, seed_batches * batch ids, ready in work_stream order
 *   rng_seeds    host, seed_batches values
 *   n_input      host, steps values: input nodes per batch
 *   n_hit        host, steps values: cache hits per batch; page-locked memory
 *                when the pipeline has no host tier (the device writes them)
 *   n_hit_tier   host, steps values or null: hits in the host tier
 *   on_batch     may be null
 * Returns after a device synchronisation: every batch is complete, the last
 * batch's rows are in out_rows.
 * Errors: those of the calls named above; after an error the cache and the tier
 * may be between two batches (destroy them).
 */
int bgl_pipeline_run(bgl_pipeline_t *p, const int32_t *seeds, int64_t seed_batches,
                     const uint64_t *rng_seeds, int64_t steps, int64_t first_step, int64_t *n_input,
                     int64_t *n_hit, int64_t *n_hit_tier, bgl_batch_fn on_batch, void *user);

#ifdef __cplusplus
}
#endif
#endif /* BGL_H */
