// GPU-resident FIFO feature cache (BGL paper, Sec. 3.2: dynamic FIFO policy,
// cache map + cache buffer per GPU, lookup / gather / fetch / update workflow;
// Sec. 4 "Feature Cache Engine": circular buffer addressed through a running
// tail, the occupant of the next position is evicted from the map and its row
// overwritten, cache work on a dedicated stream).
//
// Cache map: open addressing over 128-byte buckets.  A bucket is 16 64-bit
// words = exactly one cache line: words 0..14 hold (node id << 32 | slot) or
// EMPTY, word 15 counts the live entries that rest in a later bucket although
// their id hashes to this one or to an earlier one, i.e. whose walk from their
// home bucket to their resting bucket passed over this bucket.  A lookup reads
// its id's bucket (one line) and goes on to the next bucket only while that
// count is not zero (one id per lane: a wavefront keeps 64 independent line
// reads in flight; a 16-lanes-per-id lookup that found the id with a ballot was
// measured at half the speed, the lookup being latency bound).  An insertion is
// done by a group of 16 lanes that reads the bucket with one coalesced request,
// picks a free word with a wavefront ballot and claims it with a CAS; every full
// bucket it walks past gets its count raised by one.  An eviction blanks its
// word (slot_to_entry[slot] remembers the word that maps a slot's occupant, so
// no search) and lowers the counts of the buckets between the evicted id's home
// bucket (recomputed from the id) and that word's bucket: what one insertion
// added, the eviction of the same entry takes away.  So the counts always say
// exactly which buckets a live entry was pushed past, however long the cache
// has been churning under the FIFO policy: no tombstones, no rebuilds, and the
// length of a lookup depends on the load only (full buckets are rare at load
// <= 1/2 of 15 words per bucket), not on the cache's age.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include <hip/hip_ext.h>

#include "bgl_host_tier.h"
#include "bgl_internal.h"

namespace {

using namespace bgl;

constexpr uint64_t EMPTY64 = ~0ull;
constexpr int BUCKET = 16;       // 64-bit words per bucket (15 entries + the count of entries pushed past it)
constexpr int KEYS_PER_TILE = 256;  // ids per workgroup in probe / miss-list kernels
constexpr int PROF_RING = 4096;

struct CacheDev {          // device-resident scalars
    // tail is kept twice: FIFO update number k reads tail[k & 1] in every
    // workgroup while one lane writes tail[(k + 1) & 1], so no launch is needed
    // just to advance it.  The host counts the updates (bgl_cache::insert_calls).
    unsigned long long tail[2];
    unsigned long long lookups, hits;
    long long n_miss_last;  // miss count of the most recent lookup
    long long n_miss_gen[2];  // the same, kept per call parity for early lookups (the previous call's fetch still reads its own)
    long long n_hit_last;   // hit count of the most recent lookup
    int status;
    unsigned long long probe_lines;  // bucket lines read by all map lookups so far
    unsigned long long census[2];    // bgl_cache_map_stats: buckets with a count, sum of the counts
};

}  // namespace

struct bgl_cache {
    int64_t capacity = 0;
    int32_t row_bytes = 0;
    int64_t num_nodes = 0;
    const char *features = nullptr;  // device-visible backing store
    bool features_in_hbm = false;    // backing store is device memory (then the fetch is an HBM gather)
    int device = 0;
    int64_t rows = 0;                // row positions of the buffer: capacity + spare positions (see RowRing)
    char *buffer = nullptr;          // rows * row_bytes
    uint64_t *table = nullptr;       // num_buckets * BUCKET words
    uint32_t num_buckets = 0;        // power of two
    int32_t *slot_to_node = nullptr;  // capacity
    uint32_t *slot_to_entry = nullptr;
    CacheDev *dev = nullptr;
    int32_t *mbs = nullptr;          // per-tile miss counts of the most recent lookup (mbs_cap of them), then mbs_cap prefixes,
                                     // then mbs_cap counts of bucket lines read
    int64_t mbs_cap = 0;
    int32_t *hit_pos = nullptr;      // hits of the most recent lookup: hit_cap positions, then hit_cap slots
    int64_t hit_cap = 0;
    int64_t last_n = 0;              // n of the most recent lookup
    int32_t *mpos_copy[2] = {nullptr, nullptr};  // early lookups: the library's own copy of miss_pos, alternating between calls
    int64_t mpos_cap[2] = {0, 0};
    int32_t *src_of[2] = {nullptr, nullptr};  // assembled output: where each position's row comes from, alternating between calls
    int64_t src_cap[2] = {0, 0};
    uint64_t lookup_calls = 0;
    uint64_t insert_calls = 0;       // FIFO updates enqueued so far (selects the live copy of tail)
    hipStream_t own_side = nullptr;  // the miss fetch's stream when the caller names none; created on first use
                                     // (a process has few hardware queues: a stream that is never used should not take one)
    // Ordering between streams.  ev_listed: lists and hit rows of the last lookup are complete
    // (recorded on that lookup's main stream); ev_miss: its miss rows are complete (recorded on
    // the stream the fetch ran on); ev_map: the last FIFO update is complete (recorded on the
    // update's stream when that is not the lookup's main stream).
    hipEvent_t ev_listed = nullptr, ev_miss = nullptr, ev_map = nullptr;
    hipEvent_t ev_ids = nullptr;     // the lists of a lookup are complete (tiered: the missed ids have reached the host)
    hipStream_t last_main = nullptr, fetch_stream = nullptr, map_stream = nullptr;
    bool fetch_pending = false;      // ev_miss marks a miss fetch that later work may have to wait for
    bool fetch_reads_caller_lists = true;  // that fetch reads the caller's miss_pos (not the library's copy)
    bool map_pending = false;        // ev_map marks a FIFO update the next lookup has to wait for
    bool ev_listed_valid = false;    // a lookup has recorded ev_listed
    bool write_through = false;      // the miss fetch also fills the cache buffer (see bgl_cache_set_write_through)
    bool awaiting_insert = false;    // write-through: a lookup's misses are in the buffer but not in the map yet
    const void *wt_ids = nullptr, *wt_miss_pos = nullptr;  // arguments of that lookup
    // A tiered lookup between its two halves (bgl_cache_lookup_tiered_begin / _finish): the host threads
    // are packing its rows, the kernels that take them to their places have not been enqueued yet.
    struct TieredCall {
        bool active = false;
        bgl_host_tier *t = nullptr;
        bgl::TierPlan plan;
        hipStream_t ms = nullptr, ss = nullptr, ls = nullptr;
        const int32_t *ids = nullptr, *mpos = nullptr, *src_of = nullptr;
        int32_t *miss_pos = nullptr;
        void *out_rows = nullptr;
        int64_t n = 0;
        int par = 0, gen = 0;
    } tiered;
    // profiling
    unsigned profiling = 0;          // bit s set: stage s is timed
    hipEvent_t timed_start = nullptr, timed_stop = nullptr;  // events the next launch() hands to the kernel dispatch itself
    std::vector<hipEvent_t> prof_ev;  // pairs
    struct Rec { int stage; int ev; };
    std::vector<Rec> prof_rec;
    double prof_overhead_ms = 0;     // event pair around an (almost) empty kernel
    int64_t prof_dropped = 0;        // timed launches that got no events (event creation failed)
    int prof_every[BGL_NUM_STAGES];  // stage s is timed only in calls whose ordinal is a multiple of this
    double prof_ms[BGL_NUM_STAGES] = {};
    int64_t prof_n[BGL_NUM_STAGES] = {};

    bgl_cache() { std::fill(prof_every, prof_every + BGL_NUM_STAGES, 1); }
};

namespace {

// ------------------------------------------------------------------ kernels
__global__ void k_fill_u64(uint64_t *p, int64_t n, uint64_t v, int mark_stride)
{
    // every mark_stride-th word (the buckets' pushed-past counts) starts at 0
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = ((i % mark_stride) == mark_stride - 1) ? 0ull : v;
}

__global__ void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// Map lookup, one id per lane.  A lane reads its id's whole bucket (one 128-byte
// line, eight 16-byte loads issued together) and compares the 15 entries in
// registers; the chain continues only past a bucket whose pushed-past count is
// not zero.  A wavefront thus keeps 64 independent line reads in flight, which is
// what a latency-bound random lookup needs.  The misses of a wavefront are
// counted with one ballot; the bucket lines read are summed per workgroup for
// the map statistics (the list kernel adds the sums up).
__global__ __launch_bounds__(KEYS_PER_TILE) void k_probe(const int32_t *__restrict__ ids, int64_t n,
                                                         int64_t num_nodes,
                                                         const uint64_t *__restrict__ table,
                                                         uint32_t bucket_mask, int32_t *out_slot,
                                                         int32_t *mbs, int32_t *tile_lines, CacheDev *dev)
{
    __shared__ int sh_miss[KEYS_PER_TILE / kWave];
    __shared__ int sh_lines[KEYS_PER_TILE / kWave];
    const int64_t i = (int64_t)blockIdx.x * KEYS_PER_TILE + threadIdx.x;
    int slot = -1;
    int lines = 0;
    if (i < n) {
        const int32_t id = ids[i];
        if (id < 0 || (int64_t)id >= num_nodes) {
            dev->status = BGL_EINVAL;
        } else {
            const uint32_t key = (uint32_t)id;
            uint32_t b = hash32(key) & bucket_mask;
            for (uint32_t tries = 0; tries <= bucket_mask; ++tries) {
                const ulonglong2 *bp = reinterpret_cast<const ulonglong2 *>(table + (size_t)b * BUCKET);
                ulonglong2 w[BUCKET / 2];
#pragma unroll
                for (int k = 0; k < BUCKET / 2; ++k) w[k] = bp[k];
                bool found = false;
#pragma unroll
                for (int k = 0; k < BUCKET / 2; ++k) {
                    if ((uint32_t)(w[k].x >> 32) == key) { slot = (int)(uint32_t)w[k].x; found = true; }
                    if (k < BUCKET / 2 - 1 && (uint32_t)(w[k].y >> 32) == key) {
                        slot = (int)(uint32_t)w[k].y;
                        found = true;
                    }
                }
                ++lines;
                if (found || w[BUCKET / 2 - 1].y == 0) break;  // count zero: no live entry was pushed past this bucket
                b = (b + 1) & bucket_mask;
            }
        }
        out_slot[i] = slot;
    }
    const uint64_t missed = __ballot(i < n && slot < 0);
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) lines += __shfl_down(lines, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) {
        sh_miss[threadIdx.x / kWave] = __popcll(missed);
        sh_lines[threadIdx.x / kWave] = lines;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0, ln = 0;
#pragma unroll
        for (int k = 0; k < KEYS_PER_TILE / kWave; ++k) { t += sh_miss[k]; ln += sh_lines[k]; }
        mbs[blockIdx.x] = t;
        tile_lines[blockIdx.x] = ln;  // (summed by the list kernel: one atomic per workgroup on one counter
                                      // costs this kernel a third of its time)
    }
}

__global__ __launch_bounds__(kScanThreads) void k_scan_tiles(const int32_t *mbs, int64_t tiles, int32_t *prefix)
{
    __shared__ int sh[kScanThreads / kWave];
    scan_tile_counts<kScanThreads>(mbs, tiles, prefix, sh);
}

// Counters of an empty lookup (n = 0); with n > 0 k_split_list publishes them.
__global__ void k_empty_lookup(CacheDev *dev, int64_t *n_hit_host, int gen)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        dev->n_miss_last = 0;
        dev->n_miss_gen[gen] = 0;
        dev->n_hit_last = 0;
        if (n_hit_host) *n_hit_host = 0;
    }
}

// Where the rows live.  The cache buffer has `rows` >= capacity row positions.  Insertion
// number k (counted from the cache's creation, k = tail at the time) is written to position
// k mod rows, while its slot, which is what the map, out_slot and slot_to_node speak of, is
// k mod capacity.  With rows == capacity the two are the same number.  With spare positions
// (bgl_cache_set_spare_rows) a batch's new rows go to positions that hold no live row as long
// as the batch has no more misses than there are spare positions: the rows its own
// insertions evict stay readable until the next batch, so nothing has to be read "before it
// is overwritten".  The live rows are the last min(tail, capacity) insertions; slot and
// position of a live row follow from each other and tail by additions alone.
struct RowRing {
    int64_t capacity, rows;
    int64_t newest_slot, newest_pos;  // of insertion tail - 1 (tail > 0)
    // this call's insertions: ranks start <= r < start + count stay, rank r goes to position first_pos + (r - start)
    int64_t start, count, first_pos;
    __device__ __forceinline__ RowRing(unsigned long long tail, int64_t capacity_, int64_t rows_, int64_t n_miss = 0)
        : capacity(capacity_), rows(rows_)
    {
        const unsigned long long newest = tail > 0 ? tail - 1 : 0;
        newest_slot = (int64_t)(newest % (unsigned long long)capacity);
        newest_pos = (int64_t)(newest % (unsigned long long)rows);
        start = n_miss > capacity ? n_miss - capacity : 0;
        count = n_miss - start;
        first_pos = (int64_t)((tail + (unsigned long long)start) % (unsigned long long)rows);
    }
    __device__ __forceinline__ int64_t pos_of_slot(int64_t slot) const  // an occupied slot
    {
        int64_t age = newest_slot - slot;  // insertions since
        if (age < 0) age += capacity;
        const int64_t pos = newest_pos - age;
        return pos < 0 ? pos + rows : pos;
    }
    __device__ __forceinline__ int64_t pos_of_rank(int64_t r) const  // start <= r < start + count
    {
        const int64_t pos = first_pos + (r - start);
        return pos >= rows ? pos - rows : pos;
    }
    __device__ __forceinline__ bool overwritten(int64_t pos) const  // by this call's insertions
    {
        int64_t d = pos - first_pos;
        if (d < 0) d += rows;
        return d < count;
    }
};

// Ordered lists of the miss positions and of the hits (position and slot side by
// side, so the gather needs no dependent lookup).  A hit's rank is its position
// minus the number of misses before it.  Every workgroup sums the miss counts of
// the tiles before it (a few thousand ints at most), or reads the sum from
// tile_prefix where the call has so many tiles that k_scan_tiles ran first; the
// last one also publishes the call's counters.
__global__ __launch_bounds__(KEYS_PER_TILE) void k_split_list(const int32_t *__restrict__ out_slot,
                                                              int64_t n,
                                                              const int32_t *__restrict__ mbs,
                                                              const int32_t *__restrict__ tile_prefix,
                                                              const int32_t *__restrict__ tile_lines,
                                                              int32_t *miss_pos, int32_t *hit_pos,
                                                              int32_t *hit_slot, CacheDev *dev,
                                                              int64_t *n_hit_host,
                                                              const int32_t *__restrict__ ids,
                                                              int64_t num_nodes, int32_t *miss_ids_host,
                                                              int32_t *miss_pos_copy, int gen, int32_t *src_of,
                                                              int64_t capacity, int64_t rows, int par)
{
    __shared__ int sh_scan[KEYS_PER_TILE / kWave];
    __shared__ int sh_base;
    int tot;
    if (tile_prefix) {
        if (threadIdx.x == 0) sh_base = tile_prefix[blockIdx.x];
    } else {
        int part = 0;
        for (int t = threadIdx.x; t < (int)blockIdx.x; t += KEYS_PER_TILE) part += mbs[t];
        (void)block_excl_scan<KEYS_PER_TILE>(part, sh_scan, tot);
        if (threadIdx.x == 0) sh_base = tot;
    }
    const int64_t i = (int64_t)blockIdx.x * KEYS_PER_TILE + threadIdx.x;
    const int slot = i < n ? out_slot[i] : 0;
    const int flag = (i < n && slot < 0) ? 1 : 0;
    const int ex = block_excl_scan<KEYS_PER_TILE>(flag, sh_scan, tot);  // its barriers publish sh_base
    const int mrank = sh_base + ex;
    if (flag) {
        miss_pos[mrank] = (int32_t)i;
        if (miss_pos_copy) miss_pos_copy[mrank] = (int32_t)i;
        if (miss_ids_host) {  // a host tier that keeps nothing: it only wants the ids of the misses, in order
            const int32_t id = ids[i];
            miss_ids_host[mrank] = id;
            if (id < 0 || (int64_t)id >= num_nodes) n_hit_host[3] = 1;  // the host refuses the batch
        }
    } else if (i < n) {
        // the kernels that read the row get its position in the cache buffer (see RowRing)
        const int32_t pos = (int32_t)RowRing(dev->tail[par], capacity, rows).pos_of_slot(slot);
        if (!src_of) {
            hit_pos[i - mrank] = (int32_t)i;
            hit_slot[i - mrank] = pos;
        } else {
            src_of[i] = pos;
        }
    }
    // assembled output (k_assemble_rows): the source of every position's row, a row position of the
    // cache buffer (>= 0) or, as -(r + 1), miss number r, whose row comes in with the packed miss rows
    if (src_of && flag) src_of[i] = -(mrank + 1);
    if (blockIdx.x != gridDim.x - 1) return;
    // the last workgroup publishes the call's counters
    int lines = 0, all_lines;
    for (int t = threadIdx.x; t < (int)gridDim.x; t += KEYS_PER_TILE) lines += tile_lines[t];
    (void)block_excl_scan<KEYS_PER_TILE>(lines, sh_scan, all_lines);
    if (threadIdx.x == 0) {
        const long long n_miss = sh_base + tot;
        dev->probe_lines += (unsigned long long)all_lines;
        dev->n_miss_last = n_miss;
        dev->n_miss_gen[gen] = n_miss;
        dev->n_hit_last = n - n_miss;
        dev->lookups += (unsigned long long)n;
        dev->hits += (unsigned long long)(n - n_miss);
        // page-locked host memory: visible to the host once the kernel has completed
        if (n_hit_host) *n_hit_host = n - n_miss;
        if (miss_ids_host) {  // the tier's counts: nothing found there, everything to be brought in
            n_hit_host[1] = 0;
            n_hit_host[2] = n_miss;
        }
    }
}

// Row copies move 16-byte chunks; a row has Q = row_bytes / 16 of them.  Chunk
// index -> (row, chunk in row) with a compile-time Q where the width is a
// common one, so the division is a multiply.
template <int Q>
struct RowSplit {
    __device__ __forceinline__ static void split(int64_t idx, int q, int64_t &row, int &c)
    {
        if constexpr (Q > 0) { row = idx / Q; c = (int)(idx - row * Q); }
        else { row = idx / q; c = (int)(idx - row * q); }
    }
};

constexpr int COPY_THREADS = 256;
constexpr int COPY_UNROLL = 4;  // (the kernels name the four chunks of a lane by hand)
// Workgroups of a kernel that reads rows over the host link.  Each lane keeps
// four 16-byte loads in flight, so 64 x 256 lanes hold 1 MiB: that saturates
// the link for rows read in place (whole 128-byte lines, partly unused), and
// much more queues host reads in front of the concurrent kernels' HBM reads and
// slows those by an order of magnitude.  The packed ring is read densely and
// needs half as much in flight; with 64 workgroups there the next batch's
// lookup, and with it the packing of its rows, starts late.
constexpr int FETCH_BLOCKS = 64;
constexpr int RING_FETCH_BLOCKS = 32;
// Tiered lookup: rows the host threads copy per chunk before that chunk's fetch is launched.
constexpr int64_t TIER_CHUNK_ROWS = 49152;
constexpr int64_t TIER_FIRST_CHUNK_ROWS = 3072;
// Assembled output: largest out_rows of a call that is still written with ordinary stores.
constexpr int64_t ASSEMBLE_CACHED_OUTPUT_BYTES = 128ll << 20;

// out[i] = the cached row of ids[i] for every hit i (taken from the hit list, which holds the
// rows' positions in the cache buffer, so the work is proportional to the hits).  Consecutive lanes take consecutive
// 16-byte chunks of a row, so the loads and stores of one row are contiguous;
// four independent chunks per lane keep loads in flight.  The grid is sized for
// n rows; workgroups beyond the hit count leave at once.
template <int Q>
__global__ __launch_bounds__(COPY_THREADS) void k_gather_hits(
    const int32_t *__restrict__ hit_pos, const int32_t *__restrict__ hit_slot, int q,
    const uint4 *__restrict__ buffer, uint4 *__restrict__ out, const CacheDev *dev)
{
    static_assert(COPY_UNROLL == 4, "the four chunks of a lane are written out by hand");
    const int qq = Q > 0 ? Q : q;
    const int64_t total = (int64_t)dev->n_hit_last * qq;
    const int64_t base = (int64_t)blockIdx.x * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
    if (base - threadIdx.x >= total) return;
    // Three phases without a branch in between, so that the four list reads of a lane are in flight
    // together, then its four row reads, then its stores: chunk numbers beyond the end are clamped
    // to the last chunk, which those lanes then copy once more (same bytes to the same place).
    // (Written chunk by chunk with a branch each, every read waited for the one before it; with only
    // the stores under a branch the compiler moved reads back in there; and as an array `uint4 v[4]`
    // the values were put into LDS instead of registers.)
    const int64_t last = total - 1;
    int64_t r0, r1, r2, r3;
    int c0, c1, c2, c3;
    RowSplit<Q>::split(min(base, last), q, r0, c0);
    RowSplit<Q>::split(min(base + COPY_THREADS, last), q, r1, c1);
    RowSplit<Q>::split(min(base + 2 * COPY_THREADS, last), q, r2, c2);
    RowSplit<Q>::split(min(base + 3 * COPY_THREADS, last), q, r3, c3);
    const int32_t s0 = hit_slot[r0], s1 = hit_slot[r1], s2 = hit_slot[r2], s3 = hit_slot[r3];
    const int32_t p0 = hit_pos[r0], p1 = hit_pos[r1], p2 = hit_pos[r2], p3 = hit_pos[r3];
    const uint4 v0 = buffer[(int64_t)s0 * qq + c0];
    const uint4 v1 = buffer[(int64_t)s1 * qq + c1];
    const uint4 v2 = buffer[(int64_t)s2 * qq + c2];
    const uint4 v3 = buffer[(int64_t)s3 * qq + c3];
    out[(int64_t)p0 * qq + c0] = v0;
    out[(int64_t)p1 * qq + c1] = v1;
    out[(int64_t)p2 * qq + c2] = v2;
    out[(int64_t)p3 * qq + c3] = v3;
}

// out[miss_pos[r]] = features[ids[miss_pos[r]]] for every miss r; the loads cross
// the host link when the backing store is page-locked host memory.  The link
// needs little data in flight compared with HBM, and waves blocked on it would
// otherwise hold the wave slots the concurrent hit gather needs, so this kernel
// runs as a small fixed grid that strides over the miss list.
//
// Write-through variant (WT): the same loaded chunk is also stored into the cache
// buffer slot the row will get from the FIFO update that follows, so that update
// needs no row copy: miss r goes to slot (tail + r) mod capacity, ranks that a
// later miss of the same batch would overwrite are skipped.
template <int Q, bool WT>
__global__ __launch_bounds__(COPY_THREADS) void k_fetch_miss(
    const int32_t *__restrict__ miss_pos, const int32_t *__restrict__ ids, int q,
    int64_t num_nodes, const uint4 *__restrict__ features, uint4 *__restrict__ out,
    const CacheDev *dev, uint4 *__restrict__ buffer, int64_t capacity, int64_t rows, int par, int gen)
{
    static_assert(COPY_UNROLL == 4, "the four chunks of a lane are written out by hand");
    const int qq = Q > 0 ? Q : q;
    const int64_t n_miss = dev->n_miss_gen[gen];
    const int64_t total = n_miss * qq;
    const int64_t last = total - 1;
    // (the ranks that stay cover less than one turn of the buffer: the wrap-around is one subtraction)
    const RowRing ring(WT ? dev->tail[par] : 0ull, capacity, rows, n_miss);
    const int64_t start = ring.start;
    const int64_t step = (int64_t)gridDim.x * (COPY_THREADS * COPY_UNROLL);
    for (int64_t base = (int64_t)blockIdx.x * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
         base - threadIdx.x < total; base += step) {
        // Phase by phase for the lane's four chunks, as in k_gather_hits: positions, ids, rows, stores;
        // chunk numbers beyond the end are clamped to the last chunk, which is then copied again.
        int64_t r0, r1, r2, r3;
        int c0, c1, c2, c3;
        RowSplit<Q>::split(min(base, last), q, r0, c0);
        RowSplit<Q>::split(min(base + COPY_THREADS, last), q, r1, c1);
        RowSplit<Q>::split(min(base + 2 * COPY_THREADS, last), q, r2, c2);
        RowSplit<Q>::split(min(base + 3 * COPY_THREADS, last), q, r3, c3);
        const int32_t m0 = miss_pos[r0], m1 = miss_pos[r1], m2 = miss_pos[r2], m3 = miss_pos[r3];
        const int32_t i0 = ids[m0], i1 = ids[m1], i2 = ids[m2], i3 = ids[m3];
        // an id outside the table (reported by the lookup) reads row 0 and stores nothing
        const bool ok0 = i0 >= 0 && (int64_t)i0 < num_nodes, ok1 = i1 >= 0 && (int64_t)i1 < num_nodes;
        const bool ok2 = i2 >= 0 && (int64_t)i2 < num_nodes, ok3 = i3 >= 0 && (int64_t)i3 < num_nodes;
        uint4 v0 = features[(int64_t)(ok0 ? i0 : 0) * qq + c0];
        uint4 v1 = features[(int64_t)(ok1 ? i1 : 0) * qq + c1];
        uint4 v2 = features[(int64_t)(ok2 ? i2 : 0) * qq + c2];
        uint4 v3 = features[(int64_t)(ok3 ? i3 : 0) * qq + c3];
        // (the four reads stay above the branches that follow: the values are needed here)
        asm volatile("" : "+v"(v0.x), "+v"(v0.y), "+v"(v0.z), "+v"(v0.w), "+v"(v1.x), "+v"(v1.y), "+v"(v1.z), "+v"(v1.w),
                          "+v"(v2.x), "+v"(v2.y), "+v"(v2.z), "+v"(v2.w), "+v"(v3.x), "+v"(v3.y), "+v"(v3.z), "+v"(v3.w));
        auto store = [&](bool ok, int64_t r, int32_t m, int c, const uint4 &v) {
            if (!ok) return;
            out[(int64_t)m * qq + c] = v;
            if (WT && r >= start) buffer[ring.pos_of_rank(r) * qq + c] = v;
        };
        store(ok0, r0, m0, c0, v0);
        store(ok1, r1, m1, c1, v1);
        store(ok2, r2, m2, c2, v2);
        store(ok3, r3, m3, c3, v3);
    }
}

// 16-byte accesses that say "not needed again soon" (NT) or nothing.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ void st16(uint4 *p, const uint4 &v)
{
    if (NT) __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
    else *p = v;
}
template <bool NT>
__device__ __forceinline__ uint4 ld16(const uint4 *p)
{
    if (NT) {
        const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        return uint4{t.x, t.y, t.z, t.w};
    }
    return *p;
}

// Tiered lookup: out[miss_pos[r]] = rows[(first + l) mod ring] for listed misses
// l0 <= l < l0 + count of the GPU cache, r = rank[l] (r = l without a list: a tier
// that keeps nothing lists every miss).  rows are page-locked host rows that the
// host threads have just packed in list order: the host tier's ring (rows it
// brought in from the store) or its staging rows (rows it held), or the device
// memory the copy engine has moved those rows to (NT: these are read once, and
// what is written is for a later kernel, so neither should displace the lines
// the next hit gather works on; measured, that gather takes 24 instead of 28
// microseconds and this kernel 69 instead of 74).  Same launch shape and
// write-through rule as k_fetch_miss.
template <int Q, bool WT, bool NT>
__global__ __launch_bounds__(COPY_THREADS) void k_fetch_rows(
    const int32_t *__restrict__ rank, int64_t l0, int64_t count, unsigned long long first, int64_t ring,
    const int32_t *__restrict__ miss_pos, int q, const uint4 *__restrict__ rows, uint4 *__restrict__ out,
    const CacheDev *dev, uint4 *__restrict__ buffer, int64_t capacity, int64_t buffer_rows, int par, int64_t n_miss)
{
    static_assert(COPY_UNROLL == 4, "the four chunks of a lane are written out by hand");
    const int qq = Q > 0 ? Q : q;
    const int64_t total = count * qq;
    const int64_t last = total - 1;
    // the two wrap-arounds without a division per chunk: the launch covers less than one turn of
    // the ring, and the ranks it stores (start <= r < n_miss) less than one turn of the buffer
    const int64_t first_pos = (int64_t)((first + (unsigned long long)l0) % (unsigned long long)ring) - l0;
    const RowRing dst(WT ? dev->tail[par] : 0ull, capacity, buffer_rows, n_miss);
    const int64_t start = dst.start;
    const int64_t step = (int64_t)gridDim.x * (COPY_THREADS * COPY_UNROLL);
    for (int64_t base = (int64_t)blockIdx.x * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
         base - threadIdx.x < total; base += step) {
        // Phase by phase for the lane's four chunks, as in k_gather_hits: ranks, positions, rows,
        // stores; chunk numbers beyond the end are clamped to the last chunk, which is then copied again.
        int64_t l_0, l_1, l_2, l_3;
        int c0, c1, c2, c3;
        RowSplit<Q>::split(min(base, last), q, l_0, c0);
        RowSplit<Q>::split(min(base + COPY_THREADS, last), q, l_1, c1);
        RowSplit<Q>::split(min(base + 2 * COPY_THREADS, last), q, l_2, c2);
        RowSplit<Q>::split(min(base + 3 * COPY_THREADS, last), q, l_3, c3);
        l_0 += l0; l_1 += l0; l_2 += l0; l_3 += l0;
        int64_t r0 = l_0, r1 = l_1, r2 = l_2, r3 = l_3;
        if (rank) { r0 = rank[l_0]; r1 = rank[l_1]; r2 = rank[l_2]; r3 = rank[l_3]; }
        const int32_t m0 = miss_pos[r0], m1 = miss_pos[r1], m2 = miss_pos[r2], m3 = miss_pos[r3];
        auto wrapped = [](int64_t x, int64_t turn) { return x >= turn ? x - turn : x; };
        uint4 v0 = ld16<NT>(&rows[wrapped(first_pos + l_0, ring) * qq + c0]);
        uint4 v1 = ld16<NT>(&rows[wrapped(first_pos + l_1, ring) * qq + c1]);
        uint4 v2 = ld16<NT>(&rows[wrapped(first_pos + l_2, ring) * qq + c2]);
        uint4 v3 = ld16<NT>(&rows[wrapped(first_pos + l_3, ring) * qq + c3]);
        st16<NT>(&out[(int64_t)m0 * qq + c0], v0);
        st16<NT>(&out[(int64_t)m1 * qq + c1], v1);
        st16<NT>(&out[(int64_t)m2 * qq + c2], v2);
        st16<NT>(&out[(int64_t)m3 * qq + c3], v3);
        if (WT) {
            if (start == 0) {  // every rank gets a slot (the usual case: fewer misses than slots)
                st16<NT>(&buffer[dst.pos_of_rank(r0) * qq + c0], v0);
                st16<NT>(&buffer[dst.pos_of_rank(r1) * qq + c1], v1);
                st16<NT>(&buffer[dst.pos_of_rank(r2) * qq + c2], v2);
                st16<NT>(&buffer[dst.pos_of_rank(r3) * qq + c3], v3);
            } else {
                if (r0 >= start) st16<NT>(&buffer[dst.pos_of_rank(r0) * qq + c0], v0);
                if (r1 >= start) st16<NT>(&buffer[dst.pos_of_rank(r1) * qq + c1], v1);
                if (r2 >= start) st16<NT>(&buffer[dst.pos_of_rank(r2) * qq + c2], v2);
                if (r3 >= start) st16<NT>(&buffer[dst.pos_of_rank(r3) * qq + c3], v3);
            }
        }
    }
}

// ---- assembled output
// With the packed miss rows of a call already in device memory (the copy engine
// has landed them, in miss order), one pass over the output in its own order can
// write every row: a hit's row comes from the cache buffer, a miss's row from the
// landed rows, and the miss rows also go to the buffer slots the FIFO rule gives
// them (write-through).  Every output line is then written whole by one stream of
// stores, and the hit gather and the scatter of the landed rows are one launch
// large enough to fill the memory system.  One hazard: a hit whose row lies
// where this call's own misses are written must be read before it is
// overwritten.  Those rows (few when a batch's misses are few against the
// capacity, all of the hits when they outnumber it) are copied by
// k_assemble_pre, which runs first; k_assemble_rows leaves them alone.
// With enough spare row positions in the buffer (RowRing) no live row lies where this call
// writes, and the first pass is not launched at all.
// The hits inside the window, copied before the window is written.  Each wavefront scans 64
// positions (one per lane), packs the ones concerned into LDS with a ballot and copies their rows
// with all its lanes, four 16-byte chunks in flight per lane.
template <int Q>
__global__ __launch_bounds__(COPY_THREADS) void k_assemble_pre(
    const int32_t *__restrict__ src_of, int64_t n, int q, const uint4 *__restrict__ buffer,
    uint4 *__restrict__ out, const CacheDev *dev, int64_t capacity, int64_t rows, int par, int64_t n_miss)
{
    constexpr int WAVES = COPY_THREADS / kWave;
    __shared__ int32_t sh_pos[WAVES][kWave];
    __shared__ int32_t sh_slot[WAVES][kWave];
    const int qq = Q > 0 ? Q : q;
    const RowRing ring(dev->tail[par], capacity, rows, n_miss);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t step = (int64_t)gridDim.x * COPY_THREADS;
    for (int64_t base = (int64_t)blockIdx.x * COPY_THREADS + wave * kWave; base < n; base += step) {
        const int64_t i = base + lane;
        const int32_t s = i < n ? src_of[i] : -1;
        const bool mine = s >= 0 && ring.overwritten(s);
        const uint64_t mask = __ballot(mine);
        if (mask == 0) continue;  // (uniform in the wavefront)
        const int m = __popcll(mask);
        if (mine) {
            const int at = __popcll(mask & ((1ull << lane) - 1ull));
            sh_pos[wave][at] = (int32_t)i;
            sh_slot[wave][at] = s;
        }
        // (the lists are written and read by this wavefront only)
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int total = m * qq;
        for (int k0 = 0; k0 < total; k0 += 4 * kWave) {
            const int last = total - 1;
            const int k[4] = {min(k0 + lane, last), min(k0 + kWave + lane, last), min(k0 + 2 * kWave + lane, last),
                              min(k0 + 3 * kWave + lane, last)};
            int j[4], cc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if constexpr (Q > 0) { j[u] = k[u] / Q; cc[u] = k[u] - j[u] * Q; }
                else { j[u] = k[u] / q; cc[u] = k[u] - j[u] * q; }
            }
            const uint4 v0 = buffer[(int64_t)sh_slot[wave][j[0]] * qq + cc[0]];
            const uint4 v1 = buffer[(int64_t)sh_slot[wave][j[1]] * qq + cc[1]];
            const uint4 v2 = buffer[(int64_t)sh_slot[wave][j[2]] * qq + cc[2]];
            const uint4 v3 = buffer[(int64_t)sh_slot[wave][j[3]] * qq + cc[3]];
            out[(int64_t)sh_pos[wave][j[0]] * qq + cc[0]] = v0;
            out[(int64_t)sh_pos[wave][j[1]] * qq + cc[1]] = v1;
            out[(int64_t)sh_pos[wave][j[2]] * qq + cc[2]] = v2;
            out[(int64_t)sh_pos[wave][j[3]] * qq + cc[3]] = v3;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// Every other row, in output order: chunk number -> (position, chunk in row); the position's
// source decides where the chunk is read.  Phases as in k_gather_hits: the four sources of a lane,
// then its four chunks, then the stores; chunk numbers beyond the end are clamped to the last
// chunk, which is then copied again.  A chunk of a hit inside the window is read (from a slot that
// may be changing: the value is not used) and not stored.
template <int Q, bool NTO>
__global__ __launch_bounds__(COPY_THREADS) void k_assemble_rows(
    const int32_t *__restrict__ src_of, int64_t n, int q, const uint4 *__restrict__ landed,
    uint4 *buffer, uint4 *__restrict__ out, const CacheDev *dev, int64_t capacity, int64_t rows, int par,
    int64_t n_miss)
{
    static_assert(COPY_UNROLL == 4, "the four chunks of a lane are written out by hand");
    const int qq = Q > 0 ? Q : q;
    const int64_t total = n * qq;
    const int64_t last = total - 1;
    const RowRing ring(dev->tail[par], capacity, rows, n_miss);
    const int64_t step = (int64_t)gridDim.x * (COPY_THREADS * COPY_UNROLL);
    for (int64_t base = (int64_t)blockIdx.x * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
         base - threadIdx.x < total; base += step) {
        const int64_t x0 = min(base, last), x1 = min(base + COPY_THREADS, last),
                      x2 = min(base + 2 * COPY_THREADS, last), x3 = min(base + 3 * COPY_THREADS, last);
        int64_t i0, i1, i2, i3;
        int c0, c1, c2, c3;
        RowSplit<Q>::split(x0, q, i0, c0);
        RowSplit<Q>::split(x1, q, i1, c1);
        RowSplit<Q>::split(x2, q, i2, c2);
        RowSplit<Q>::split(x3, q, i3, c3);
        const int32_t s0 = src_of[i0], s1 = src_of[i1], s2 = src_of[i2], s3 = src_of[i3];
        auto source = [&](int32_t s, int c) -> const uint4 * {
            return s >= 0 ? buffer + (int64_t)s * qq + c : landed + (int64_t)(-s - 1) * qq + c;
        };
        uint4 v0 = *source(s0, c0);
        uint4 v1 = *source(s1, c1);
        uint4 v2 = *source(s2, c2);
        uint4 v3 = *source(s3, c3);
        // (the four reads stay above the branches that follow: the values are needed here)
        asm volatile("" : "+v"(v0.x), "+v"(v0.y), "+v"(v0.z), "+v"(v0.w), "+v"(v1.x), "+v"(v1.y), "+v"(v1.z), "+v"(v1.w),
                          "+v"(v2.x), "+v"(v2.y), "+v"(v2.z), "+v"(v2.w), "+v"(v3.x), "+v"(v3.y), "+v"(v3.z), "+v"(v3.w));
        auto store = [&](int32_t s, int c, int64_t x, const uint4 &v) {
            if (s >= 0) {
                if (!ring.overwritten(s)) st16<NTO>(&out[x], v);
            } else {
                st16<NTO>(&out[x], v);
                const int64_t r = -(int64_t)s - 1;
                if (r >= ring.start) st16<true>(&buffer[ring.pos_of_rank(r) * qq + c], v);
            }
        };
        store(s0, c0, x0, v0);
        store(s1, c1, x1, v1);
        store(s2, c2, x2, v2);
        store(s3, c3, x3, v3);
    }
}

// Map update: 16 lanes per inserted row.  Evict the slot's occupant (blank its
// word, found through slot_to_entry, and take one off the pushed-past count of
// every bucket from the evicted id's home bucket up to the word's bucket), then
// read the new id's bucket with one coalesced request, pick a free word with a
// wavefront ballot and claim it with a CAS; a bucket without a free word gets
// one added to its count before the group moves on.  Counts change by atomic
// adds only and no lookup runs beside an update, so after the launch every
// count is exact whatever the order of the groups.  Bucket words are read with
// device-scope atomic loads so that the retry after a lost CAS sees the winner's
// word.  (One row per lane was measured too: no faster, the update is bound by
// its random lines, not by lane count.)
__device__ __forceinline__ void insert_map_part(
    int64_t block, const int32_t *__restrict__ ids, const int32_t *__restrict__ miss_pos,
    int64_t n_miss, int64_t start, unsigned long long tail, int64_t capacity, int64_t num_nodes,
    uint64_t *table, uint32_t bucket_mask, int32_t *slot_to_node, uint32_t *slot_to_entry,
    CacheDev *dev)
{
    const int l = threadIdx.x & (BUCKET - 1);
    const int gshift = (threadIdx.x & (kWave - 1)) & ~(BUCKET - 1);
    const int64_t r = start + (block * COPY_THREADS + threadIdx.x) / BUCKET;
    if (r >= n_miss) return;  // uniform inside the group
    const int64_t slot = (int64_t)((tail + (unsigned long long)r) % (unsigned long long)capacity);
    const int32_t key = ids[miss_pos[r]];
    const int32_t old = slot_to_node[slot];
    if (old >= 0 && l == 0) {
        const uint32_t word = slot_to_entry[slot];
        __hip_atomic_store(&table[word], EMPTY64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the buckets this entry had been pushed past (none for an entry in its home bucket)
        const uint32_t rest = word / BUCKET;
        for (uint32_t b = hash32((uint32_t)old) & bucket_mask; b != rest; b = (b + 1) & bucket_mask)
            atomicAdd((unsigned long long *)&table[(size_t)b * BUCKET + (BUCKET - 1)], ~0ull);  // -1
    }
    if (key < 0 || (int64_t)key >= num_nodes) {
        // reported by the lookup already: the slot's row will be overwritten, so
        // leave the slot unmapped rather than mapped to the wrong bytes
        if (l == 0) {
            slot_to_node[slot] = -1;
            dev->status = BGL_EINVAL;
        }
        return;
    }
    const uint64_t mine = ((uint64_t)(uint32_t)key << 32) | (uint32_t)slot;
    uint32_t b = hash32((uint32_t)key) & bucket_mask;
    uint32_t entry = 0;
    bool done = false;
    // every lost CAS means another group filled a word: at most 15 retries per
    // bucket, and a table at load <= 1/2 always has a bucket with a free word
    for (uint32_t tries = 0; tries < 16u * (bucket_mask + 1u) && !done; ++tries) {
        const uint64_t e = __hip_atomic_load(&table[(size_t)b * BUCKET + l], __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        const bool free_word = l < BUCKET - 1 && e == EMPTY64;
        const uint32_t fm = (uint32_t)(__ballot(free_word) >> gshift) & 0xffffu;
        if (fm) {
            const int t = __ffs(fm) - 1;
            int won = 0;
            if (l == t) {
                unsigned long long prev = atomicCAS(
                    (unsigned long long *)&table[(size_t)b * BUCKET + t], EMPTY64, mine);
                won = prev == EMPTY64;
            }
            won = __shfl(won, t, BUCKET);
            if (won) {
                entry = b * BUCKET + (uint32_t)t;
                done = true;
            }
        } else {
            // full: this entry will rest beyond bucket b (its eviction takes the one off again)
            if (l == BUCKET - 1) atomicAdd((unsigned long long *)&table[(size_t)b * BUCKET + l], 1ull);
            b = (b + 1) & bucket_mask;
        }
    }
    if (l == 0) {
        if (done) {
            slot_to_node[slot] = key;
            slot_to_entry[slot] = entry;
        } else {
            dev->status = BGL_ECAPACITY;
        }
    }
}

// buffer[(tail + r) % capacity] = out[miss_pos[r]]: the destination is a
// contiguous (wrapping) run of slots, so the stores stream.
template <int Q>
__device__ __forceinline__ void insert_rows_part(
    int64_t block, const int32_t *__restrict__ miss_pos, int64_t n_miss, int64_t start,
    unsigned long long tail, int64_t capacity, int64_t rows, int q, const uint4 *__restrict__ out,
    uint4 *__restrict__ buffer)
{
    static_assert(COPY_UNROLL == 4, "the four chunks of a lane are written out by hand");
    const int qq = Q > 0 ? Q : q;
    const int64_t total = (n_miss - start) * qq;
    const int64_t base = block * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
    if (base - threadIdx.x >= total) return;
    // Phase by phase for the lane's four chunks, as in k_gather_hits: positions, rows, stores; chunk
    // numbers beyond the end are clamped to the last chunk, which is then copied again.
    const int64_t last = total - 1;
    // (start <= r < n_miss covers at most one turn of the buffer: the wrap-around is one subtraction)
    const RowRing ring(tail, capacity, rows, n_miss);
    int64_t r0, r1, r2, r3;
    int c0, c1, c2, c3;
    RowSplit<Q>::split(min(base, last), q, r0, c0);
    RowSplit<Q>::split(min(base + COPY_THREADS, last), q, r1, c1);
    RowSplit<Q>::split(min(base + 2 * COPY_THREADS, last), q, r2, c2);
    RowSplit<Q>::split(min(base + 3 * COPY_THREADS, last), q, r3, c3);
    const int32_t m0 = miss_pos[start + r0], m1 = miss_pos[start + r1], m2 = miss_pos[start + r2],
                  m3 = miss_pos[start + r3];
    const uint4 v0 = out[(int64_t)m0 * qq + c0];
    const uint4 v1 = out[(int64_t)m1 * qq + c1];
    const uint4 v2 = out[(int64_t)m2 * qq + c2];
    const uint4 v3 = out[(int64_t)m3 * qq + c3];
    buffer[ring.pos_of_rank(start + r0) * qq + c0] = v0;
    buffer[ring.pos_of_rank(start + r1) * qq + c1] = v1;
    buffer[ring.pos_of_rank(start + r2) * qq + c2] = v2;
    buffer[ring.pos_of_rank(start + r3) * qq + c3] = v3;
}

// The FIFO update is two launches because only the row copy needs the fetched
// rows: the map update is enqueued ahead of the wait for the miss fetch and runs
// while the host link is still busy.  Both read tail[par]; the row copy stores the
// advanced value in tail[par ^ 1] for the next update.
__global__ __launch_bounds__(COPY_THREADS) void k_insert_map(
    const int32_t *__restrict__ ids, const int32_t *__restrict__ miss_pos, int64_t n_miss_arg,
    int64_t capacity, int64_t num_nodes, uint64_t *table, uint32_t bucket_mask,
    int32_t *slot_to_node, uint32_t *slot_to_entry, CacheDev *dev, int par, int advance)
{
    const int64_t n_miss = n_miss_arg >= 0 ? n_miss_arg : dev->n_miss_last;
    const int64_t start = n_miss > capacity ? n_miss - capacity : 0;  // earlier ranks would be overwritten
    const unsigned long long tail = dev->tail[par];
    // write-through mode has no row-copy launch: then this one advances tail
    if (advance && blockIdx.x == 0 && threadIdx.x == 0) dev->tail[par ^ 1] = tail + (unsigned long long)n_miss;
    insert_map_part(blockIdx.x, ids, miss_pos, n_miss, start, tail, capacity, num_nodes,
                    table, bucket_mask, slot_to_node, slot_to_entry, dev);
}

template <int Q>
__global__ __launch_bounds__(COPY_THREADS) void k_insert_rows(
    const int32_t *__restrict__ miss_pos, int64_t n_miss_arg, int64_t capacity, int64_t rows, int q,
    const uint4 *__restrict__ out, uint4 *__restrict__ buffer, CacheDev *dev, int par)
{
    const int64_t n_miss = n_miss_arg >= 0 ? n_miss_arg : dev->n_miss_last;
    const int64_t start = n_miss > capacity ? n_miss - capacity : 0;
    const unsigned long long tail = dev->tail[par];
    if (blockIdx.x == 0 && threadIdx.x == 0) dev->tail[par ^ 1] = tail + (unsigned long long)n_miss;
    insert_rows_part<Q>(blockIdx.x, miss_pos, n_miss, start, tail, capacity, rows, q, out, buffer);
}

// FIFO update when the launches above are skipped (nothing can be inserted).
__global__ void k_advance_tail(CacheDev *dev, int64_t n_miss_arg, int par)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const long long n = n_miss_arg >= 0 ? n_miss_arg : dev->n_miss_last;
        dev->tail[par ^ 1] = dev->tail[par] + (unsigned long long)n;
    }
}

__global__ void k_noop() {}

// Census of the pushed-past counts for bgl_cache_map_stats: how many buckets a
// lookup would walk past, and how many (entry, bucket) pairs that is.
__global__ void k_map_census(const uint64_t *__restrict__ table, uint32_t num_buckets, CacheDev *dev)
{
    unsigned long long nz = 0, sum = 0;
    for (uint32_t b = blockIdx.x * blockDim.x + threadIdx.x; b < num_buckets; b += gridDim.x * blockDim.x) {
        const uint64_t cnt = table[(size_t)b * BUCKET + (BUCKET - 1)];
        nz += cnt != 0;
        sum += cnt;
    }
    if (nz) atomicAdd(&dev->census[0], nz);
    if (sum) atomicAdd(&dev->census[1], sum);
}

// ------------------------------------------------------------------ host helpers
// Stage timers.  A stage that is one kernel is timed by the dispatch itself: the
// pair of events goes into the launch (launch() below) and records the kernel's
// own begin and end on the device.  A stage of several launches (exact = false)
// is bracketed by two event records on the stream, which also times the launch
// gaps around it.
struct Prof {
    bgl_cache *c;
    hipStream_t st;
    int ev = -1;
    bool exact;
    Prof(bgl_cache *c_, int stage, hipStream_t st_, bool exact_ = true) : c(c_), st(st_), exact(exact_)
    {
        if (!(c->profiling & (1u << stage))) return;
        const bool of_update = stage == BGL_STAGE_INSERT_MAP || stage == BGL_STAGE_INSERT_ROWS;
        const uint64_t call = of_update ? c->insert_calls + 1 : c->lookup_calls;
        if (c->prof_every[stage] > 1 && call % (uint64_t)c->prof_every[stage] != 0) return;
        if (2 * (c->prof_rec.size() + 1) > c->prof_ev.size()) {  // more timed launches than events: add some
            const size_t old = c->prof_ev.size();
            c->prof_ev.resize(old + 2 * PROF_RING, nullptr);
            for (size_t k = old; k < c->prof_ev.size(); ++k)
                if (hipEventCreate(&c->prof_ev[k]) != hipSuccess) {
                    for (size_t j = old; j < k; ++j) (void)hipEventDestroy(c->prof_ev[j]);
                    c->prof_ev.resize(old);
                    c->prof_dropped += 1;
                    return;
                }
        }
        ev = (int)c->prof_rec.size() * 2;
        c->prof_rec.push_back({stage, ev});
        if (exact) {
            c->timed_start = c->prof_ev[ev];
            c->timed_stop = c->prof_ev[ev + 1];
        } else {
            (void)hipEventRecord(c->prof_ev[ev], st);
        }
    }
    ~Prof()
    {
        if (ev < 0) return;
        if (exact) c->timed_start = c->timed_stop = nullptr;  // (already taken by the launch)
        else (void)hipEventRecord(c->prof_ev[ev + 1], st);
    }
};

// Kernel launch; inside a Prof scope of a one-kernel stage the dispatch records its
// own begin and end into that scope's events.
template <typename... P, typename... A>
void launch(bgl_cache *c, hipStream_t st, void (*kernel)(P...), dim3 grid, dim3 block, A &&...a)
{
    if (c->timed_start) {
        hipEvent_t e0 = c->timed_start, e1 = c->timed_stop;
        c->timed_start = c->timed_stop = nullptr;
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, e0, e1, 0, static_cast<P>(a)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, st, static_cast<P>(a)...);
    }
}

void drain_profile(bgl_cache *c)
{
    for (auto &r : c->prof_rec) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->prof_ev[r.ev], c->prof_ev[r.ev + 1]) == hipSuccess) {
            c->prof_ms[r.stage] += ms;
            c->prof_n[r.stage] += 1;
        }
    }
    c->prof_rec.clear();
}

template <typename F>
void dispatch_q(int q, F &&f)
{
    switch (q) {
    case 25: f(std::integral_constant<int, 25>{}); break;  // 100 x fp32
    case 32: f(std::integral_constant<int, 32>{}); break;  // 128 x fp32
    case 64: f(std::integral_constant<int, 64>{}); break;  // 512 x bf16
    default: f(std::integral_constant<int, 0>{}); break;
    }
}

int copy_blocks(int64_t rows, int q)
{
    return (int)bgl::ceil_div(rows * q, (int64_t)COPY_THREADS * COPY_UNROLL);
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" int bgl_cache_create(int64_t capacity_rows, int32_t row_bytes,
                                const void *host_features, int64_t num_nodes, bgl_cache_t **out)
try {
    if (!out) BGL_FAIL(BGL_EINVAL, "out is null");
    *out = nullptr;
    if (capacity_rows < 1 || capacity_rows > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "capacity_rows must be in [1, 2^31) (got %lld)", (long long)capacity_rows);
    if (row_bytes < 16 || row_bytes % 16 != 0)
        BGL_FAIL(BGL_EINVAL, "row_bytes must be a positive multiple of 16 (got %d)", row_bytes);
    if (num_nodes < 1 || num_nodes > INT32_MAX) BGL_FAIL(BGL_EINVAL, "num_nodes out of range");
    if (!bgl::aligned(host_features, 16)) BGL_FAIL(BGL_EINVAL, "host_features is not 16-byte aligned");

    hipPointerAttribute_t attr;
    attr.type = hipMemoryTypeHost;
    const char *feat_dev = nullptr;
    if (host_features) {  // null: misses are served through a host tier only
        if (hipPointerGetAttributes(&attr, host_features) != hipSuccess) {
            (void)hipGetLastError();
            BGL_FAIL(BGL_EINVAL, "host_features is neither page-locked host memory nor device memory");
        }
        if (attr.type == hipMemoryTypeHost || attr.type == hipMemoryTypeDevice ||
            attr.type == hipMemoryTypeManaged) {
            feat_dev = static_cast<const char *>(attr.devicePointer);
        }
        if (!feat_dev)
            BGL_FAIL(BGL_EINVAL, "host_features is neither page-locked host memory nor device memory");
    }

    bgl_cache *c = new (std::nothrow) bgl_cache();
    if (!c) BGL_FAIL(BGL_ENOMEM, "out of host memory");
    c->capacity = capacity_rows;
    c->rows = capacity_rows;
    c->row_bytes = row_bytes;
    c->num_nodes = num_nodes;
    c->features = feat_dev;
    c->features_in_hbm = attr.type == hipMemoryTypeDevice;
    // load <= 1/2 of the 15 usable words per bucket
    uint64_t nbk = 1;
    while (nbk * 15 < (uint64_t)capacity_rows * 2) nbk <<= 1;
    c->num_buckets = (uint32_t)nbk;

    auto fail = [&](int code) { bgl_cache_destroy(c); return code; };
    hipError_t e;
    if (hipGetDevice(&c->device) != hipSuccess) { bgl::set_error("hipGetDevice failed"); return fail(BGL_EHIP); }
#define TRY_ALLOC(ptr, bytes)                                                              \
    if ((e = hipMalloc((void **)&(ptr), (bytes))) != hipSuccess) {                         \
        bgl::set_error("hipMalloc of %zu bytes failed: %s", (size_t)(bytes), hipGetErrorString(e)); \
        return fail(e == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP);                     \
    }
    TRY_ALLOC(c->buffer, (size_t)c->rows * row_bytes);
    TRY_ALLOC(c->table, (size_t)nbk * BUCKET * sizeof(uint64_t));
    TRY_ALLOC(c->slot_to_node, (size_t)capacity_rows * sizeof(int32_t));
    TRY_ALLOC(c->slot_to_entry, (size_t)capacity_rows * sizeof(uint32_t));
    TRY_ALLOC(c->dev, sizeof(CacheDev));
#undef TRY_ALLOC
    if (hipEventCreateWithFlags(&c->ev_listed, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_miss, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_map, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_ids, hipEventDisableTiming) != hipSuccess) {
        bgl::set_error("stream/event creation failed");
        return fail(BGL_EHIP);
    }
    hipLaunchKernelGGL(k_fill_u64, dim3(2048), dim3(256), 0, 0, c->table, (int64_t)nbk * BUCKET,
                       EMPTY64, BUCKET);
    hipLaunchKernelGGL(k_fill_i32, dim3(1024), dim3(256), 0, 0, c->slot_to_node, capacity_rows, -1);
    if (hipMemset(c->dev, 0, sizeof(CacheDev)) != hipSuccess ||
        hipMemset(c->buffer, 0, (size_t)c->rows * row_bytes) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
        bgl::set_error("cache initialisation failed: %s", hipGetErrorString(hipGetLastError()));
        return fail(BGL_EHIP);
    }
    *out = c;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_destroy(bgl_cache_t *c)
try {
    if (!c) return BGL_OK;
    (void)hipDeviceSynchronize();
    for (auto ev : c->prof_ev) (void)hipEventDestroy(ev);
    if (c->ev_listed) (void)hipEventDestroy(c->ev_listed);
    if (c->ev_miss) (void)hipEventDestroy(c->ev_miss);
    if (c->ev_map) (void)hipEventDestroy(c->ev_map);
    if (c->ev_ids) (void)hipEventDestroy(c->ev_ids);
    if (c->own_side) (void)hipStreamDestroy(c->own_side);
    (void)hipFree(c->buffer);
    (void)hipFree(c->table);
    (void)hipFree(c->slot_to_node);
    (void)hipFree(c->slot_to_entry);
    (void)hipFree(c->dev);
    (void)hipFree(c->mbs);
    (void)hipFree(c->hit_pos);
    (void)hipFree(c->mpos_copy[0]);
    (void)hipFree(c->mpos_copy[1]);
    (void)hipFree(c->src_of[0]);
    (void)hipFree(c->src_of[1]);
    delete c;
    return BGL_OK;
} BGL_NOTHROW_END

namespace {

// The lists one lookup leaves for its own later kernels: per-tile miss counts (mbs_cap of them)
// followed by mbs_cap prefixes and mbs_cap counts of bucket lines read, and the hits as hit_cap
// positions followed by hit_cap slots.
struct LookupLists {
    int32_t *mbs;
    int64_t mbs_cap;
    int32_t *hit_pos;
    int64_t hit_cap;
};

// First half of a lookup: map lookup and lists on stream ls, with a host tier its
// lookup for the misses (followed by ev_ids), then the hit gather on stream ms,
// ev_listed.  ls == ms unless the lookup runs early (see the tiered call): then
// the lists go to *mpos_used, the library's own copy of miss_pos, because the
// caller's miss_pos of the previous call is still being read by that call's
// fetch while this one's lists are written.
int lookup_phase(bgl_cache *c, const int32_t *ids, int64_t n, void *out_rows, int32_t *out_slot,
                 int32_t *miss_pos, int64_t *n_hit_dev, hipStream_t ms, hipStream_t ls, bgl_host_tier *tier,
                 const int32_t **mpos_used, int *gen_used, const LookupLists *fixed = nullptr,
                 const int32_t **src_of_used = nullptr)
{
    const bool early = ls != ms;
    const int gen = (int)(c->lookup_calls & 1);  // which copy of the per-call device state this call owns
    *gen_used = gen;
    const int64_t tiles = bgl::ceil_div(n, KEYS_PER_TILE);
    // the per-call lists: the cache's own, grown on demand, or the ones the caller of this function brings
    if (!fixed && tiles + 1 > c->mbs_cap) {
        BGL_HIP(hipDeviceSynchronize());
        (void)hipFree(c->mbs);
        c->mbs = nullptr;
        c->mbs_cap = 0;
        const int64_t cap = std::max<int64_t>(2 * tiles + 1, 1024);
        BGL_HIP(hipMalloc((void **)&c->mbs, 3 * sizeof(int32_t) * (size_t)cap));  // counts, their prefixes, lines read
        c->mbs_cap = cap;
    }
    if (!fixed && n > c->hit_cap) {
        BGL_HIP(hipDeviceSynchronize());
        (void)hipFree(c->hit_pos);
        c->hit_pos = nullptr;
        c->hit_cap = 0;
        const int64_t cap = std::max<int64_t>(n + n / 2, 4096);
        BGL_HIP(hipMalloc((void **)&c->hit_pos, 2 * sizeof(int32_t) * (size_t)cap));  // positions, then slots
        c->hit_cap = cap;
    }
    int32_t *mpos_copy = nullptr;
    if (early) {
        const int g = gen;
        if (n > c->mpos_cap[g]) {
            BGL_HIP(hipDeviceSynchronize());
            (void)hipFree(c->mpos_copy[g]);
            c->mpos_copy[g] = nullptr;
            c->mpos_cap[g] = 0;
            const int64_t cap = std::max<int64_t>(n + n / 2, 4096);
            BGL_HIP(hipMalloc((void **)&c->mpos_copy[g], sizeof(int32_t) * (size_t)cap));
            c->mpos_cap[g] = cap;
        }
        mpos_copy = c->mpos_copy[g];
    }
    *mpos_used = early ? mpos_copy : miss_pos;
    // Assembled output (the caller launches k_assemble_pre / k_assemble_rows once the miss rows have
    // landed): the list kernel records every position's source, and there is no hit gather here.
    int32_t *src_of = nullptr;
    if (src_of_used) {
        const int g = gen;
        if (n > c->src_cap[g]) {
            BGL_HIP(hipDeviceSynchronize());
            (void)hipFree(c->src_of[g]);
            c->src_of[g] = nullptr;
            c->src_cap[g] = 0;
            const int64_t cap = std::max<int64_t>(n + n / 2, 4096);
            BGL_HIP(hipMalloc((void **)&c->src_of[g], sizeof(int32_t) * (size_t)cap));
            c->src_cap[g] = cap;
        }
        src_of = c->src_of[g];
        *src_of_used = src_of;
    }
    int32_t *const mbs = fixed ? fixed->mbs : c->mbs;
    const int64_t mbs_cap = fixed ? fixed->mbs_cap : c->mbs_cap;
    int32_t *const hit_pos = fixed ? fixed->hit_pos : c->hit_pos;
    const int64_t hit_cap = fixed ? fixed->hit_cap : c->hit_cap;
    c->lookup_calls += 1;
    c->last_n = n;
    const int q = c->row_bytes / 16;
    if (tier) bgl::tier_prepare(tier);
    if (c->map_pending && c->map_stream != ls) BGL_HIP(hipStreamWaitEvent(ls, c->ev_map, 0));
    if (!early && c->fetch_pending && c->fetch_stream != ms) {
        // the previous call's fetch still reads that call's lists
        BGL_HIP(hipStreamWaitEvent(ms, c->ev_miss, 0));
    }
    if (early && c->fetch_pending && c->fetch_reads_caller_lists) {
        // so does it when that call was not an early one: then this one cannot be early either
        BGL_HIP(hipStreamWaitEvent(ls, c->ev_miss, 0));
    }
    if (n > 0) {
        {
            Prof p(c, BGL_STAGE_PROBE, ls);
            launch(c, ls, k_probe, dim3((unsigned)tiles), dim3(KEYS_PER_TILE), ids, n, c->num_nodes, c->table,
                   c->num_buckets - 1, out_slot, mbs, mbs + 2 * mbs_cap, c->dev);
        }
        {
            Prof p(c, BGL_STAGE_MISS_LIST, ls, false);
            int32_t *tile_prefix = nullptr;
            if (tiles >= kSelfSumTiles) {
                tile_prefix = mbs + mbs_cap;
                hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(kScanThreads), 0, ls, mbs, tiles, tile_prefix);
            }
            hipLaunchKernelGGL(k_split_list, dim3((unsigned)tiles), dim3(KEYS_PER_TILE), 0, ls, out_slot,
                               n, mbs, tile_prefix, mbs + 2 * mbs_cap, miss_pos, hit_pos, hit_pos + hit_cap, c->dev,
                               n_hit_dev, ids, c->num_nodes,
                               tier ? bgl::tier_ids_device_if_passthrough(tier) : nullptr, mpos_copy, gen, src_of,
                               c->capacity, c->rows, (int)(c->insert_calls & 1));
        }
    } else {
        hipLaunchKernelGGL(k_empty_lookup, dim3(1), dim3(64), 0, ls, c->dev, n_hit_dev, gen);
    }
    if (tier) {
        const int rc = bgl::tier_enqueue_lookup(tier, ids, miss_pos, &c->dev->n_miss_last, n, gen, ls);
        if (rc != BGL_OK) return rc;
    }
    if (tier || early) BGL_HIP(hipEventRecord(c->ev_ids, ls));  // the lists are complete
    if (early) {
        // the hit gather reads rows the previous fetch may still be writing, and needs the lists
        if (c->fetch_pending && c->fetch_stream != ms) BGL_HIP(hipStreamWaitEvent(ms, c->ev_miss, 0));
        BGL_HIP(hipStreamWaitEvent(ms, c->ev_ids, 0));
    }
    c->fetch_pending = false;
    c->map_pending = false;
    c->last_main = ms;
    c->ev_listed_valid = true;
    if (n > 0 && !src_of) {
        Prof p(c, BGL_STAGE_GATHER_HIT, ms);
        dispatch_q(q, [&](auto Q) {
            launch(c, ms, k_gather_hits<decltype(Q)::value>, dim3(copy_blocks(n, q)), dim3(COPY_THREADS),
                   hit_pos, hit_pos + hit_cap, q, reinterpret_cast<const uint4 *>(c->buffer),
                   reinterpret_cast<uint4 *>(out_rows), c->dev);
        });
    }
    // The miss fetch starts once the hit gather is done: host-link reads
    // queued in the memory pipeline would otherwise stall the gather's HBM
    // reads, and the fetch (milliseconds) loses nothing by starting a few
    // tens of microseconds later.
    BGL_HIP(hipEventRecord(c->ev_listed, ms));
    return BGL_OK;
}

// The stream of the miss fetch: the caller's, or one of the cache's own.
int side_stream_of(bgl_cache *c, void *side_stream, hipStream_t *out)
{
    if (side_stream) {
        *out = static_cast<hipStream_t>(side_stream);
        return BGL_OK;
    }
    if (!c->own_side) BGL_HIP(hipStreamCreateWithFlags(&c->own_side, hipStreamNonBlocking));
    *out = c->own_side;
    return BGL_OK;
}

int check_lookup_args(bgl_cache *c, const int32_t *ids, int64_t n, void *out_rows, int32_t *out_slot,
                      int32_t *miss_pos)
{
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (n < 0 || n > INT32_MAX) BGL_FAIL(BGL_EINVAL, "n must be in [0, 2^31) (got %lld)", (long long)n);
    if (n > 0 && (!ids || !out_rows || !out_slot || !miss_pos))
        BGL_FAIL(BGL_EINVAL, "ids, out_rows, out_slot and miss_pos must not be null");
    if (!bgl::aligned(out_rows, 16)) BGL_FAIL(BGL_EINVAL, "out_rows is not 16-byte aligned");
    if (c->tiered.active)
        BGL_FAIL(BGL_EINVAL, "a tiered lookup has been begun: bgl_cache_lookup_tiered_finish comes first");
    if (c->write_through && c->awaiting_insert)
        BGL_FAIL(BGL_EINVAL, "write-through mode: the previous lookup's misses have not been inserted yet");
    return BGL_OK;
}

}  // namespace

namespace {

int lookup_gather_impl(bgl_cache_t *c, const int32_t *ids, int64_t n, void *out_rows, int32_t *out_slot,
                       int32_t *miss_pos, int64_t *n_hit_host, void *main_stream, void *side_stream,
                       void *lookup_stream, bool early, const LookupLists *fixed = nullptr)
{
    int rc = check_lookup_args(c, ids, n, out_rows, out_slot, miss_pos);
    if (rc != BGL_OK) return rc;
    if (early && !c->write_through)
        BGL_FAIL(BGL_EINVAL, "an early lookup needs write-through mode");
    if (!c->features) BGL_FAIL(BGL_EINVAL, "the cache has no backing store: use bgl_cache_lookup_gather_tiered");
    hipStream_t ms = static_cast<hipStream_t>(main_stream);
    hipStream_t ss = nullptr;
    if (fixed) {
        ss = side_stream ? static_cast<hipStream_t>(side_stream) : ms;  // (no stream is created here)
    } else {
        rc = side_stream_of(c, side_stream, &ss);
        if (rc != BGL_OK) return rc;
    }
    // the hit count goes straight into the caller's page-locked word (no copy launch)
    int64_t *n_hit_dev = nullptr;
    if (n_hit_host) {
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, n_hit_host) != hipSuccess || attr.type != hipMemoryTypeHost ||
            !attr.devicePointer) {
            (void)hipGetLastError();
            BGL_FAIL(BGL_EINVAL, "n_hit_host must be page-locked host memory");
        }
        n_hit_dev = static_cast<int64_t *>(attr.devicePointer);
    }
    const int q = c->row_bytes / 16;
    hipStream_t ls = early ? static_cast<hipStream_t>(lookup_stream) : ms;
    const int32_t *mpos = nullptr;
    int gen = 0;
    rc = lookup_phase(c, ids, n, out_rows, out_slot, miss_pos, n_hit_dev, ms, ls, nullptr, &mpos, &gen, fixed);
    if (rc != BGL_OK) return rc;
    if (n > 0) {
        if (ss != ms) BGL_HIP(hipStreamWaitEvent(ss, c->ev_listed, 0));
        {
            Prof p(c, BGL_STAGE_FETCH_MISS, ss);
            // the small grid is for the host link only; an HBM-resident store wants the whole chip
            const int blocks = (int)std::min<int64_t>(copy_blocks(n, q), c->features_in_hbm ? 8192 : FETCH_BLOCKS);
            const int par = (int)(c->insert_calls & 1);
            dispatch_q(q, [&](auto Q) {
                auto k = c->write_through ? k_fetch_miss<decltype(Q)::value, true>
                                          : k_fetch_miss<decltype(Q)::value, false>;
                launch(c, ss, k, dim3(blocks), dim3(COPY_THREADS), mpos, ids, q, c->num_nodes,
                       reinterpret_cast<const uint4 *>(c->features), reinterpret_cast<uint4 *>(out_rows), c->dev,
                       reinterpret_cast<uint4 *>(c->buffer), c->capacity, c->rows, par, gen);
            });
        }
        BGL_HIP(hipEventRecord(c->ev_miss, ss));
        c->fetch_pending = true;
        c->fetch_stream = ss;
        c->fetch_reads_caller_lists = mpos == miss_pos;
    }
    BGL_HIP(hipGetLastError());
    if (c->write_through) {
        c->awaiting_insert = true;
        c->wt_ids = ids;
        c->wt_miss_pos = miss_pos;
    }
    return BGL_OK;
}

}  // namespace

extern "C" int bgl_cache_lookup_gather(bgl_cache_t *c, const int32_t *ids, int64_t n,
                                       void *out_rows, int32_t *out_slot, int32_t *miss_pos,
                                       int64_t *n_hit_host, void *main_stream, void *side_stream)
try {
    return lookup_gather_impl(c, ids, n, out_rows, out_slot, miss_pos, n_hit_host, main_stream, side_stream,
                              nullptr, false);
} BGL_NOTHROW_END

// ---- the lookup that allocates nothing
// Its lists live in a fixed array in device memory that is part of the library's code object
// (every GPU the library runs on holds its own copy until the process ends).  The array's name
// is only a host-side stand-in: the address the kernels get is asked for once per device.
namespace {

constexpr int64_t NOALLOC_MAX_IDS = BGL_NOALLOC_MAX_IDS;
constexpr int64_t NOALLOC_TILES = (NOALLOC_MAX_IDS + KEYS_PER_TILE - 1) / KEYS_PER_TILE + 1;
constexpr size_t NOALLOC_MBS_BYTES = (3 * sizeof(int32_t) * (size_t)NOALLOC_TILES + 255) / 256 * 256;
constexpr size_t NOALLOC_BYTES = NOALLOC_MBS_BYTES + 2 * sizeof(int32_t) * (size_t)NOALLOC_MAX_IDS;
constexpr int NOALLOC_MAX_DEVICES = 64;

static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];

void *g_scratch_ptr[NOALLOC_MAX_DEVICES];  // device address of `scratch` on each device, once asked for
std::mutex g_scratch_mutex;

int scratch_of_current_device(int device, void **out)
{
    if (device < 0 || device >= NOALLOC_MAX_DEVICES) BGL_FAIL(BGL_EUNSUPPORTED, "device ordinal %d is out of range", device);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        BGL_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) BGL_FAIL(BGL_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return BGL_OK;
}

}  // namespace

extern "C" int bgl_cache_lookup_gather_noalloc(bgl_cache_t *c, const int32_t *ids, int64_t n,
                                               void *out_rows, int32_t *out_slot, int32_t *miss_pos,
                                               int64_t *n_hit_host, void *main_stream, void *side_stream)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (n > NOALLOC_MAX_IDS)
        BGL_FAIL(BGL_ECAPACITY, "n = %lld exceeds BGL_NOALLOC_MAX_IDS = %lld: use bgl_cache_lookup_gather",
                 (long long)n, (long long)NOALLOC_MAX_IDS);
    int device = -1;
    BGL_HIP(hipGetDevice(&device));
    if (device != c->device)
        BGL_FAIL(BGL_EINVAL, "the cache lives on device %d, the current device is %d", c->device, device);
    void *ptr = nullptr;
    int rc = scratch_of_current_device(device, &ptr);
    if (rc != BGL_OK) return rc;
    unsigned char *base = static_cast<unsigned char *>(ptr);
    const LookupLists lists{reinterpret_cast<int32_t *>(base), NOALLOC_TILES,
                            reinterpret_cast<int32_t *>(base + NOALLOC_MBS_BYTES), NOALLOC_MAX_IDS};
    // (a timed launch may have to create events: this call's kernels are not timed)
    struct Untimed {
        bgl_cache *c;
        unsigned saved;
        explicit Untimed(bgl_cache *c_) : c(c_), saved(c_->profiling) { c->profiling = 0; }
        ~Untimed() { c->profiling = saved; }
    } untimed(c);
    return lookup_gather_impl(c, ids, n, out_rows, out_slot, miss_pos, n_hit_host, main_stream, side_stream,
                              nullptr, false, &lists);
} BGL_NOTHROW_END

extern "C" int bgl_cache_lookup_gather_early(bgl_cache_t *c, const int32_t *ids, int64_t n,
                                             void *out_rows, int32_t *out_slot, int32_t *miss_pos,
                                             int64_t *n_hit_host, void *main_stream, void *side_stream,
                                             void *lookup_stream)
try {
    return lookup_gather_impl(c, ids, n, out_rows, out_slot, miss_pos, n_hit_host, main_stream, side_stream,
                              lookup_stream, static_cast<hipStream_t>(lookup_stream) != static_cast<hipStream_t>(main_stream));
} BGL_NOTHROW_END

namespace {

// The packed rows of one tiered lookup on their way to out_rows (and, in write-through mode, to the
// cache buffer).  Host threads pack them as one sequence: first the rows the tier holds (into its
// staging rows, in list order), then the others (from the store into consecutive ring positions).
struct TieredRows {
    bgl_cache *c;
    bgl_host_tier *t;
    const bgl::TierPlan *plan;
    hipStream_t ss;        // the stream of the kernels that write the rows to their places
    const int32_t *mpos;   // this call's miss positions (the caller's list, or the library's copy)
    void *out_rows;
    int64_t n;
    int par;               // which copy of the cache's tail the kernels read
    bool early;            // the lookup ran early: the host is ahead of the link
    const int32_t *src_of; // assembled output: the source of every position's row (else null)

    // out[mpos[rank[l]]] = base[(first + l) mod ring] for l0 <= l < l0 + count.  landed: the rows are in
    // device memory (whole chip; rows read once, and written for a later kernel: non-temporal accesses, so
    // that they do not push the cache buffer's and the output's lines out of the chip's caches in front of
    // the next hit gather); else they are read over the host link (small grid).
    void launch_rows(const char *base, unsigned long long first, int64_t ring, const int32_t *rank, int64_t l0,
                     int64_t count, bool landed) const
    {
        if (count == 0) return;
        const int q = c->row_bytes / 16;
        Prof p(c, BGL_STAGE_FETCH_MISS, ss);
        const int blocks = (int)std::min<int64_t>(copy_blocks(count, q), landed ? 8192 : RING_FETCH_BLOCKS);
        dispatch_q(q, [&](auto Q) {
            constexpr int QQ = decltype(Q)::value;
            auto k = landed ? (c->write_through ? k_fetch_rows<QQ, true, true> : k_fetch_rows<QQ, false, true>)
                            : (c->write_through ? k_fetch_rows<QQ, true, false> : k_fetch_rows<QQ, false, false>);
            launch(c, ss, k, dim3(blocks), dim3(COPY_THREADS), rank, l0, count, first, ring, mpos, q,
                   reinterpret_cast<const uint4 *>(base), reinterpret_cast<uint4 *>(out_rows), c->dev,
                   reinterpret_cast<uint4 *>(c->buffer), c->capacity, c->rows, par, n - plan->n_hit_gpu);
        });
    }
    // Assembled output, first launch: the hits whose slots this call's misses are about to take.
    void launch_assemble_pre() const
    {
        const int q = c->row_bytes / 16;
        Prof p(c, BGL_STAGE_ASSEMBLE_PRE, ss);
        const int blocks = (int)std::min<int64_t>(bgl::ceil_div(n, COPY_THREADS), 2048);
        dispatch_q(q, [&](auto Q) {
            launch(c, ss, k_assemble_pre<decltype(Q)::value>, dim3(blocks), dim3(COPY_THREADS), src_of, n, q,
                   reinterpret_cast<const uint4 *>(c->buffer), reinterpret_cast<uint4 *>(out_rows), c->dev,
                   c->capacity, c->rows, par, n - plan->n_hit_gpu);
        });
    }
    // Second launch, once the packed miss rows are in `land`: every other row of the output, and
    // the miss rows into the cache buffer.
    void launch_assemble_rows(const char *land) const
    {
        const int q = c->row_bytes / 16;
        Prof p(c, BGL_STAGE_ASSEMBLE, ss);
        // One workgroup per 1,024 chunks (a grid capped at 8,192 workgroups that strides was measured 2 % slower
        // on 400- and 1,024-byte rows).  The output is written with ordinary stores while a batch's rows fit
        // the chip's last-level cache with room to spare (the next batch overwrites them there, and whoever
        // consumes them reads them there), with non-temporal ones beyond that; the rows that go into the
        // cache buffer are always written non-temporally.  (Measured, fraction of HBM peak with ordinary /
        // non-temporal output stores: 61 MB of output 0.68 / 0.64, 102 MB 0.77 / 0.67, 171 MB 0.66 / 0.66,
        // 310 MB 0.68 / 0.70.)
        const bool nto = (int64_t)n * c->row_bytes > ASSEMBLE_CACHED_OUTPUT_BYTES;
        const int blocks = (int)std::min<int64_t>(copy_blocks(n, q), 1 << 20);
        dispatch_q(q, [&](auto Q) {
            constexpr int QQ = decltype(Q)::value;
            auto k = nto ? k_assemble_rows<QQ, true> : k_assemble_rows<QQ, false>;
            launch(c, ss, k, dim3(blocks), dim3(COPY_THREADS), src_of, n, q,
                   reinterpret_cast<const uint4 *>(land), reinterpret_cast<uint4 *>(c->buffer),
                   reinterpret_cast<uint4 *>(out_rows), c->dev, c->capacity, c->rows, par, n - plan->n_hit_gpu);
        });
    }
};

// Copy-engine transport: the packed rows go to device memory (`land`) with plain copies on the tier's
// copy stream, as soon as they are packed and whatever the kernels of this cache are doing (the
// previous call's rows may still be on their way); kernels then scatter them from there, after the
// hit gather.  The link carries one batch after the other.
int rows_by_copy_engine(const TieredRows &r, char *land)
{
    bgl_cache *c = r.c;
    bgl_host_tier *t = r.t;
    const bgl::TierPlan &plan = *r.plan;
    const int64_t total = plan.n_hit + plan.n_miss;
    const size_t rb = (size_t)c->row_bytes;
    hipStream_t cs = bgl::tier_copy_stream(t);
    const char *ring_rows = bgl::tier_rows_device(t);
    auto copy = [&](char *dst, const char *src, int64_t count) -> int {
        Prof p(c, BGL_STAGE_LINK_COPY, cs, false);
        BGL_HIP(hipMemcpyAsync(dst, src, (size_t)count * rb, hipMemcpyDefault, cs));
        return BGL_OK;
    };
    // rows x0 <= x < x1 of the packed sequence: the tier's hits (staging rows), then its misses (ring)
    auto copy_rows = [&](int64_t x0, int64_t x1) -> int {
        if (x0 < plan.n_hit) {
            const int64_t e = std::min(x1, plan.n_hit);
            const int r1 = copy(land + (size_t)x0 * rb, plan.stage + (size_t)x0 * rb, e - x0);
            if (r1 != BGL_OK) return r1;
        }
        const int64_t a = std::max(x0, plan.n_hit) - plan.n_hit, b = x1 - plan.n_hit;
        if (b > a) {
            const int64_t pos = (int64_t)((plan.ptail + (uint64_t)a) % (uint64_t)plan.ring);
            const int64_t len1 = std::min(b - a, plan.ring - pos);  // up to the end of the ring
            const int r1 = copy(land + (size_t)(plan.n_hit + a) * rb, ring_rows + (size_t)pos * rb, len1);
            if (r1 != BGL_OK) return r1;
            if (len1 < b - a) {
                const int r2 = copy(land + (size_t)(plan.n_hit + a + len1) * rb, ring_rows, b - a - len1);
                if (r2 != BGL_OK) return r2;
            }
        }
        return BGL_OK;
    };
    // A copy costs the link a few microseconds whatever its size, so while earlier copies (the
    // previous call's, or this call's) still occupy the link the packed rows pile up for one larger
    // copy; when the link is free a chunk goes at once.
    // (`land` was last read by the kernels of the call before the previous one.  They are over: this call's
    // lists, which the host has just waited for, follow the previous call's map update, which follows that
    // call's lists, which were recorded behind the wait for those kernels.)
    // (an early lookup is ahead of the link as a rule: large chunks from the start, but a short batch is
    // not held back for one)
    int64_t chunk = r.early ? std::min(TIER_CHUNK_ROWS, std::max<int64_t>(total / 4, 4 * TIER_FIRST_CHUNK_ROWS))
                            : TIER_FIRST_CHUNK_ROWS;
    bool link_busy = bgl::tier_copy_event_recorded(t);
    for (int64_t launched = 0; launched < total;) {
        const int64_t ready = bgl::tier_copy_progress(t);
        bool go = ready > launched && ready == total;
        if (!go && ready - launched >= chunk) {
            if (link_busy) {
                link_busy = hipEventQuery(bgl::tier_copy_event(t)) != hipSuccess;
                (void)hipGetLastError();  // "not ready" is no error
            }
            go = !link_busy;
        }
        if (go) {
            const int rc = copy_rows(launched, ready);
            if (rc != BGL_OK) return rc;
            BGL_HIP(hipEventRecord(bgl::tier_copy_event(t), cs));
            bgl::tier_set_copy_event_recorded(t);
            link_busy = true;
            launched = ready;
            chunk = std::min<int64_t>(2 * chunk, TIER_CHUNK_ROWS);
        } else if (!bgl::tier_copy_help(t)) {  // nothing to send: pack a few rows too
            __builtin_ia32_pause();
        }
    }
    bgl::tier_copy_wait(t);
    if (r.src_of) {  // (the tier keeps nothing: plan.n_hit == 0, the landed rows are in miss order)
        // The first pass is needed only if this call's rows may land on live ones: not when the buffer
        // has a spare position for every miss of the call (the misses that do not stay advance the
        // position too).  (It needs no landed row: it runs while the copies are still on their way.)
        if (r.n - plan.n_hit_gpu > c->rows - c->capacity) r.launch_assemble_pre();
        BGL_HIP(hipStreamWaitEvent(r.ss, bgl::tier_copy_event(t), 0));
        r.launch_assemble_rows(land);
        return BGL_OK;
    }
    BGL_HIP(hipStreamWaitEvent(r.ss, bgl::tier_copy_event(t), 0));  // (recorded behind the last copy)
    r.launch_rows(land, 0ull, (int64_t)INT64_MAX, plan.hit_rank, 0, plan.n_hit, true);
    r.launch_rows(land + (size_t)plan.n_hit * rb, 0ull, (int64_t)INT64_MAX, plan.miss_rank, 0, plan.n_miss, true);
    return BGL_OK;
}

// Kernel transport: the kernels read the page-locked rows over the host link themselves, chunk by
// chunk as the rows are packed.  Small chunks first, so that the link starts early; the copy threads
// outrun the link only by a little, so the chunks grow until a launch is a few per cent of its kernel.
int rows_by_kernels(const TieredRows &r)
{
    bgl_cache *c = r.c;
    bgl_host_tier *t = r.t;
    const bgl::TierPlan &plan = *r.plan;
    const int64_t total = plan.n_hit + plan.n_miss;
    const char *ring_rows = bgl::tier_rows_device(t);
    // (an early lookup is ahead of the link anyway: full chunks from the start)
    int64_t chunk = r.early ? TIER_CHUNK_ROWS : TIER_FIRST_CHUNK_ROWS;
    bool gather_done = false;
    for (int64_t launched = 0; launched < total;) {
        const int64_t ready = bgl::tier_copy_progress(t);
        // a chunk does not straddle the two kinds of rows
        const int64_t limit = launched < plan.n_hit ? std::min(ready, plan.n_hit) : ready;
        bool go = limit > launched && (limit == plan.n_hit || limit == total);
        if (!go && limit - launched >= chunk) {
            // An early lookup's fetch cannot start before its hit gather has run, which waits for
            // the previous call's fetch: until then the packed rows pile up for one larger launch.
            if (r.early && !gather_done) {
                gather_done = hipEventQuery(c->ev_listed) == hipSuccess;
                (void)hipGetLastError();  // "not ready" is no error
            }
            go = gather_done || !r.early;
        }
        if (go) {
            if (launched < plan.n_hit)
                r.launch_rows(plan.stage, 0ull, (int64_t)INT64_MAX, plan.hit_rank, launched, limit - launched,
                              false);
            else
                r.launch_rows(ring_rows, (unsigned long long)plan.ptail, plan.ring, plan.miss_rank,
                              launched - plan.n_hit, limit - launched, false);
            launched = limit;
            chunk = std::min<int64_t>(2 * chunk, TIER_CHUNK_ROWS);
        } else if (!bgl::tier_copy_help(t)) {  // nothing to send: pack a few rows too
            __builtin_ia32_pause();
        }
    }
    bgl::tier_copy_wait(t);
    return BGL_OK;
}

}  // namespace

namespace {

// First half of a tiered lookup: the map lookup and the lists (and, unless one pass will write the whole
// output, the hit gather) are enqueued, the host waits for the lists and its threads start packing rows.
int tiered_begin(bgl_cache_t *c, bgl_host_tier_t *t, const int32_t *ids, int64_t n, void *out_rows,
                 int32_t *out_slot, int32_t *miss_pos, void *main_stream, void *side_stream, void *lookup_stream,
                 int early_lookup)
{
    int rc = check_lookup_args(c, ids, n, out_rows, out_slot, miss_pos);
    if (rc != BGL_OK) return rc;
    if (!t) BGL_FAIL(BGL_EINVAL, "tier handle is null");
    if (bgl::tier_row_bytes(t) != c->row_bytes || bgl::tier_num_nodes(t) != c->num_nodes)
        BGL_FAIL(BGL_EINVAL, "cache and host tier differ in row_bytes or num_nodes");
    if (n > bgl::tier_max_batch(t))
        BGL_FAIL(BGL_ECAPACITY, "n = %lld exceeds the tier's max_batch_rows", (long long)n);
    hipStream_t ms = static_cast<hipStream_t>(main_stream);
    hipStream_t ss = nullptr;
    rc = side_stream_of(c, side_stream, &ss);
    if (rc != BGL_OK) return rc;
    // Early lookup: only in write-through mode (otherwise the previous call's row copy still reads
    // the caller's miss_pos).
    hipStream_t ls = ms;
    if (early_lookup && static_cast<hipStream_t>(lookup_stream) != ms) {
        if (!c->write_through) BGL_FAIL(BGL_EINVAL, "early_lookup needs write-through mode");
        ls = static_cast<hipStream_t>(lookup_stream);
    }
    const int32_t *mpos = nullptr;
    int gen = 0;
    // One pass that writes the whole output (k_assemble_rows) instead of a hit gather now and a scatter of
    // the landed miss rows later: when the tier was asked for it, keeps nothing (its packed rows are then
    // in miss order), lands them in device memory, and the cache is in write-through mode.
    const bool assemble = bgl::tier_assemble(t) && bgl::tier_capacity(t) == 0 && c->write_through &&
                          bgl::tier_landing(t, (int)(c->lookup_calls & 1)) != nullptr;
    const int32_t *src_of = nullptr;
    rc = lookup_phase(c, ids, n, out_rows, out_slot, miss_pos, bgl::tier_count_device(t), ms, ls, t, &mpos, &gen,
                      nullptr, assemble ? &src_of : nullptr);
    if (rc != BGL_OK) return rc;
    BGL_HIP(hipGetLastError());
    struct Guard {  // whatever goes wrong below, the copy threads are released and the batch is dropped
        bgl_host_tier *t;
        bool armed = true;
        ~Guard() { if (armed) bgl::tier_abort(t); }
    } guard{t};
    // the host continues as soon as the lists are there; the hit gather runs meanwhile
    BGL_HIP(hipEventSynchronize(c->ev_ids));
    bgl_cache::TieredCall &tc = c->tiered;
    rc = bgl::tier_begin(t, n, &tc.plan);
    if (rc != BGL_OK) return rc;
    // (Waking the copy threads earlier, to have them spin until the ids arrive, was measured:
    // slower, the spinning threads get in the way of the wait for the lookup.)
    if (ss != ms) BGL_HIP(hipStreamWaitEvent(ss, c->ev_listed, 0));
    if (tc.plan.n_hit + tc.plan.n_miss > 0) {
        rc = bgl::tier_copy_start(t);  // host threads start packing
        if (rc != BGL_OK) return rc;
    }
    guard.armed = false;
    tc.active = true;
    tc.t = t;
    tc.ms = ms;
    tc.ss = ss;
    tc.ls = ls;
    tc.ids = ids;
    tc.mpos = mpos;
    tc.src_of = src_of;
    tc.miss_pos = miss_pos;
    tc.out_rows = out_rows;
    tc.n = n;
    tc.par = (int)(c->insert_calls & 1);  // (the map update of this batch may be enqueued before the second half)
    tc.gen = gen;
    if (c->write_through) {
        c->awaiting_insert = true;
        c->wt_ids = ids;
        c->wt_miss_pos = miss_pos;
    }
    return BGL_OK;
}

// Second half: the packed rows go on their way as the host threads finish them, and the kernels that take
// them to their places are enqueued.  Returns when the last row is packed and everything is enqueued.
int tiered_finish(bgl_cache_t *c, int64_t *n_hit)
{
    bgl_cache::TieredCall &tc = c->tiered;
    bgl_host_tier *t = tc.t;
    tc.active = false;
    struct Guard {
        bgl_host_tier *t;
        bool armed = true;
        ~Guard() { if (armed) bgl::tier_abort(t); }
    } guard{t};
    const bgl::TierPlan &plan = tc.plan;
    const TieredRows rows{c, t, &plan, tc.ss, tc.mpos, tc.out_rows, tc.n, tc.par, tc.ls != tc.ms, tc.src_of};
    int rc;
    if (plan.n_hit + plan.n_miss > 0) {
        char *land = bgl::tier_landing(t, tc.gen);  // device memory the copy engine fills, if that transport is on
        rc = land ? rows_by_copy_engine(rows, land) : rows_by_kernels(rows);
        if (rc != BGL_OK) return rc;
    } else if (tc.src_of && tc.n > 0) {
        rows.launch_assemble_rows(nullptr);  // every id hit: the pass only gathers (no landed row is read)
    }
    BGL_HIP(hipEventRecord(c->ev_miss, tc.ss));
    // the tier's map changes after this call's lists are final and before the next lookup,
    // which runs on the lookup stream
    rc = bgl::tier_enqueue_update(t, tc.ids, tc.miss_pos, tc.ls);
    if (rc != BGL_OK) return rc;
    guard.armed = false;
    BGL_HIP(hipGetLastError());
    c->fetch_pending = true;
    c->fetch_stream = tc.ss;
    c->fetch_reads_caller_lists = tc.mpos == tc.miss_pos;
    if (n_hit) {
        n_hit[0] = plan.n_hit_gpu;
        n_hit[1] = plan.n_hit;
    }
    return BGL_OK;
}

}  // namespace

extern "C" int bgl_cache_lookup_gather_tiered(bgl_cache_t *c, bgl_host_tier_t *t, const int32_t *ids,
                                              int64_t n, void *out_rows, int32_t *out_slot,
                                              int32_t *miss_pos, int64_t *n_hit, void *main_stream,
                                              void *side_stream, void *lookup_stream, int early_lookup)
try {
    const int rc = tiered_begin(c, t, ids, n, out_rows, out_slot, miss_pos, main_stream, side_stream, lookup_stream,
                                early_lookup);
    if (rc != BGL_OK) return rc;
    return tiered_finish(c, n_hit);
} BGL_NOTHROW_END

extern "C" int bgl_cache_lookup_tiered_begin(bgl_cache_t *c, bgl_host_tier_t *t, const int32_t *ids, int64_t n,
                                             void *out_rows, int32_t *out_slot, int32_t *miss_pos,
                                             int64_t *n_hit, void *main_stream, void *side_stream,
                                             void *lookup_stream, int early_lookup)
try {
    const int rc = tiered_begin(c, t, ids, n, out_rows, out_slot, miss_pos, main_stream, side_stream, lookup_stream,
                                early_lookup);
    if (rc != BGL_OK) return rc;
    if (n_hit) {  // known already: the lists are on the host
        n_hit[0] = c->tiered.plan.n_hit_gpu;
        n_hit[1] = c->tiered.plan.n_hit;
    }
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_lookup_tiered_finish(bgl_cache_t *c)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (!c->tiered.active) BGL_FAIL(BGL_EINVAL, "no tiered lookup has been begun");
    return tiered_finish(c, nullptr);
} BGL_NOTHROW_END

extern "C" int bgl_cache_insert_fifo(bgl_cache_t *c, const int32_t *ids, const int32_t *miss_pos,
                                     int64_t n_miss, const void *out_rows, void *stream)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (n_miss < -1 || n_miss > INT32_MAX) BGL_FAIL(BGL_EINVAL, "n_miss out of range");
    const int64_t bound = n_miss >= 0 ? n_miss : c->last_n;  // launch size
    if (bound > 0 && (!ids || !miss_pos || !out_rows))
        BGL_FAIL(BGL_EINVAL, "ids, miss_pos and out_rows must not be null");
    if (!bgl::aligned(out_rows, 16)) BGL_FAIL(BGL_EINVAL, "out_rows is not 16-byte aligned");
    if (c->tiered.active && !c->write_through)
        BGL_FAIL(BGL_EINVAL, "a tiered lookup has been begun: without write-through mode the FIFO update copies "
                             "rows that bgl_cache_lookup_tiered_finish has yet to bring in");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int q = c->row_bytes / 16;
    const int64_t eff = std::min<int64_t>(bound, c->capacity);
    const int par = (int)(c->insert_calls & 1);
    const bool other_stream = st != c->last_main;
    if (other_stream && c->ev_listed_valid) BGL_HIP(hipStreamWaitEvent(st, c->ev_listed, 0));  // the lookup's lists
    if (c->write_through) {
        // the rows are already on their way into the buffer: only the map changes here,
        // and nothing has to wait for the miss fetch
        if (!c->awaiting_insert || n_miss != -1 || ids != c->wt_ids || miss_pos != c->wt_miss_pos)
            BGL_FAIL(BGL_EINVAL, "write-through mode: insert_fifo must follow its lookup_gather with the same "
                                 "ids and miss_pos and n_miss = -1");
        c->awaiting_insert = false;
        if (eff > 0) {
            Prof p(c, BGL_STAGE_INSERT_MAP, st);
            launch(c, st, k_insert_map, dim3((unsigned)bgl::ceil_div(eff * BUCKET, COPY_THREADS)),
                   dim3(COPY_THREADS), ids, miss_pos, n_miss, c->capacity, c->num_nodes, c->table,
                   c->num_buckets - 1, c->slot_to_node, c->slot_to_entry, c->dev, par, 1);
        } else {
            hipLaunchKernelGGL(k_advance_tail, dim3(1), dim3(64), 0, st, c->dev, n_miss, par);
        }
        c->insert_calls += 1;
        BGL_HIP(hipGetLastError());
        // (recorded on every stream: the next lookup may run on another one than this call's lookup did)
        BGL_HIP(hipEventRecord(c->ev_map, st));
        c->map_pending = true;
        c->map_stream = st;
        return BGL_OK;
    }
    if (eff > 0) {
        {
            Prof p(c, BGL_STAGE_INSERT_MAP, st);
            launch(c, st, k_insert_map, dim3((unsigned)bgl::ceil_div(eff * BUCKET, COPY_THREADS)),
                   dim3(COPY_THREADS), ids, miss_pos, n_miss, c->capacity, c->num_nodes, c->table,
                   c->num_buckets - 1, c->slot_to_node, c->slot_to_entry, c->dev, par, 0);
        }
        if (c->fetch_pending && c->fetch_stream != st)
            BGL_HIP(hipStreamWaitEvent(st, c->ev_miss, 0));  // rows of the misses
        {
            Prof p(c, BGL_STAGE_INSERT_ROWS, st);
            dispatch_q(q, [&](auto Q) {
                launch(c, st, k_insert_rows<decltype(Q)::value>, dim3(copy_blocks(eff, q)), dim3(COPY_THREADS),
                       miss_pos, n_miss, c->capacity, c->rows, q, reinterpret_cast<const uint4 *>(out_rows),
                       reinterpret_cast<uint4 *>(c->buffer), c->dev, par);
            });
        }
    } else {
        if (c->fetch_pending && c->fetch_stream != st) BGL_HIP(hipStreamWaitEvent(st, c->ev_miss, 0));
        hipLaunchKernelGGL(k_advance_tail, dim3(1), dim3(64), 0, st, c->dev, n_miss, par);
    }
    c->insert_calls += 1;
    BGL_HIP(hipGetLastError());
    BGL_HIP(hipEventRecord(c->ev_map, st));
    c->map_pending = true;
    c->map_stream = st;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_set_spare_rows(bgl_cache_t *c, int64_t spare_rows)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (spare_rows < 0 || c->capacity + spare_rows > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "spare_rows must be >= 0 and capacity + spare_rows < 2^31 (got %lld)", (long long)spare_rows);
    if (c->insert_calls != 0 || c->awaiting_insert || c->tiered.active)
        BGL_FAIL(BGL_EINVAL, "the spare rows can only be set before the first insertion");
    BGL_HIP(hipDeviceSynchronize());
    const int64_t rows = c->capacity + spare_rows;
    if (rows == c->rows) return BGL_OK;
    char *buf = nullptr;
    const hipError_t e = hipMalloc((void **)&buf, (size_t)rows * c->row_bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        bgl::set_error("hipMalloc of %zu bytes failed: %s", (size_t)rows * c->row_bytes, hipGetErrorString(e));
        return e == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP;
    }
    if (hipMemset(buf, 0, (size_t)rows * c->row_bytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        (void)hipFree(buf);
        BGL_FAIL(BGL_EHIP, "clearing the cache buffer failed: %s", hipGetErrorString(hipGetLastError()));
    }
    (void)hipFree(c->buffer);
    c->buffer = buf;
    c->rows = rows;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_set_write_through(bgl_cache_t *c, int enable)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (c->awaiting_insert) BGL_FAIL(BGL_EINVAL, "a lookup's misses are still waiting for their insert_fifo");
    if (c->tiered.active) BGL_FAIL(BGL_EINVAL, "a tiered lookup has been begun: bgl_cache_lookup_tiered_finish comes first");
    c->write_through = enable != 0;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_wait_rows(bgl_cache_t *c, void *stream)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (c->fetch_pending && c->fetch_stream != st) BGL_HIP(hipStreamWaitEvent(st, c->ev_miss, 0));
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_wait_lists(bgl_cache_t *c, void *stream)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (c->ev_listed_valid && st != c->last_main)
        BGL_HIP(hipStreamWaitEvent(st, c->ev_listed, 0));
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_export_state(bgl_cache_t *c, int32_t *slot_to_node, uint64_t *tail,
                                      void *buffer)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    BGL_HIP(hipDeviceSynchronize());
    if (slot_to_node)
        BGL_HIP(hipMemcpy(slot_to_node, c->slot_to_node, sizeof(int32_t) * (size_t)c->capacity,
                          hipMemcpyDeviceToHost));
    if (tail) {
        CacheDev h;
        BGL_HIP(hipMemcpy(&h, c->dev, sizeof(h), hipMemcpyDeviceToHost));
        *tail = h.tail[c->insert_calls & 1];
    }
    if (buffer) {
        // rows by slot: the live rows are the last min(tail, capacity) insertions, insertion k sits at
        // position k mod rows and belongs to slot k mod capacity; runs of consecutive insertions are
        // copied whole (they break where either number wraps), empty slots read as zeros
        CacheDev h;
        BGL_HIP(hipMemcpy(&h, c->dev, sizeof(h), hipMemcpyDeviceToHost));
        const uint64_t t = h.tail[c->insert_calls & 1];
        const uint64_t cap = (uint64_t)c->capacity, rows = (uint64_t)c->rows, rb = (uint64_t)c->row_bytes;
        const uint64_t live = std::min<uint64_t>(t, cap);
        char *dst = static_cast<char *>(buffer);
        if (live < cap) std::memset(dst + live * rb, 0, (size_t)((cap - live) * rb));  // (then t < capacity: slots 0 .. t-1 are live)
        for (uint64_t k = t - live; k < t;) {
            const uint64_t slot = k % cap, pos = k % rows;
            const uint64_t run = std::min<uint64_t>(std::min<uint64_t>(cap - slot, rows - pos), t - k);
            BGL_HIP(hipMemcpy(dst + slot * rb, c->buffer + pos * rb, (size_t)(run * rb), hipMemcpyDeviceToHost));
            k += run;
        }
    }
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_stats(bgl_cache_t *c, uint64_t *lookups, uint64_t *hits, uint64_t *inserts,
                               uint64_t *evictions, int32_t *status)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    BGL_HIP(hipDeviceSynchronize());
    CacheDev h;
    BGL_HIP(hipMemcpy(&h, c->dev, sizeof(h), hipMemcpyDeviceToHost));
    if (lookups) *lookups = h.lookups;
    if (hits) *hits = h.hits;
    const uint64_t tail = h.tail[c->insert_calls & 1];
    if (inserts) *inserts = tail;  // every insertion advances tail by one
    // every insertion beyond the first `capacity` ones overwrote an occupied slot
    if (evictions) *evictions = tail > (uint64_t)c->capacity ? tail - (uint64_t)c->capacity : 0;
    if (status) *status = h.status;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_map_stats(bgl_cache_t *c, uint64_t *ids_looked_up, uint64_t *bucket_lines_read,
                                   uint64_t *num_buckets, uint64_t *buckets_passed, uint64_t *passes)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    BGL_HIP(hipDeviceSynchronize());
    CacheDev h;
    if (buckets_passed || passes) {
        BGL_HIP(hipMemset(&c->dev->census[0], 0, sizeof(h.census)));
        hipLaunchKernelGGL(k_map_census, dim3(256), dim3(256), 0, 0, c->table, c->num_buckets, c->dev);
        BGL_HIP(hipGetLastError());
        BGL_HIP(hipDeviceSynchronize());
    }
    BGL_HIP(hipMemcpy(&h, c->dev, sizeof(h), hipMemcpyDeviceToHost));
    if (ids_looked_up) *ids_looked_up = h.lookups;
    if (bucket_lines_read) *bucket_lines_read = h.probe_lines;
    if (num_buckets) *num_buckets = c->num_buckets;
    if (buckets_passed) *buckets_passed = h.census[0];
    if (passes) *passes = h.census[1];
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_set_profiling(bgl_cache_t *c, int enable)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    BGL_HIP(hipDeviceSynchronize());
    if (enable && c->prof_ev.empty()) {
        c->prof_ev.resize(2 * PROF_RING, nullptr);
        for (auto &ev : c->prof_ev) BGL_HIP(hipEventCreate(&ev));
    }
    c->prof_rec.clear();
    c->prof_rec.reserve(PROF_RING);
    c->prof_dropped = 0;
    for (int s = 0; s < BGL_NUM_STAGES; ++s) { c->prof_ms[s] = 0; c->prof_n[s] = 0; }
    c->profiling = (unsigned)enable;
    if (enable) {
        // What an event pair reads for a kernel that does nothing:
        // the launch gap that every bracketed stage time includes.
        double sum = 0;
        const int reps = 16;
        for (int r = 0; r < reps + 2; ++r) {
            BGL_HIP(hipEventRecord(c->prof_ev[0], 0));
            hipLaunchKernelGGL(k_noop, dim3(1), dim3(64), 0, 0);
            BGL_HIP(hipEventRecord(c->prof_ev[1], 0));
            BGL_HIP(hipEventSynchronize(c->prof_ev[1]));
            float ms = 0.f;
            BGL_HIP(hipEventElapsedTime(&ms, c->prof_ev[0], c->prof_ev[1]));
            if (r >= 2) sum += ms;
        }
        c->prof_overhead_ms = sum / reps;
    }
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_set_profiling_every(bgl_cache_t *c, int stage, int every)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (stage < 0 || stage >= BGL_NUM_STAGES) BGL_FAIL(BGL_EINVAL, "unknown stage %d", stage);
    if (every < 1) BGL_FAIL(BGL_EINVAL, "every must be >= 1 (got %d)", every);
    c->prof_every[stage] = every;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_cache_profile(bgl_cache_t *c, int stage, double *total_ms, int64_t *launches)
try {
    if (!c) BGL_FAIL(BGL_EINVAL, "cache handle is null");
    if (stage == BGL_STAGE_EVENT_OVERHEAD) {
        if (total_ms) *total_ms = c->prof_overhead_ms;
        if (launches) *launches = 1;
        return BGL_OK;
    }
    if (stage < 0 || stage >= BGL_NUM_STAGES) BGL_FAIL(BGL_EINVAL, "unknown stage %d", stage);
    BGL_HIP(hipDeviceSynchronize());
    drain_profile(c);
    if (c->prof_dropped > 0)
        BGL_FAIL(BGL_ENOMEM, "%lld timed launches could not get events; the stage totals are incomplete",
                 (long long)c->prof_dropped);
    if (total_ms) *total_ms = c->prof_ms[stage];
    if (launches) *launches = c->prof_n[stage];
    return BGL_OK;
} BGL_NOTHROW_END
