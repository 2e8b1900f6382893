// Second cache level in host memory (BGL paper, Sec. 3.2.3: the CPU cache behind
// the GPU cache uses the same policy as the GPU cache, i.e. FIFO; the misses of
// both levels come from the feature store, the graph store servers' stand-in).
//
// Only the tier's ROWS live in host memory (page-locked).  Its bookkeeping lives
// in HBM, where random access is cheap: node ids are dense, so the map is a
// plain array node -> row position (4 bytes per node), looked up by a kernel
// for the GPU cache's misses right behind that cache's own lookup; the same kernels list the rows the tier holds and the ids
// it does not.  The host only feeds rows, always packed, because rows that are
// not multiples of 128 bytes cross the link a quarter faster packed than read in
// place: its threads copy the rows the tier holds into staging rows, in list
// order, and the missing rows from the store into the positions first-in
// first-out assigns (consecutive), and the calling thread sends each chunk on
// as soon as its rows are in place: a plain copy into device memory on the copy
// stream (the copy-engine transport), or a fetch kernel that reads the chunk
// over the link.
//
// Rows sit in a ring of capacity_rows + 2 * max_batch_rows positions, filled in
// insertion order.  The newest capacity_rows insertions are the tier's content
// (logical slot = insertion number mod capacity_rows, as in the GPU cache); a
// row's position is reused only after capacity_rows + 2 * max_batch_rows further
// insertions, so a row found by a batch's lookup is still intact after that
// batch's and the next batch's insertions (which an early lookup brings in while
// this batch is still being fetched) have evicted it, and no copy ever has to
// wait for a fetch.  A tier that keeps nothing (capacity 0) is just the ring:
// rows pass through, packed, on their way over the link.
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "bgl_host_tier.h"
#include "bgl_internal.h"
#include "bgl_pool.h"

namespace {

constexpr int TT = 256;            // lookups per workgroup
constexpr int64_t COPY_TASK = 128;  // rows per host task

using namespace bgl;

__global__ void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// Map lookup for the GPU cache's misses: rank r (r-th entry of miss_pos) -> row
// position in the ring or -1; per-workgroup count of the -1s.
__global__ __launch_bounds__(TT) void k_tier_probe(const int32_t *__restrict__ ids,
                                                   const int32_t *__restrict__ miss_pos,
                                                   const long long *__restrict__ n_ranks,
                                                   int64_t num_nodes, const int32_t *__restrict__ node_pos,
                                                   int32_t *rank_pos, int32_t *tile_miss, int64_t *counts_host)
{
    __shared__ int sh[TT / kWave];
    const int64_t m = *n_ranks;
    if ((int64_t)blockIdx.x * TT >= m) return;
    const int64_t r = (int64_t)blockIdx.x * TT + threadIdx.x;
    int p = -1;
    if (r < m) {
        const int32_t id = ids[miss_pos[r]];
        if (id < 0 || (int64_t)id >= num_nodes) counts_host[3] = 1;  // the host refuses the batch
        else if (node_pos) p = node_pos[id];
        rank_pos[r] = p;
    }
    const uint64_t missed = __ballot(r < m && p < 0);
    if ((threadIdx.x & (kWave - 1)) == 0) sh[threadIdx.x / kWave] = __popcll(missed);
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < TT / kWave; ++k) t += sh[k];
        tile_miss[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(kScanThreads) void k_tier_scan_tiles(const long long *__restrict__ n_ranks,
                                                                  const int32_t *tile_miss, int32_t *prefix)
{
    __shared__ int sh[kScanThreads / kWave];
    scan_tile_counts<kScanThreads>(tile_miss, (*n_ranks + TT - 1) / TT, prefix, sh);
}

// Ordered lists: ranks the tier holds, ranks it does not; the ring positions of
// the former and the node ids of the latter go to page-locked host memory for
// the copy threads.  The last workgroup publishes both counts to the host.
__global__ __launch_bounds__(TT) void k_tier_lists(const int32_t *__restrict__ ids,
                                                   const int32_t *__restrict__ miss_pos,
                                                   const long long *__restrict__ n_ranks,
                                                   const int32_t *__restrict__ rank_pos,
                                                   const int32_t *__restrict__ tile_miss,
                                                   const int32_t *__restrict__ tile_prefix,
                                                   int32_t *hit_rank, int32_t *hit_pos_host, int32_t *miss_rank,
                                                   int32_t *miss_ids_host, int64_t *counts_host)
{
    __shared__ int sh_scan[TT / kWave];
    __shared__ int sh_base;
    const int64_t m = *n_ranks;
    const int64_t tiles = (m + TT - 1) / TT;
    if ((int64_t)blockIdx.x >= tiles) {
        if (m == 0 && blockIdx.x == 0 && threadIdx.x == 0) { counts_host[1] = 0; counts_host[2] = 0; }
        return;
    }
    int tot;
    if (tile_prefix) {  // calls of many tiles: k_tier_scan_tiles has summed the counts
        if (threadIdx.x == 0) sh_base = tile_prefix[blockIdx.x];
    } else {
        int part = 0;
        for (int t = threadIdx.x; t < (int)blockIdx.x; t += TT) part += tile_miss[t];
        (void)block_excl_scan<TT>(part, sh_scan, tot);
        if (threadIdx.x == 0) sh_base = tot;
    }
    const int64_t r = (int64_t)blockIdx.x * TT + threadIdx.x;
    const int p = r < m ? rank_pos[r] : 0;
    const int flag = (r < m && p < 0) ? 1 : 0;
    const int ex = block_excl_scan<TT>(flag, sh_scan, tot);  // its barriers publish sh_base
    const int j = sh_base + ex;
    if (flag) {
        miss_rank[j] = (int32_t)r;
        miss_ids_host[j] = ids[miss_pos[r]];
    } else if (r < m) {
        hit_rank[r - j] = (int32_t)r;
        hit_pos_host[r - j] = p;
    }
    if ((int64_t)blockIdx.x == tiles - 1 && threadIdx.x == 0) {
        const long long n_miss = sh_base + tot;
        counts_host[1] = m - n_miss;
        counts_host[2] = n_miss;
    }
}

// First-in first-out update of the bookkeeping: miss j >= start takes logical
// slot (tail + j) mod capacity and ring position (ptail + j) mod ring; the
// slot's former occupant leaves the map.  The ids of a batch are distinct and an
// occupant is never one of them, so no two lanes write the same entry.
__global__ __launch_bounds__(TT) void k_tier_update(const int32_t *__restrict__ ids,
                                                    const int32_t *__restrict__ miss_pos,
                                                    const int32_t *__restrict__ miss_rank, int64_t start,
                                                    int64_t n_miss, unsigned long long tail,
                                                    unsigned long long ptail, int64_t capacity, int64_t ring,
                                                    int32_t *node_pos, int32_t *slot_node, int32_t *slot_pos)
{
    const int64_t j = start + (int64_t)blockIdx.x * TT + threadIdx.x;
    if (j >= n_miss) return;
    const int32_t id = ids[miss_pos[miss_rank[j]]];
    const int64_t s = (int64_t)((tail + (unsigned long long)j) % (unsigned long long)capacity);
    const int32_t pp = (int32_t)((ptail + (unsigned long long)j) % (unsigned long long)ring);
    const int32_t old = slot_node[s];
    if (old >= 0) node_pos[old] = -1;
    slot_node[s] = id;
    slot_pos[s] = pp;
    node_pos[id] = pp;
}

}  // namespace

struct bgl_host_tier {
    const char *store = nullptr;  // num_nodes rows, ordinary host memory
    int64_t num_nodes = 0;
    int32_t row_bytes = 0;
    int64_t capacity = 0;   // logical slots
    int64_t max_batch = 0;
    int64_t ring = 0;       // row positions: capacity + 2 * max_batch
    int device = 0;
    char *rows = nullptr;   // page-locked, ring rows
    char *rows_dev = nullptr;
    char *pinned = nullptr;  // page-locked: counts[8] | miss ids[max_batch] | ring positions of the found rows[max_batch]
    char *stage = nullptr;   // page-locked: 2 x max_batch rows (one half per call parity): found rows, packed
    char *stage_dev = nullptr;
    char *pinned_dev = nullptr;
    // copy-engine transport: device memory the packed rows land in (one per call parity), its stream and event
    char *landing[2] = {nullptr, nullptr};
    bool assemble = false;     // copy-engine transport, mode 2: the cache writes its whole output in one pass
    hipStream_t copy_stream = nullptr;  // shared by all tiers of the process (not owned)
    hipEvent_t copy_event = nullptr;
    bool copy_event_recorded = false;
    // device: bookkeeping and per-batch lists
    int32_t *node_pos = nullptr, *slot_node = nullptr, *slot_pos = nullptr;
    int32_t *rank_pos = nullptr, *tile_miss = nullptr;
    // the lists a batch's fetch kernels read, alternating between calls: an early lookup writes the next
    // batch's while the previous batch's are still in use
    int32_t *hit_rank[2] = {nullptr, nullptr}, *miss_rank[2] = {nullptr, nullptr};
    int cur_gen = 0;
    uint64_t tail = 0;      // insertions so far (host mirrors of what the kernels are told)
    uint64_t ptail = 0;     // next ring position
    uint64_t lookups = 0, hits = 0;
    double copy_ms = 0;
    uint64_t batches = 0;
    // the batch being served
    int64_t cur_m = 0, cur_hit = 0, cur_miss = 0;
    bool serving = false;
    bgl::Pool *pool = nullptr;
    bgl::Pool::Fn copy_fn;
    bool copying = false;
    bool copy_timed = false;  // this batch's copy time has been added to copy_ms
    std::chrono::steady_clock::time_point copy_t0;

    volatile int64_t *counts() const { return reinterpret_cast<volatile int64_t *>(pinned); }
    const int32_t *miss_ids() const { return reinterpret_cast<const int32_t *>(pinned + 64); }
    const int32_t *hit_positions() const { return reinterpret_cast<const int32_t *>(pinned + 64 + 4 * (size_t)max_batch); }
};

namespace bgl {

int64_t *tier_count_device(bgl_host_tier *t) { return reinterpret_cast<int64_t *>(t->pinned_dev); }
const char *tier_rows_device(bgl_host_tier *t) { return t->rows_dev; }
int64_t tier_max_batch(const bgl_host_tier *t) { return t->max_batch; }
int64_t tier_capacity(const bgl_host_tier *t) { return t->capacity; }
int32_t *tier_ids_device_if_passthrough(bgl_host_tier *t)
{
    return t->capacity == 0 ? reinterpret_cast<int32_t *>(t->pinned_dev + 64) : nullptr;
}
int32_t tier_row_bytes(const bgl_host_tier *t) { return t->row_bytes; }
char *tier_landing(bgl_host_tier *t, int gen) { return t->landing[gen & 1]; }
bool tier_assemble(const bgl_host_tier *t) { return t->assemble; }
hipStream_t tier_copy_stream(bgl_host_tier *t) { return t->copy_stream; }
hipEvent_t tier_copy_event(bgl_host_tier *t) { return t->copy_event; }
bool tier_copy_event_recorded(const bgl_host_tier *t) { return t->copy_event_recorded; }
void tier_set_copy_event_recorded(bgl_host_tier *t) { t->copy_event_recorded = true; }
int64_t tier_num_nodes(const bgl_host_tier *t) { return t->num_nodes; }

int tier_enqueue_lookup(bgl_host_tier *t, const int32_t *ids, const int32_t *miss_pos,
                        const long long *n_ranks_dev, int64_t n_upper, int gen, hipStream_t st)
{
    if (t->serving) BGL_FAIL(BGL_EINVAL, "host tier: the previous batch has not been finished");
    if (n_upper > t->max_batch)
        BGL_FAIL(BGL_ECAPACITY, "%lld ids exceed the tier's max_batch_rows %lld", (long long)n_upper,
                 (long long)t->max_batch);
    t->cur_gen = gen & 1;
    if (t->capacity == 0) return BGL_OK;  // the cache's own list kernel has sent ids and counts (tier_prepare)
    if (n_upper == 0) {
        t->counts()[1] = 0;
        t->counts()[2] = 0;
        return BGL_OK;
    }
    const unsigned tiles = (unsigned)bgl::ceil_div(n_upper, TT);
    hipLaunchKernelGGL(k_tier_probe, dim3(tiles), dim3(TT), 0, st, ids, miss_pos, n_ranks_dev, t->num_nodes,
                       t->node_pos, t->rank_pos, t->tile_miss, reinterpret_cast<int64_t *>(t->pinned_dev));
    int32_t *tile_prefix = nullptr;
    if (tiles >= kSelfSumTiles) {
        tile_prefix = t->tile_miss + bgl::ceil_div(t->max_batch, TT) + 1;
        hipLaunchKernelGGL(k_tier_scan_tiles, dim3(1), dim3(kScanThreads), 0, st, n_ranks_dev, t->tile_miss,
                           tile_prefix);
    }
    hipLaunchKernelGGL(k_tier_lists, dim3(tiles), dim3(TT), 0, st, ids, miss_pos, n_ranks_dev, t->rank_pos,
                       t->tile_miss, tile_prefix, t->hit_rank[t->cur_gen],
                       reinterpret_cast<int32_t *>(t->pinned_dev + 64 + 4 * (size_t)t->max_batch),
                       t->miss_rank[t->cur_gen], reinterpret_cast<int32_t *>(t->pinned_dev + 64),
                       reinterpret_cast<int64_t *>(t->pinned_dev));
    BGL_HIP(hipGetLastError());
    return BGL_OK;
}

void tier_prepare(bgl_host_tier *t)
{
    // set by the lookup kernels when they meet an id outside [0, num_nodes)
    t->counts()[3] = 0;
    t->counts()[1] = 0;
    t->counts()[2] = 0;
}

int tier_begin(bgl_host_tier *t, int64_t n, TierPlan *plan)
{
    const int64_t n_hit_gpu = t->counts()[0];
    const int64_t m = n - n_hit_gpu;
    const int64_t n_hit = t->counts()[1], n_miss = t->counts()[2];
    if (n_hit_gpu < 0 || m < 0 || n_hit + n_miss != m)
        BGL_FAIL(BGL_EHIP, "host tier: inconsistent counts from the device (%lld, %lld, %lld of %lld)",
                 (long long)n_hit_gpu, (long long)n_hit, (long long)n_miss, (long long)n);
    if (t->counts()[3] != 0) BGL_FAIL(BGL_EINVAL, "host tier: node id outside [0, num_nodes)");
    t->cur_m = m;
    t->cur_hit = n_hit;
    t->cur_miss = n_miss;
    t->serving = true;
    plan->n_hit_gpu = n_hit_gpu;
    plan->n_hit = n_hit;
    plan->n_miss = n_miss;
    plan->hit_rank = t->hit_rank[t->cur_gen];
    plan->stage = t->stage_dev ? t->stage_dev + (size_t)t->cur_gen * (size_t)t->max_batch * (size_t)t->row_bytes
                               : nullptr;
    plan->miss_rank = t->capacity > 0 ? t->miss_rank[t->cur_gen] : nullptr;  // capacity 0: every rank, in order
    plan->ptail = t->ptail;
    plan->ring = t->ring;
    return BGL_OK;
}

int tier_copy_start(bgl_host_tier *t)
{
    if (!t->serving) BGL_FAIL(BGL_EINVAL, "host tier: no batch is being served");
    t->copy_t0 = std::chrono::steady_clock::now();
    // one sequence of rows: the found ones first (ring -> this call's half of the staging rows, packed in
    // list order), then the missing ones (store -> their ring positions, consecutive)
    t->copy_fn = [t](int64_t k) {
        const size_t rb = (size_t)t->row_bytes;
        const int32_t *mi = t->miss_ids();
        const int32_t *hp = t->hit_positions();
        char *stage = t->stage + (size_t)t->cur_gen * (size_t)t->max_batch * rb;
        const int64_t n_hit = t->cur_hit;
        const int64_t hi = std::min<int64_t>(n_hit + t->cur_miss, (k + 1) * COPY_TASK);
        // (asking for the scattered source rows a few rows ahead was measured: no faster, a dozen threads
        // already keep enough reads in flight; writing the packed rows with 16-byte streaming stores was
        // measured too: 20-80 % slower than the library's memcpy)
        for (int64_t x = k * COPY_TASK; x < hi; ++x) {
            if (x < n_hit) {
                std::memcpy(stage + (size_t)x * rb, t->rows + (size_t)hp[x] * rb, rb);
            } else {
                const int64_t j = x - n_hit;
                const uint64_t pp = (t->ptail + (uint64_t)j) % (uint64_t)t->ring;
                std::memcpy(t->rows + (size_t)pp * rb, t->store + (size_t)mi[j] * rb, rb);
            }
        }
    };
    t->copying = true;
    t->copy_timed = false;
    t->pool->start(bgl::ceil_div(t->cur_hit + t->cur_miss, COPY_TASK), t->copy_fn);
    return BGL_OK;
}

int64_t tier_copy_progress(bgl_host_tier *t)
{
    const int64_t total = t->cur_hit + t->cur_miss;
    const int64_t ready = std::min<int64_t>(total, t->pool->done_prefix() * COPY_TASK);
    if (ready == total && t->copying && !t->copy_timed) {  // the moment the calling thread sees the last row in place
        t->copy_timed = true;
        t->copy_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t->copy_t0).count();
    }
    return ready;
}

bool tier_copy_help(bgl_host_tier *t) { return t->copying && t->pool->help_one(); }

void tier_copy_wait(bgl_host_tier *t)
{
    if (!t->copying) return;
    t->pool->wait();
    (void)tier_copy_progress(t);
    t->copying = false;
}

int tier_enqueue_update(bgl_host_tier *t, const int32_t *ids, const int32_t *miss_pos, hipStream_t st)
{
    if (!t->serving) BGL_FAIL(BGL_EINVAL, "host tier: no batch is being served");
    const int64_t n_miss = t->cur_miss;
    const int64_t start = n_miss > t->capacity ? n_miss - t->capacity : 0;
    if (n_miss > start) {  // never with capacity 0
        hipLaunchKernelGGL(k_tier_update, dim3((unsigned)bgl::ceil_div(n_miss - start, TT)), dim3(TT), 0, st, ids,
                           miss_pos, t->miss_rank[t->cur_gen], start, n_miss, (unsigned long long)t->tail,
                           (unsigned long long)t->ptail, t->capacity, t->ring, t->node_pos, t->slot_node,
                           t->slot_pos);
        BGL_HIP(hipGetLastError());
    }
    t->tail += (uint64_t)n_miss;
    t->ptail = (t->ptail + (uint64_t)n_miss) % (uint64_t)t->ring;
    t->lookups += (uint64_t)t->cur_m;
    t->hits += (uint64_t)t->cur_hit;
    t->batches += 1;
    t->serving = false;
    return BGL_OK;
}

void tier_abort(bgl_host_tier *t)
{
    tier_copy_wait(t);  // copies already under way land in ring positions nothing refers to
    t->serving = false;
}

}  // namespace bgl

extern "C" int bgl_host_tier_create(const void *store, int64_t num_nodes, int32_t row_bytes,
                                    int64_t capacity_rows, int64_t max_batch_rows, int32_t num_threads,
                                    bgl_host_tier_t **out)
try {
    if (!out) BGL_FAIL(BGL_EINVAL, "out is null");
    *out = nullptr;
    if (!store) BGL_FAIL(BGL_EINVAL, "store is null");
    if (num_nodes < 1 || num_nodes > INT32_MAX) BGL_FAIL(BGL_EINVAL, "num_nodes out of range");
    if (row_bytes < 16 || row_bytes % 16 != 0)
        BGL_FAIL(BGL_EINVAL, "row_bytes must be a positive multiple of 16 (got %d)", row_bytes);
    if (capacity_rows < 0 || capacity_rows > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "capacity_rows must be in [0, 2^31) (got %lld)", (long long)capacity_rows);
    if (max_batch_rows < 1 || max_batch_rows > INT32_MAX / 2 || capacity_rows + 2 * max_batch_rows > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "max_batch_rows must be >= 1 and capacity_rows + 2 * max_batch_rows < 2^31 (got %lld)",
                 (long long)max_batch_rows);
    if (num_threads < 0 || num_threads > 256) BGL_FAIL(BGL_EINVAL, "num_threads must be in [0, 256]");
    if (num_threads == 0) {
        const unsigned hw = std::thread::hardware_concurrency();
        // Three quarters of the cores, 16 at most: measured with 9 to 15 threads on a 16-core share,
        // 9-12 pack a batch in time and leave the copies over the link 1 % faster than 15 do.
        num_threads = (int32_t)std::max<unsigned>(1, std::min<unsigned>(hw ? hw : 2, 16) * 3 / 4);
    }
    bgl_host_tier *t = new (std::nothrow) bgl_host_tier();
    if (!t) BGL_FAIL(BGL_ENOMEM, "out of host memory");
    t->store = static_cast<const char *>(store);
    t->num_nodes = num_nodes;
    t->row_bytes = row_bytes;
    t->capacity = capacity_rows;
    t->max_batch = max_batch_rows;
    // two batches of room beyond the content: the next batch may be brought in (early lookup) while the
    // previous one is still being fetched
    t->ring = capacity_rows + 2 * max_batch_rows;
    const size_t mb = (size_t)max_batch_rows;
    const size_t row_total = (size_t)t->ring * (size_t)row_bytes;
    auto fail = [&](int code) { bgl_host_tier_destroy(t); return code; };
    hipError_t e;
    if (hipGetDevice(&t->device) != hipSuccess) { bgl::set_error("hipGetDevice failed"); return fail(BGL_EHIP); }
    if ((e = hipHostMalloc((void **)&t->rows, row_total, hipHostMallocDefault)) != hipSuccess) {
        (void)hipGetLastError();
        t->rows = nullptr;
        bgl::set_error("page-locked allocation of %zu bytes failed: %s", row_total, hipGetErrorString(e));
        return fail(BGL_ENOMEM);
    }
    if ((e = hipHostMalloc((void **)&t->pinned, 64 + 8 * mb, hipHostMallocDefault)) != hipSuccess) {
        (void)hipGetLastError();
        t->pinned = nullptr;
        bgl::set_error("page-locked allocation of %zu bytes failed: %s", 64 + 8 * mb, hipGetErrorString(e));
        return fail(BGL_ENOMEM);
    }
    if (capacity_rows > 0) {  // a tier that keeps nothing never finds a row
        const size_t stage_total = 2 * mb * (size_t)row_bytes;
        if ((e = hipHostMalloc((void **)&t->stage, stage_total, hipHostMallocDefault)) != hipSuccess) {
            (void)hipGetLastError();
            t->stage = nullptr;
            bgl::set_error("page-locked allocation of %zu bytes failed: %s", stage_total, hipGetErrorString(e));
            return fail(BGL_ENOMEM);
        }
        if (hipHostGetDevicePointer((void **)&t->stage_dev, t->stage, 0) != hipSuccess) {
            bgl::set_error("hipHostGetDevicePointer failed");
            return fail(BGL_EHIP);
        }
    }
    if (hipHostGetDevicePointer((void **)&t->rows_dev, t->rows, 0) != hipSuccess ||
        hipHostGetDevicePointer((void **)&t->pinned_dev, t->pinned, 0) != hipSuccess) {
        bgl::set_error("hipHostGetDevicePointer failed");
        return fail(BGL_EHIP);
    }
    std::memset(t->pinned, 0, 64);
#define TRY_ALLOC(ptr, count)                                                                            \
    if ((e = hipMalloc((void **)&(ptr), sizeof(int32_t) * (size_t)(count))) != hipSuccess) {              \
        (void)hipGetLastError();                                                                         \
        (ptr) = nullptr;                                                                                 \
        bgl::set_error("hipMalloc of %zu bytes failed: %s", sizeof(int32_t) * (size_t)(count),           \
                       hipGetErrorString(e));                                                            \
        return fail(e == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP);                                   \
    }
    if (capacity_rows > 0) {  // capacity 0: nothing is kept, every row passes through the ring
        TRY_ALLOC(t->node_pos, num_nodes);
        TRY_ALLOC(t->slot_node, capacity_rows);
        TRY_ALLOC(t->slot_pos, capacity_rows);
    }
    TRY_ALLOC(t->rank_pos, mb);
    TRY_ALLOC(t->tile_miss, 2 * (bgl::ceil_div((int64_t)mb, TT) + 1));  // counts, then their prefixes
    for (int g = 0; g < 2; ++g) {
        TRY_ALLOC(t->hit_rank[g], mb);
        TRY_ALLOC(t->miss_rank[g], mb);
    }
#undef TRY_ALLOC
    if (capacity_rows > 0) {
        hipLaunchKernelGGL(k_fill_i32, dim3(2048), dim3(256), 0, 0, t->node_pos, num_nodes, -1);
        hipLaunchKernelGGL(k_fill_i32, dim3(1024), dim3(256), 0, 0, t->slot_node, capacity_rows, -1);
        hipLaunchKernelGGL(k_fill_i32, dim3(1024), dim3(256), 0, 0, t->slot_pos, capacity_rows, 0);
    }
    if (hipDeviceSynchronize() != hipSuccess) {
        bgl::set_error("tier initialisation failed: %s", hipGetErrorString(hipGetLastError()));
        return fail(BGL_EHIP);
    }
    try {
        t->pool = new bgl::Pool(num_threads);
    } catch (const std::exception &) {
        bgl::set_error("could not start the host threads");
        return fail(BGL_ENOMEM);
    }
    if (t->stage) {
        const size_t stage_total = 2 * mb * (size_t)row_bytes;
        t->pool->run((int64_t)bgl::ceil_div((int64_t)stage_total, 1 << 20), [&](int64_t k) {
            const size_t lo = (size_t)k << 20;
            std::memset(t->stage + lo, 0, std::min<size_t>((size_t)1 << 20, stage_total - lo));
        });
    }
    // touch every page of the ring now rather than inside the first batches' copies
    t->pool->run((int64_t)bgl::ceil_div((int64_t)row_total, 1 << 20), [&](int64_t k) {
        const size_t lo = (size_t)k << 20;
        std::memset(t->rows + lo, 0, std::min<size_t>((size_t)1 << 20, row_total - lo));
    });
    *out = t;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_host_tier_set_copy_engine(bgl_host_tier_t *t, int enable)
try {
    if (!t) BGL_FAIL(BGL_EINVAL, "tier handle is null");
    if (t->serving) BGL_FAIL(BGL_EINVAL, "host tier: a batch is being served");
    if (enable < 0 || enable > 2) BGL_FAIL(BGL_EINVAL, "the transport is 0, 1 or 2 (got %d)", enable);
    BGL_HIP(hipDeviceSynchronize());  // earlier batches may still use what this call changes
    t->assemble = enable == 2;
    if (!enable) {
        for (int g = 0; g < 2; ++g) {
            (void)hipFree(t->landing[g]);
            t->landing[g] = nullptr;
        }
        return BGL_OK;
    }
    if (t->landing[0]) return BGL_OK;
    if (!t->copy_stream) {
        // One copy stream per process, shared by all tiers and never destroyed: a process has only a
        // few hardware queues, and streams that map onto the same one run one after the other.
        static std::mutex guard;  // (tiers of different callers may get here at the same time)
        static hipStream_t shared_copy_stream = nullptr;
        std::lock_guard<std::mutex> lk(guard);
        if (!shared_copy_stream) BGL_HIP(hipStreamCreateWithFlags(&shared_copy_stream, hipStreamNonBlocking));
        t->copy_stream = shared_copy_stream;
    }
    if (!t->copy_event) BGL_HIP(hipEventCreateWithFlags(&t->copy_event, hipEventDisableTiming));
    const size_t bytes = (size_t)t->max_batch * (size_t)t->row_bytes;
    for (int g = 0; g < 2; ++g) {
        const hipError_t e = hipMalloc((void **)&t->landing[g], bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            t->landing[g] = nullptr;
            (void)hipFree(t->landing[0]);
            t->landing[0] = nullptr;
            bgl::set_error("hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
            return e == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP;
        }
    }
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_host_tier_destroy(bgl_host_tier_t *t)
try {
    if (!t) return BGL_OK;
    (void)hipDeviceSynchronize();  // kernels may still read the rows
    delete t->pool;
    (void)hipFree(t->landing[0]);
    (void)hipFree(t->landing[1]);
    if (t->copy_event) (void)hipEventDestroy(t->copy_event);
    if (t->rows) (void)hipHostFree(t->rows);
    if (t->pinned) (void)hipHostFree(t->pinned);
    if (t->stage) (void)hipHostFree(t->stage);
    (void)hipFree(t->node_pos);
    (void)hipFree(t->slot_node);
    (void)hipFree(t->slot_pos);
    (void)hipFree(t->rank_pos);
    (void)hipFree(t->tile_miss);
    for (int g = 0; g < 2; ++g) {
        (void)hipFree(t->hit_rank[g]);
        (void)hipFree(t->miss_rank[g]);
    }
    delete t;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_host_tier_export_state(bgl_host_tier_t *t, int32_t *slot_to_node, uint64_t *tail,
                                          void *buffer_rows)
try {
    if (!t) BGL_FAIL(BGL_EINVAL, "tier handle is null");
    BGL_HIP(hipDeviceSynchronize());
    std::vector<int32_t> node, pos;
    try {
        node.resize((size_t)t->capacity);
        pos.resize((size_t)t->capacity);
    } catch (const std::bad_alloc &) {
        BGL_FAIL(BGL_ENOMEM, "out of host memory");
    }
    if (t->capacity > 0) {
        BGL_HIP(hipMemcpy(node.data(), t->slot_node, sizeof(int32_t) * (size_t)t->capacity, hipMemcpyDeviceToHost));
        BGL_HIP(hipMemcpy(pos.data(), t->slot_pos, sizeof(int32_t) * (size_t)t->capacity, hipMemcpyDeviceToHost));
    }
    if (slot_to_node) std::memcpy(slot_to_node, node.data(), sizeof(int32_t) * (size_t)t->capacity);
    if (tail) *tail = t->tail;
    if (buffer_rows) {
        const size_t rb = (size_t)t->row_bytes;
        char *dst = static_cast<char *>(buffer_rows);
        for (int64_t s = 0; s < t->capacity; ++s) {
            if (node[(size_t)s] >= 0) std::memcpy(dst + (size_t)s * rb, t->rows + (size_t)pos[(size_t)s] * rb, rb);
            else std::memset(dst + (size_t)s * rb, 0, rb);
        }
    }
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_host_tier_stats(bgl_host_tier_t *t, uint64_t *lookups, uint64_t *hits, double *copy_ms,
                                   uint64_t *batches, int32_t *threads)
try {
    if (!t) BGL_FAIL(BGL_EINVAL, "tier handle is null");
    if (lookups) *lookups = t->lookups;
    if (hits) *hits = t->hits;
    if (copy_ms) *copy_ms = t->copy_ms;
    if (batches) *batches = t->batches;
    if (threads) *threads = t->pool->threads();
    return BGL_OK;
} BGL_NOTHROW_END
