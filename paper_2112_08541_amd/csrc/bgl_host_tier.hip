// Second cache level in host memory (BGL paper, Sec. 3.2.3: the CPU cache behind
// the GPU cache uses the same policy as the GPU cache, i.e. FIFO; the misses of
// both levels come from the feature store, the graph store servers' stand-in).
//
// Host code only.  The tier's rows live in page-locked memory that kernels read
// in place over the host link, so a row found here is never copied by the CPU; a
// row brought in from the store is copied once, into the slot FIFO assigns to it
// (or into a staging row when it does not enter the tier), and read from there.
// Node ids are dense, so the map is a plain array node -> slot (4 bytes per
// node of host memory).  The loops over a batch's ids run on a small pool of
// threads; a batch's ids are distinct, which makes every parallel loop here
// write disjoint entries.
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "bgl_host_tier.h"
#include "bgl_internal.h"

namespace {

// parallel_for over [0, n) in chunks; the caller works too and returns when all chunks are done.
class Pool {
public:
    explicit Pool(int threads)
    {
        for (int i = 1; i < threads; ++i) workers_.emplace_back([this] { loop(); });
    }
    ~Pool()
    {
        {
            std::lock_guard<std::mutex> lk(m_);
            stop_ = true;
        }
        cv_.notify_all();
        for (auto &t : workers_) t.join();
    }
    int threads() const { return (int)workers_.size() + 1; }

    void run(int64_t n, int64_t chunk, const std::function<void(int64_t, int64_t, int64_t)> &fn)
    {
        if (n <= 0) return;
        const int64_t chunks = (n + chunk - 1) / chunk;
        if (chunks == 1 || workers_.empty()) {
            for (int64_t k = 0; k < chunks; ++k) fn(k, k * chunk, std::min(n, (k + 1) * chunk));
            return;
        }
        {
            std::lock_guard<std::mutex> lk(m_);
            fn_ = &fn;
            n_ = n;
            chunk_ = chunk;
            chunks_ = chunks;
            next_.store(0);
            busy_ = (int)workers_.size();
            ++gen_;
        }
        cv_.notify_all();
        work();
        std::unique_lock<std::mutex> lk(m_);
        done_.wait(lk, [this] { return busy_ == 0; });
        fn_ = nullptr;
    }

private:
    void work()
    {
        for (;;) {
            const int64_t k = next_.fetch_add(1);
            if (k >= chunks_) return;
            (*fn_)(k, k * chunk_, std::min(n_, (k + 1) * chunk_));
        }
    }
    void loop()
    {
        uint64_t seen = 0;
        for (;;) {
            {
                std::unique_lock<std::mutex> lk(m_);
                cv_.wait(lk, [&] { return stop_ || gen_ != seen; });
                if (stop_) return;
                seen = gen_;
            }
            work();
            {
                std::lock_guard<std::mutex> lk(m_);
                if (--busy_ == 0) done_.notify_one();
            }
        }
    }

    std::vector<std::thread> workers_;
    std::mutex m_;
    std::condition_variable cv_, done_;
    const std::function<void(int64_t, int64_t, int64_t)> *fn_ = nullptr;
    int64_t n_ = 0, chunk_ = 1, chunks_ = 0;
    std::atomic<int64_t> next_{0};
    int busy_ = 0;
    uint64_t gen_ = 0;
    bool stop_ = false;
};

constexpr int64_t CHUNK = 2048;  // ids per task

}  // namespace

struct bgl_host_tier {
    const char *store = nullptr;  // num_nodes rows, ordinary host memory
    int64_t num_nodes = 0;
    int32_t row_bytes = 0;
    int64_t capacity = 0;
    int64_t max_batch = 0;
    // page-locked: capacity tier rows, then max_batch staging rows
    char *rows = nullptr;
    char *rows_dev = nullptr;
    // page-locked lists: ids | hit_rank | miss_rank | hit_src | miss_src | GPU hit count
    char *lists = nullptr;
    char *lists_dev = nullptr;
    int32_t *ids = nullptr, *hit_rank = nullptr, *miss_rank = nullptr;
    int64_t *hit_src = nullptr, *miss_src = nullptr;
    std::vector<int32_t> node_to_slot, slot_to_node, slot_rank;
    std::vector<uint32_t> slot_epoch;  // batch number of the last lookup that found the slot's row
    std::vector<int64_t> src_row;      // per rank, while a batch is being served
    std::vector<int64_t> chunk_hits;
    uint64_t tail = 0;
    uint32_t epoch = 0;
    uint64_t lookups = 0, hits = 0;
    std::atomic<uint64_t> kept_aside{0};  // found rows copied to staging before their slot was reused
    // between tier_lookup and tier_insert
    int64_t cur_m = 0, cur_hit = 0, cur_miss = 0;
    bool serving = false;
    Pool *pool = nullptr;
};

namespace bgl {

int32_t *tier_ids_device(bgl_host_tier *t) { return reinterpret_cast<int32_t *>(t->lists_dev); }
int64_t *tier_count_device(bgl_host_tier *t) { return reinterpret_cast<int64_t *>(t->lists_dev + 28 * (size_t)t->max_batch); }
const volatile int64_t *tier_count_host(bgl_host_tier *t) { return reinterpret_cast<const volatile int64_t *>(t->lists + 28 * (size_t)t->max_batch); }
const char *tier_rows_device(bgl_host_tier *t) { return t->rows_dev; }
int64_t tier_max_batch(const bgl_host_tier *t) { return t->max_batch; }
int32_t tier_row_bytes(const bgl_host_tier *t) { return t->row_bytes; }
int64_t tier_num_nodes(const bgl_host_tier *t) { return t->num_nodes; }

int tier_lookup(bgl_host_tier *t, int64_t m, TierPlan *plan)
{
    if (m < 0 || m > t->max_batch) BGL_FAIL(BGL_ECAPACITY, "%lld ids exceed the tier's max_batch_rows %lld",
                                            (long long)m, (long long)t->max_batch);
    if (t->serving) BGL_FAIL(BGL_EINVAL, "host tier: the previous batch has not been inserted");
    t->epoch += 1;
    if (t->epoch == 0) {  // wrapped: forget old marks
        std::fill(t->slot_epoch.begin(), t->slot_epoch.end(), 0u);
        t->epoch = 1;
    }
    const uint32_t epoch = t->epoch;
    const int64_t chunks = bgl::ceil_div(m, CHUNK);
    t->chunk_hits.assign((size_t)chunks + 1, 0);
    std::atomic<int> bad{0};
    // map lookup; a found slot remembers which rank found it
    t->pool->run(m, CHUNK, [&](int64_t k, int64_t lo, int64_t hi) {
        int64_t h = 0;
        for (int64_t r = lo; r < hi; ++r) {
            const int32_t id = t->ids[r];
            if (id < 0 || (int64_t)id >= t->num_nodes) { bad.store(1); t->src_row[r] = -1; continue; }
            const int32_t s = t->node_to_slot[id];
            t->src_row[r] = s;
            if (s >= 0) {
                t->slot_epoch[s] = epoch;
                t->slot_rank[s] = (int32_t)r;
                ++h;
            }
        }
        t->chunk_hits[(size_t)k] = h;
    });
    if (bad.load()) BGL_FAIL(BGL_EINVAL, "host tier: node id outside [0, num_nodes)");
    int64_t n_hit = 0;
    for (int64_t k = 0; k < chunks; ++k) {
        const int64_t h = t->chunk_hits[(size_t)k];
        t->chunk_hits[(size_t)k] = n_hit;
        n_hit += h;
    }
    const int64_t n_miss = m - n_hit;
    // Rows found now whose slot this batch's insertions will reuse: keep a copy in the
    // staging row of their rank, so the copy from the store may overwrite the slot at once.
    const int64_t start = n_miss > t->capacity ? n_miss - t->capacity : 0;
    const size_t rb = (size_t)t->row_bytes;
    t->pool->run(n_miss - start, CHUNK, [&](int64_t, int64_t lo, int64_t hi) {
        for (int64_t j = start + lo; j < start + hi; ++j) {
            const int64_t s = (int64_t)((t->tail + (uint64_t)j) % (uint64_t)t->capacity);
            if (t->slot_epoch[(size_t)s] == epoch) {
                const int64_t r = t->slot_rank[(size_t)s];
                std::memcpy(t->rows + (size_t)(t->capacity + r) * rb, t->rows + (size_t)s * rb, rb);
                t->src_row[(size_t)r] = t->capacity + r;
                t->kept_aside.fetch_add(1, std::memory_order_relaxed);
            }
        }
    });
    // ordered lists of both kinds
    t->pool->run(m, CHUNK, [&](int64_t k, int64_t lo, int64_t hi) {
        int64_t h = t->chunk_hits[(size_t)k];
        int64_t ms = lo - h;
        for (int64_t r = lo; r < hi; ++r) {
            const int64_t s = t->src_row[(size_t)r];
            if (s >= 0) {
                t->hit_rank[h] = (int32_t)r;
                t->hit_src[h] = s;
                ++h;
            } else {
                t->miss_rank[ms++] = (int32_t)r;
            }
        }
    });
    t->cur_m = m;
    t->cur_hit = n_hit;
    t->cur_miss = n_miss;
    t->serving = true;
    const size_t mb = (size_t)t->max_batch;
    plan->hit_rank = reinterpret_cast<const int32_t *>(t->lists_dev + 4 * mb);
    plan->miss_rank = reinterpret_cast<const int32_t *>(t->lists_dev + 8 * mb);
    plan->hit_src = reinterpret_cast<const int64_t *>(t->lists_dev + 12 * mb);
    plan->miss_src = reinterpret_cast<const int64_t *>(t->lists_dev + 20 * mb);
    plan->n_hit = n_hit;
    plan->n_miss = n_miss;
    return BGL_OK;
}

int tier_insert(bgl_host_tier *t)
{
    if (!t->serving) BGL_FAIL(BGL_EINVAL, "host tier: no batch is being served");
    const int64_t n_miss = t->cur_miss;
    const int64_t start = n_miss > t->capacity ? n_miss - t->capacity : 0;
    const size_t rb = (size_t)t->row_bytes;
    t->pool->run(n_miss, CHUNK / 4, [&](int64_t, int64_t lo, int64_t hi) {
        for (int64_t j = lo; j < hi; ++j) {
            const int64_t r = t->miss_rank[j];
            const int32_t id = t->ids[r];
            const char *src = t->store + (size_t)id * rb;
            if (j < start) {  // more misses than slots: the early ones pass through staging only
                std::memcpy(t->rows + (size_t)(t->capacity + r) * rb, src, rb);
                t->miss_src[j] = t->capacity + r;
                continue;
            }
            const int64_t s = (int64_t)((t->tail + (uint64_t)j) % (uint64_t)t->capacity);
            const int32_t old = t->slot_to_node[(size_t)s];
            if (old >= 0) t->node_to_slot[(size_t)old] = -1;
            std::memcpy(t->rows + (size_t)s * rb, src, rb);
            t->slot_to_node[(size_t)s] = id;
            t->node_to_slot[(size_t)id] = (int32_t)s;
            t->miss_src[j] = s;
        }
    });
    t->tail += (uint64_t)n_miss;
    t->lookups += (uint64_t)t->cur_m;
    t->hits += (uint64_t)t->cur_hit;
    t->serving = false;
    return BGL_OK;
}

}  // namespace bgl

extern "C" int bgl_host_tier_create(const void *store, int64_t num_nodes, int32_t row_bytes,
                                    int64_t capacity_rows, int64_t max_batch_rows, int32_t num_threads,
                                    bgl_host_tier_t **out)
{
    if (!out) BGL_FAIL(BGL_EINVAL, "out is null");
    *out = nullptr;
    if (!store) BGL_FAIL(BGL_EINVAL, "store is null");
    if (num_nodes < 1 || num_nodes > INT32_MAX) BGL_FAIL(BGL_EINVAL, "num_nodes out of range");
    if (row_bytes < 16 || row_bytes % 16 != 0)
        BGL_FAIL(BGL_EINVAL, "row_bytes must be a positive multiple of 16 (got %d)", row_bytes);
    if (capacity_rows < 1 || capacity_rows > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "capacity_rows must be in [1, 2^31) (got %lld)", (long long)capacity_rows);
    if (max_batch_rows < 1 || max_batch_rows > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "max_batch_rows must be in [1, 2^31) (got %lld)", (long long)max_batch_rows);
    if (num_threads < 0 || num_threads > 256) BGL_FAIL(BGL_EINVAL, "num_threads must be in [0, 256]");
    if (num_threads == 0) {
        const unsigned hw = std::thread::hardware_concurrency();
        num_threads = (int32_t)std::min<unsigned>(hw ? hw : 1, 16);
    }
    bgl_host_tier *t = new (std::nothrow) bgl_host_tier();
    if (!t) BGL_FAIL(BGL_ENOMEM, "out of host memory");
    t->store = static_cast<const char *>(store);
    t->num_nodes = num_nodes;
    t->row_bytes = row_bytes;
    t->capacity = capacity_rows;
    t->max_batch = bgl::round_up((size_t)max_batch_rows, 4);  // keeps the 8-byte lists aligned
    const size_t mb = (size_t)t->max_batch;
    const size_t row_total = ((size_t)capacity_rows + mb) * (size_t)row_bytes;
    auto fail = [&](int code) { bgl_host_tier_destroy(t); return code; };
    hipError_t e = hipHostMalloc((void **)&t->rows, row_total, hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        t->rows = nullptr;
        bgl::set_error("page-locked allocation of %zu bytes failed: %s", row_total, hipGetErrorString(e));
        return fail(BGL_ENOMEM);
    }
    e = hipHostMalloc((void **)&t->lists, 28 * mb + 64, hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        t->lists = nullptr;
        bgl::set_error("page-locked allocation of %zu bytes failed: %s", 28 * mb, hipGetErrorString(e));
        return fail(BGL_ENOMEM);
    }
    if (hipHostGetDevicePointer((void **)&t->rows_dev, t->rows, 0) != hipSuccess ||
        hipHostGetDevicePointer((void **)&t->lists_dev, t->lists, 0) != hipSuccess) {
        bgl::set_error("hipHostGetDevicePointer failed");
        return fail(BGL_EHIP);
    }
    t->ids = reinterpret_cast<int32_t *>(t->lists);
    t->hit_rank = reinterpret_cast<int32_t *>(t->lists + 4 * mb);
    t->miss_rank = reinterpret_cast<int32_t *>(t->lists + 8 * mb);
    t->hit_src = reinterpret_cast<int64_t *>(t->lists + 12 * mb);
    t->miss_src = reinterpret_cast<int64_t *>(t->lists + 20 * mb);
    try {
        t->node_to_slot.assign((size_t)num_nodes, -1);
        t->slot_to_node.assign((size_t)capacity_rows, -1);
        t->slot_rank.assign((size_t)capacity_rows, 0);
        t->slot_epoch.assign((size_t)capacity_rows, 0u);
        t->src_row.assign(mb, -1);
        t->pool = new Pool(num_threads);
    } catch (const std::exception &) {
        bgl::set_error("out of host memory");
        return fail(BGL_ENOMEM);
    }
    std::memset(t->rows, 0, (size_t)capacity_rows * (size_t)row_bytes);
    *out = t;
    return BGL_OK;
}

extern "C" int bgl_host_tier_destroy(bgl_host_tier_t *t)
{
    if (!t) return BGL_OK;
    (void)hipDeviceSynchronize();  // kernels may still read the rows
    delete t->pool;
    if (t->rows) (void)hipHostFree(t->rows);
    if (t->lists) (void)hipHostFree(t->lists);
    delete t;
    return BGL_OK;
}

extern "C" int bgl_host_tier_export_state(bgl_host_tier_t *t, int32_t *slot_to_node, uint64_t *tail,
                                          void *buffer_rows)
{
    if (!t) BGL_FAIL(BGL_EINVAL, "tier handle is null");
    if (slot_to_node) std::memcpy(slot_to_node, t->slot_to_node.data(), sizeof(int32_t) * (size_t)t->capacity);
    if (tail) *tail = t->tail;
    if (buffer_rows) std::memcpy(buffer_rows, t->rows, (size_t)t->capacity * (size_t)t->row_bytes);
    return BGL_OK;
}

extern "C" int bgl_host_tier_stats(bgl_host_tier_t *t, uint64_t *lookups, uint64_t *hits,
                                   uint64_t *kept_aside, int32_t *threads)
{
    if (!t) BGL_FAIL(BGL_EINVAL, "tier handle is null");
    if (lookups) *lookups = t->lookups;
    if (hits) *hits = t->hits;
    if (kept_aside) *kept_aside = t->kept_aside.load();
    if (threads) *threads = t->pool->threads();
    return BGL_OK;
}
