// Proximity-aware ordering of the training nodes (BGL paper, Sec. 3.2.2):
// several BFS sequences over the training nodes from given roots, each read from
// a given offset, merged into batches in turn.  The traversals run on the GPU;
// the merge (a strictly sequential scan over a few hundred thousand ids) and the
// shuffling-error statistic run on the host.
//
// BFS order is the first-in-first-out queue order (neighbors in CSR row order,
// restart at the smallest unvisited id).  The queue order of a level is fixed by
// the previous one: a node's place is given by the first (rank of the parent in
// its level, edge position in the parent's row) that reaches it.  So a
// level-synchronous traversal reproduces it exactly: expand (16 lanes walk one
// frontier node's row; atomicMin of that 64-bit key per newly seen neighbor, and
// a bit in the next-level bitmap), compact the bitmap to a candidate list, sort
// the candidates by key (rocPRIM radix sort, a plain library primitive), append
// the level's training nodes to the sequence.  Restarts: nodes all of whose
// out-neighbors are visited ("closed") would each be a one-node traversal; all
// closed nodes below the smallest open node are taken in one step, in id order,
// which is what the sequential rule does.
#include <algorithm>
#include <climits>
#include <cstring>
#include <vector>

#include "bgl_internal.h"

#include <rocprim/rocprim.hpp>

namespace {

using namespace bgl;

constexpr int BT = 256;
constexpr uint64_t NO_KEY = ~0ull;

struct OrderDev {
    int fsize;      // size of the list the last bitmap compaction wrote
    int seq_len;    // training nodes recorded so far
    int open_min;   // smallest unvisited node that has an unvisited out-neighbor
    int status;
};

__device__ __forceinline__ bool test_bit(const uint32_t *bm, uint32_t v) { return (bm[v >> 5] >> (v & 31)) & 1u; }

__global__ void k_fill_u32(uint32_t *p, int64_t n, uint32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

__global__ void k_fill_key(uint64_t *p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = NO_KEY;
}

__global__ void k_set_bits(const int32_t *ids, int64_t n, int64_t num_nodes, uint32_t *bm, OrderDev *dev)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t v = ids[i];
    if (v < 0 || (int64_t)v >= num_nodes) { dev->status = BGL_EINVAL; return; }
    const uint32_t old = atomicOr(&bm[(uint32_t)v >> 5], 1u << (v & 31));
    if (old & (1u << (v & 31))) dev->status = BGL_EINVAL;  // listed twice
}

// A fresh traversal: bits at and above num_nodes count as visited.
__global__ void k_reset(uint32_t *visited, uint32_t *next, int64_t words, int64_t num_nodes, OrderDev *dev)
{
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w == 0) { dev->fsize = 0; dev->seq_len = 0; dev->open_min = INT_MAX; }
    if (w >= words) return;
    uint32_t v = 0;
    const int64_t base = w * 32;
    if (base + 32 > num_nodes) v = num_nodes > base ? ~0u << (uint32_t)(num_nodes - base) : ~0u;
    visited[w] = v;
    next[w] = 0;
}

// Start (or restart) a traversal at one node; node < 0 means "at dev->open_min".
__global__ void k_start_at(int32_t node, uint32_t *visited, const uint32_t *train, int32_t *frontier,
                           int32_t *seq, OrderDev *dev)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int32_t v = node >= 0 ? node : dev->open_min;
    visited[(uint32_t)v >> 5] |= 1u << (v & 31);
    frontier[0] = v;
    dev->fsize = 1;
    if (test_bit(train, (uint32_t)v)) seq[dev->seq_len++] = v;
    dev->open_min = INT_MAX;
}

// 16 lanes per frontier node walk its row.  `visited` holds the earlier levels
// only; a neighbor outside it gets the smallest (parent rank, edge position) key
// of this level and a bit in `next`.
template <typename RP>
__global__ __launch_bounds__(BT) void k_expand(const RP *__restrict__ row_ptr, const int32_t *__restrict__ col,
                                               const int32_t *__restrict__ frontier, int fsize,
                                               const uint32_t *__restrict__ visited, uint32_t *next, uint64_t *key)
{
    const int64_t g = ((int64_t)blockIdx.x * BT + threadIdx.x) >> 4;
    const int l = threadIdx.x & 15;
    if (g >= fsize) return;
    const int32_t v = frontier[g];
    const int64_t lo = (int64_t)row_ptr[v], hi = (int64_t)row_ptr[v + 1];
    for (int64_t e = lo + l; e < hi; e += 16) {
        const uint32_t u = (uint32_t)col[e];
        const uint32_t bit = 1u << (u & 31);
        if (visited[u >> 5] & bit) continue;
        const uint64_t k = ((uint64_t)g << 32) | (uint64_t)(e - lo);
        if (__hip_atomic_load(&key[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > k)
            atomicMin((unsigned long long *)&key[u], (unsigned long long)k);
        if (!(__hip_atomic_load(&next[u >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit))
            atomicOr(&next[u >> 5], bit);
    }
}

// Bitmap -> ascending id list, three steps.  One bitmap word per lane.
__global__ __launch_bounds__(BT) void k_bm_count(const uint32_t *__restrict__ next, int64_t words, int32_t *bs)
{
    __shared__ int sh[BT / kWave];
    const int64_t w = (int64_t)blockIdx.x * BT + threadIdx.x;
    int tot;
    (void)block_excl_scan<BT>(w < words ? __popc(next[w]) : 0, sh, tot);
    if (threadIdx.x == 0) bs[blockIdx.x] = tot;
}

// Exclusive prefix of per-workgroup counts (in place); the total goes to
// dev->fsize (to_seq = 0) or extends the sequence (to_seq = 1, base in *seq_base).
__global__ __launch_bounds__(1024) void k_scan_counts(int32_t *bs, int nb, OrderDev *dev, int to_seq, int32_t *seq_base)
{
    __shared__ int sh[1024 / kWave];
    int carry = 0;
    for (int base = 0; base < nb; base += 1024) {
        const int i = base + threadIdx.x;
        int tot;
        const int ex = block_excl_scan<1024>(i < nb ? bs[i] : 0, sh, tot);
        if (i < nb) bs[i] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) {
        if (to_seq) { *seq_base = dev->seq_len; dev->seq_len += carry; }
        else dev->fsize = carry;
    }
}

__global__ __launch_bounds__(BT) void k_bm_write(uint32_t *next, uint32_t *visited, int64_t words,
                                                 const int32_t *__restrict__ pre, int32_t *cand)
{
    __shared__ int sh[BT / kWave];
    const int64_t w = (int64_t)blockIdx.x * BT + threadIdx.x;
    uint32_t m = w < words ? next[w] : 0u;
    int tot;
    int o = pre[blockIdx.x] + block_excl_scan<BT>(__popc(m), sh, tot);
    if (m) { next[w] = 0; visited[w] |= m; }
    const int32_t base = (int32_t)(w * 32);
    while (m) { cand[o++] = base + (__ffs(m) - 1); m &= m - 1; }
}

__global__ __launch_bounds__(BT) void k_gather_keys(const int32_t *__restrict__ cand, int n,
                                                    const uint64_t *__restrict__ key, uint64_t *out)
{
    const int i = blockIdx.x * BT + threadIdx.x;
    if (i < n) out[i] = key[cand[i]];
}

// Append the training nodes of a list to the sequence, keeping the list's order.
__global__ __launch_bounds__(BT) void k_list_count(const int32_t *__restrict__ list, int n,
                                                   const uint32_t *__restrict__ train, int32_t *bs)
{
    __shared__ int sh[BT / kWave];
    const int i = blockIdx.x * BT + threadIdx.x;
    int tot;
    (void)block_excl_scan<BT>((i < n && test_bit(train, (uint32_t)list[i])) ? 1 : 0, sh, tot);
    if (threadIdx.x == 0) bs[blockIdx.x] = tot;
}

__global__ __launch_bounds__(BT) void k_list_write(const int32_t *__restrict__ list, int n,
                                                   const uint32_t *__restrict__ train,
                                                   const int32_t *__restrict__ pre,
                                                   const int32_t *__restrict__ seq_base, int32_t *seq)
{
    __shared__ int sh[BT / kWave];
    const int i = blockIdx.x * BT + threadIdx.x;
    const int flag = (i < n && test_bit(train, (uint32_t)list[i])) ? 1 : 0;
    int tot;
    const int ex = block_excl_scan<BT>(flag, sh, tot);
    if (flag) seq[*seq_base + pre[blockIdx.x] + ex] = list[i];
}

// Smallest unvisited node with an unvisited out-neighbor other than itself.  The search runs at every
// restart of the traversal, and the visited set only grows: an edge that once led to a visited node
// (or back to its own node) always will, so every node keeps the number of leading edges of its row
// that are known to (`cursor`) and the next search goes on from there.  Over a whole traversal a row
// is walked once, however many restarts there are.
template <typename RP>
__global__ __launch_bounds__(BT) void k_open_min(const RP *__restrict__ row_ptr, const int32_t *__restrict__ col,
                                                 const uint32_t *__restrict__ visited, int64_t num_nodes,
                                                 int32_t *cursor, OrderDev *dev)
{
    const int64_t v = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (v >= num_nodes || test_bit(visited, (uint32_t)v)) return;
    if (v >= dev->open_min) return;  // cannot improve the minimum
    const int64_t lo = (int64_t)row_ptr[v], hi = (int64_t)row_ptr[v + 1];
    int64_t e = lo + cursor[v];
    for (; e < hi; ++e) {
        const uint32_t u = (uint32_t)col[e];
        if ((int64_t)u != v && !test_bit(visited, u)) break;
    }
    cursor[v] = (int32_t)(e - lo);
    if (e < hi) atomicMin(&dev->open_min, (int)v);
}

// Every unvisited node below dev->open_min is closed: mark them all for the next compaction.
__global__ __launch_bounds__(BT) void k_take_closed(const uint32_t *__restrict__ visited, uint32_t *next,
                                                    int64_t words, const OrderDev *dev)
{
    const int64_t w = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (w >= words) return;
    const int64_t limit = dev->open_min;  // INT_MAX: take everything
    const int64_t base = w * 32;
    if (base >= limit) return;
    uint32_t free_bits = ~visited[w];
    if (limit < base + 32) free_bits &= (1u << (uint32_t)(limit - base)) - 1u;
    if (free_bits) next[w] = free_bits;
}

struct OrderWork {
    uint32_t *visited = nullptr, *next = nullptr, *train = nullptr;
    int32_t *frontier = nullptr, *cand = nullptr, *seq = nullptr, *train_ids = nullptr, *bs = nullptr, *seq_base = nullptr;
    int32_t *cursor = nullptr;  // per node: leading edges of its row known to end at visited nodes (k_open_min)
    uint64_t *key = nullptr, *keys_in = nullptr, *keys_out = nullptr;
    void *sort_tmp = nullptr;
    size_t sort_tmp_bytes = 0;
    OrderDev *dev = nullptr;
    OrderDev *host = nullptr;  // page-locked mirror
    char *block = nullptr;     // the one device allocation all of the above are carved from
    ~OrderWork()
    {
        (void)hipFree(block);
        if (host) (void)hipHostFree(host);
    }
};

int read_dev(OrderWork &w, hipStream_t st)
{
    BGL_HIP(hipMemcpyAsync(w.host, w.dev, sizeof(OrderDev), hipMemcpyDeviceToHost, st));
    BGL_HIP(hipStreamSynchronize(st));
    return BGL_OK;
}

int prepare(const bgl_graph *g, const int32_t *train_nodes, int64_t num_train, OrderWork &w, hipStream_t st)
{
    const int64_t N = g->num_nodes, words = ceil_div(N, 32);
    const int64_t nb = std::max(ceil_div(words, BT), ceil_div(N, BT));
    // one device allocation for the whole call, sized up front and carved into 256-byte aligned parts
    BGL_HIP(rocprim::radix_sort_pairs(nullptr, w.sort_tmp_bytes, w.keys_in, w.keys_out, w.cand, w.frontier,
                                      (size_t)N, 0, 64, st));
    const size_t nt = (size_t)std::max<int64_t>(num_train, 1);
    const size_t sizes[] = {(size_t)words * 4, (size_t)words * 4, (size_t)words * 4, (size_t)N * 4, (size_t)N * 4,
                            (size_t)N * 8, (size_t)N * 8, (size_t)N * 8, nt * 4, nt * 4, (size_t)(nb + 1) * 4, 4,
                            sizeof(OrderDev), std::max<size_t>(w.sort_tmp_bytes, 16), (size_t)N * 4};
    size_t total = 0;
    for (size_t sz : sizes) total += round_up(sz, 256);
    BGL_HIP(hipMalloc((void **)&w.block, total));
    char *at = w.block;
    auto take = [&](size_t k) { char *p = at; at += round_up(sizes[k], 256); return p; };
    w.visited = reinterpret_cast<uint32_t *>(take(0));
    w.next = reinterpret_cast<uint32_t *>(take(1));
    w.train = reinterpret_cast<uint32_t *>(take(2));
    w.frontier = reinterpret_cast<int32_t *>(take(3));
    w.cand = reinterpret_cast<int32_t *>(take(4));
    w.key = reinterpret_cast<uint64_t *>(take(5));
    w.keys_in = reinterpret_cast<uint64_t *>(take(6));
    w.keys_out = reinterpret_cast<uint64_t *>(take(7));
    w.seq = reinterpret_cast<int32_t *>(take(8));
    w.train_ids = reinterpret_cast<int32_t *>(take(9));
    w.bs = reinterpret_cast<int32_t *>(take(10));
    w.seq_base = reinterpret_cast<int32_t *>(take(11));
    w.dev = reinterpret_cast<OrderDev *>(take(12));
    w.sort_tmp = take(13);
    w.cursor = reinterpret_cast<int32_t *>(take(14));
    BGL_HIP(hipHostMalloc((void **)&w.host, sizeof(OrderDev), hipHostMallocDefault));
    BGL_HIP(hipMemsetAsync(w.dev, 0, sizeof(OrderDev), st));
    BGL_HIP(hipMemcpyAsync(w.train_ids, train_nodes, num_train * 4, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(k_fill_u32, dim3(std::min<int64_t>(ceil_div(words, BT), 4096)), dim3(BT), 0, st, w.train, words, 0u);
    if (num_train > 0)
        hipLaunchKernelGGL(k_set_bits, dim3((unsigned)ceil_div(num_train, BT)), dim3(BT), 0, st, w.train_ids,
                           num_train, N, w.train, w.dev);
    int rc = read_dev(w, st);
    if (rc != BGL_OK) return rc;
    if (w.host->status != 0) BGL_FAIL(BGL_EINVAL, "train_nodes holds an id outside [0, num_nodes) or a repeated id");
    return BGL_OK;
}

// One traversal; leaves the sequence (num_train ids) in w.seq.
template <typename RP>
int bfs_sequence(const bgl_graph *g, int64_t root, int64_t num_train, OrderWork &w, hipStream_t st)
{
    const int64_t N = g->num_nodes, words = ceil_div(N, 32);
    const int nbw = (int)ceil_div(words, BT);
    const RP *rp = static_cast<const RP *>(g->row_ptr);
    hipLaunchKernelGGL(k_reset, dim3(nbw), dim3(BT), 0, st, w.visited, w.next, words, N, w.dev);
    hipLaunchKernelGGL(k_fill_key, dim3((unsigned)std::min<int64_t>(ceil_div(N, BT), 8192)), dim3(BT), 0, st, w.key, N);
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)std::min<int64_t>(ceil_div(N, BT), 8192)), dim3(BT), 0, st,
                       reinterpret_cast<uint32_t *>(w.cursor), N, 0u);
    hipLaunchKernelGGL(k_start_at, dim3(1), dim3(64), 0, st, (int32_t)root, w.visited, w.train, w.frontier, w.seq, w.dev);
    int64_t visited_count = 1;
    int fsize = 1;
    // next-level bitmap -> w.cand (ascending ids), marks them visited; returns the count
    auto compact = [&](int &count) -> int {
        hipLaunchKernelGGL(k_bm_count, dim3(nbw), dim3(BT), 0, st, w.next, words, w.bs);
        hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, st, w.bs, nbw, w.dev, 0, w.seq_base);
        hipLaunchKernelGGL(k_bm_write, dim3(nbw), dim3(BT), 0, st, w.next, w.visited, words, w.bs, w.cand);
        int rc = read_dev(w, st);
        if (rc != BGL_OK) return rc;
        count = w.host->fsize;
        return BGL_OK;
    };
    auto append_training = [&](const int32_t *list, int n) {
        if (n <= 0) return;
        const int nb = (int)ceil_div(n, BT);
        hipLaunchKernelGGL(k_list_count, dim3(nb), dim3(BT), 0, st, list, n, w.train, w.bs);
        hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, st, w.bs, nb, w.dev, 1, w.seq_base);
        hipLaunchKernelGGL(k_list_write, dim3(nb), dim3(BT), 0, st, list, n, w.train, w.bs, w.seq_base, w.seq);
    };
    for (;;) {
        while (fsize > 0) {
            const int parents = fsize;
            hipLaunchKernelGGL((k_expand<RP>), dim3((unsigned)ceil_div((int64_t)fsize * 16, BT)), dim3(BT), 0, st, rp,
                               g->col, w.frontier, fsize, w.visited, w.next, w.key);
            int rc = compact(fsize);
            if (rc != BGL_OK) return rc;
            visited_count += fsize;
            if (fsize == 0) break;
            // queue order of the new level: sort the candidates by (parent rank, edge position)
            hipLaunchKernelGGL(k_gather_keys, dim3((unsigned)ceil_div(fsize, BT)), dim3(BT), 0, st, w.cand, fsize, w.key, w.keys_in);
            int parent_bits = 1;
            while ((1ll << parent_bits) < parents) ++parent_bits;
            size_t tmp = w.sort_tmp_bytes;
            BGL_HIP(rocprim::radix_sort_pairs(w.sort_tmp, tmp, w.keys_in, w.keys_out, w.cand, w.frontier,
                                              (size_t)fsize, 0, (unsigned)std::min(64, 32 + parent_bits), st));
            append_training(w.frontier, fsize);
        }
        if (visited_count >= N) break;
        hipLaunchKernelGGL((k_open_min<RP>), dim3((unsigned)ceil_div(N, BT)), dim3(BT), 0, st, rp, g->col, w.visited, N, w.cursor,
                           w.dev);
        hipLaunchKernelGGL(k_take_closed, dim3(nbw), dim3(BT), 0, st, w.visited, w.next, words, w.dev);
        int closed = 0;
        int rc = compact(closed);       // one-node traversals, in id order
        if (rc != BGL_OK) return rc;
        visited_count += closed;
        append_training(w.cand, closed);
        if (w.host->open_min == INT_MAX) break;  // everything that was left was closed
        hipLaunchKernelGGL(k_start_at, dim3(1), dim3(64), 0, st, (int32_t)-1, w.visited, w.train, w.frontier, w.seq, w.dev);
        fsize = 1;
        visited_count += 1;
    }
    BGL_HIP(hipGetLastError());
    int rc = read_dev(w, st);
    if (rc != BGL_OK) return rc;
    if (visited_count != N || w.host->seq_len != num_train)
        BGL_FAIL(BGL_EHIP, "traversal ended with %lld of %lld nodes and %d of %lld training nodes",
                 (long long)visited_count, (long long)N, w.host->seq_len, (long long)num_train);
    return BGL_OK;
}

int check_order_args(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train)
{
    if (!g) BGL_FAIL(BGL_EINVAL, "graph handle is null");
    if (num_train < 1 || num_train > g->num_nodes) BGL_FAIL(BGL_EINVAL, "num_train must be in [1, num_nodes]");
    if (!train_nodes) BGL_FAIL(BGL_EINVAL, "train_nodes is null");
    return BGL_OK;
}

}  // namespace

extern "C" int bgl_order_bfs_sequence(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                                      int64_t root, int32_t *seq, void *stream)
try {
    int rc = check_order_args(g, train_nodes, num_train);
    if (rc != BGL_OK) return rc;
    if (root < 0 || root >= g->num_nodes) BGL_FAIL(BGL_EINVAL, "root is outside [0, num_nodes)");
    if (!seq) BGL_FAIL(BGL_EINVAL, "seq is null");
    hipStream_t st = static_cast<hipStream_t>(stream);
    OrderWork w;
    if ((rc = prepare(g, train_nodes, num_train, w, st)) != BGL_OK) return rc;
    rc = g->bits == 64 ? bfs_sequence<int64_t>(g, root, num_train, w, st) : bfs_sequence<int32_t>(g, root, num_train, w, st);
    if (rc != BGL_OK) return rc;
    BGL_HIP(hipMemcpyAsync(seq, w.seq, num_train * 4, hipMemcpyDeviceToHost, st));
    BGL_HIP(hipStreamSynchronize(st));
    return BGL_OK;
} BGL_NOTHROW_END

namespace {

int check_proximity_args(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                         int32_t num_sequences, const int64_t *roots, const int64_t *shifts)
{
    int rc = check_order_args(g, train_nodes, num_train);
    if (rc != BGL_OK) return rc;
    if (num_sequences < 1 || !roots || !shifts) BGL_FAIL(BGL_EINVAL, "need at least one sequence with a root and a shift");
    for (int j = 0; j < num_sequences; ++j) {
        if (roots[j] < 0 || roots[j] >= g->num_nodes) BGL_FAIL(BGL_EINVAL, "roots[%d] is outside [0, num_nodes)", j);
        if (shifts[j] < 0 || shifts[j] >= num_train) BGL_FAIL(BGL_EINVAL, "shifts[%d] is outside [0, num_train)", j);
    }
    return BGL_OK;
}

int compute_sequences(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train, int32_t num_sequences,
                      const int64_t *roots, hipStream_t st, std::vector<std::vector<int32_t>> &seqs)
{
    OrderWork w;
    int rc = prepare(g, train_nodes, num_train, w, st);
    if (rc != BGL_OK) return rc;
    seqs.assign((size_t)num_sequences, std::vector<int32_t>());
    for (int j = 0; j < num_sequences; ++j) {
        rc = g->bits == 64 ? bfs_sequence<int64_t>(g, roots[j], num_train, w, st)
                           : bfs_sequence<int32_t>(g, roots[j], num_train, w, st);
        if (rc != BGL_OK) return rc;
        seqs[(size_t)j].resize((size_t)num_train);
        BGL_HIP(hipMemcpyAsync(seqs[(size_t)j].data(), w.seq, num_train * 4, hipMemcpyDeviceToHost, st));
        BGL_HIP(hipStreamSynchronize(st));
    }
    return BGL_OK;
}

// turn t takes the next node of sequence t mod S that no earlier turn has taken
void merge_sequences(const std::vector<std::vector<int32_t>> &seqs, int32_t num_sequences, const int64_t *shifts,
                     int64_t num_train, int64_t num_nodes, int64_t num_out, int32_t *order)
{
    std::vector<uint8_t> used((size_t)num_nodes, 0);
    std::vector<int64_t> cursor((size_t)num_sequences, 0);
    for (int64_t k = 0, turn = 0; k < num_out; ++k, ++turn) {
        const size_t j = (size_t)(turn % num_sequences);
        int32_t v;
        do {
            v = seqs[j][(size_t)((shifts[j] + cursor[j]) % num_train)];
            cursor[j] += 1;
        } while (used[(size_t)v]);
        used[(size_t)v] = 1;
        order[k] = v;
    }
}

}  // namespace

extern "C" int bgl_order_proximity(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                                   int32_t num_sequences, const int64_t *roots, const int64_t *shifts,
                                   int64_t num_out, int32_t *order, void *stream)
try {
    int rc = check_proximity_args(g, train_nodes, num_train, num_sequences, roots, shifts);
    if (rc != BGL_OK) return rc;
    if (num_out < 0 || num_out > num_train) BGL_FAIL(BGL_EINVAL, "num_out must be in [0, num_train]");
    if (num_out > 0 && !order) BGL_FAIL(BGL_EINVAL, "order is null");
    std::vector<std::vector<int32_t>> seqs;
    rc = compute_sequences(g, train_nodes, num_train, num_sequences, roots, static_cast<hipStream_t>(stream), seqs);
    if (rc != BGL_OK) return rc;
    merge_sequences(seqs, num_sequences, shifts, num_train, g->num_nodes, num_out, order);
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_order_choose_sequences(const bgl_graph_t *g, const int32_t *train_nodes, int64_t num_train,
                                          int32_t max_sequences, const int64_t *roots, const int64_t *shifts,
                                          int32_t batch, const int32_t *labels, int32_t num_classes,
                                          double threshold, int32_t *chosen, double *mean_tv_per_count,
                                          int32_t *order, void *stream)
try {
    int rc = check_proximity_args(g, train_nodes, num_train, max_sequences, roots, shifts);
    if (rc != BGL_OK) return rc;
    if (!labels || !chosen || !order) BGL_FAIL(BGL_EINVAL, "labels, chosen and order must not be null");
    std::vector<std::vector<int32_t>> seqs;
    rc = compute_sequences(g, train_nodes, num_train, max_sequences, roots, static_cast<hipStream_t>(stream), seqs);
    if (rc != BGL_OK) return rc;
    for (int32_t s = 1; s <= max_sequences; ++s) {
        merge_sequences(seqs, s, shifts, num_train, g->num_nodes, num_train, order);
        double mean_tv = 0.0, max_tv = 0.0;
        rc = bgl_order_shuffling_error(order, num_train, batch, labels, g->num_nodes, num_classes, &mean_tv, &max_tv);
        if (rc != BGL_OK) return rc;
        if (mean_tv_per_count) mean_tv_per_count[s - 1] = mean_tv;
        *chosen = s;
        if (mean_tv <= threshold) break;   // `order` holds the order for this count
    }
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_order_shuffling_error(const int32_t *order, int64_t n, int32_t batch, const int32_t *labels,
                                         int64_t num_nodes, int32_t num_classes, double *mean_tv, double *max_tv)
try {
    if (!order || !labels || !mean_tv || !max_tv) BGL_FAIL(BGL_EINVAL, "null argument");
    if (n < 1 || batch < 1 || num_classes < 1 || num_nodes < 1) BGL_FAIL(BGL_EINVAL, "sizes must be positive");
    std::vector<int64_t> global((size_t)num_classes, 0), local((size_t)num_classes);
    for (int64_t i = 0; i < n; ++i) {
        if (order[i] < 0 || order[i] >= num_nodes) BGL_FAIL(BGL_EINVAL, "order[%lld] is not a node id", (long long)i);
        const int32_t c = labels[order[i]];
        if (c < 0 || c >= num_classes) BGL_FAIL(BGL_EINVAL, "label of node %d is outside [0, num_classes)", order[i]);
        global[(size_t)c] += 1;
    }
    double sum = 0.0, mx = 0.0;
    int64_t batches = 0;
    for (int64_t s = 0; s < n; s += batch, ++batches) {
        const int64_t e = std::min<int64_t>(s + batch, n);
        std::fill(local.begin(), local.end(), 0);
        for (int64_t i = s; i < e; ++i) local[(size_t)labels[order[i]]] += 1;
        double tv = 0.0;
        for (int32_t c = 0; c < num_classes; ++c) {
            const double pb = (double)local[(size_t)c] / (double)(e - s), pg = (double)global[(size_t)c] / (double)n;
            tv += 0.5 * (pb > pg ? pb - pg : pg - pb);
        }
        sum += tv;
        mx = std::max(mx, tv);
    }
    *mean_tv = sum / (double)batches;
    *max_tv = mx;
    return BGL_OK;
} BGL_NOTHROW_END
