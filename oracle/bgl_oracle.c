/*
 * CPU oracle for minibatch preparation as described in the BGL paper
 * (arXiv 2112.08541): k-hop fanout neighbor sampling (Sec. 2.1 stage 1,
 * Sec. 5.1 "Mini-batch Sampling Algorithms") followed by feature retrieval
 * through a FIFO feature cache (Sec. 3.2 "Feature Cache Engine", Sec. 4
 * "Feature Cache Engine" paragraph on the circular buffer and `tail`).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is deliberately plain, single-threaded and
 * slow: one loop per step of the method, no blocking, no fusion, direct-mapped
 * arrays instead of hash tables.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.  It shares no code, header,
 * table or constant generator with the HIP library.
 *
 * Everything here is integer or byte work, so results are exact.
 *
 * Where the paper is silent the canonical reading is stated at the function
 * that implements it.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Random numbers.  The paper does not name a generator for neighbor sampling;
 * the canonical choice is a counter-based one keyed on (call seed, hop, node,
 * slot) so that a draw does not depend on how the node was reached.  The
 * mixing function is the published SplitMix64 output function (Steele, Lea,
 * Flood 2014; Vigna's reference splitmix64.c): three xor-shifts and two odd
 * multiplications, all mod 2^64. */

#define BGLO_GOLDEN 0x9E3779B97F4A7C15ULL

uint64_t bglo_mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

/* 64-bit word for (call seed, hop, node, slot): hop and node select a stream,
 * slot is the counter inside it.  The three steps are functions of their own so
 * that each can be checked against the published SplitMix64 outputs:
 *   hop key   = output number hop+1 of the SplitMix64 generator seeded with the
 *               call seed (the generator adds the golden-ratio constant to its
 *               state before every output);
 *   node key  = the hop key with the node id xor-ed in, mixed once;
 *   draw      = output number slot+1 of the generator seeded with the node key. */
uint64_t bglo_hop_key(uint64_t rng_seed, int32_t hop)
{
    return bglo_mix64(rng_seed + BGLO_GOLDEN * (uint64_t)(hop + 1));
}

uint64_t bglo_node_key(uint64_t hop_key, int32_t node)
{
    return bglo_mix64(hop_key ^ (uint64_t)(uint32_t)node);
}

uint64_t bglo_slot_draw(uint64_t node_key, int32_t slot)
{
    return bglo_mix64(node_key + BGLO_GOLDEN * (uint64_t)(slot + 1));
}

uint64_t bglo_draw(uint64_t rng_seed, int32_t hop, int32_t node, int32_t slot)
{
    return bglo_slot_draw(bglo_node_key(bglo_hop_key(rng_seed, hop), node), slot);
}

/* Map a 64-bit word to [0, m): floor(x * m / 2^64).  No rejection step, so
 * the bias is at most m / 2^64. */
uint64_t bglo_mulhi64(uint64_t x, uint64_t m)
{
    return (uint64_t)(((unsigned __int128)x * (unsigned __int128)m) >> 64);
}

/* ------------------------------------------------------------------------- */
/* Uniform k-subset of {0..d-1} from given bounded integers (Robert Floyd's
 * algorithm, CACM 1987): for s = 0..k-1 with J = d-k+s, t[s] must lie in
 * [0, J]; position s is t[s] unless that value was already chosen, in which
 * case it is J.  Output order is slot order, not sorted. */
void bglo_floyd_from_t(int64_t d, int32_t k, const int64_t *t, int64_t *pos)
{
    for (int32_t s = 0; s < k; ++s) {
        int64_t J = d - k + s;
        int64_t cand = t[s];
        int seen = 0;
        for (int32_t j = 0; j < s; ++j)
            if (pos[j] == cand) seen = 1;
        pos[s] = seen ? J : cand;
    }
}

/* Edge positions sampled for one node: GraphSAGE-style neighbor sampling
 * (Sec. 5.1) without replacement over edge positions; a node with at most
 * `fanout` edges keeps all of them in CSR order (so the count is
 * min(fanout, degree)).  Returns the count. */
int32_t bglo_sample_positions(uint64_t rng_seed, int32_t hop, int32_t node,
                              int64_t d, int32_t fanout, int64_t *pos)
{
    if (d <= (int64_t)fanout) {
        for (int64_t s = 0; s < d; ++s) pos[s] = s;
        return (int32_t)d;
    }
    int64_t *t = (int64_t *)malloc(sizeof(int64_t) * (size_t)fanout);
    for (int32_t s = 0; s < fanout; ++s) {
        int64_t J = d - fanout + s;
        t[s] = (int64_t)bglo_mulhi64(bglo_draw(rng_seed, hop, node, s), (uint64_t)(J + 1));
    }
    bglo_floyd_from_t(d, fanout, t, pos);
    free(t);
    return fanout;
}

static int64_t rp_at(const void *row_ptr, int bits, int64_t i)
{
    return bits == 64 ? ((const int64_t *)row_ptr)[i] : (int64_t)((const int32_t *)row_ptr)[i];
}

/* ------------------------------------------------------------------------- */
/* k-hop sampling ("iteratively sampling next-hop neighbors", Sec. 3.1; batch
 * of seeds, one fanout per hop, Sec. 5.1).
 *
 * frontier_0 = seeds with repeats removed, first occurrence kept.
 * For hop h: every node of frontier_h, in frontier order, is sampled with
 * fanouts[h] (fanouts[0] applies at the seeds).  The sampled neighbor ids, in
 * (frontier index, slot) order, are appended to frontier_h with repeats
 * removed (first occurrence kept) to give frontier_{h+1}; frontier_h is a
 * prefix of frontier_{h+1}, so a node's local id never changes.
 *
 * Outputs (caller-allocated):
 *   input_nodes[cap_nodes]         frontier_K, global ids
 *   n_frontier[num_hops+1]         |frontier_h|
 *   hop_row_ptr[h][n_frontier[h]+1]  prefix sum of per-node sample counts
 *   hop_col_local[h][nnz_h]        local id (index in frontier_{h+1}) per edge
 *   hop_col_global[h][nnz_h]       global id per edge (may be NULL)
 *   nnz[num_hops]
 * Returns 0, or -1 on bad arguments, -4 if an output capacity is too small.
 */
int bglo_sample_khop(const void *row_ptr, int row_ptr_bits, const int32_t *col,
                     int64_t num_nodes,
                     const int32_t *seeds, int32_t num_seeds,
                     const int32_t *fanouts, int32_t num_hops, uint64_t rng_seed,
                     int32_t *input_nodes, int64_t cap_nodes,
                     int32_t *n_frontier,
                     int32_t **hop_row_ptr, int32_t **hop_col_local,
                     int32_t **hop_col_global, const int64_t *cap_edges,
                     int64_t *nnz)
{
    if (num_hops <= 0 || num_seeds < 0) return -1;
    /* node id -> local id, -1 = not in the frontier yet */
    int32_t *local_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(num_nodes > 0 ? num_nodes : 1));
    if (!local_of) return -2;
    for (int64_t v = 0; v < num_nodes; ++v) local_of[v] = -1;

    int rc = 0;
    int64_t n = 0;
    for (int32_t i = 0; i < num_seeds; ++i) {
        int32_t v = seeds[i];
        if (v < 0 || (int64_t)v >= num_nodes) { rc = -1; goto done; }
        if (local_of[v] < 0) {
            if (n >= cap_nodes) { rc = -4; goto done; }
            local_of[v] = (int32_t)n;
            input_nodes[n++] = v;
        }
    }
    n_frontier[0] = (int32_t)n;

    for (int32_t h = 0; h < num_hops; ++h) {
        int32_t k = fanouts[h];
        if (k <= 0) { rc = -1; goto done; }
        int64_t n_dst = n;
        int64_t e = 0;
        int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
        hop_row_ptr[h][0] = 0;
        for (int64_t i = 0; i < n_dst; ++i) {
            int32_t v = input_nodes[i];
            int64_t lo = rp_at(row_ptr, row_ptr_bits, v);
            int64_t d = rp_at(row_ptr, row_ptr_bits, (int64_t)v + 1) - lo;
            int32_t c = bglo_sample_positions(rng_seed, h, v, d, k, pos);
            for (int32_t s = 0; s < c; ++s) {
                int32_t u = col[lo + pos[s]];
                if (e >= cap_edges[h]) { free(pos); rc = -4; goto done; }
                if (local_of[u] < 0) {
                    if (n >= cap_nodes) { free(pos); rc = -4; goto done; }
                    local_of[u] = (int32_t)n;
                    input_nodes[n++] = u;
                }
                hop_col_local[h][e] = local_of[u];
                if (hop_col_global && hop_col_global[h]) hop_col_global[h][e] = u;
                ++e;
            }
            hop_row_ptr[h][i + 1] = (int32_t)e;
        }
        free(pos);
        nnz[h] = e;
        n_frontier[h + 1] = (int32_t)n;
    }
done:
    free(local_of);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* FIFO feature cache (Sec. 3.2.1 policy; Sec. 3.2.3 cache map + cache buffer
 * and the lookup / gather / fetch / update workflow; Sec. 4: the buffer is a
 * circular queue addressed through a running `tail`, the old occupant of a
 * position is evicted from the map and its row overwritten).
 *
 * State: slot_to_node[C] (-1 = empty), node_to_slot[N] (-1 = not cached; the
 * "contiguous 1D array as a hashmap" of the Sec. 3.2.1 footnote), tail = number
 * of insertions so far, buffer[C][row_bytes].  The backing store is one host
 * feature table (the CPU cache and the graph store of Sec. 3.2.3 collapsed
 * into one level).
 *
 * Reading of the slot formula: the r-th insertion overall (r counted from 0)
 * lands in slot r mod C, i.e. the first insertion uses slot 0.
 */
typedef struct {
    int64_t capacity;
    int32_t row_bytes;
    int64_t num_nodes;
    const uint8_t *features; /* not owned */
    int32_t *slot_to_node;
    int32_t *node_to_slot;
    uint8_t *buffer;
    uint64_t tail;
    uint64_t lookups, hits;
    uint32_t *seen_in_call; /* [N]: number of the last lookup call that contained the id */
    uint32_t call;
} bglo_cache;

bglo_cache *bglo_cache_create(int64_t capacity_rows, int32_t row_bytes,
                              const void *host_features, int64_t num_nodes)
{
    if (capacity_rows <= 0 || row_bytes <= 0 || num_nodes <= 0 || !host_features) return NULL;
    bglo_cache *c = (bglo_cache *)calloc(1, sizeof(bglo_cache));
    if (!c) return NULL;
    c->capacity = capacity_rows;
    c->row_bytes = row_bytes;
    c->num_nodes = num_nodes;
    c->features = (const uint8_t *)host_features;
    c->slot_to_node = (int32_t *)malloc(sizeof(int32_t) * (size_t)capacity_rows);
    c->node_to_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)num_nodes);
    c->buffer = (uint8_t *)calloc((size_t)capacity_rows, (size_t)row_bytes);
    c->seen_in_call = (uint32_t *)calloc((size_t)num_nodes, sizeof(uint32_t));
    if (!c->slot_to_node || !c->node_to_slot || !c->buffer || !c->seen_in_call) {
        free(c->slot_to_node); free(c->node_to_slot); free(c->buffer); free(c->seen_in_call); free(c);
        return NULL;
    }
    for (int64_t s = 0; s < capacity_rows; ++s) c->slot_to_node[s] = -1;
    for (int64_t v = 0; v < num_nodes; ++v) c->node_to_slot[v] = -1;
    return c;
}

void bglo_cache_destroy(bglo_cache *c)
{
    if (!c) return;
    free(c->slot_to_node); free(c->node_to_slot); free(c->buffer); free(c->seen_in_call); free(c);
}

/* Lookup against the state at entry, then serve every row: hits from the cache
 * buffer, misses from the host table.  No state change (FIFO: a hit does not
 * refresh a row's position).  miss_pos receives the positions i of the misses
 * in ascending order.  The ids of one call must be distinct (they are the
 * deduplicated nodes of one sampled subgraph): a repeated id would be inserted
 * twice by the update that follows.  Returns the number of hits, -1 on an id
 * outside the table, -2 on a repeated id; nothing is counted in those cases. */
int64_t bglo_cache_lookup_gather(bglo_cache *c, const int32_t *ids, int64_t n,
                                 void *out_rows, int32_t *out_slot,
                                 int32_t *miss_pos)
{
    uint8_t *out = (uint8_t *)out_rows;
    size_t rb = (size_t)c->row_bytes;
    int64_t n_hit = 0, n_miss = 0;
    c->call += 1;
    if (c->call == 0) { /* the call number wrapped: forget the old marks */
        memset(c->seen_in_call, 0, sizeof(uint32_t) * (size_t)c->num_nodes);
        c->call = 1;
    }
    for (int64_t i = 0; i < n; ++i) {
        int32_t v = ids[i];
        if (v < 0 || (int64_t)v >= c->num_nodes) return -1;
        if (c->seen_in_call[v] == c->call) return -2;
        c->seen_in_call[v] = c->call;
    }
    for (int64_t i = 0; i < n; ++i) {
        int32_t v = ids[i];
        int32_t slot = c->node_to_slot[v];
        out_slot[i] = slot;
        if (slot >= 0) {
            memcpy(out + (size_t)i * rb, c->buffer + (size_t)slot * rb, rb);
            ++n_hit;
        } else {
            memcpy(out + (size_t)i * rb, c->features + (size_t)v * rb, rb);
            miss_pos[n_miss++] = (int32_t)i;
        }
    }
    c->lookups += (uint64_t)n;
    c->hits += (uint64_t)n_hit;
    return n_hit;
}

/* Insert the missed rows one after another, in miss_pos order: take the next
 * position of the circular buffer, evict its occupant from the map, record the
 * new node, copy its row from out_rows.  With more misses than slots the later
 * insertions simply overwrite the earlier ones of the same call. */
void bglo_cache_insert_fifo(bglo_cache *c, const int32_t *ids, const int32_t *miss_pos,
                            int64_t n_miss, const void *out_rows)
{
    const uint8_t *out = (const uint8_t *)out_rows;
    size_t rb = (size_t)c->row_bytes;
    for (int64_t r = 0; r < n_miss; ++r) {
        int64_t slot = (int64_t)((c->tail + (uint64_t)r) % (uint64_t)c->capacity);
        int32_t old = c->slot_to_node[slot];
        if (old >= 0) c->node_to_slot[old] = -1;
        int32_t v = ids[miss_pos[r]];
        c->slot_to_node[slot] = v;
        c->node_to_slot[v] = (int32_t)slot;
        memcpy(c->buffer + (size_t)slot * rb, out + (size_t)miss_pos[r] * rb, rb);
    }
    c->tail += (uint64_t)n_miss;
}

/* Accessors for tests. */
uint64_t bglo_cache_tail(const bglo_cache *c) { return c->tail; }
const int32_t *bglo_cache_slot_to_node(const bglo_cache *c) { return c->slot_to_node; }
const int32_t *bglo_cache_node_to_slot(const bglo_cache *c) { return c->node_to_slot; }
const uint8_t *bglo_cache_buffer(const bglo_cache *c) { return c->buffer; }
void bglo_cache_stats(const bglo_cache *c, uint64_t *lookups, uint64_t *hits)
{
    *lookups = c->lookups;
    *hits = c->hits;
}

/* ------------------------------------------------------------------------- */
/* Proximity-aware ordering (Sec. 3.2.2): training-node sequences in BFS order
 * from several roots, each sequence rotated by a random offset, batches filled
 * from the sequences in turn.  The random roots and offsets are inputs.
 *
 * BFS order: the textbook first-in-first-out queue traversal, the neighbors of a
 * node taken in CSR row order; when a traversal is exhausted it restarts at the
 * smallest node id not visited yet (small components end up at the end of the
 * sequence, as Sec. 3.2.2 observes).  Only training nodes are recorded. */

/* Returns the number of training nodes recorded in seq, or -1 on bad arguments. */
int64_t bglo_bfs_sequence(const void *row_ptr, int row_ptr_bits, const int32_t *col,
                          int64_t num_nodes, const uint8_t *is_train, int64_t root,
                          int32_t *seq)
{
    if (num_nodes <= 0 || root < 0 || root >= num_nodes) return -1;
    uint8_t *seen = (uint8_t *)calloc((size_t)num_nodes, 1);
    int32_t *queue = (int32_t *)malloc(sizeof(int32_t) * (size_t)num_nodes);
    if (!seen || !queue) { free(seen); free(queue); return -1; }
    int64_t head = 0, tail = 0, n_out = 0, scan = 0;
    int64_t start = root;
    for (;;) {
        seen[start] = 1;
        queue[tail++] = (int32_t)start;
        while (head < tail) {
            int32_t v = queue[head++];
            if (is_train[v]) seq[n_out++] = v;
            int64_t lo = rp_at(row_ptr, row_ptr_bits, v);
            int64_t hi = rp_at(row_ptr, row_ptr_bits, (int64_t)v + 1);
            for (int64_t e = lo; e < hi; ++e) {
                int32_t u = col[e];
                if (!seen[u]) { seen[u] = 1; queue[tail++] = u; }
            }
        }
        while (scan < num_nodes && seen[scan]) ++scan;   /* smallest unvisited id */
        if (scan >= num_nodes) break;
        start = scan;
    }
    free(seen); free(queue);
    return n_out;
}

/* Merge: sequence j is read from offset shifts[j] (cyclically); turn t takes the
 * next node of sequence t mod S that no earlier turn has taken.  seqs holds the S
 * sequences back to back (each num_train long).  Writes num_out <= num_train ids. */
int bglo_po_merge(const int32_t *seqs, int64_t num_train, int32_t num_seq, const int64_t *shifts,
                  int64_t num_nodes, int64_t num_out, int32_t *order)
{
    if (num_seq < 1 || num_out > num_train) return -1;
    uint8_t *used = (uint8_t *)calloc((size_t)num_nodes, 1);
    int64_t *cursor = (int64_t *)calloc((size_t)num_seq, sizeof(int64_t));
    if (!used || !cursor) { free(used); free(cursor); return -2; }
    int64_t turn = 0;
    for (int64_t k = 0; k < num_out; ++k, ++turn) {
        int32_t j = (int32_t)(turn % num_seq);
        const int32_t *s = seqs + (size_t)j * (size_t)num_train;
        int32_t v;
        for (;;) {
            v = s[(shifts[j] + cursor[j]) % num_train];
            cursor[j] += 1;
            if (!used[v]) break;
        }
        used[v] = 1;
        order[k] = v;
    }
    free(used); free(cursor);
    return 0;
}

/* Shuffling error (Sec. 3.2.2, after Meng et al.): total variation distance
 * between the label distribution of a batch and that of all ordered nodes;
 * reading: reported as the mean and the maximum over the batches (the paper
 * "estimates the probability of each label as the frequency per mini-batch"
 * without saying how batches are combined). */
int bglo_shuffling_error(const int32_t *order, int64_t n, int32_t batch, const int32_t *labels,
                         int32_t num_classes, double *mean_tv, double *max_tv)
{
    if (n <= 0 || batch <= 0 || num_classes <= 0) return -1;
    /* integer counts first, so that equal frequencies compare equal */
    int64_t *g = (int64_t *)calloc((size_t)num_classes, sizeof(int64_t));
    int64_t *b = (int64_t *)calloc((size_t)num_classes, sizeof(int64_t));
    for (int64_t i = 0; i < n; ++i) g[labels[order[i]]] += 1;
    int64_t nb = 0;
    double sum = 0.0, mx = 0.0;
    for (int64_t s = 0; s < n; s += batch, ++nb) {
        int64_t e = s + batch < n ? s + batch : n;
        for (int32_t c = 0; c < num_classes; ++c) b[c] = 0;
        for (int64_t i = s; i < e; ++i) b[labels[order[i]]] += 1;
        double tv = 0.0;
        for (int32_t c = 0; c < num_classes; ++c) {
            double pb = (double)b[c] / (double)(e - s), pg = (double)g[c] / (double)n;
            tv += 0.5 * (pb > pg ? pb - pg : pg - pb);
        }
        sum += tv;
        if (tv > mx) mx = tv;
    }
    *mean_tv = sum / (double)nb;
    *max_tv = mx;
    free(g); free(b);
    return 0;
}
