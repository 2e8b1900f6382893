// k-hop fanout neighbor sampling with per-hop deduplication and relabelling
// (BGL paper, Sec. 3.1: samplers iteratively sample next-hop neighbors of the
// training nodes; Sec. 5.1: Neighbor Sampling with one fanout per hop).
//
// One call runs 1 + num_hops stages on one stream without any host round trip:
// stage 0 removes repeated seeds, stage h+1 samples hop h.  Every stage is four
// kernels:
//   sample/insert  a group of G lanes (G = power of two >= fanout) per frontier
//                  node draws the node's edge positions (Floyd's subset
//                  algorithm resolved with wavefront ballots), reads the
//                  neighbor ids, removes repeats inside the workgroup in an LDS
//                  hash table and enters the survivors in a global hash table
//                  with atomicMin on their position, so that the entry of every
//                  id ends up holding its first position in (node, slot) order
//   flag           marks the positions that are first occurrences of a new id
//                  and ranks them inside each tile
//   scan           one workgroup turns the per-tile totals into prefixes and
//                  publishes the stage's sizes
//   finalize       gives every new id its local id (old frontier size + rank),
//                  appends it to the frontier, and writes the hop's CSR block
// A stage of at most TILE tiles (262,144 padded positions) has no scan launch:
// every workgroup of finalize turns the tile totals into prefixes itself, in LDS
// (one block scan), and the first one publishes the sizes.
// Launches are sized by upper bounds; the real sizes stay on the device.
#include "bgl_internal.h"

namespace {

using namespace bgl;

constexpr int TILE = 512;                      // threads (= padded positions) per workgroup
constexpr uint64_t EMPTY64 = ~0ull;
constexpr uint32_t TENT = 0x80000000u;         // value is a tentative position, not yet a local id
constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;
constexpr int STATUS = BGL_COUNTS_LEN - 1;
constexpr int NNZ0 = BGL_MAX_HOPS + 1;

// SplitMix64 output function (Steele, Lea, Flood 2014): the mixing step of the
// counter-based generator keyed on (call seed, hop, node, slot).
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// Start of a call: empty table, counts at zero.
__global__ void k_prepare(uint64_t *p, int64_t n, uint64_t v, int32_t *cnt)
{
    if (blockIdx.x == 0 && threadIdx.x < BGL_COUNTS_LEN) cnt[threadIdx.x] = 0;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// Enter (key, val) in the global table, keeping the smallest val per key.
// Entries are (key << 32 | val); returns the entry index.
__device__ __forceinline__ int table_insert_min(uint64_t *tab, uint32_t mask, uint32_t key,
                                                uint32_t val, int32_t *cnt)
{
    const uint64_t mine = ((uint64_t)key << 32) | val;
    uint32_t s = hash32(key) & mask;
    for (uint32_t tries = 0; tries <= mask; ++tries) {
        uint64_t cur = __hip_atomic_load(&tab[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cur == EMPTY64) {
            unsigned long long old = atomicCAS((unsigned long long *)&tab[s], EMPTY64, mine);
            if (old == EMPTY64) return (int)s;
            cur = old;
        }
        if ((uint32_t)(cur >> 32) == key) {
            if ((uint32_t)cur > val) atomicMin((unsigned long long *)&tab[s], mine);
            return (int)s;
        }
        s = (s + 1) & mask;
    }
    cnt[STATUS] = BGL_ECAPACITY;  // cannot happen: the table outsizes the frontier bound
    return -1;
}

// Second half of a sample/insert kernel: workgroup-local dedup in LDS, then one
// global insert per distinct id of the workgroup.  sh_tab (2*TILE entries) must
// be EMPTY64 and visible to the whole workgroup on entry.
__device__ __forceinline__ void dedup_and_insert(bool valid, uint32_t key, uint32_t p,
                                                 uint64_t *tab, uint32_t mask,
                                                 int32_t *slotidx, uint64_t *sh_tab,
                                                 int32_t *sh_gs, int32_t *cnt)
{
    constexpr uint32_t LM = 2 * TILE - 1;
    uint32_t ls = 0;
    if (valid) {
        const uint64_t mine = ((uint64_t)key << 32) | threadIdx.x;
        ls = (hash32(key) >> 8) & LM;
        for (;;) {
            unsigned long long old = atomicCAS((unsigned long long *)&sh_tab[ls], EMPTY64, mine);
            if (old == EMPTY64) break;
            if ((uint32_t)(old >> 32) == key) {
                atomicMin((unsigned long long *)&sh_tab[ls], mine);
                break;
            }
            ls = (ls + 1) & LM;
        }
    }
    __syncthreads();
    if (valid && (uint32_t)sh_tab[ls] == threadIdx.x)
        sh_gs[ls] = table_insert_min(tab, mask, key, TENT | p, cnt);
    __syncthreads();
    slotidx[p] = valid ? sh_gs[ls] : -1;
}

// Stage 0: the seeds themselves are the keys, position = index in the seed list.
__global__ __launch_bounds__(TILE) void k_seed_insert(const int32_t *seeds, int32_t num_seeds,
                                                      int64_t num_nodes, uint64_t *tab,
                                                      uint32_t mask, int32_t *slotidx,
                                                      int32_t *cnt)
{
    __shared__ uint64_t sh_tab[2 * TILE];
    __shared__ int32_t sh_gs[2 * TILE];
    for (int i = threadIdx.x; i < 2 * TILE; i += TILE) sh_tab[i] = EMPTY64;
    __syncthreads();
    const uint32_t p = blockIdx.x * TILE + threadIdx.x;
    bool valid = p < (uint32_t)num_seeds;
    int32_t v = valid ? seeds[p] : 0;
    if (valid && (v < 0 || (int64_t)v >= num_nodes)) {
        cnt[STATUS] = BGL_EINVAL;
        valid = false;
    }
    dedup_and_insert(valid, (uint32_t)v, p, tab, mask, slotidx, sh_tab, sh_gs, cnt);
}

// Stage h+1: sample hop h.  G lanes per frontier node; lane s owns slot s.
template <int G, typename RP>
__global__ __launch_bounds__(TILE) void k_sample_insert(
    const RP *__restrict__ row_ptr, const int32_t *__restrict__ col,
    const int32_t *__restrict__ frontier, int32_t *cnt, int hop, int fanout, uint64_t h0,
    uint64_t *tab, uint32_t mask, int32_t *slotidx, int32_t *lrow, int32_t *cbs)
{
    __shared__ uint64_t sh_tab[2 * TILE];
    __shared__ int32_t sh_gs[2 * TILE];
    __shared__ int sh_scan[TILE / kWave];

    const int n_dst = cnt[hop];
    const uint32_t p = blockIdx.x * TILE + threadIdx.x;
    if ((int64_t)blockIdx.x * TILE >= (int64_t)n_dst * G) return;  // whole workgroup

    for (int i = threadIdx.x; i < 2 * TILE; i += TILE) sh_tab[i] = EMPTY64;

    const int i = (int)(p / G);
    const int s = (int)(p & (G - 1));
    const int lane = threadIdx.x & (kWave - 1);
    const int gshift = lane & ~(G - 1);
    const bool active = i < n_dst;

    int64_t lo = 0, d = 0;
    uint32_t v = 0;
    if (active) {
        v = (uint32_t)frontier[i];
        // both ends of the row with one read (the pair is only 4 or 8 bytes aligned)
        typedef RP Ends __attribute__((ext_vector_type(2), aligned(sizeof(RP))));
        const Ends ends = *reinterpret_cast<const Ends *>(row_ptr + v);
        lo = (int64_t)ends.x;
        d = (int64_t)ends.y - lo;
    }
    const int c = (int)(d < (int64_t)fanout ? d : (int64_t)fanout);
    const bool need = active && d > (int64_t)fanout;  // Floyd's algorithm, else the whole row
    const int64_t J = d - fanout + s;
    uint32_t pos = (uint32_t)s;
    if (need && s < fanout) {
        const uint64_t h1 = mix64(h0 ^ (uint64_t)v);
        const uint64_t w = mix64(h1 + GOLDEN * (uint64_t)(s + 1));
        pos = (uint32_t)__umul64hi(w, (uint64_t)(J + 1));
    }
    if (__ballot(need) != 0) {
        // Slot q keeps its draw unless an earlier slot already holds that
        // position, in which case it takes J_q.  Lanes below q are final.
        for (int q = 1; q < fanout; ++q) {
            const uint32_t tq = __shfl(pos, q, G);
            const bool coll = need && s < q && pos == tq;
            const uint64_t bal = __ballot(coll);
            const bool any = (G == kWave) ? (bal != 0)
                                          : (((bal >> gshift) & ((1ull << (G & 63)) - 1ull)) != 0);
            if (need && s == q && any) pos = (uint32_t)J;
        }
    }
    const bool valid = active && s < c;
    uint32_t u = 0;
    if (valid) u = (uint32_t)col[lo + (int64_t)pos];

    // per-node counts -> row starts inside this tile, tile total
    int total;
    const int ex = block_excl_scan<TILE>((active && s == 0) ? c : 0, sh_scan, total);
    if (active && s == 0) lrow[i] = ex;
    if (threadIdx.x == 0) cbs[blockIdx.x] = total;
    // (block_excl_scan ended with a barrier: sh_tab is initialised for everyone)
    dedup_and_insert(valid, u, p, tab, mask, slotidx, sh_tab, sh_gs, cnt);
}

// Which positions introduced a new id?  Rank them inside the tile.
__global__ __launch_bounds__(TILE) void k_flag(const int32_t *cnt, int stage, int G,
                                               int32_t num_seeds, const uint64_t *tab,
                                               const int32_t *slotidx, int32_t *lrank,
                                               int32_t *fbs)
{
    __shared__ int sh_scan[TILE / kWave];
    const int64_t P = stage == 0 ? (int64_t)num_seeds : (int64_t)cnt[stage - 1] * G;
    if ((int64_t)blockIdx.x * TILE >= P) return;
    const uint32_t p = blockIdx.x * TILE + threadIdx.x;
    int flag = 0;
    if ((int64_t)p < P) {
        const int gs = slotidx[p];
        if (gs >= 0) flag = ((uint32_t)tab[gs] == (TENT | p)) ? 1 : 0;
    }
    int total;
    const int ex = block_excl_scan<TILE>(flag, sh_scan, total);
    if ((int64_t)p < P) lrank[p] = ex;
    if (threadIdx.x == 0) fbs[blockIdx.x] = total;
}

// Prefixes over tiles and the sizes of this stage.
__global__ __launch_bounds__(1024) void k_scan_sums(int32_t *cnt, int stage, int G,
                                                    int32_t num_seeds, const int32_t *fbs,
                                                    const int32_t *cbs, int32_t *fpre,
                                                    int32_t *cpre, int32_t *row_ptr_h)
{
    __shared__ int sh_scan[1024 / kWave];
    const int n_dst = stage == 0 ? 0 : cnt[stage - 1];
    const int64_t P = stage == 0 ? (int64_t)num_seeds : (int64_t)n_dst * G;
    const int nb = (int)((P + TILE - 1) / TILE);
    int carry_f = 0, carry_c = 0;
    for (int base = 0; base < nb; base += 1024) {
        const int idx = base + threadIdx.x;
        const int f = idx < nb ? fbs[idx] : 0;
        const int c = (cbs && idx < nb) ? cbs[idx] : 0;
        int tf, tc;
        const int ef = block_excl_scan<1024>(f, sh_scan, tf);
        const int ec = block_excl_scan<1024>(c, sh_scan, tc);
        if (idx < nb) {
            fpre[idx] = carry_f + ef;
            cpre[idx] = carry_c + ec;
        }
        carry_f += tf;
        carry_c += tc;
    }
    if (threadIdx.x == 0) {
        cnt[stage] = n_dst + carry_f;
        if (stage > 0) {
            cnt[NNZ0 + stage - 1] = carry_c;
            row_ptr_h[n_dst] = carry_c;
        }
    }
}

// Local ids, frontier append, CSR block.  SELF_SCAN: the stage has at most TILE tiles and no scan
// launch; fpre / cpre then hold the tile TOTALS (what k_flag and k_sample_insert wrote), every
// workgroup scans them in LDS, and workgroup 0 publishes the stage's sizes.
template <bool SELF_SCAN>
__global__ __launch_bounds__(TILE) void k_finalize(int32_t *cnt, int stage, int logG,
                                                   int32_t num_seeds, uint64_t *tab,
                                                   const int32_t *slotidx, const int32_t *lrank,
                                                   const int32_t *fpre, const int32_t *cpre,
                                                   const int32_t *lrow, int32_t *frontier,
                                                   int32_t *row_ptr_h, int32_t *col_local)
{
    __shared__ int sh_scan[TILE / kWave];
    __shared__ int32_t sh_f[SELF_SCAN ? TILE : 1], sh_c[SELF_SCAN ? TILE : 1];
    const int n_dst = stage == 0 ? 0 : cnt[stage - 1];
    const int64_t P = stage == 0 ? (int64_t)num_seeds : ((int64_t)n_dst << logG);
    // (whole workgroups; the one that publishes the sizes stays, also for an empty stage)
    if ((int64_t)blockIdx.x * TILE >= P && !(SELF_SCAN && blockIdx.x == 0)) return;
    if constexpr (SELF_SCAN) {
        const int nb = (int)((P + TILE - 1) / TILE);  // <= TILE
        const int t = threadIdx.x;
        int tf, tc;
        sh_f[t] = block_excl_scan<TILE>(t < nb ? fpre[t] : 0, sh_scan, tf);
        sh_c[t] = block_excl_scan<TILE>((stage > 0 && t < nb) ? cpre[t] : 0, sh_scan, tc);
        __syncthreads();
        if (blockIdx.x == 0 && t == 0) {
            cnt[stage] = n_dst + tf;
            if (stage > 0) {
                cnt[NNZ0 + stage - 1] = tc;
                row_ptr_h[n_dst] = tc;
            }
        }
        fpre = sh_f;
        cpre = sh_c;
    }
    const uint32_t p = blockIdx.x * TILE + threadIdx.x;
    if ((int64_t)p >= P) return;
    const int gs = slotidx[p];
    int local = -1;
    if (gs >= 0) {
        const uint64_t e = __hip_atomic_load(&tab[gs], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t val = (uint32_t)e;
        if (val & TENT) {
            const uint32_t q = val & ~TENT;  // first position of this id
            local = n_dst + fpre[q / TILE] + lrank[q];
            if (q == p) {
                frontier[local] = (int32_t)(e >> 32);
                // Other positions of the same id may read the entry while it
                // turns from "first position" into "local id"; both forms
                // decode to the same local id.
                __hip_atomic_store(reinterpret_cast<uint32_t *>(&tab[gs]), (uint32_t)local,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            local = (int)val;
        }
    }
    if (stage > 0) {
        const int i = (int)(p >> logG);
        const int s = (int)(p & ((1u << logG) - 1));
        const int base = cpre[p / TILE] + lrow[i];
        if (s == 0) row_ptr_h[i] = base;
        if (gs >= 0) col_local[base + s] = local;
    }
}

// ------------------------------------------------------------------ host side
struct Layout {
    int K;
    int G[BGL_MAX_HOPS], logG[BGL_MAX_HOPS];
    int64_t ubf[BGL_MAX_HOPS + 1], ube[BGL_MAX_HOPS];
    int64_t P[BGL_MAX_HOPS + 1];  // padded positions per stage
    int64_t table_entries;
    size_t off_counts, off_frontier, off_row_ptr[BGL_MAX_HOPS], off_col[BGL_MAX_HOPS];
    size_t off_table, off_slotidx, off_lrank, off_lrow, off_fbs, off_cbs, off_fpre, off_cpre;
    size_t bytes;
};

int make_layout(int32_t num_seeds, const int32_t *fanouts, int32_t num_hops, int64_t num_nodes,
                Layout &L)
{
    if (num_seeds < 1) BGL_FAIL(BGL_EINVAL, "num_seeds must be >= 1 (got %d)", num_seeds);
    if (num_hops < 1 || num_hops > BGL_MAX_HOPS)
        BGL_FAIL(BGL_EINVAL, "num_hops must be in [1, %d] (got %d)", BGL_MAX_HOPS, num_hops);
    if (!fanouts) BGL_FAIL(BGL_EINVAL, "fanouts is null");
    if (num_nodes < 1 || num_nodes > INT32_MAX) BGL_FAIL(BGL_EINVAL, "num_nodes out of range");
    L.K = num_hops;
    L.ubf[0] = num_seeds < num_nodes ? num_seeds : num_nodes;
    L.P[0] = num_seeds;
    int64_t pmax = num_seeds, fmax = L.ubf[0];
    for (int h = 0; h < num_hops; ++h) {
        const int f = fanouts[h];
        if (f < 1) BGL_FAIL(BGL_EINVAL, "fanouts[%d] = %d must be >= 1", h, f);
        if (f > BGL_MAX_FANOUT)
            BGL_FAIL(BGL_EUNSUPPORTED, "fanouts[%d] = %d exceeds BGL_MAX_FANOUT = %d", h, f,
                     BGL_MAX_FANOUT);
        int g = 4, lg = 2;
        while (g < f) { g <<= 1; ++lg; }
        L.G[h] = g;
        L.logG[h] = lg;
        L.ube[h] = L.ubf[h] * f;
        L.P[h + 1] = L.ubf[h] * g;
        int64_t nxt = L.ubf[h] * (1 + (int64_t)f);
        L.ubf[h + 1] = nxt < num_nodes ? nxt : num_nodes;
        if (L.P[h + 1] > pmax) pmax = L.P[h + 1];
        if (L.ubf[h] > fmax) fmax = L.ubf[h];
        if (L.P[h + 1] >= (int64_t)TENT || L.ube[h] >= (int64_t)TENT)
            BGL_FAIL(BGL_EUNSUPPORTED, "hop %d is too large for 31-bit positions", h);
    }
    int64_t need = L.ubf[num_hops] + L.ubf[num_hops] / 3 + 1;
    int64_t ts = 1024;
    while (ts < need) ts <<= 1;
    L.table_entries = ts;
    const int64_t nbmax = bgl::ceil_div(pmax, TILE) + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += bgl::round_up(bytes, 256); return o; };
    L.off_counts = take(sizeof(int32_t) * BGL_COUNTS_LEN);
    L.off_frontier = take(sizeof(int32_t) * (size_t)L.ubf[num_hops]);
    for (int h = 0; h < num_hops; ++h) {
        L.off_row_ptr[h] = take(sizeof(int32_t) * (size_t)(L.ubf[h] + 1));
        L.off_col[h] = take(sizeof(int32_t) * (size_t)L.ube[h]);
    }
    L.off_table = take(sizeof(uint64_t) * (size_t)ts);
    const size_t ppad = bgl::round_up((size_t)pmax, TILE);
    L.off_slotidx = take(sizeof(int32_t) * ppad);
    L.off_lrank = take(sizeof(int32_t) * ppad);
    L.off_lrow = take(sizeof(int32_t) * (size_t)fmax);
    L.off_fbs = take(sizeof(int32_t) * (size_t)nbmax);
    L.off_cbs = take(sizeof(int32_t) * (size_t)nbmax);
    L.off_fpre = take(sizeof(int32_t) * (size_t)nbmax);
    L.off_cpre = take(sizeof(int32_t) * (size_t)nbmax);
    L.bytes = off;
    return BGL_OK;
}

template <int G, typename RP>
void launch_sample(const bgl_graph *g, int blocks, hipStream_t st, const int32_t *frontier,
                   int32_t *cnt, int hop, int fanout, uint64_t h0, uint64_t *tab, uint32_t mask,
                   int32_t *slotidx, int32_t *lrow, int32_t *cbs)
{
    hipLaunchKernelGGL((k_sample_insert<G, RP>), dim3(blocks), dim3(TILE), 0, st,
                       static_cast<const RP *>(g->row_ptr), g->col, frontier, cnt, hop, fanout,
                       h0, tab, mask, slotidx, lrow, cbs);
}

template <typename RP>
void launch_sample_g(int G, const bgl_graph *g, int blocks, hipStream_t st,
                     const int32_t *frontier, int32_t *cnt, int hop, int fanout, uint64_t h0,
                     uint64_t *tab, uint32_t mask, int32_t *slotidx, int32_t *lrow, int32_t *cbs)
{
    switch (G) {
    case 4: launch_sample<4, RP>(g, blocks, st, frontier, cnt, hop, fanout, h0, tab, mask, slotidx, lrow, cbs); break;
    case 8: launch_sample<8, RP>(g, blocks, st, frontier, cnt, hop, fanout, h0, tab, mask, slotidx, lrow, cbs); break;
    case 16: launch_sample<16, RP>(g, blocks, st, frontier, cnt, hop, fanout, h0, tab, mask, slotidx, lrow, cbs); break;
    case 32: launch_sample<32, RP>(g, blocks, st, frontier, cnt, hop, fanout, h0, tab, mask, slotidx, lrow, cbs); break;
    default: launch_sample<64, RP>(g, blocks, st, frontier, cnt, hop, fanout, h0, tab, mask, slotidx, lrow, cbs); break;
    }
}

}  // namespace

extern "C" int bgl_sample_workspace_bytes(int32_t num_seeds, const int32_t *fanouts,
                                          int32_t num_hops, int64_t num_nodes, size_t *bytes)
try {
    if (!bytes) BGL_FAIL(BGL_EINVAL, "bytes is null");
    Layout L;
    int rc = make_layout(num_seeds, fanouts, num_hops, num_nodes, L);
    if (rc != BGL_OK) return rc;
    *bytes = L.bytes;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_sample_khop(const bgl_graph_t *g, const int32_t *seeds, int32_t num_seeds,
                               const int32_t *fanouts, int32_t num_hops, uint64_t rng_seed,
                               void *workspace, size_t workspace_bytes, bgl_subgraph_t *out,
                               int32_t *counts_host, void *stream)
try {
    if (!g) BGL_FAIL(BGL_EINVAL, "graph handle is null");
    if (!seeds) BGL_FAIL(BGL_EINVAL, "seeds is null");
    if (!out) BGL_FAIL(BGL_EINVAL, "out is null");
    if (!workspace || !bgl::aligned(workspace, 256))
        BGL_FAIL(BGL_EINVAL, "workspace is null or not 256-byte aligned");
    Layout L;
    int rc = make_layout(num_seeds, fanouts, num_hops, g->num_nodes, L);
    if (rc != BGL_OK) return rc;
    if (workspace_bytes < L.bytes)
        BGL_FAIL(BGL_ECAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, L.bytes);

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    int32_t *cnt = reinterpret_cast<int32_t *>(ws + L.off_counts);
    int32_t *frontier = reinterpret_cast<int32_t *>(ws + L.off_frontier);
    uint64_t *tab = reinterpret_cast<uint64_t *>(ws + L.off_table);
    int32_t *slotidx = reinterpret_cast<int32_t *>(ws + L.off_slotidx);
    int32_t *lrank = reinterpret_cast<int32_t *>(ws + L.off_lrank);
    int32_t *lrow = reinterpret_cast<int32_t *>(ws + L.off_lrow);
    int32_t *fbs = reinterpret_cast<int32_t *>(ws + L.off_fbs);
    int32_t *cbs = reinterpret_cast<int32_t *>(ws + L.off_cbs);
    int32_t *fpre = reinterpret_cast<int32_t *>(ws + L.off_fpre);
    int32_t *cpre = reinterpret_cast<int32_t *>(ws + L.off_cpre);
    const uint32_t mask = (uint32_t)(L.table_entries - 1);

    out->num_hops = num_hops;
    out->input_nodes = frontier;
    out->counts = cnt;
    for (int h = 0; h <= BGL_MAX_HOPS; ++h) out->cap_nodes[h] = h <= num_hops ? L.ubf[h] : 0;
    for (int h = 0; h < BGL_MAX_HOPS; ++h) {
        out->row_ptr[h] = h < num_hops ? reinterpret_cast<int32_t *>(ws + L.off_row_ptr[h]) : nullptr;
        out->col_local[h] = h < num_hops ? reinterpret_cast<int32_t *>(ws + L.off_col[h]) : nullptr;
        out->cap_edges[h] = h < num_hops ? L.ube[h] : 0;
    }

    {
        int blocks = (int)std::min<int64_t>(bgl::ceil_div(L.table_entries, 1024), 4096);
        hipLaunchKernelGGL(k_prepare, dim3(blocks), dim3(256), 0, st, tab, L.table_entries, EMPTY64, cnt);
    }
    // stage 0: unique seeds
    {
        const int blocks = (int)bgl::ceil_div(L.P[0], TILE);
        hipLaunchKernelGGL(k_seed_insert, dim3(blocks), dim3(TILE), 0, st, seeds, num_seeds,
                           g->num_nodes, tab, mask, slotidx, cnt);
        hipLaunchKernelGGL(k_flag, dim3(blocks), dim3(TILE), 0, st, cnt, 0, 1, num_seeds, tab,
                           slotidx, lrank, fbs);
        if (blocks <= TILE) {
            hipLaunchKernelGGL(k_finalize<true>, dim3(blocks), dim3(TILE), 0, st, cnt, 0, 0, num_seeds, tab,
                               slotidx, lrank, fbs, cbs, lrow, frontier, (int32_t *)nullptr, (int32_t *)nullptr);
        } else {
            hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(1024), 0, st, cnt, 0, 1, num_seeds, fbs,
                               (const int32_t *)nullptr, fpre, cpre, (int32_t *)nullptr);
            hipLaunchKernelGGL(k_finalize<false>, dim3(blocks), dim3(TILE), 0, st, cnt, 0, 0, num_seeds, tab,
                               slotidx, lrank, fpre, cpre, lrow, frontier, (int32_t *)nullptr,
                               (int32_t *)nullptr);
        }
    }
    for (int h = 0; h < num_hops; ++h) {
        const int blocks = (int)bgl::ceil_div(L.P[h + 1], TILE);
        const uint64_t h0 = mix64(rng_seed + GOLDEN * (uint64_t)(h + 1));
        if (g->bits == 64)
            launch_sample_g<int64_t>(L.G[h], g, blocks, st, frontier, cnt, h, fanouts[h], h0, tab,
                                     mask, slotidx, lrow, cbs);
        else
            launch_sample_g<int32_t>(L.G[h], g, blocks, st, frontier, cnt, h, fanouts[h], h0, tab,
                                     mask, slotidx, lrow, cbs);
        hipLaunchKernelGGL(k_flag, dim3(blocks), dim3(TILE), 0, st, cnt, h + 1, L.G[h], num_seeds,
                           tab, slotidx, lrank, fbs);
        if (blocks <= TILE) {
            hipLaunchKernelGGL(k_finalize<true>, dim3(blocks), dim3(TILE), 0, st, cnt, h + 1, L.logG[h],
                               num_seeds, tab, slotidx, lrank, fbs, cbs, lrow, frontier,
                               out->row_ptr[h], out->col_local[h]);
        } else {
            hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(1024), 0, st, cnt, h + 1, L.G[h], num_seeds,
                               fbs, cbs, fpre, cpre, out->row_ptr[h]);
            hipLaunchKernelGGL(k_finalize<false>, dim3(blocks), dim3(TILE), 0, st, cnt, h + 1, L.logG[h],
                               num_seeds, tab, slotidx, lrank, fpre, cpre, lrow, frontier,
                               out->row_ptr[h], out->col_local[h]);
        }
    }
    BGL_HIP(hipGetLastError());
    if (counts_host)
        BGL_HIP(hipMemcpyAsync(counts_host, cnt, sizeof(int32_t) * BGL_COUNTS_LEN,
                               hipMemcpyDeviceToHost, st));
    return BGL_OK;
} BGL_NOTHROW_END
