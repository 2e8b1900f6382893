/*
 * Seeded synthetic inputs for the minibatch-preparation path: power-law CSR
 * graphs and feature tables.  These are inputs
 * only: nothing here belongs to the sampling or caching method, and this file
 * has its own random-number generator (a counter hash built on the MurmurHash3
 * 64-bit finaliser) so that it shares no arithmetic with either the HIP library
 * or the CPU oracle.
 *
 * Results depend only on the arguments, never on the number of threads: every
 * node (or feature row) owns a private random stream.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t fmix64(uint64_t k)
{
    k ^= k >> 33;
    k *= 0xff51afd7ed558ccdULL;
    k ^= k >> 33;
    k *= 0xc4ceb9fe1a85ec53ULL;
    k ^= k >> 33;
    return k;
}

/* counter-based word: (seed, stream, counter) -> 64 bits */
static inline uint64_t gen_word(uint64_t seed, uint64_t stream, uint64_t counter)
{
    uint64_t a = fmix64(seed ^ 0x243F6A8885A308D3ULL);
    uint64_t b = fmix64(a + 0xD1B54A32D192ED03ULL * (stream + 1));
    return fmix64(b ^ (0x8CB92BA72F3D8DD7ULL * (counter + 1)));
}

static inline double gen_unit(uint64_t w) /* (0,1) */
{
    return ((double)(w >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

/* mean of the truncated discrete power law P(d) ~ d^-alpha on [dmin, dmax] */
static double powerlaw_mean(double alpha, int64_t dmin, int64_t dmax)
{
    double num = 0.0, den = 0.0;
    for (int64_t d = dmin; d <= dmax; ++d) {
        double w = pow((double)d, -alpha);
        num += w * (double)d;
        den += w;
    }
    return num / den;
}

/* Out-degrees from a truncated power law whose exponent is solved (bisection)
 * for the requested mean.  deg[N] receives the degrees; returns their sum, or
 * -1 on bad arguments. */
int64_t bglgen_degrees(int64_t num_nodes, double mean_degree, int64_t dmin, int64_t dmax,
                       uint64_t seed, int32_t *deg)
{
    if (num_nodes <= 0 || dmin < 1 || dmax < dmin || mean_degree < (double)dmin ||
        mean_degree > (double)dmax) return -1;
    double lo = 0.0, hi = 12.0; /* mean decreases as alpha grows */
    for (int it = 0; it < 60; ++it) {
        double mid = 0.5 * (lo + hi);
        if (powerlaw_mean(mid, dmin, dmax) > mean_degree) lo = mid; else hi = mid;
    }
    double alpha = 0.5 * (lo + hi);
    int64_t span = dmax - dmin + 1;
    double *cdf = (double *)malloc(sizeof(double) * (size_t)span);
    if (!cdf) return -1;
    double acc = 0.0;
    for (int64_t d = dmin; d <= dmax; ++d) { acc += pow((double)d, -alpha); cdf[d - dmin] = acc; }
    for (int64_t d = 0; d < span; ++d) cdf[d] /= acc;
    int64_t total = 0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (int64_t v = 0; v < num_nodes; ++v) {
        double u = gen_unit(gen_word(seed, (uint64_t)v, 0));
        int64_t a = 0, b = span - 1;
        while (a < b) { int64_t m = (a + b) >> 1; if (cdf[m] < u) a = m + 1; else b = m; }
        deg[v] = (int32_t)(a + dmin);
        total += a + dmin;
    }
    free(cdf);
    return total;
}

/* exclusive prefix sum of deg into row_ptr (32- or 64-bit); returns the total */
int64_t bglgen_row_ptr(int64_t num_nodes, const int32_t *deg, void *row_ptr, int bits)
{
    int64_t acc = 0;
    for (int64_t v = 0; v < num_nodes; ++v) {
        if (bits == 64) ((int64_t *)row_ptr)[v] = acc; else ((int32_t *)row_ptr)[v] = (int32_t)acc;
        acc += deg[v];
    }
    if (bits == 64) ((int64_t *)row_ptr)[num_nodes] = acc; else ((int32_t *)row_ptr)[num_nodes] = (int32_t)acc;
    return acc;
}

/* seeded Fisher-Yates permutation of 0..N-1 and its inverse */
void bglgen_permutation(int64_t n, uint64_t seed, int32_t *perm, int32_t *inv)
{
    for (int64_t i = 0; i < n; ++i) perm[i] = (int32_t)i;
    for (int64_t i = n - 1; i > 0; --i) {
        uint64_t w = gen_word(seed, 0x5eed, (uint64_t)i);
        int64_t j = (int64_t)(((unsigned __int128)w * (unsigned __int128)(i + 1)) >> 64);
        int32_t t = perm[i]; perm[i] = perm[j]; perm[j] = t;
    }
    if (inv) for (int64_t i = 0; i < n; ++i) inv[perm[i]] = (int32_t)i;
}

/* Zipf-like rank in [0, n): density ~ (r+1)^-beta, by inverting the continuous CDF */
static inline int64_t zipf_rank(double u, int64_t n, double beta)
{
    double r;
    if (fabs(beta - 1.0) < 1e-9) {
        r = exp(u * log((double)n + 1.0)) - 1.0;
    } else {
        double e = 1.0 - beta;
        r = pow(u * (pow((double)n + 1.0, e) - 1.0) + 1.0, 1.0 / e) - 1.0;
    }
    int64_t k = (int64_t)r;
    if (k < 0) k = 0;
    if (k >= n) k = n - 1;
    return k;
}

/* Edge destinations.  Nodes live, in a hidden "generation order", on a ring of
 * num_nodes positions.  With probability p_local an edge is a short-range one: it
 * goes to the position at a signed distance from the source drawn from an
 * exponential law of mean `reach` (of two such draws the one that lands on the
 * more "popular" position is kept, popularity being a fixed hash of the
 * position: a mild local skew of the in-degree).  Otherwise it goes to one of
 * num_hubs hub positions scattered over the ring, chosen by a Zipf law over
 * their ranks (heavy-tailed in-degree).  The
 * short-range edges give the graph a geometry: a breadth-first traversal grows
 * region by region over many levels instead of reaching everything in two or
 * three, so that nodes that follow each other in a breadth-first order have
 * neighborhoods that overlap, which is the property of real graphs that
 * proximity-aware ordering (Sec. 3.2.2 of the paper) relies on; a graph whose
 * edges all go to ranks of a large block, or a pure configuration model, is an
 * expander and shows none of it.  perm maps generation order -> node id, inv is
 * its inverse, so that node ids carry no locality.  Rows are not sorted;
 * repeated edges and self loops stay. */
int bglgen_edges(int64_t num_nodes, const void *row_ptr, int bits, int32_t *col,
                 uint64_t seed, int64_t reach, double p_local, double beta, int64_t num_hubs,
                 const int32_t *perm, const int32_t *inv)
{
    if (num_nodes <= 0 || reach <= 0 || num_hubs <= 0) return -1;
    if (num_hubs > num_nodes) num_hubs = num_nodes;
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t v = 0; v < num_nodes; ++v) {
        int64_t lo = bits == 64 ? ((const int64_t *)row_ptr)[v] : ((const int32_t *)row_ptr)[v];
        int64_t hi = bits == 64 ? ((const int64_t *)row_ptr)[v + 1] : ((const int32_t *)row_ptr)[v + 1];
        int64_t g = inv[v];
        for (int64_t e = lo; e < hi; ++e) {
            uint64_t c = (uint64_t)(e - lo);
            uint64_t w0 = gen_word(seed, (uint64_t)v, 3 * c + 1);
            double u1 = gen_unit(gen_word(seed, (uint64_t)v, 3 * c + 2));
            int64_t dst_g;
            if (gen_unit(w0) < p_local) {
                double u2 = gen_unit(gen_word(seed, (uint64_t)v, 3 * c + 3));
                int64_t best = g;
                uint64_t best_pop = 0;
                for (int k = 0; k < 2; ++k) {
                    double u = k == 0 ? u1 : u2;
                    int64_t d = 1 + (int64_t)(-(double)reach * log(u));
                    if (d >= num_nodes) d = num_nodes - 1;
                    int64_t cand = ((w0 >> k) & 1) ? g + d : g - d;
                    cand %= num_nodes;
                    if (cand < 0) cand += num_nodes;
                    uint64_t pop = fmix64((uint64_t)cand * 0x9FB21C651E98DF25ULL + seed);
                    if (k == 0 || pop > best_pop) { best = cand; best_pop = pop; }
                }
                dst_g = best;
            } else {
                /* one of num_hubs hub positions, Zipf-ranked; the hubs are scattered over the ring */
                dst_g = (int64_t)(fmix64((uint64_t)zipf_rank(u1, num_hubs, beta) + 0x632BE59BD9B4E019ULL * (seed | 1)) %
                                  (uint64_t)num_nodes);
            }
            col[e] = perm[dst_g];
        }
    }
    return 0;
}

/* Features ~ N(0,1) by Box-Muller.  elem_bytes 4: IEEE fp32; 2: bfloat16
 * (round to nearest even of the fp32 value). */
int bglgen_features(int64_t num_rows, int32_t dim, int32_t elem_bytes, uint64_t seed, void *out)
{
    if (num_rows < 0 || dim <= 0 || (elem_bytes != 4 && elem_bytes != 2)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < num_rows; ++r) {
        for (int32_t j = 0; j < dim; j += 2) {
            double u1 = gen_unit(gen_word(seed, (uint64_t)r, (uint64_t)j));
            double u2 = gen_unit(gen_word(seed, (uint64_t)r, (uint64_t)j + 1));
            double rad = sqrt(-2.0 * log(u1));
            float z[2] = {(float)(rad * cos(6.283185307179586 * u2)),
                          (float)(rad * sin(6.283185307179586 * u2))};
            for (int q = 0; q < 2 && j + q < dim; ++q) {
                if (elem_bytes == 4) {
                    ((float *)out)[r * dim + j + q] = z[q];
                } else {
                    uint32_t b;
                    memcpy(&b, &z[q], 4);
                    b += 0x7FFFu + ((b >> 16) & 1u);
                    ((uint16_t *)out)[r * dim + j + q] = (uint16_t)(b >> 16);
                }
            }
        }
    }
    return 0;
}
