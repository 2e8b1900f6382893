/*
 * Hit-ratio simulators for the cache policies the BGL paper compares FIFO with
 * (Sec. 2.3 and Sec. 3.2.1: a static degree-based cache as in PaGraph, LRU and
 * LFU).  Analysis tools for the policy study only: they track which node ids
 * are cached, not feature rows, and are not part of the minibatch path (the
 * library's cache is FIFO, as the paper chooses).
 *
 * Every simulator consumes one batch of distinct ids at a time.  Lookups see the
 * state at batch entry (as the FIFO cache's lookup does); then the batch's ids
 * update the state in order.
 */
#include <stdint.h>
#include <stdlib.h>

#define NIL (-1)

typedef struct {
    int kind;          /* 0 static, 1 LRU, 2 LFU */
    int64_t n, cap, size;
    /* LRU / LFU: doubly linked lists over node ids */
    int32_t *prev, *next;
    uint8_t *in;       /* cached? */
    int32_t head, tail; /* LRU: head = most recent, tail = least recent */
    /* LFU: per-frequency lists; freq[v]; list f has fhead[f] (most recent) / ftail[f] */
    int32_t *freq, *fhead, *ftail;
    int64_t fcap;      /* allocated frequencies */
    int32_t minf;
    uint8_t *hitbuf;
    int64_t hitcap;
} psim;

psim *psim_create(int kind, int64_t num_nodes, int64_t capacity)
{
    psim *s = (psim *)calloc(1, sizeof(psim));
    s->kind = kind; s->n = num_nodes; s->cap = capacity;
    s->in = (uint8_t *)calloc((size_t)num_nodes, 1);
    s->prev = (int32_t *)malloc(sizeof(int32_t) * (size_t)num_nodes);
    s->next = (int32_t *)malloc(sizeof(int32_t) * (size_t)num_nodes);
    s->head = s->tail = NIL;
    if (kind == 2) {
        s->freq = (int32_t *)calloc((size_t)num_nodes, sizeof(int32_t));
        s->fcap = 1024;
        s->fhead = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->fcap);
        s->ftail = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->fcap);
        for (int64_t f = 0; f < s->fcap; ++f) s->fhead[f] = s->ftail[f] = NIL;
        s->minf = 1;
    }
    return s;
}

void psim_destroy(psim *s)
{
    if (!s) return;
    free(s->in); free(s->prev); free(s->next); free(s->freq); free(s->fhead); free(s->ftail); free(s->hitbuf); free(s);
}

/* static policy: the cached set is fixed up front */
void psim_static_fill(psim *s, const int32_t *ids, int64_t count)
{
    for (int64_t i = 0; i < count && i < s->cap; ++i) s->in[ids[i]] = 1;
}

static void lru_unlink(psim *s, int32_t v)
{
    if (s->prev[v] != NIL) s->next[s->prev[v]] = s->next[v]; else s->head = s->next[v];
    if (s->next[v] != NIL) s->prev[s->next[v]] = s->prev[v]; else s->tail = s->prev[v];
}

static void lru_push_front(psim *s, int32_t v)
{
    s->prev[v] = NIL; s->next[v] = s->head;
    if (s->head != NIL) s->prev[s->head] = v; else s->tail = v;
    s->head = v;
}

static void lfu_grow(psim *s, int64_t f)
{
    if (f < s->fcap) return;
    int64_t nc = s->fcap;
    while (nc <= f) nc *= 2;
    s->fhead = (int32_t *)realloc(s->fhead, sizeof(int32_t) * (size_t)nc);
    s->ftail = (int32_t *)realloc(s->ftail, sizeof(int32_t) * (size_t)nc);
    for (int64_t k = s->fcap; k < nc; ++k) s->fhead[k] = s->ftail[k] = NIL;
    s->fcap = nc;
}

static void lfu_unlink(psim *s, int32_t v)
{
    int32_t f = s->freq[v];
    if (s->prev[v] != NIL) s->next[s->prev[v]] = s->next[v]; else s->fhead[f] = s->next[v];
    if (s->next[v] != NIL) s->prev[s->next[v]] = s->prev[v]; else s->ftail[f] = s->prev[v];
}

static void lfu_push_front(psim *s, int32_t v, int32_t f)
{
    lfu_grow(s, f);
    s->freq[v] = f;
    s->prev[v] = NIL; s->next[v] = s->fhead[f];
    if (s->fhead[f] != NIL) s->prev[s->fhead[f]] = v; else s->ftail[f] = v;
    s->fhead[f] = v;
}

/* One batch of distinct ids; returns the number of hits. */
int64_t psim_batch(psim *s, const int32_t *ids, int64_t n)
{
    if (n > s->hitcap) { free(s->hitbuf); s->hitbuf = (uint8_t *)malloc((size_t)n); s->hitcap = n; }
    int64_t hits = 0;
    for (int64_t i = 0; i < n; ++i) { s->hitbuf[i] = s->in[ids[i]]; hits += s->hitbuf[i]; }
    if (s->kind == 0) return hits;
    for (int64_t i = 0; i < n; ++i) {
        int32_t v = ids[i];
        if (s->kind == 1) {                    /* LRU */
            if (s->in[v]) { lru_unlink(s, v); lru_push_front(s, v); continue; }
            if (s->size == s->cap) { int32_t t = s->tail; lru_unlink(s, t); s->in[t] = 0; s->size--; }
            lru_push_front(s, v); s->in[v] = 1; s->size++;
        } else {                               /* LFU, ties evict the least recently used */
            if (s->in[v]) {
                int32_t f = s->freq[v];
                lfu_unlink(s, v);
                if (f == s->minf && s->fhead[f] == NIL) s->minf = f + 1;
                lfu_push_front(s, v, f + 1);
                continue;
            }
            if (s->size == s->cap) {
                while (s->ftail[s->minf] == NIL) s->minf++;
                int32_t t = s->ftail[s->minf];
                lfu_unlink(s, t); s->in[t] = 0; s->size--;
            }
            lfu_push_front(s, v, 1); s->in[v] = 1; s->size++; s->minf = 1;
        }
    }
    return hits;
}
