/*
 * CPU oracle for the cache-enabled embedding step of HET (arXiv 2112.07221).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, one-key-at-a-time execution of the
 * paper's client protocol on host arrays.  It exists so that tests and the benchmark's CPU
 * baseline leg can check and time the rules themselves; nothing in the GPU library includes,
 * links or calls it, and it includes nothing from the GPU library.
 *
 * What it follows (all from the paper):
 *   Section 3.1  Cache Management: global clock c_g per global row, start clock c_s and
 *                local clock c_c per cached row; Fetch, Evict(key), Evict(), CheckValid.
 *   Algorithm 1  client loop: unique key set of the minibatch, Read, Write.
 *   Algorithm 2  Read: Find, CheckValid, Evict+Fetch of an invalid row, Fetch of an absent one, Get.
 *   Algorithm 3  Write: Update + Clock per key, then Evict() of the overflow.
 *   Section 4.3  cache policies LRU and LFU.
 *
 * Readings where the paper is silent (single worker, one cache, one server table):
 *   - Update applies the optimizer step to the cached row; Evict copies the row (and the
 *     Adagrad accumulator) to the global table.  With one writer this equals pushing the
 *     accumulated change and having the server add it.
 *   - c_c grows by one per Write call per unique key, whatever the key's multiplicity.
 *   - Evict(k)+Fetch(k) of a resident row keeps its slot and its policy counters.
 *   - Rows fetched on a miss are added beyond the capacity; the overflow is trimmed by Evict()
 *     at the end of Write (or at the start of a Read that follows a Read).
 *   - A "use" is membership in the unique key set of a Read.  LRU orders by (last_use, slot),
 *     LFU by (freq, last_use, slot), ascending; the first size-C entries are evicted.
 *   - Missed keys in ascending key order take free slots in ascending slot order.
 *   - A row with c_c == c_s has accumulated nothing and is not written back.
 *   - Duplicate gradients of one key are summed in order of increasing position.
 *   - Adagrad: a += g*g; x -= lr * g / (sqrt(a) + eps); the accumulator travels with the row.
 *   - flush() writes every dirty resident row back (the paper allows dropping them instead).
 *
 * Several workers (het_oracle_set_many_writers): the literal form of Evict in Section 3.1.  Every
 * worker has a cache of its own over the one global table.  Evict pushes what the worker has
 * accumulated on the row since it fetched it (row now minus row as fetched; for SGD exactly the
 * scaled sum of its gradients) and the server adds that to the global row, c_g = max(c_g, c_c).
 * Fetch therefore keeps a copy of the row as fetched.  After a flush the replica keeps its own
 * view and counts further changes from there.  CheckValid's second condition, c_g <= c_c + s, now
 * matters: another worker's pushes advance c_g (Lemma 1 bounds the replicas' clocks through it).
 * het_oracle_foreign_update is a push by a worker that is not modelled otherwise: the server adds
 * a delta to the global row and advances its clock by one.
 *
 * Row-wise Adagrad (not in the paper; a common half-state variant for embedding tables): one
 * accumulator per row, a += mean_j(g_j^2); x_j -= lr * g_j / (sqrt(a) + eps).  The accumulator
 * arrays then hold one value per row (A[V], one per cached row) and travel with the row as before.
 *
 * Light-weight LFU (Section 4.3: once an embedding's frequency is "high enough" it is accessed
 * directly and its frequency is no longer maintained; the paper gives no threshold): LFU whose
 * use counter stops at a cap (het_oracle_set_lfu_cap, default 16).  A row whose counter has
 * reached the cap is no longer touched by Reads: neither its counter nor its last-use stamp moves.
 * It is an approximation of LFU by design; tests compare its miss rate with exact LFU's.
 *
 * Floating point is HET_REAL (double unless overridden at compile time); compile with
 * -ffp-contract=off so that every operation rounds once.
 *
 * Pins (tests/test_oracle_*.py): a hand-worked trace, a list-based brute-force twin on tiny
 * inputs, a dense uncached trainer, the SGD closed form, a library Adagrad, clock-drift and
 * size invariants, the closed-form refresh count when nothing is evicted, and c_g equal to the
 * number of iterations that touched the key.  Several workers (tests/test_oracle_multiwriter.py):
 * with one worker the delta push equals the write-back; with two workers and SGD the flushed table
 * equals the initial one minus lr times the sum of all gradients of both; CheckValid's bounds
 * after every Read and Lemma 1's 2s bound at a common global clock; a two-worker brute-force twin.
 * Which IDs LRU/LFU evict on the paper's own datasets is "parity unpinned": the paper prints no
 * worked example for it.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifndef HET_REAL
#define HET_REAL double
#endif
typedef HET_REAL real;

enum { POLICY_LRU = 0, POLICY_LFU = 1, POLICY_LFU_LIGHT = 3 };   /* (2 is the GPU library's "no cache") */
enum { OPT_SGD = 0, OPT_ADAGRAD = 1, OPT_ADAGRAD_ROW = 2 };
enum { CLS_HIT = 0, CLS_STALE = 1, CLS_MISS = 2 };
enum { ERR_NONE = 0, ERR_RANGE = 1, ERR_STATE = 2, ERR_ARG = 4 };

typedef struct {
    int64_t n, U, hit, stale, miss, evicted, evicted_dirty, stale_dirty, flushed;
} call_stats;

typedef struct het_oracle {
    /* configuration */
    int64_t C, P, max_ids, s;
    int32_t dim, policy, opt;
    int32_t sdim;            /* optimizer state per row: dim (Adagrad), 1 (row-wise Adagrad); unused for SGD */
    int32_t many;            /* several workers write the global table: Evict pushes deltas */
    uint32_t lfu_cap;        /* light-weight LFU: the use counter stops here */
    real eps;
    /* global table (caller's arrays) */
    real *W, *A;
    uint32_t *Cg;
    int64_t V;
    /* cache slots 0..P-1 */
    int64_t *key;            /* -1 = free */
    real *row, *acc;
    real *row0, *acc0;       /* many writers: the row (accumulator) as it was fetched */
    uint32_t *cs, *cc, *last_use, *freq;
    int64_t *slot_of;        /* [V], -1 = not cached: Cache.Find */
    int64_t size;
    uint32_t t;              /* number of non-empty Reads so far */
    /* records of the last calls, for comparison */
    int64_t *lk_key;
    int32_t *lk_cls;
    int64_t *lk_slot;
    int64_t lk_U;
    int64_t *ev_id;
    int64_t ev_n;
    call_stats last, total;
    int32_t err;
} het_oracle;

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

het_oracle *het_oracle_create(int64_t capacity, int32_t dim, int64_t s, int32_t policy,
                              int64_t max_batch_ids, int32_t optimizer, double eps)
{
    if (capacity <= 0 || dim <= 0 || s < 0 || max_batch_ids <= 0) return NULL;
    if (policy != POLICY_LRU && policy != POLICY_LFU && policy != POLICY_LFU_LIGHT) return NULL;
    if (optimizer != OPT_SGD && optimizer != OPT_ADAGRAD && optimizer != OPT_ADAGRAD_ROW) return NULL;
    het_oracle *o = (het_oracle *)calloc(1, sizeof(*o));
    o->lfu_cap = 16;
    o->sdim = optimizer == OPT_ADAGRAD_ROW ? 1 : dim;
    o->C = capacity; o->dim = dim; o->s = s; o->policy = policy;
    o->max_ids = max_batch_ids; o->opt = optimizer; o->eps = (real)eps;
    o->P = capacity + max_batch_ids;
    o->key = (int64_t *)malloc(sizeof(int64_t) * o->P);
    for (int64_t i = 0; i < o->P; ++i) o->key[i] = -1;
    o->row = (real *)calloc((size_t)o->P * dim, sizeof(real));
    o->acc = (real *)calloc((size_t)o->P * dim, sizeof(real));
    o->cs = (uint32_t *)calloc(o->P, sizeof(uint32_t));
    o->cc = (uint32_t *)calloc(o->P, sizeof(uint32_t));
    o->last_use = (uint32_t *)calloc(o->P, sizeof(uint32_t));
    o->freq = (uint32_t *)calloc(o->P, sizeof(uint32_t));
    o->lk_key = (int64_t *)malloc(sizeof(int64_t) * max_batch_ids);
    o->lk_cls = (int32_t *)malloc(sizeof(int32_t) * max_batch_ids);
    o->lk_slot = (int64_t *)malloc(sizeof(int64_t) * max_batch_ids);
    o->ev_id = (int64_t *)malloc(sizeof(int64_t) * o->P);
    return o;
}

/* W[V][dim], A[V][dim] (may be NULL for SGD), Cg[V] zero-initialised; all owned by the caller. */
int het_oracle_attach(het_oracle *o, real *W, real *A, uint32_t *Cg, int64_t V)
{
    if (!o || !W || !Cg || V <= 0) return ERR_ARG;
    if (o->opt != OPT_SGD && !A) return ERR_ARG;
    o->W = W; o->A = A; o->Cg = Cg; o->V = V;
    free(o->slot_of);
    o->slot_of = (int64_t *)malloc(sizeof(int64_t) * V);
    for (int64_t k = 0; k < V; ++k) o->slot_of[k] = -1;
    return ERR_NONE;
}

void het_oracle_destroy(het_oracle *o)
{
    if (!o) return;
    free(o->key); free(o->row); free(o->acc); free(o->row0); free(o->acc0); free(o->cs); free(o->cc);
    free(o->last_use); free(o->freq); free(o->slot_of);
    free(o->lk_key); free(o->lk_cls); free(o->lk_slot); free(o->ev_id);
    free(o);
}

/* Light-weight LFU: where the use counter stops (at least 1). */
int het_oracle_set_lfu_cap(het_oracle *o, uint32_t cap)
{
    if (!o || cap == 0) return ERR_ARG;
    o->lfu_cap = cap;
    return ERR_NONE;
}

/* Call right after create: this cache is one of several workers' over one global table. */
int het_oracle_set_many_writers(het_oracle *o)
{
    if (!o || o->W) return ERR_ARG;
    o->many = 1;
    o->row0 = (real *)calloc((size_t)o->P * o->dim, sizeof(real));
    o->acc0 = (real *)calloc((size_t)o->P * o->dim, sizeof(real));
    return ERR_NONE;
}

/* Evict's push: the server takes the row and c_g = max(c_g, c_c)   (Section 3.1, Evict).
 * Several workers: it takes what this worker accumulated since its Fetch and adds it. */
static int write_back(het_oracle *o, int64_t slot)
{
    int64_t k = o->key[slot];
    if (o->cc[slot] == o->cs[slot]) return 0;          /* nothing accumulated */
    if (o->many) {
        for (int32_t j = 0; j < o->dim; ++j) {
            real d = o->row[(size_t)slot * o->dim + j] - o->row0[(size_t)slot * o->dim + j];
            o->W[(size_t)k * o->dim + j] = o->W[(size_t)k * o->dim + j] + d;
            if (o->opt != OPT_SGD && j < o->sdim) {
                real da = o->acc[(size_t)slot * o->sdim + j] - o->acc0[(size_t)slot * o->sdim + j];
                o->A[(size_t)k * o->sdim + j] = o->A[(size_t)k * o->sdim + j] + da;
            }
        }
    } else {
        memcpy(o->W + (size_t)k * o->dim, o->row + (size_t)slot * o->dim, sizeof(real) * o->dim);
        if (o->opt != OPT_SGD)
            memcpy(o->A + (size_t)k * o->sdim, o->acc + (size_t)slot * o->sdim, sizeof(real) * o->sdim);
    }
    if (o->cc[slot] > o->Cg[k]) o->Cg[k] = o->cc[slot];
    return 1;
}

/* Several workers: from here on the replica counts its changes anew. */
static void rebase(het_oracle *o, int64_t slot)
{
    if (!o->many) return;
    memcpy(o->row0 + (size_t)slot * o->dim, o->row + (size_t)slot * o->dim, sizeof(real) * o->dim);
    if (o->opt != OPT_SGD)
        memcpy(o->acc0 + (size_t)slot * o->sdim, o->acc + (size_t)slot * o->sdim, sizeof(real) * o->sdim);
}

/* Fetch: read the global row, c_s = c_c = c_g   (Section 3.1, Fetch) */
static void fetch_into(het_oracle *o, int64_t k, int64_t slot)
{
    memcpy(o->row + (size_t)slot * o->dim, o->W + (size_t)k * o->dim, sizeof(real) * o->dim);
    if (o->opt != OPT_SGD)
        memcpy(o->acc + (size_t)slot * o->sdim, o->A + (size_t)k * o->sdim, sizeof(real) * o->sdim);
    o->cs[slot] = o->cc[slot] = o->Cg[k];
    rebase(o, slot);
}

/* CheckValid: c_c <= c_s + s  and  c_g <= c_c + s   (Section 3.1, CheckValid).  Written as
 * differences so that s = INT64_MAX ("never stale") does not overflow. */
static int check_valid(const het_oracle *o, int64_t slot)
{
    int64_t k = o->key[slot];
    int64_t ahead = (int64_t)o->cc[slot] - (int64_t)o->cs[slot];
    int64_t behind = (int64_t)o->Cg[k] - (int64_t)o->cc[slot];
    return ahead <= o->s && behind <= o->s;
}

typedef struct { uint32_t freq, last_use; int64_t slot; int32_t policy; } victim_key;

static int cmp_victim(const void *a, const void *b)
{
    const victim_key *x = (const victim_key *)a, *y = (const victim_key *)b;
    if (x->policy != POLICY_LRU && x->freq != y->freq) return x->freq < y->freq ? -1 : 1;
    if (x->last_use != y->last_use) return x->last_use < y->last_use ? -1 : 1;
    return (x->slot > y->slot) - (x->slot < y->slot);
}

/* Evict() without a key: drop the overflow chosen by the policy   (Section 3.1; Algorithm 3) */
static void trim(het_oracle *o, call_stats *st)
{
    o->ev_n = 0;
    int64_t m = o->size - o->C;
    if (m <= 0) return;
    victim_key *v = (victim_key *)malloc(sizeof(victim_key) * o->size);
    int64_t r = 0;
    for (int64_t slot = 0; slot < o->P; ++slot)
        if (o->key[slot] >= 0) {
            v[r].freq = o->freq[slot]; v[r].last_use = o->last_use[slot];
            v[r].slot = slot; v[r].policy = o->policy; ++r;
        }
    qsort(v, (size_t)r, sizeof(victim_key), cmp_victim);
    for (int64_t j = 0; j < m; ++j) {
        int64_t slot = v[j].slot, k = o->key[slot];
        st->evicted_dirty += write_back(o, slot);
        st->evicted += 1;
        o->ev_id[o->ev_n++] = k;
        o->slot_of[k] = -1;
        o->key[slot] = -1;
        o->size -= 1;
    }
    free(v);
}

static void add_stats(call_stats *t, const call_stats *c)
{
    t->n += c->n; t->U += c->U; t->hit += c->hit; t->stale += c->stale; t->miss += c->miss;
    t->evicted += c->evicted; t->evicted_dirty += c->evicted_dirty;
    t->stale_dirty += c->stale_dirty; t->flushed += c->flushed;
}

/* Sorted distinct valid keys of ids[n] into K (capacity n); returns U.  Sets ERR_RANGE if an id
 * lies outside [0, V).   (Algorithm 1: the unique key set of the minibatch) */
static int64_t unique_keys(het_oracle *o, const int64_t *ids, int64_t n, int64_t *K)
{
    int64_t m = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= o->V) { o->err |= ERR_RANGE; continue; }
        K[m++] = ids[i];
    }
    qsort(K, (size_t)m, sizeof(int64_t), cmp_i64);
    int64_t U = 0;
    for (int64_t i = 0; i < m; ++i)
        if (i == 0 || K[i] != K[i - 1]) K[U++] = K[i];
    return U;
}

/* Read (Algorithm 2) on the unique keys of ids; leaves every valid id resident. */
static int read_keys(het_oracle *o, const int64_t *ids, int64_t n)
{
    if (!o || !o->W || !ids || n < 0 || n > o->max_ids) return ERR_ARG;
    call_stats st; memset(&st, 0, sizeof(st));
    o->t += 1;
    if (o->size > o->C) trim(o, &st);          /* a Read that follows a Read */
    int64_t *K = o->lk_key;
    int64_t U = unique_keys(o, ids, n, K);
    st.n = n; st.U = U; o->lk_U = U;

    int64_t cursor = 0;                         /* smallest free slot: only moves up in a Read */
    for (int64_t u = 0; u < U; ++u) {           /* Algorithm 2's loop over the key set */
        int64_t k = K[u], slot = o->slot_of[k];                 /* Find */
        if (slot >= 0) {
            if (!check_valid(o, slot)) {                        /* CheckValid */
                st.stale_dirty += write_back(o, slot);          /* Evict(k) */
                fetch_into(o, k, slot);                         /* Fetch(k), in place */
                o->lk_cls[u] = CLS_STALE; st.stale += 1;
            } else {
                o->lk_cls[u] = CLS_HIT; st.hit += 1;
            }
        } else {                                                /* Fetch(k) into a new slot */
            while (o->key[cursor] >= 0) ++cursor;
            slot = cursor;
            o->key[slot] = k;
            o->slot_of[k] = slot;
            fetch_into(o, k, slot);
            o->freq[slot] = 0;
            o->size += 1;
            o->lk_cls[u] = CLS_MISS; st.miss += 1;
        }
    }
    for (int64_t u = 0; u < U; ++u) {           /* one use per key per Read */
        int64_t slot = o->slot_of[K[u]];
        o->lk_slot[u] = slot;
        if (o->policy == POLICY_LFU_LIGHT && o->freq[slot] >= o->lfu_cap) continue;   /* frequent enough: no upkeep */
        o->last_use[slot] = o->t;
        o->freq[slot] += 1;
    }
    o->last = st; add_stats(&o->total, &st);
    return ERR_NONE;
}

/* out[n][dim]: the cached row of every id (zeros for an id outside the vocabulary). */
int het_oracle_lookup(het_oracle *o, const int64_t *ids, int64_t n, real *out)
{
    if (n == 0) return ERR_NONE;
    if (!out) return ERR_ARG;
    int rc = read_keys(o, ids, n);
    if (rc) return rc;
    for (int64_t i = 0; i < n; ++i) {           /* Get */
        real *dst = out + (size_t)i * o->dim;
        if (ids[i] < 0 || ids[i] >= o->V) { memset(dst, 0, sizeof(real) * o->dim); continue; }
        memcpy(dst, o->row + (size_t)o->slot_of[ids[i]] * o->dim, sizeof(real) * o->dim);
    }
    return o->err;
}

/* Pooled read: out[b] = sum of the rows of ids[offsets[b] .. offsets[b+1]) in bag order. */
int het_oracle_lookup_pooled(het_oracle *o, const int64_t *ids, int64_t n, const int64_t *offsets,
                             int64_t n_bags, real *out)
{
    if (n == 0) return ERR_NONE;
    if (!out || !offsets || n_bags <= 0) return ERR_ARG;
    int rc = read_keys(o, ids, n);
    if (rc) return rc;
    for (int64_t b = 0; b < n_bags; ++b) {
        real *dst = out + (size_t)b * o->dim;
        for (int32_t j = 0; j < o->dim; ++j) dst[j] = 0;
        for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
            if (ids[i] < 0 || ids[i] >= o->V) continue;
            const real *src = o->row + (size_t)o->slot_of[ids[i]] * o->dim;
            for (int32_t j = 0; j < o->dim; ++j) dst[j] = dst[j] + src[j];
        }
    }
    return o->err;
}

/* Write (Algorithm 3).  grad_row[i] = index of the gradient row of position i (i itself, or the
 * bag of i for the pooled form). */
static int write_keys(het_oracle *o, const int64_t *ids, int64_t n, const real *grads,
                      const int64_t *offsets, int64_t n_bags, real lr)
{
    if (!o || !o->W || !ids || !grads || n < 0 || n > o->max_ids) return ERR_ARG;
    call_stats st; memset(&st, 0, sizeof(st));
    int64_t *K = (int64_t *)malloc(sizeof(int64_t) * (n > 0 ? n : 1));
    int64_t U = unique_keys(o, ids, n, K);
    st.n = n; st.U = U;
    real *G = (real *)calloc((size_t)(U > 0 ? U : 1) * o->dim, sizeof(real));
    int64_t b = 0;
    for (int64_t i = 0; i < n; ++i) {           /* G_k = sum of the gradients of key k */
        if (offsets) while (b + 1 < n_bags && i >= offsets[b + 1]) ++b;
        if (ids[i] < 0 || ids[i] >= o->V) continue;
        int64_t *p = (int64_t *)bsearch(&ids[i], K, (size_t)U, sizeof(int64_t), cmp_i64);
        real *g = G + (size_t)(p - K) * o->dim;
        const real *src = grads + (size_t)(offsets ? b : i) * o->dim;
        for (int32_t j = 0; j < o->dim; ++j) g[j] = g[j] + src[j];
    }
    for (int64_t u = 0; u < U; ++u) {           /* Update + Clock */
        int64_t slot = o->slot_of[K[u]];
        if (slot < 0) { o->err |= ERR_STATE; continue; }
        real *x = o->row + (size_t)slot * o->dim, *a = o->acc + (size_t)slot * o->sdim;
        const real *g = G + (size_t)u * o->dim;
        real row_denom = 0;
        if (o->opt == OPT_ADAGRAD_ROW) {        /* one accumulator for the row: the mean of the squares */
            real ss = 0;
            for (int32_t j = 0; j < o->dim; ++j) { real sq = g[j] * g[j]; ss = ss + sq; }
            ss = ss / (real)o->dim;
            a[0] = a[0] + ss;
            row_denom = (real)sqrt((double)a[0]) + o->eps;
        }
        for (int32_t j = 0; j < o->dim; ++j) {
            if (o->opt == OPT_ADAGRAD_ROW) {
                real step = lr * g[j];
                step = step / row_denom;
                x[j] = x[j] - step;
            } else if (o->opt == OPT_SGD) {
                real step = lr * g[j];
                x[j] = x[j] - step;
            } else {
                real sq = g[j] * g[j];
                a[j] = a[j] + sq;
                real denom = (real)sqrt((double)a[j]) + o->eps;
                real step = lr * g[j];
                step = step / denom;
                x[j] = x[j] - step;
            }
        }
        o->cc[slot] += 1;
    }
    free(G); free(K);
    trim(o, &st);                               /* Evict() */
    o->last = st; add_stats(&o->total, &st);
    return o->err;
}

int het_oracle_update(het_oracle *o, const int64_t *ids, const real *grads, int64_t n, real lr)
{
    if (n == 0) return ERR_NONE;
    return write_keys(o, ids, n, grads, NULL, 0, lr);
}

int het_oracle_update_pooled(het_oracle *o, const int64_t *ids, int64_t n, const int64_t *offsets,
                             const real *bag_grads, int64_t n_bags, real lr)
{
    if (n == 0) return ERR_NONE;
    if (!offsets || n_bags <= 0) return ERR_ARG;
    return write_keys(o, ids, n, bag_grads, offsets, n_bags, lr);
}

/* Write every dirty resident row back; rows stay cached and become clean. */
int het_oracle_flush(het_oracle *o)
{
    if (!o || !o->W) return ERR_ARG;
    call_stats st; memset(&st, 0, sizeof(st));
    for (int64_t slot = 0; slot < o->P; ++slot)
        if (o->key[slot] >= 0 && write_back(o, slot)) {
            o->cs[slot] = o->cc[slot] = o->Cg[o->key[slot]];
            rebase(o, slot);
            st.flushed += 1;
        }
    o->last = st; add_stats(&o->total, &st);
    return o->err;
}

/* A push by a worker that is not modelled otherwise (Section 3.1, Evict, the server's side): the
 * server adds deltas[i][:] to the global row ids[i] and advances its clock by one. */
int het_oracle_foreign_update(het_oracle *o, const int64_t *ids, const real *deltas, int64_t n)
{
    if (!o || !o->W || !ids || !deltas || n < 0) return ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= o->V) { o->err |= ERR_RANGE; continue; }
        for (int32_t j = 0; j < o->dim; ++j)
            o->W[(size_t)ids[i] * o->dim + j] = o->W[(size_t)ids[i] * o->dim + j] + deltas[(size_t)i * o->dim + j];
        o->Cg[ids[i]] += 1;
    }
    return o->err;
}

/* Resident rows in ascending slot order. Arrays need room for capacity + max_batch_ids entries. */
int64_t het_oracle_export_state(const het_oracle *o, int64_t *keys, int64_t *slots, uint32_t *cs,
                                uint32_t *cc, uint32_t *last_use, uint32_t *freq)
{
    int64_t r = 0;
    for (int64_t slot = 0; slot < o->P; ++slot)
        if (o->key[slot] >= 0) {
            keys[r] = o->key[slot]; slots[r] = slot; cs[r] = o->cs[slot]; cc[r] = o->cc[slot];
            last_use[r] = o->last_use[slot]; freq[r] = o->freq[slot]; ++r;
        }
    return r;
}

/* Cached row values (and accumulators if acc != NULL) of the resident rows, same order. */
int64_t het_oracle_export_rows(const het_oracle *o, real *rows, real *acc)
{
    int64_t r = 0;
    for (int64_t slot = 0; slot < o->P; ++slot)
        if (o->key[slot] >= 0) {
            memcpy(rows + (size_t)r * o->dim, o->row + (size_t)slot * o->dim, sizeof(real) * o->dim);
            if (acc) memcpy(acc + (size_t)r * o->sdim, o->acc + (size_t)slot * o->sdim,
                            sizeof(real) * o->sdim);
            ++r;
        }
    return r;
}

/* Unique keys of the last Read with their class (0 hit, 1 stale, 2 miss) and slot. */
int64_t het_oracle_last_lookup(const het_oracle *o, int64_t *keys, int32_t *cls, int64_t *slots)
{
    memcpy(keys, o->lk_key, sizeof(int64_t) * o->lk_U);
    memcpy(cls, o->lk_cls, sizeof(int32_t) * o->lk_U);
    memcpy(slots, o->lk_slot, sizeof(int64_t) * o->lk_U);
    return o->lk_U;
}

/* IDs evicted by the last trim, in eviction order. */
int64_t het_oracle_last_evicted(const het_oracle *o, int64_t *ids)
{
    memcpy(ids, o->ev_id, sizeof(int64_t) * o->ev_n);
    return o->ev_n;
}

/* out[0..8] = last call, out[9..17] = totals; order as in call_stats. */
void het_oracle_stats(const het_oracle *o, int64_t *out)
{
    memcpy(out, &o->last, sizeof(call_stats));
    memcpy(out + 9, &o->total, sizeof(call_stats));
}

int64_t het_oracle_size(const het_oracle *o) { return o->size; }
int64_t het_oracle_iteration(const het_oracle *o) { return (int64_t)o->t; }
int32_t het_oracle_error(const het_oracle *o) { return o->err; }
void het_oracle_clear_error(het_oracle *o) { o->err = 0; }
int32_t het_oracle_real_bytes(void) { return (int32_t)sizeof(real); }
