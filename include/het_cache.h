/*
 * het_cache.h - C ABI of the MI355X embedding-cache step.
 *
 * One cache object serves one worker's share of a huge embedding table: the global
 * ("server") table stays in a backing store, a bounded number of rows is cached in HBM, and
 * every cached row carries a start clock c_s and a local clock c_c next to the global clock
 * c_g of its global row (HET, arXiv 2112.07221, Section 3.1).  het_lookup is the client's
 * Read (Algorithm 2) on the unique key set of a minibatch (Algorithm 1), het_update is its
 * Write (Algorithm 3), including the policy-driven Evict() of the overflow (Section 3.1,
 * Section 4.3).  All steps run in HIP kernels on the configured stream.
 *
 * Conventions
 *   - Every function returns an int status: HET_OK (0) or a negative het_status.
 *   - "device" pointers are HIP device allocations of the current device, owned by the caller
 *     and only borrowed for the duration stated; "host" pointers are ordinary host memory.
 *   - het_lookup* / het_update* only enqueue work on the configured stream and return; their
 *     results are valid in the order of that stream (the library uses no other stream).
 *     het_flush, het_stats, het_export_*, het_last_* and het_cache_destroy wait for the stream.
 *   - Errors the host can see (NULL, sizes out of range, wrong call order) are returned at
 *     once and change nothing.  Errors only the device can see (an id outside [0, vocab), an
 *     update of an id that is not cached) set a sticky bit that the next waiting call returns
 *     (HET_ERANGE / HET_ESTATE) and het_stats reports; the offending ids are skipped (their
 *     lookup rows are zero).  het_clear_error resets the bits.
 *   - The library allocates device memory only in het_cache_configure / het_attach_backing and
 *     frees it in het_cache_destroy; lookup/update/flush allocate nothing.
 *   - A cache object is not thread-safe; use it from one host thread at a time.
 */
#ifndef HET_CACHE_H
#define HET_CACHE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct het_cache het_cache;

typedef enum het_status {
    HET_OK = 0,
    HET_EINVAL = -1,  /* bad argument or call order; nothing was done */
    HET_ENOMEM = -2,  /* a device or host allocation failed */
    HET_EHIP = -3,    /* a HIP runtime call failed */
    HET_ERANGE = -4,  /* sticky: some id was outside [0, vocab) */
    HET_ESTATE = -5   /* sticky: het_update saw an id that is not cached (no het_lookup before) */
} het_status;

enum { HET_POLICY_LRU = 0, HET_POLICY_LFU = 1,          /* Section 4.3 */
       HET_POLICY_NONE = 2,                              /* no cache at all: the baseline "Hybrid (w/o Cache)" of Section 5 */
       HET_POLICY_LFU_LIGHT = 3 };                       /* the light-weight LFU of Section 4.3, an approximation of LFU: see het_cache_set_lfu_cap */
enum { HET_OPT_SGD = 0, HET_OPT_ADAGRAD = 1,
       HET_OPT_ADAGRAD_ROWWISE = 2 };   /* one accumulator per row: a += mean_j(G_j^2); x_j -= lr * G_j / (sqrt(a) + eps) */
enum { HET_BACKING_HBM = 0, HET_BACKING_PINNED_HOST = 1 };
enum { HET_CLASS_HIT = 0, HET_CLASS_STALE = 1, HET_CLASS_MISS = 2 };
#define HET_S_INFINITE INT64_MAX /* staleness bound that never invalidates a row */

/* Counters of the most recent lookup/update/flush call and running totals since creation. */
typedef struct het_counters {
    int64_t n;             /* ids passed in */
    int64_t unique;        /* distinct valid ids (size of the key set K) */
    int64_t hit;           /* keys found valid in the cache */
    int64_t stale;         /* keys found but failing CheckValid: synchronised in place */
    int64_t miss;          /* keys fetched from the backing store into a new slot */
    int64_t evicted;       /* rows dropped by the policy trim */
    int64_t evicted_dirty; /* ... of which were written back (c_c > c_s) */
    int64_t stale_dirty;   /* stale rows written back before their refresh */
    int64_t flushed;       /* rows written back by het_flush */
} het_counters;

typedef struct het_stats_t {
    het_counters last;
    het_counters total;
    int64_t resident;      /* rows in the cache now */
    int64_t iteration;     /* number of non-empty lookups so far (the LRU time stamp) */
    int32_t error_bits;    /* 1: id out of range, 2: update of an id that is not cached */
} het_stats_t;

/*
 * Creates an empty cache for `capacity` rows of `dim` floats with staleness bound `s`
 * (CheckValid, Section 3.1: a cached row is valid iff c_c <= c_s + s and c_g <= c_c + s) and
 * eviction `policy`.  s may be HET_S_INFINITE.  No device memory is taken yet.
 * With HET_POLICY_NONE there is no cache (capacity and s are ignored, vocab must stay below
 * 2^31): het_lookup gathers from the global table, het_update applies the coalesced gradients
 * to it, nothing is ever cached, there are no clocks, and het_flush has nothing to do.  It is
 * the yardstick for what the cache buys (table in host memory) or costs (table in HBM).
 * HET_EINVAL: out == NULL, capacity <= 0, dim <= 0, s < 0, unknown policy.
 */
int het_cache_create(het_cache **out, int64_t capacity, int32_t dim, int64_t s, int32_t policy);

/*
 * HET_POLICY_LFU_LIGHT (Section 4.3: an embedding whose frequency is high enough is accessed
 * directly, without the upkeep of its frequency; the paper names no threshold): LFU whose use
 * counter stops at `cap` (default 16).  A row that has been used that often is no longer touched by
 * lookups: neither its counter nor its last-use stamp is written, and it leaves the cache only
 * after every row used less often.  It evicts other rows than exact LFU does where counts beyond
 * the cap would have decided; on skewed streams the miss rate is about the same (bench.py
 * --policy-study).  Call between het_cache_create and het_cache_configure.  HET_EINVAL: cap == 0,
 * another policy, already configured.
 */
int het_cache_set_lfu_cap(het_cache *c, uint32_t cap);

/*
 * Several workers over one global table (Section 3.1; Lemma 1).  Call between het_cache_create and
 * het_cache_configure.  The cache then keeps every row as it was fetched, and Evict (of a stale
 * row at a lookup, of the overflow at an update, and het_flush) pushes what the worker accumulated
 * since its Fetch: the global row takes row - row_as_fetched (the Adagrad accumulator likewise) and
 * c_g = max(c_g, c_c), as the paper words Evict, instead of being overwritten.  A stale row is
 * then really fetched again (other workers' pushes are in the global row), so CheckValid's second
 * condition c_g <= c_c + s matters.  Several caches of one process may be attached to the same
 * table, state and cg arrays if they are configured on the same stream: their calls then take
 * effect in the order they are made.  Costs one more copy of the cached rows in HBM.  The table
 * must be in HBM.  HET_EINVAL: already configured, or HET_POLICY_NONE.
 */
int het_cache_set_many_writers(het_cache *c);

/*
 * Fixes the largest number of ids one call may carry, the optimizer het_update applies and the
 * HIP stream (a hipStream_t, NULL = the default stream) all work is enqueued on, and allocates
 * the cache in HBM: capacity + max_batch_ids row slots (rows fetched on a miss are added beyond
 * the capacity and the overflow is trimmed at the end of the update, Algorithm 2 / 3), the
 * id->slot hash table and the per-call workspaces.  Must be called once, before attach.
 * eps is Adagrad's epsilon (ignored for SGD).  HET_OPT_ADAGRAD_ROWWISE keeps one accumulator per row
 * instead of one per element (half the optimizer state of an embedding table): `state` of
 * het_attach_backing is then float[vocab] and het_export_rows' acc float[n_resident]; the table
 * must be in HBM.
 * HET_EINVAL: max_batch_ids <= 0 or above 2^20, unknown optimizer, eps < 0, a second call, or
 * rows wider than the kernels take (dim above 4096, or above 1024 if dim is no multiple of 4; for
 * HET_OPT_ADAGRAD_ROWWISE dim above 256, or above 64 if dim is no multiple of 4), row-wise Adagrad
 * together with het_cache_set_many_writers.
 * HET_ENOMEM: the device allocation failed.
 */
int het_cache_configure(het_cache *c, int64_t max_batch_ids, int32_t optimizer, float eps,
                        void *hip_stream);

/*
 * Names the global embedding table this cache fronts (Section 3.1):
 *   table  float[vocab][dim], row-major: the global rows;
 *   state  float[vocab][dim]: Adagrad accumulators, travelling with the rows (NULL for SGD;
 *          float[vocab] for row-wise Adagrad);
 *   cg     uint32[vocab]: global clock c_g per row, zero-initialised by the caller.
 * location HET_BACKING_HBM: device pointers.  HET_BACKING_PINNED_HOST: pointers to pinned,
 * device-mapped host memory (hipHostMalloc); kernels read and write it over the host link.
 * The caller owns the arrays; the library reads and writes them during lookup/update/flush and
 * they must outlive the cache.  Between a lookup and the update that follows it the caller must
 * not write them (with the table in HBM the rows a lookup misses are read from it for the output
 * at once and for the cache by that update); writes by other workers go through
 * het_backing_foreign_update.  vocab must be below 2^32 - 1.
 */
int het_attach_backing(het_cache *c, float *table, float *state, uint32_t *cg, int64_t vocab,
                       int32_t location);

/*
 * Read (Algorithm 2) of the unique keys of ids[n] (device, int64), then out[i][:] = cached row
 * of ids[i] (device, float[n][dim], row-major).  Keys not cached are fetched from the backing
 * store into the smallest free slots in ascending key order with c_s = c_c = c_g (Fetch); keys
 * cached but invalid are written back if they hold updates (Evict: c_g = max(c_g, c_c)) and
 * refreshed in place; every key of the batch counts as one use for LRU/LFU.  n == 0 is a
 * complete no-op.  n > max_batch_ids: HET_EINVAL.  If the previous call was also a lookup, the
 * overflow it left is trimmed first.
 */
int het_lookup(het_cache *c, const int64_t *ids, int64_t n, float *out);

/*
 * Optional: announces the ids of a coming lookup (Section 4.2: the indices of the next minibatch
 * are known in advance).  Their sort, the dedup of Algorithm 1, touches no cache state, so the
 * kernels of the calls made between this call and that lookup carry it in extra workgroups, one
 * stage per kernel (two, if two announced batches are under way); whatever is still missing runs
 * when the lookup comes.  A sort has two stages per eight bits of the vocabulary's width, a
 * lookup plus an update have four kernels that can carry: announce two batches ahead (before the
 * lookup of batch t, the ids of batch t + 2) and the sort is never seen.  ids[n] (device) must be
 * complete in stream order when this call is made and stay unchanged until the lookup that
 * passes the same pointer and n (that lookup checks the order sorted ahead against the ids as
 * they are then; ids that changed set error bit 2, HET_ESTATE, and its results are not
 * meaningful).  Three batches can stand announced at a time (a fourth replaces
 * the oldest).  Results are identical with and without the announcement; a lookup with other
 * ids leaves it standing for a later one.  Nothing is launched by this call.
 * Lifetime of the buffer: the kernels of LATER calls read it (the first sort stage converts the
 * ids), so it must stay allocated until its lookup has been enqueued, or until
 * het_prefetch_cancel / het_flush has withdrawn the announcement and the work enqueued before
 * that has completed.  An announcement is matched by pointer and n alone: a new buffer that an
 * allocator places at the same address with the same n while the old announcement stands is
 * taken for the old one (and then flagged HET_ESTATE by the check above); cancel first.
 */
int het_prefetch(het_cache *c, const int64_t *ids, int64_t n);

/* Withdraws every standing announcement: sort stages not yet enqueued never run, the buffers are
 * not read by anything enqueued after this call.  het_flush does the same. */
int het_prefetch_cancel(het_cache *c);

/*
 * The server's side of Evict for a worker that is not one of this process's caches (Section 3.1):
 * table[ids[i]][:] += deltas[i][:] and cg[ids[i]] += 1, on the cache's stream.  ids (device,
 * int64[n]) must be distinct; deltas is device, float[n][dim].  Ids outside the vocabulary are
 * skipped and set error bit 1.  The table must be in HBM.  Cached copies of these rows turn stale
 * by CheckValid's second condition once c_g has run more than s ahead of their clock.
 */
int het_backing_foreign_update(het_cache *c, const int64_t *ids, const float *deltas, int64_t n);

/*
 * Pooled Read for multi-hot inputs: bag b holds ids[offsets[b] .. offsets[b+1]) and
 * out[b][:] = sum of its rows, added in bag order in fp64 and rounded once (device,
 * float[n_bags][dim]).
 * offsets: device, int64[n_bags + 1], non-decreasing, offsets[0] = 0, offsets[n_bags] = n.
 */
int het_lookup_pooled(het_cache *c, const int64_t *ids, int64_t n, const int64_t *offsets,
                      int64_t n_bags, float *out);

/*
 * Write (Algorithm 3) for the ids of the preceding lookup: per unique key k the gradients
 * grads[i][:] (device, float[n][dim]) of all positions i with ids[i] == k are summed in order
 * of increasing i, the optimizer step is applied to the cached row
 *   SGD      x -= lr * G
 *   Adagrad  a += G*G;  x -= lr * G / (sqrt(a) + eps)
 * and c_c grows by one (once per key per call).  Then Evict(): while more than `capacity` rows
 * are cached, the rows smallest in (last_use, slot) for LRU or (freq, last_use, slot) for LFU
 * are dropped, those with c_c > c_s being written back first (c_g = max(c_g, c_c)).
 * ids (device, int64[n]) may be any buffer that holds ids cached by that lookup, in any order
 * and number: they are sorted afresh.  If it is the very pointer and n of the preceding lookup,
 * the lookup's sorted order is reused instead, so the buffer must still hold what it held then.
 * Every id is checked against that order on the device; a buffer whose contents changed sets
 * error bit 2 (HET_ESTATE at the next status query) and the gradients have gone to the wrong
 * rows: the cache and what it later writes back are then no longer meaningful.  An id that is
 * not cached sets the same bit and is skipped; ids outside the vocabulary set error bit 1.
 */
int het_update(het_cache *c, const int64_t *ids, const float *grads, int64_t n, float lr);

/* Pooled Write: the gradient of every position of bag b is bag_grads[b][:] (device,
 * float[n_bags][dim]); ids/offsets as in het_lookup_pooled. */
int het_update_pooled(het_cache *c, const int64_t *ids, int64_t n, const int64_t *offsets,
                      const float *bag_grads, int64_t n_bags, float lr);

/*
 * Writes every cached row that holds updates back to the backing store (as Evict does) and
 * marks it clean (c_s = c_c = c_g); rows stay cached.  Afterwards the backing store alone holds
 * the trained table.  (The paper lets updates left in the cache at the end of training be
 * dropped, Section 3.3; this call keeps them instead.)  Waits for the stream.
 */
int het_flush(het_cache *c);

/* Waits for the stream and fills *out (host). */
int het_stats(het_cache *c, het_stats_t *out);

/* Resets the sticky device error bits. */
int het_clear_error(het_cache *c);

/*
 * Parity helpers (wait for the stream; all pointers are host memory; any may be NULL).
 * het_export_state: the cached rows in ascending slot order; arrays need room for
 *   capacity + max_batch_ids entries; *n_resident receives the count.
 * het_export_rows: their values (and Adagrad accumulators), float[n_resident][dim], same order.
 * het_last_lookup: the sorted unique keys of the last lookup with class (HET_CLASS_*) and slot;
 *   arrays need room for max_batch_ids entries.
 * het_last_evicted: the ids dropped by the most recent trim, in no particular order; room for
 *   capacity + max_batch_ids entries.
 */
int het_export_state(het_cache *c, int64_t *keys, int32_t *slots, uint32_t *cs, uint32_t *cc,
                     uint32_t *last_use, uint32_t *freq, int64_t *n_resident);
int het_export_rows(het_cache *c, float *rows, float *acc);
int het_last_lookup(het_cache *c, int64_t *keys, int32_t *cls, int32_t *slots, int64_t *n_unique);
int het_last_evicted(het_cache *c, int64_t *ids, int64_t *n);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): het_lookup of a cache created with HET_POLICY_NONE,
 * without a cache object.  out[i][:] = table[ids[i]][:] for ids (device, int64[n]) inside
 * [0, vocab), zero rows for the others; table is float[vocab][dim] (device, or pinned host memory
 * mapped into the device), out float[n][dim] (device).  The ids go through the same sort, run
 * marking and gather kernels as het_lookup; their workspaces (sort buffers, per-position arrays,
 * scalars) live in a static device array of about 1.8 MB that every GPU the library runs on holds
 * until the process ends, so the call allocates and frees nothing, on the device or through any
 * library.  n may be at most HET_NOALLOC_MAX_IDS; dim as for het_cache_configure; vocab below
 * 2^31.  The work is enqueued on hip_stream (a hipStream_t, NULL = the default stream) and the
 * call returns without waiting.  err_bits (device, uint32, may be NULL) receives, in stream order,
 * 1 if some id was outside the vocabulary, else 0.  All calls on one GPU share the array: calls
 * whose work overlaps on one GPU (two streams, two threads) race and must be serialised by the
 * caller.  HET_EINVAL: a size out of range or a NULL pointer.  HET_EHIP: the runtime refused.
 */
#define HET_NOALLOC_MAX_IDS 65536
int het_lookup_nocache_static(const float *table, int64_t vocab, int32_t dim, const int64_t *ids, int64_t n,
                              float *out, uint32_t *err_bits, void *hip_stream);

/*
 * Per-kernel timing for benchmarks.  Between het_profile_begin and het_profile_end every kernel
 * the library launches for this cache is bracketed by a pair of HIP events on the cache's
 * stream (this slows the calls down slightly and creates events: not for timed regions).
 * het_profile_end waits for the stream and adds up, per kernel index, the elapsed milliseconds
 * into total_ms[n_kernels] and the launch count into launches[n_kernels] (host arrays).
 * het_profile_kernel_count / het_profile_kernel_name give the index space.
 */
int het_profile_begin(het_cache *c);
int het_profile_end(het_cache *c, double *total_ms, int64_t *launches, int32_t n_kernels);
int het_profile_kernel_count(void);
const char *het_profile_kernel_name(int index);

/*
 * Time stamps inside the two heavy kernels, for finding out where their time goes.  `kernel` is the
 * index (het_profile_kernel_name) of "apply_kernel" (het_update's main kernel) or of
 * "fill_gather_kernel" (het_lookup's second kernel).  While `records` (device memory,
 * HET_TRACE_WORDS uint64 per workgroup, room for `capacity` workgroups, zeroed by the caller) is
 * set, every launch of that kernel writes per workgroup: [0] start, [5] the last wave's end,
 * [6] role.  apply_kernel: roles 1 carried sort stage, 2 select stage, 3 id check, 4 tile of the
 * update; for role 4 also [1] tile loaded and segments listed, [2] short segments done, [3] long
 * segments done, [4] past the barrier before the runs that cross tile borders (as far as the
 * workgroup got).  fill_gather_kernel: roles 1 carried sort stage, 2 fetch, 3 the fetched keys'
 * bookkeeping, 4 select stage, 5 gather, 6 host link.  Clock: the GPU's constant 100 MHz counter.
 * A later launch overwrites the records.  capacity 0 (records ignored) switches the stamps off
 * again.  They cost a few stores per workgroup: not for timed regions.  HET_EINVAL for a bad
 * argument.
 */
#define HET_TRACE_WORDS 8
int het_profile_trace(het_cache *c, int32_t kernel, uint64_t *records, int64_t capacity);

/*
 * Reference points for the roofline (not part of the path): runs, `reps` times in a row on
 * hip_stream (after two launches that are not timed), a plain kernel that has the memory access
 * pattern of one of the path's heavy steps and nothing else, and gives the average milliseconds
 * per launch between two HIP events in *avg_ms (host).  All pointers but avg_ms are device memory;
 * rows have `dim` floats (4, 8, 16, ... 128, or a multiple of 4 above 256); idx holds n row numbers
 * (uint32).
 *   HET_PATTERN_COPY    x[i] = src[i], i < n: a streaming copy (idx unused)
 *   HET_PATTERN_GATHER  x[i] = src[idx[i]]: the gather (Get of Algorithm 2)
 *   HET_PATTERN_UPDATE  rows idx[i] (distinct) of x, and of a unless it is NULL, read, changed and
 *                       written back: the optimizer step on cached rows (Update of Algorithm 3).
 *                       With per = 2 or 3 every row also reads `per` rows of src, numbers
 *                       gidx[i * per ...]: the gradients of its key's lookups (per = 0: none)
 * The caller owns every buffer and makes them large enough for the row numbers it passes.
 * HET_EINVAL for a bad size or a missing pointer, HET_EHIP if the runtime refused.
 */
#define HET_PATTERN_COPY 0
#define HET_PATTERN_GATHER 1
#define HET_PATTERN_UPDATE 2
int het_profile_rows(int32_t pattern, float *x, float *a, const float *src, const uint32_t *idx, int64_t n, int32_t dim,
                     const uint32_t *gidx, int32_t per, int32_t reps, double *avg_ms, void *hip_stream);

/* Waits for the stream, frees everything the library allocated.  NULL is allowed. */
int het_cache_destroy(het_cache *c);

/* Short hash of the sources this library was built from (set by the build script; "unknown"
 * otherwise): lets a stored measurement say which build it belongs to. */
const char *het_build_id(void);

/* Static description of a status code. */
const char *het_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* HET_CACHE_H */
