// Kernels of the cache step proper: Read (Algorithm 2 of the paper), Write (Algorithm 3), the
// policy trim Evict() (Section 3.1, Section 4.3) and flush.
//
// Device-side counts never travel to the host inside a call.  Where a kernel needs the number
// of items an earlier kernel found in other tiles (misses, stale rows, free slots, rows tied at
// the eviction threshold), the earlier kernel leaves one count per tile and the later kernel
// adds up the counts of the tiles before its own: "count at the producer, prefix at the
// consumer".  That keeps every ordering decision (which miss takes which free slot, which of
// several equal policy keys is evicted) a function of sorted order alone, never of the arrival
// order of atomics, and no workgroup ever waits for another.
#pragma once
#include "common.hpp"
#include "hash_table.hpp"
#include "sort_unique.hpp"

namespace het {

// Everything a kernel needs to know about one cache, passed by value.
struct CacheView {
    // global table (Section 3.1): rows, optimizer state, global clock c_g
    float *W, *A;
    uint32_t *Cg;
    uint32_t vocab;
    // cache slots
    float *rows, *acc;
    uint32_t *slot_key, *cs, *cc, *last_use, *freq;
    uint32_t n_slots;     // capacity + max_batch_ids
    uint32_t capacity;
    uint32_t max_ids;
    int64_t s;            // staleness bound
    HashTable ht;
    uint32_t *free_list;  // free slots in ascending order (first max_ids of them)
    DState *ds;
    RowGeom geom;
    int adagrad;
};

constexpr int32_t SRC_BACKING = -1;   // gather reads the global row: the key was not cached (or is refetched)
constexpr int32_t SRC_ZERO = -2;      // id outside the vocabulary: the output row is zero

constexpr int PT_THREADS = 1024;                // probe tiles: 1024 sorted positions per workgroup,
constexpr int PT_WAVES = PT_THREADS / WAVE;     // one per thread, so every probe's loads are in flight at once
constexpr int PT_TILE = PT_THREADS;
constexpr int CHUNK = 16;                       // sorted positions per row group in the apply kernel

// Per-call workspaces (sized by max_batch_ids unless noted).  Per-key facts are stored at the
// key's head position in the sorted order.
struct Workspace {
    uint32_t *skey, *perm;        // sorted keys and their original positions
    int32_t *src;                 // per sorted position: slot to gather from, or SRC_*
    int32_t *head_slot;           // at heads: slot of the key (set by fill for a missed key)
    uint8_t *cls;                 // at heads: HIT / STALE / MISS (lookup)
    uint32_t *tile_miss, *tile_stale;     // per probe tile counts
    uint32_t *miss_stage, *stale_stage;   // per probe tile: head positions of its missed / stale keys
    uint32_t *bag_of;             // pooled: bag of each original position
    double *partial;              // apply: [chunks][2][dim] partial gradient sums of runs that cross chunk borders
};

// CheckValid (Section 3.1): c_c <= c_s + s and c_g <= c_c + s, as differences so that an
// "infinite" s cannot overflow.
__device__ __forceinline__ bool check_valid(uint32_t cs, uint32_t cc, uint32_t cg, int64_t s)
{
    return (int64_t)cc - (int64_t)cs <= s && (int64_t)cg - (int64_t)cc <= s;
}

__device__ __forceinline__ void count2(unsigned long long *a, unsigned long long *b, uint32_t v)
{
    if (v) { atomicAdd(a, (unsigned long long)v); atomicAdd(b, (unsigned long long)v); }
}

// Find for every sorted position; at the head of every run of equal keys also CheckValid and
// the policy's use count.  LOOKUP: classifies HIT / STALE / MISS, stages missed and stale keys
// per tile for the fill kernel and tells the gather where each position's row comes from.
// Otherwise (update that sorted its own ids): only resolves slots and flags keys not cached.
template <bool LOOKUP>
__global__ __launch_bounds__(PT_THREADS) void probe_kernel(CacheView cv, Workspace ws, uint32_t n)
{
    __shared__ uint32_t lds[PT_WAVES + 1];
    const uint32_t tile = blockIdx.x;
    const uint32_t vocab = cv.vocab;
    const uint32_t j = tile * PT_TILE + threadIdx.x;
    DState *ds = cv.ds;

    bool head = false, miss = false, stale = false, hit = false, absent = false;
    if (j < n) {
        const uint32_t key = ws.skey[j];
        if (key == vocab) {                                   // id outside the vocabulary
            if (LOOKUP) ws.src[j] = SRC_ZERO;
            ws.head_slot[j] = SLOT_NONE;
        } else {
            head = j == 0 || ws.skey[j - 1] != key;
            if (j + 1 == n || ws.skey[j + 1] == vocab) ds->n_valid = j + 1;    // one writer: the last valid position
            const int32_t slot = ht_find(cv.ht, key);
            int32_t src = slot == SLOT_NONE ? SRC_BACKING : slot;
            bool valid = true;
            if (LOOKUP && slot != SLOT_NONE) {
                const uint32_t cs = cv.cs[slot], cc = cv.cc[slot];
                valid = check_valid(cs, cc, cv.Cg[key], cv.s);
                // A stale row that holds no updates of its own is refetched: its value is the
                // global row.  (One with updates is pushed first, so its own value stays current.)
                if (!valid && !(cc > cs)) src = SRC_BACKING;
            }
            if (LOOKUP) ws.src[j] = src;
            if (head) {
                ws.head_slot[j] = slot;
                if (LOOKUP) {
                    if (slot == SLOT_NONE) miss = true;
                    else {
                        hit = valid; stale = !valid;
                        cv.last_use[slot] = ds->t;            // one use per key per Read
                        cv.freq[slot] += 1;
                    }
                    ws.cls[j] = (uint8_t)(miss ? CLS_MISS : (stale ? CLS_STALE : CLS_HIT));
                } else {
                    absent = slot == SLOT_NONE;
                }
            }
        }
    }

    if (LOOKUP) {
        // stage this tile's missed and stale keys, in key order, for the fill kernel
        uint32_t tot_miss, tot_stale;
        const uint32_t mo = block_excl_scan<PT_WAVES>(miss ? 1u : 0u, lds, tot_miss);
        const uint32_t so = block_excl_scan<PT_WAVES>(stale ? 1u : 0u, lds, tot_stale);
        if (miss) ws.miss_stage[tile * PT_TILE + mo] = j;
        if (stale) ws.stale_stage[tile * PT_TILE + so] = j;
        const uint32_t tot_hit = block_sum<PT_WAVES>(hit ? 1u : 0u, lds);
        const uint32_t tot_heads = block_sum<PT_WAVES>(head ? 1u : 0u, lds);
        if (threadIdx.x == 0) {
            ws.tile_miss[tile] = tot_miss;
            ws.tile_stale[tile] = tot_stale;
            count2(&ds->last.hit, &ds->total.hit, tot_hit);
            count2(&ds->last.stale, &ds->total.stale, tot_stale);
            count2(&ds->last.miss, &ds->total.miss, tot_miss);
            count2(&ds->last.unique, &ds->total.unique, tot_heads);
            if (tot_miss) atomicAdd(&ds->size, (int32_t)tot_miss);
        }
    } else {
        if (__any(absent) && lane_id() == 0) atomicOr(&ds->err, ERRBIT_STATE);
        const uint32_t tot_heads = block_sum<PT_WAVES>(head ? 1u : 0u, lds);
        if (threadIdx.x == 0) count2(&ds->last.unique, &ds->total.unique, tot_heads);
    }
}

// Evict's push for one row (Section 3.1): copy the row (and the accumulator) to the global
// table; the group's first lane sets c_g = max(c_g, c_c).  Called by a whole row group.
template <int VEC>
__device__ __forceinline__ void push_row(const CacheView &cv, uint32_t key, uint32_t slot, int gl)
{
    const RowGeom g = cv.geom;
    row_copy<VEC>(cv.W + (size_t)key * g.dim, cv.rows + (size_t)slot * g.dim, g.chunks, g.lanes, gl);
    if (cv.adagrad)
        row_copy<VEC>(cv.A + (size_t)key * g.dim, cv.acc + (size_t)slot * g.dim, g.chunks, g.lanes, gl);
    if (gl == 0) { const uint32_t cc = cv.cc[slot]; if (cc > cv.Cg[key]) cv.Cg[key] = cc; }
}

// Fetch's pull for one row: copy the global row (and the accumulator) into the slot.
template <int VEC>
__device__ __forceinline__ void pull_row(const CacheView &cv, uint32_t key, uint32_t slot, int gl)
{
    const RowGeom g = cv.geom;
    row_copy<VEC>(cv.rows + (size_t)slot * g.dim, cv.W + (size_t)key * g.dim, g.chunks, g.lanes, gl);
    if (cv.adagrad)
        row_copy<VEC>(cv.acc + (size_t)slot * g.dim, cv.A + (size_t)key * g.dim, g.chunks, g.lanes, gl);
}

// Exclusive prefix of per-tile counts into LDS (ntiles <= capacity of `pre`), total returned.
template <int NW>
__device__ __forceinline__ uint32_t tile_prefix_to_lds(const uint32_t *counts, uint32_t ntiles, uint32_t *pre, uint32_t *scan)
{
    uint32_t carry = 0;
    for (uint32_t b = 0; b < ntiles; b += NW * WAVE) {
        const uint32_t i = b + threadIdx.x;
        const uint32_t v = i < ntiles ? counts[i] : 0u;
        uint32_t tot;
        const uint32_t e = block_excl_scan<NW>(v, scan, tot);
        if (i < ntiles) pre[i] = carry + e;
        carry += tot;
    }
    __syncthreads();
    return carry;
}

// Largest t with pre[t] <= m (pre ascending, pre[0] = 0).
__device__ __forceinline__ uint32_t tile_of(const uint32_t *pre, uint32_t ntiles, uint32_t m)
{
    uint32_t lo = 0, hi = ntiles;
    while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (pre[mid] <= m) lo = mid; else hi = mid; }
    return lo;
}

constexpr int MAX_PROBE_TILES = 1024;     // max_batch_ids <= 2^20 per call

// Fetch of the missed keys, Evict + Fetch of the stale ones (Algorithm 2), and Get.  One row
// group per item.  The i-th missed key in ascending key order takes the i-th free slot in
// ascending slot order.  The gather reads a missed key's row from the global table (the same
// values the fetch copies), so it does not have to wait for the fetch.
// POOLED: out[b] = sum of the bag's rows in bag order; else out[perm[j]] = row of position j.
template <int VEC, bool POOLED>
__global__ __launch_bounds__(256) void fill_gather_kernel(CacheView cv, Workspace ws, uint32_t n, uint32_t ptiles, float *__restrict__ out,
                                                          const int64_t *__restrict__ offsets, uint32_t n_bags,
                                                          const uint32_t *__restrict__ inv)
{
    using V = typename VecT<VEC>::type;
    __shared__ uint32_t pre_miss[MAX_PROBE_TILES], pre_stale[MAX_PROBE_TILES];
    __shared__ uint32_t scan[4 + 1];
    const RowGeom g = cv.geom;
    const uint32_t tot_miss = tile_prefix_to_lds<4>(ws.tile_miss, ptiles, pre_miss, scan);
    const uint32_t tot_stale = tile_prefix_to_lds<4>(ws.tile_stale, ptiles, pre_stale, scan);
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    const uint32_t t = cv.ds->t;

    for (uint32_t m = gid; m < tot_miss; m += ngroups) {                 // Fetch(k) into a new slot
        const uint32_t tl = tile_of(pre_miss, ptiles, m);
        const uint32_t j = ws.miss_stage[tl * PT_TILE + (m - pre_miss[tl])];
        const uint32_t key = ws.skey[j];
        const uint32_t slot = cv.free_list[m];
        pull_row<VEC>(cv, key, slot, gl);
        if (gl == 0) {
            const uint32_t cg = cv.Cg[key];
            cv.cs[slot] = cg; cv.cc[slot] = cg;                          // c_s = c_c = c_g
            cv.slot_key[slot] = key;
            cv.last_use[slot] = t;
            cv.freq[slot] = 1;
            ws.head_slot[j] = (int32_t)slot;
            if (!ht_insert(cv.ht, key, slot)) atomicOr(&cv.ds->err, ERRBIT_INTERNAL);
        }
    }
    for (uint32_t m = gid; m < tot_stale; m += ngroups) {                // Evict(k); Fetch(k) in place
        const uint32_t tl = tile_of(pre_stale, ptiles, m);
        const uint32_t j = ws.stale_stage[tl * PT_TILE + (m - pre_stale[tl])];
        const uint32_t key = ws.skey[j];
        const uint32_t slot = (uint32_t)ws.head_slot[j];
        const bool has_updates = cv.cc[slot] > cv.cs[slot];
        if (has_updates) push_row<VEC>(cv, key, slot, gl);               // now the global row equals the cached one
        else pull_row<VEC>(cv, key, slot, gl);
        if (gl == 0) {
            const uint32_t cg = cv.Cg[key];
            cv.cs[slot] = cg; cv.cc[slot] = cg;
            if (has_updates) count2(&cv.ds->last.stale_dirty, &cv.ds->total.stale_dirty, 1u);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) cv.ds->n_unique = (uint32_t)cv.ds->last.unique;   // for an update that reuses this order

    if (!POOLED) {
        for (uint32_t j = gid; j < n; j += ngroups) {                    // Get
            const int32_t s = ws.src[j];
            float *dst = out + (size_t)ws.perm[j] * g.dim;
            if (s == SRC_ZERO) row_zero<VEC>(dst, g.chunks, g.lanes, gl);
            else if (s == SRC_BACKING) row_copy<VEC>(dst, cv.W + (size_t)ws.skey[j] * g.dim, g.chunks, g.lanes, gl);
            else row_copy<VEC>(dst, cv.rows + (size_t)(uint32_t)s * g.dim, g.chunks, g.lanes, gl);
        }
    } else {
        for (uint32_t b = gid; b < n_bags; b += ngroups) {
            int64_t lo = offsets[b], hi = offsets[b + 1];
            lo = lo < 0 ? 0 : lo; hi = hi > (int64_t)n ? (int64_t)n : hi;
            for (int c = gl; c < g.chunks; c += g.lanes) {
                V sum{};
                for (int64_t i = lo; i < hi; ++i) {
                    const uint32_t j = inv[i];
                    const int32_t s = ws.src[j];
                    if (s == SRC_ZERO) continue;
                    const float *row = s == SRC_BACKING ? cv.W + (size_t)ws.skey[j] * g.dim : cv.rows + (size_t)(uint32_t)s * g.dim;
                    const V v = reinterpret_cast<const V *>(row)[c];
                    if constexpr (VEC == 4) { sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w; }
                    else sum += v;
                }
                reinterpret_cast<V *>(out + (size_t)b * g.dim)[c] = sum;
            }
        }
    }
}

// Pooled forms: inv[perm[j]] = j (sorted position of every original position), and the bag of
// every original position.
__global__ __launch_bounds__(256) void pooled_index_kernel(Workspace ws, uint32_t n, uint32_t *__restrict__ inv,
                                                           const int64_t *__restrict__ offsets, uint32_t n_bags)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) {
        inv[ws.perm[i]] = i;
        uint32_t lo = 0, hi = n_bags;            // largest b with offsets[b] <= i
        while (hi - lo > 1) { const uint32_t mid = (lo + hi) / 2; if (offsets[mid] <= (int64_t)i) lo = mid; else hi = mid; }
        ws.bag_of[i] = lo;
    }
}

// The optimizer step on one cached row for chunk c of the row, and nothing else.
template <int VEC>
__device__ __forceinline__ void apply_step(const CacheView &cv, uint32_t slot, int c, const double *g64, float lr, float eps)
{
    using V = typename VecT<VEC>::type;
    float G[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) G[k] = (float)g64[k];           // the fp64 sum is rounded to fp32 once
    V *xp = reinterpret_cast<V *>(cv.rows + (size_t)slot * cv.geom.dim) + c;
    V xv = *xp;
    float *x = reinterpret_cast<float *>(&xv);
    if (cv.adagrad) {
        V *ap = reinterpret_cast<V *>(cv.acc + (size_t)slot * cv.geom.dim) + c;
        V av = *ap;
        float *a = reinterpret_cast<float *>(&av);
#pragma unroll
        for (int k = 0; k < VEC; ++k) { a[k] += G[k] * G[k]; x[k] -= lr * G[k] / (sqrtf(a[k]) + eps); }
        *ap = av;
    } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k) x[k] -= lr * G[k];
    }
    *xp = xv;
}

// Update + Clock (Algorithm 3), first of two kernels.  Each row group takes CHUNK consecutive
// sorted positions: it loads their keys, original positions and gradient rows up front (all
// loads in flight together), then sums the gradients of each run of equal keys in fp64 (the
// kernel is bound by reading the gradients; summing wide makes a long run of a popular key
// lose no digits) and rounds once to fp32.  A run that lies inside the chunk is applied at
// once.  A run that crosses a chunk border leaves one partial sum per chunk for the second
// kernel.
// VERIFY: the ids must be the ones the sorted order was built from (an update that reuses the
// preceding lookup's order); a position whose id differs is skipped and flagged.
// MAXC: row pieces per lane (dim / VEC / lanes, rounded up).
template <int VEC, int MAXC, bool VERIFY>
__global__ __launch_bounds__(256) void apply_kernel(CacheView cv, Workspace ws, const int64_t *__restrict__ ids,
                                                    const float *__restrict__ grads, const uint32_t *__restrict__ grad_row,
                                                    float lr, float eps, uint32_t n_ids)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    const uint32_t nv = cv.ds->n_valid;
    const uint32_t nchunks_total = (nv + CHUNK - 1) / CHUNK;
    const uint32_t *skey = ws.skey;
    if (VERIFY && blockIdx.x == 0 && threadIdx.x == 0) {
        // this call did not sort: its per-call counters start here, with the lookup's key count
        DState *ds = cv.ds;
        Counters z{};
        z.n = n_ids; z.unique = ds->n_unique;
        ds->last = z;
        atomicAdd(&ds->total.n, (unsigned long long)n_ids);
        atomicAdd(&ds->total.unique, (unsigned long long)ds->n_unique);
        if (nv < n_ids) atomicOr(&ds->err, ERRBIT_RANGE);      // the order holds ids outside the vocabulary
    }

    for (uint32_t c = gid; c < nchunks_total; c += ngroups) {
        const uint32_t j0 = c * CHUNK;
        const uint32_t cnt = min((uint32_t)CHUNK, nv - j0);
        uint32_t k[CHUNK], p[CHUNK];
        int32_t hs[CHUNK];
#pragma unroll
        for (int i = 0; i < CHUNK; ++i) {
            const bool in = (uint32_t)i < cnt;
            k[i] = in ? skey[j0 + i] : KEY_NONE;
            p[i] = in ? ws.perm[j0 + i] : 0u;
            hs[i] = in ? ws.head_slot[j0 + i] : SLOT_NONE;
        }
        const uint32_t prev_key = j0 > 0 ? skey[j0 - 1] : KEY_NONE;
        const uint32_t next_key = j0 + cnt < nv ? skey[j0 + cnt] : KEY_NONE;
        uint32_t use = 0;                                   // positions whose gradient counts
#pragma unroll
        for (int i = 0; i < CHUNK; ++i) {
            bool ok = (uint32_t)i < cnt;
            if (VERIFY && ok) ok = ids[p[i]] == (int64_t)k[i];
            use |= ok ? (1u << i) : 0u;
        }
        if (VERIFY && gl == 0 && use != (cnt >= 32 ? ~0u : ((1u << cnt) - 1u))) atomicOr(&cv.ds->err, ERRBIT_STATE);
        if (grad_row) {
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) if ((uint32_t)i < cnt) p[i] = grad_row[p[i]];
        }
#pragma unroll
        for (int q = 0; q < MAXC; ++q) {
            const int cidx = gl + q * g.lanes;
            const bool act = cidx < g.chunks;
            V v[CHUNK];
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) {
                if (act && ((use >> i) & 1u)) v[i] = reinterpret_cast<const V *>(grads + (size_t)p[i] * g.dim)[cidx];
                else v[i] = V{};
            }
            double acc64[VEC];
            int run_start = 0;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc64[e] = 0.0;
#pragma unroll
            for (int i = 0; i < CHUNK; ++i) {
                const bool in = (uint32_t)i < cnt;
                const bool begins = in && (i == 0 || k[i] != k[i - 1]);
                if (begins) {
                    run_start = i;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc64[e] = 0.0;
                }
                const float *vf = reinterpret_cast<const float *>(&v[i]);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc64[e] += (double)vf[e];       // v[i] is zero where it does not count
                bool run_ends = in && (uint32_t)(i + 1) == cnt;
                if (i + 1 < CHUNK) run_ends = run_ends || (in && (uint32_t)(i + 1) < cnt && k[i + 1] != k[i]);
                if (run_ends) {
                    const bool starts_here = run_start > 0 || prev_key != k[i];
                    const bool ends_here = (uint32_t)(i + 1) < cnt || next_key != k[i];
                    if (starts_here && ends_here) {
                        int32_t slot = SLOT_NONE;          // hs[run_start], read with compile-time indices
#pragma unroll
                        for (int h = 0; h < CHUNK; ++h) slot = (h == run_start) ? hs[h] : slot;
                        if (slot != SLOT_NONE) {
                            if (act) apply_step<VEC>(cv, (uint32_t)slot, cidx, acc64, lr, eps);
                            if (q == 0 && gl == 0) cv.cc[slot] += 1;          // Clock(k)
                        }
                    } else if (act) {
                        double *mine = ws.partial + ((size_t)c * 2 + (starts_here ? 1 : 0)) * (size_t)g.dim + (size_t)cidx * VEC;
#pragma unroll
                        for (int e = 0; e < VEC; ++e) mine[e] = acc64[e];
                    }
                }
            }
        }
    }
}

// Second kernel of Write: finishes the runs that cross chunk borders.  The group of the chunk
// in which such a run starts adds the run's partial sums in chunk order and applies the step,
// so the result does not depend on scheduling.  The kernel also prepares the trim that
// follows (clears the select histograms and the evicted-id count).
struct TrimPlan;
template <int VEC, int MAXC>
__global__ __launch_bounds__(256) void apply_finish_kernel(CacheView cv, Workspace ws, float lr, float eps, uint32_t *trim_hist,
                                                           uint32_t trim_hist_words)
{
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    const uint32_t nv = cv.ds->n_valid;
    const uint32_t nchunks_total = (nv + CHUNK - 1) / CHUNK;
    const uint32_t *skey = ws.skey;
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < trim_hist_words; i += gridDim.x * 256u) trim_hist[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) cv.ds->ev_n = 0;

    for (uint32_t c = gid; c + 1 < nchunks_total; c += ngroups) {
        const uint32_t j0 = c * CHUNK, jb = j0 + CHUNK;        // jb < nv: the border after chunk c
        const uint32_t key = skey[jb - 1];
        if (skey[jb] != key) continue;                         // no run crosses this border
        if (skey[j0] == key && j0 > 0 && skey[j0 - 1] == key) continue;   // the run started in an earlier chunk
        uint32_t head = jb - 1;
        while (head > j0 && skey[head - 1] == key) --head;
        const uint32_t tail = run_end(skey, jb, nv, key);
        const uint32_t c1 = (tail - 1) / CHUNK;
        const int32_t slot = ws.head_slot[head];
        if (slot == SLOT_NONE) continue;
#pragma unroll
        for (int q = 0; q < MAXC; ++q) {
            const int cidx = gl + q * g.lanes;
            if (cidx >= g.chunks) continue;
            double sum[VEC];
            const double *first = ws.partial + ((size_t)c * 2 + 1) * (size_t)g.dim + (size_t)cidx * VEC;
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum[e] = first[e];
            for (uint32_t cc_ = c + 1; cc_ <= c1; ++cc_) {
                const double *pp = ws.partial + ((size_t)cc_ * 2) * (size_t)g.dim + (size_t)cidx * VEC;
#pragma unroll
                for (int e = 0; e < VEC; ++e) sum[e] += pp[e];
            }
            apply_step<VEC>(cv, (uint32_t)slot, cidx, sum, lr, eps);
        }
        if (gl == 0) cv.cc[slot] += 1;                         // Clock(k)
    }
}

// ---- Evict(): policy trim ---------------------------------------------------------------------
// The victims are the m = size - capacity cached rows smallest in (last_use, slot) [LRU] or
// (freq, last_use, slot) [LFU].  A most-significant-digit radix select finds the policy key
// tau of the m-th smallest row; rows below tau go, and of the rows equal to tau the first few in
// slot order.  `bits` is the width of last_use / freq values (both are at most t).
constexpr int SEL_BITS = 11;
constexpr int SEL_BINS = 1 << SEL_BITS;
constexpr int SEL_MAX_PASSES = 6;
constexpr int TRIM_THREADS = 256;
constexpr int TRIM_WAVES = TRIM_THREADS / WAVE;
constexpr int TRIM_ITEMS = 4;
constexpr int TRIM_TILE = TRIM_THREADS * TRIM_ITEMS;   // 1024 slots per counting tile

struct TrimPlan {
    int lfu;          // policy
    int bits;         // bits per policy field
    int key_bits;     // bits of the packed policy key
    int passes;       // select passes
    uint32_t *hist;   // [SEL_MAX_PASSES][SEL_BINS], zeroed before the first pass
    uint32_t *tile_eq, *tile_free;     // per slot-tile counts
    uint32_t *ev_ids;                  // ids dropped by this trim
};

__device__ __forceinline__ uint64_t policy_key(const CacheView &cv, const TrimPlan &tp, uint32_t slot)
{
    const uint64_t lu = cv.last_use[slot];
    return tp.lfu ? (((uint64_t)cv.freq[slot] << tp.bits) | lu) : lu;
}

__device__ __forceinline__ int sel_shift(const TrimPlan &tp, int pass)
{
    const int sh = tp.key_bits - SEL_BITS * (pass + 1);
    return sh < 0 ? 0 : sh;
}
__device__ __forceinline__ int sel_width(const TrimPlan &tp, int pass)
{
    const int hi = tp.key_bits - SEL_BITS * pass;       // bits not yet decided
    return hi < SEL_BITS ? hi : SEL_BITS;
}

// Replays the select decisions of passes [0, upto): returns the key prefix chosen so far
// (in the high bits of `prefix`) and how many victims remain to be found inside it.
// Every thread of the block gets the same answer.
__device__ __forceinline__ void sel_replay(const TrimPlan &tp, int upto, uint32_t m, uint64_t &prefix,
                                           uint32_t &remaining, uint32_t *lds_pick, uint32_t *lds_scan)
{
    prefix = 0; remaining = m;
    for (int p = 0; p < upto; ++p) {
        const int width = sel_width(tp, p), bins = 1 << width;
        uint32_t local[SEL_BINS / TRIM_THREADS];
        uint32_t s = 0;
#pragma unroll
        for (int q = 0; q < SEL_BINS / TRIM_THREADS; ++q) {
            const int b = threadIdx.x * (SEL_BINS / TRIM_THREADS) + q;
            local[q] = b < bins ? tp.hist[p * SEL_BINS + b] : 0u;
            s += local[q];
        }
        uint32_t tot;
        uint32_t run = block_excl_scan<TRIM_WAVES>(s, lds_scan, tot);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < SEL_BINS / TRIM_THREADS; ++q) {
            const int b = threadIdx.x * (SEL_BINS / TRIM_THREADS) + q;
            // the digit whose cumulative count first reaches `remaining`
            if (local[q] && run < remaining && remaining <= run + local[q]) { lds_pick[0] = (uint32_t)b; lds_pick[1] = run; }
            run += local[q];
        }
        __syncthreads();
        const uint32_t digit = lds_pick[0], below = lds_pick[1];
        __syncthreads();
        prefix |= (uint64_t)digit << sel_shift(tp, p);
        remaining -= below;
    }
}

__global__ __launch_bounds__(TRIM_THREADS) void trim_begin_kernel(CacheView cv, TrimPlan tp)
{
    for (uint32_t i = blockIdx.x * TRIM_THREADS + threadIdx.x; i < SEL_MAX_PASSES * SEL_BINS; i += gridDim.x * TRIM_THREADS) tp.hist[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) cv.ds->ev_n = 0;
}

// One histogram pass of the select over the rows whose key matches the prefix chosen so far.
__global__ __launch_bounds__(TRIM_THREADS) void trim_hist_kernel(CacheView cv, TrimPlan tp, int pass)
{
    __shared__ uint32_t bins[SEL_BINS];
    __shared__ uint32_t pick[2];
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    if (over <= 0) return;
    uint64_t prefix; uint32_t remaining;
    sel_replay(tp, pass, (uint32_t)over, prefix, remaining, pick, scan);
    for (int b = threadIdx.x; b < SEL_BINS; b += TRIM_THREADS) bins[b] = 0;
    __syncthreads();
    const int shift = sel_shift(tp, pass), width = sel_width(tp, pass);
    const int decided = shift + width;                 // bits above are fixed by the prefix
    for (uint32_t slot = blockIdx.x * TRIM_THREADS + threadIdx.x; slot < cv.n_slots; slot += gridDim.x * TRIM_THREADS) {
        if (cv.slot_key[slot] == KEY_NONE) continue;
        const uint64_t k = policy_key(cv, tp, slot);
        if (decided < 64 && (k >> decided) != (prefix >> decided)) continue;
        atomicAdd(&bins[(uint32_t)(k >> shift) & ((1u << width) - 1u)], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < SEL_BINS; b += TRIM_THREADS)
        if (bins[b]) atomicAdd(&tp.hist[pass * SEL_BINS + b], bins[b]);
}

// Per slot tile: how many cached rows have a policy key equal to tau.
__global__ __launch_bounds__(TRIM_THREADS) void trim_count_kernel(CacheView cv, TrimPlan tp)
{
    __shared__ uint32_t pick[2];
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    if (over <= 0) return;
    uint64_t tau; uint32_t take_eq;
    sel_replay(tp, tp.passes, (uint32_t)over, tau, take_eq, pick, scan);
    uint32_t eq = 0;
#pragma unroll
    for (int it = 0; it < TRIM_ITEMS; ++it) {
        const uint32_t slot = blockIdx.x * TRIM_TILE + threadIdx.x * TRIM_ITEMS + it;
        if (slot < cv.n_slots && cv.slot_key[slot] != KEY_NONE && policy_key(cv, tp, slot) == tau) ++eq;
    }
    eq = block_sum<TRIM_WAVES>(eq, scan);
    if (threadIdx.x == 0) tp.tile_eq[blockIdx.x] = eq;
}

// Drops the victims among 256 consecutive slots: push if the row holds updates, erase the key,
// free the slot.  Four workgroups share a counting tile; each adds its free slots to the
// tile's count for the free-list kernel (tile_free is zero when the trim starts).
constexpr int EV_SLOTS = 256;
template <int VEC>
__global__ __launch_bounds__(TRIM_THREADS) void trim_evict_kernel(CacheView cv, TrimPlan tp)
{
    __shared__ uint32_t pick[2];
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    __shared__ uint32_t victims[EV_SLOTS];
    __shared__ uint32_t n_victims;
    const uint32_t first = blockIdx.x * EV_SLOTS;
    const uint32_t tile = first / TRIM_TILE;
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    uint64_t tau = 0; uint32_t take_eq = 0, eq_before = 0;
    if (over > 0) {
        sel_replay(tp, tp.passes, (uint32_t)over, tau, take_eq, pick, scan);
        eq_before = block_sum_array<TRIM_WAVES>(tp.tile_eq, tile, scan);
        // rows equal to tau in the same counting tile but in earlier slots
        uint32_t e = 0;
        for (uint32_t slot = tile * TRIM_TILE + threadIdx.x; slot < first; slot += TRIM_THREADS)
            if (cv.slot_key[slot] != KEY_NONE && policy_key(cv, tp, slot) == tau) ++e;
        eq_before += block_sum<TRIM_WAVES>(e, scan);
    }
    if (threadIdx.x == 0) n_victims = 0;
    const uint32_t slot = first + threadIdx.x;
    bool is_free = false, lt = false, eq = false;
    if (slot < cv.n_slots) {
        if (cv.slot_key[slot] == KEY_NONE) is_free = true;
        else if (over > 0) { const uint64_t k = policy_key(cv, tp, slot); lt = k < tau; eq = k == tau; }
    }
    uint32_t tot_eq;
    const uint32_t eq_rank = eq_before + block_excl_scan<TRIM_WAVES>(eq ? 1u : 0u, scan, tot_eq);
    __syncthreads();
    if (lt || (eq && eq_rank < take_eq)) victims[atomicAdd(&n_victims, 1u)] = slot;
    __syncthreads();
    const uint32_t nv = n_victims;
    const int lanes = cv.geom.lanes;
    const int group = threadIdx.x / lanes, gl = threadIdx.x % lanes, ngroups = TRIM_THREADS / lanes;
    __shared__ uint32_t ev_base;
    if (threadIdx.x == 0 && nv) ev_base = atomicAdd(&cv.ds->ev_n, nv);      // one append per workgroup
    __syncthreads();
    uint32_t dirty = 0;
    for (uint32_t v = group; v < nv; v += ngroups) {
        const uint32_t vs = victims[v];
        const uint32_t key = cv.slot_key[vs];
        const bool has_updates = cv.cc[vs] > cv.cs[vs];
        if (has_updates) push_row<VEC>(cv, key, vs, gl);
        if (gl == 0) {
            dirty += has_updates ? 1u : 0u;
            ht_erase(cv.ht, key);
            tp.ev_ids[ev_base + v] = key;
        }
    }
    __syncthreads();
    for (uint32_t v = threadIdx.x; v < nv; v += TRIM_THREADS) cv.slot_key[victims[v]] = KEY_NONE;
    dirty = block_sum<TRIM_WAVES>(dirty, scan);
    const uint32_t free_here = block_sum<TRIM_WAVES>(is_free ? 1u : 0u, scan);
    if (threadIdx.x == 0) {
        if (free_here + nv) atomicAdd(&tp.tile_free[tile], free_here + nv);
        count2(&cv.ds->last.evicted, &cv.ds->total.evicted, nv);
        count2(&cv.ds->last.evicted_dirty, &cv.ds->total.evicted_dirty, dirty);
    }
}

// Lists the free slots in ascending order (only the first max_ids are ever needed), settles
// the row count after the trim and clears the per-tile counts for the next trim.
__global__ __launch_bounds__(TRIM_THREADS) void trim_free_kernel(CacheView cv, TrimPlan tp, uint32_t *tile_free_next)
{
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    const uint32_t tile = blockIdx.x;
    if (tile == 0 && threadIdx.x == 0 && cv.ds->size > (int32_t)cv.capacity) cv.ds->size = (int32_t)cv.capacity;
    if (threadIdx.x == 0) tile_free_next[tile] = 0;
    const uint32_t before = block_sum_array<TRIM_WAVES>(tp.tile_free, tile, scan);
    if (before >= cv.max_ids) return;
    uint32_t mine = 0;
    bool fr[TRIM_ITEMS];
#pragma unroll
    for (int it = 0; it < TRIM_ITEMS; ++it) {
        const uint32_t slot = tile * TRIM_TILE + threadIdx.x * TRIM_ITEMS + it;
        fr[it] = slot < cv.n_slots && cv.slot_key[slot] == KEY_NONE;
        mine += fr[it] ? 1u : 0u;
    }
    uint32_t tot;
    uint32_t pos = before + block_excl_scan<TRIM_WAVES>(mine, scan, tot);
#pragma unroll
    for (int it = 0; it < TRIM_ITEMS; ++it) {
        const uint32_t slot = tile * TRIM_TILE + threadIdx.x * TRIM_ITEMS + it;
        if (fr[it]) { if (pos < cv.max_ids) cv.free_list[pos] = slot; ++pos; }
    }
}

// flush: push every cached row that holds updates and mark it clean (c_s = c_c = c_g).
template <int VEC>
__global__ __launch_bounds__(256) void flush_kernel(CacheView cv)
{
    __shared__ uint32_t lds[4];
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    uint32_t pushed = 0;
    for (uint32_t slot = gid; slot < cv.n_slots; slot += ngroups) {
        const uint32_t key = cv.slot_key[slot];
        if (key == KEY_NONE || cv.cc[slot] <= cv.cs[slot]) continue;
        push_row<VEC>(cv, key, slot, gl);
        if (gl == 0) { const uint32_t cg = cv.Cg[key]; cv.cs[slot] = cg; cv.cc[slot] = cg; ++pushed; }
    }
    pushed = block_sum<4>(pushed, lds);
    if (threadIdx.x == 0) count2(&cv.ds->last.flushed, &cv.ds->total.flushed, pushed);
}

__global__ void reset_last_kernel(DState *ds)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { Counters z{}; ds->last = z; }
}

// Initial free list (every slot free) and empty slots / hash table.
__global__ __launch_bounds__(256) void init_cache_kernel(CacheView cv, uint32_t n_entries, uint32_t n_buckets)
{
    const uint32_t i0 = blockIdx.x * 256u + threadIdx.x, stride = gridDim.x * 256u;
    for (uint32_t i = i0; i < cv.n_slots; i += stride) {
        cv.slot_key[i] = KEY_NONE; cv.cs[i] = 0; cv.cc[i] = 0; cv.last_use[i] = 0; cv.freq[i] = 0;
    }
    for (uint32_t i = i0; i < cv.max_ids; i += stride) cv.free_list[i] = i;
    for (uint32_t i = i0; i < n_entries; i += stride) cv.ht.entries[i] = ENTRY_EMPTY;
    for (uint32_t i = i0; i < n_buckets; i += stride) cv.ht.reach[i] = 0;
}

} // namespace het
