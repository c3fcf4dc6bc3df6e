// Kernels of the cache step proper: Read (Algorithm 2 of the paper), Write (Algorithm 3), the
// policy trim Evict() (Section 3.1, Section 4.3) and flush.
//
// Device-side counts never travel to the host inside a call.  Where a kernel needs the number
// of items an earlier kernel found in other tiles (unique keys, misses, free slots), the
// earlier kernel leaves one count per tile and the later kernel adds up the counts of the
// tiles before its own: "count at the producer, prefix at the consumer".  That keeps every
// ordering decision (which miss takes which free slot, which of several equal policy keys is
// evicted) a function of sorted order alone, never of the arrival order of atomics.
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

// Per-call workspaces (all sized by max_batch_ids unless noted).
struct Workspace {
    uint32_t *skey, *perm;        // sorted keys and their original positions
    uint32_t *rank;               // per sorted position: index of its key in ukey
    uint32_t *ukey, *seg;         // unique keys; start of each key's run (seg has one extra entry)
    int32_t *uslot;               // slot of each unique key
    uint8_t *ucls;                // class of each unique key (lookup)
    uint32_t *tile_heads, *tile_miss, *tile_stale;   // per unique-tile counts
    uint32_t *miss_stage, *stale_stage;              // per tile: ranks of its missed / stale keys
    uint32_t *inv;                // pooled: per original position, rank of its key
};

// CheckValid (Section 3.1): c_c <= c_s + s and c_g <= c_c + s, as differences so that an
// "infinite" s cannot overflow.
__device__ __forceinline__ bool check_valid(uint32_t cs, uint32_t cc, uint32_t cg, int64_t s)
{
    return (int64_t)cc - (int64_t)cs <= s && (int64_t)cg - (int64_t)cc <= s;
}

// Ranks the sorted positions of one tile, lists the unique keys, and looks every unique key up
// in the hash table.  LOOKUP: classifies it HIT / STALE / MISS (Find + CheckValid), counts a
// use for the policy, and stages missed and stale keys per tile for the fill kernel.
// Otherwise (update): only resolves the slot and flags keys that are not cached.
template <bool LOOKUP>
__global__ __launch_bounds__(UQ_THREADS) void rank_probe_kernel(CacheView cv, Workspace ws, uint32_t n)
{
    __shared__ uint32_t lds[UQ_WAVES + 1];
    const uint32_t tile = blockIdx.x;
    const uint32_t ntiles = gridDim.x;
    const uint32_t vocab = cv.vocab;
    const uint32_t heads_before = block_sum_array<UQ_WAVES>(ws.tile_heads, tile, lds);
    const uint32_t base = tile * UQ_TILE + threadIdx.x * UQ_ITEMS;

    uint32_t key[UQ_ITEMS];
    bool head[UQ_ITEMS];
    uint32_t mine = 0;
#pragma unroll
    for (int it = 0; it < UQ_ITEMS; ++it) {
        const uint32_t j = base + it;
        key[it] = j < n ? ws.skey[j] : vocab;
        head[it] = is_head(ws.skey, j, n, vocab);
        mine += head[it] ? 1u : 0u;
    }
    uint32_t tile_total;
    uint32_t r = heads_before + block_excl_scan<UQ_WAVES>(mine, lds, tile_total);   // heads before this thread

    uint32_t n_miss = 0, n_stale = 0, n_hit = 0, n_absent = 0;
    uint32_t miss_rank[UQ_ITEMS], stale_rank[UQ_ITEMS];
    bool is_miss[UQ_ITEMS], is_stale[UQ_ITEMS];
#pragma unroll
    for (int it = 0; it < UQ_ITEMS; ++it) {
        const uint32_t j = base + it;
        is_miss[it] = is_stale[it] = false;
        miss_rank[it] = stale_rank[it] = 0;
        if (head[it]) r += 1;                       // r = heads up to and including position j
        if (j >= n) continue;
        const bool valid = key[it] != vocab;
        ws.rank[j] = valid ? r - 1 : KEY_NONE;
        if (valid && (j + 1 == n || ws.skey[j + 1] == vocab)) ws.seg[r] = j + 1;   // end of the last run
        if (!head[it]) continue;
        const uint32_t u = r - 1;
        ws.ukey[u] = key[it];
        ws.seg[u] = j;
        const int32_t slot = ht_find(cv.ht, key[it]);
        ws.uslot[u] = slot;
        if (LOOKUP) {
            int cls;
            if (slot == SLOT_NONE) {
                cls = CLS_MISS; is_miss[it] = true; miss_rank[it] = u; ++n_miss;
            } else {
                const bool ok = check_valid(cv.cs[slot], cv.cc[slot], cv.Cg[key[it]], cv.s);
                cls = ok ? CLS_HIT : CLS_STALE;
                if (ok) ++n_hit; else { is_stale[it] = true; stale_rank[it] = u; ++n_stale; }
                cv.last_use[slot] = cv.ds->t;       // one use per key per Read
                cv.freq[slot] += 1;
            }
            ws.ucls[u] = (uint8_t)cls;
        } else if (slot == SLOT_NONE) {
            ++n_absent;
        }
    }

    if (LOOKUP) {
        // stage this tile's missed and stale keys, in key order, for the fill kernel
        uint32_t tot_miss, tot_stale;
        uint32_t mo = block_excl_scan<UQ_WAVES>(n_miss, lds, tot_miss);
        uint32_t so = block_excl_scan<UQ_WAVES>(n_stale, lds, tot_stale);
#pragma unroll
        for (int it = 0; it < UQ_ITEMS; ++it) {
            if (is_miss[it]) ws.miss_stage[tile * UQ_TILE + mo++] = miss_rank[it];
            if (is_stale[it]) ws.stale_stage[tile * UQ_TILE + so++] = stale_rank[it];
        }
        const uint32_t tot_hit = block_sum<UQ_WAVES>(n_hit, lds);
        if (threadIdx.x == 0) {
            ws.tile_miss[tile] = tot_miss;
            ws.tile_stale[tile] = tot_stale;
            DState *ds = cv.ds;
            if (tot_hit) { atomicAdd(&ds->last.hit, (unsigned long long)tot_hit); atomicAdd(&ds->total.hit, (unsigned long long)tot_hit); }
            if (tot_stale) { atomicAdd(&ds->last.stale, (unsigned long long)tot_stale); atomicAdd(&ds->total.stale, (unsigned long long)tot_stale); }
            if (tot_miss) {
                atomicAdd(&ds->last.miss, (unsigned long long)tot_miss); atomicAdd(&ds->total.miss, (unsigned long long)tot_miss);
                atomicAdd(&ds->size, (int32_t)tot_miss);
            }
        }
    } else {
        if (__any(n_absent != 0) && lane_id() == 0) atomicOr(&cv.ds->err, ERRBIT_STATE);
    }
    if (tile + 1 == ntiles && threadIdx.x == UQ_THREADS - 1) {
        // the last thread of the last tile has seen every head
        const uint32_t U = r;
        cv.ds->n_unique = U;
        cv.ds->last.unique = U;
        atomicAdd(&cv.ds->total.unique, (unsigned long long)U);
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

// Fetch of the missed keys and Evict + Fetch of the stale ones (Algorithm 2).  Workgroup b
// serves the keys that tile b of rank_probe_kernel staged.  The i-th missed key in ascending
// key order takes the i-th free slot in ascending slot order.
template <int VEC>
__global__ __launch_bounds__(UQ_THREADS) void fill_kernel(CacheView cv, Workspace ws)
{
    __shared__ uint32_t lds[UQ_WAVES];
    const uint32_t tile = blockIdx.x;
    const uint32_t miss_before = block_sum_array<UQ_WAVES>(ws.tile_miss, tile, lds);
    const uint32_t my_miss = ws.tile_miss[tile], my_stale = ws.tile_stale[tile];
    const int lanes = cv.geom.lanes;
    const int group = threadIdx.x / lanes, gl = threadIdx.x % lanes, ngroups = UQ_THREADS / lanes;
    const uint32_t t = cv.ds->t;

    for (uint32_t m = group; m < my_miss; m += ngroups) {
        const uint32_t u = ws.miss_stage[tile * UQ_TILE + m];
        const uint32_t key = ws.ukey[u];
        const uint32_t slot = cv.free_list[miss_before + m];
        pull_row<VEC>(cv, key, slot, gl);
        if (gl == 0) {
            const uint32_t cg = cv.Cg[key];
            cv.cs[slot] = cg; cv.cc[slot] = cg;           // c_s = c_c = c_g
            cv.slot_key[slot] = key;
            cv.last_use[slot] = t;
            cv.freq[slot] = 1;
            ws.uslot[u] = (int32_t)slot;
            if (!ht_insert(cv.ht, key, slot)) atomicOr(&cv.ds->err, ERRBIT_INTERNAL);
        }
    }
    uint32_t dirty = 0;
    for (uint32_t m = group; m < my_stale; m += ngroups) {
        const uint32_t u = ws.stale_stage[tile * UQ_TILE + m];
        const uint32_t key = ws.ukey[u];
        const uint32_t slot = (uint32_t)ws.uslot[u];
        const bool has_updates = cv.cc[slot] > cv.cs[slot];
        if (has_updates) push_row<VEC>(cv, key, slot, gl);     // afterwards the global row equals the cached one
        else pull_row<VEC>(cv, key, slot, gl);
        if (gl == 0) {
            const uint32_t cg = cv.Cg[key];
            cv.cs[slot] = cg; cv.cc[slot] = cg;
            dirty += has_updates ? 1u : 0u;
        }
    }
    dirty = block_sum<UQ_WAVES>(dirty, lds);
    if (threadIdx.x == 0 && dirty) {
        atomicAdd(&cv.ds->last.stale_dirty, (unsigned long long)dirty);
        atomicAdd(&cv.ds->total.stale_dirty, (unsigned long long)dirty);
    }
}

// Get: out[perm[j]] = cached row of sorted position j.  One row group per position; the
// positions of one key are adjacent, so its row is read from HBM once and from cache after.
template <int VEC>
__global__ __launch_bounds__(256) void gather_kernel(CacheView cv, Workspace ws, uint32_t n, float *__restrict__ out)
{
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    for (uint32_t j = gid; j < n; j += ngroups) {
        const uint32_t r = ws.rank[j];
        float *dst = out + (size_t)ws.perm[j] * g.dim;
        if (r == KEY_NONE) row_zero<VEC>(dst, g.chunks, g.lanes, gl);
        else row_copy<VEC>(dst, cv.rows + (size_t)(uint32_t)ws.uslot[r] * g.dim, g.chunks, g.lanes, gl);
    }
}

// Pooled forms need, per original position, the rank of its key.
__global__ __launch_bounds__(256) void invert_kernel(Workspace ws, uint32_t n)
{
    for (uint32_t j = blockIdx.x * 256u + threadIdx.x; j < n; j += gridDim.x * 256u) ws.inv[ws.perm[j]] = ws.rank[j];
}

// Pooled Get: out[b] = sum over the bag, in bag order.  One row group per bag.
template <int VEC>
__global__ __launch_bounds__(256) void pooled_gather_kernel(CacheView cv, Workspace ws, const int64_t *__restrict__ offsets,
                                                            uint32_t n, uint32_t n_bags, float *__restrict__ out)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    for (uint32_t b = gid; b < n_bags; b += ngroups) {
        int64_t lo = offsets[b], hi = offsets[b + 1];
        lo = lo < 0 ? 0 : lo; hi = hi > (int64_t)n ? (int64_t)n : hi;
        for (int c = gl; c < g.chunks; c += g.lanes) {
            V sum{};
            for (int64_t i = lo; i < hi; ++i) {
                const uint32_t r = ws.inv[i];
                if (r == KEY_NONE) continue;
                const V v = reinterpret_cast<const V *>(cv.rows + (size_t)(uint32_t)ws.uslot[r] * g.dim)[c];
                if constexpr (VEC == 4) { sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w; }
                else sum += v;
            }
            reinterpret_cast<V *>(out + (size_t)b * g.dim)[c] = sum;
        }
    }
}

// Pooled Write: bag_of[i] = bag that position i belongs to.
__global__ __launch_bounds__(256) void bag_of_kernel(const int64_t *__restrict__ offsets, uint32_t n, uint32_t n_bags, uint32_t *__restrict__ bag_of)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) {
        uint32_t lo = 0, hi = n_bags;            // largest b with offsets[b] <= i
        while (hi - lo > 1) { const uint32_t mid = (lo + hi) / 2; if (offsets[mid] <= (int64_t)i) lo = mid; else hi = mid; }
        bag_of[i] = lo;
    }
}

// Update + Clock (Algorithm 3): per unique key, the sum of its gradients in order of
// increasing position, the optimizer step on the cached row, c_c += 1.  One row group per key.
// grad_row == nullptr: the gradient of position i is grads[i]; else grads[grad_row[i]].
template <int VEC>
__global__ __launch_bounds__(256) void apply_kernel(CacheView cv, Workspace ws, const float *__restrict__ grads,
                                                    const uint32_t *__restrict__ grad_row, float lr, float eps)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t ngroups = gridDim.x * 256u / g.lanes;
    const uint32_t U = cv.ds->n_unique;
    for (uint32_t u = gid; u < U; u += ngroups) {
        const int32_t slot = ws.uslot[u];
        if (slot == SLOT_NONE) continue;
        const uint32_t lo = ws.seg[u], hi = ws.seg[u + 1];
        for (int c = gl; c < g.chunks; c += g.lanes) {
            // The sum runs in fp64 and is rounded to fp32 once: the kernel is bound by reading the
            // gradients, and a long run of a popular key no longer loses digits to its order.
            double acc64[VEC] = {};
            for (uint32_t j = lo; j < hi; ++j) {
                uint32_t src = ws.perm[j];
                if (grad_row) src = grad_row[src];
                const V v = reinterpret_cast<const V *>(grads + (size_t)src * g.dim)[c];
                if constexpr (VEC == 4) { acc64[0] += v.x; acc64[1] += v.y; acc64[2] += v.z; acc64[3] += v.w; }
                else acc64[0] += v;
            }
            V G;
            if constexpr (VEC == 4) { G.x = (float)acc64[0]; G.y = (float)acc64[1]; G.z = (float)acc64[2]; G.w = (float)acc64[3]; }
            else G = (float)acc64[0];
            V *xp = reinterpret_cast<V *>(cv.rows + (size_t)slot * g.dim) + c;
            V x = *xp;
            if (cv.adagrad) {
                V *ap = reinterpret_cast<V *>(cv.acc + (size_t)slot * g.dim) + c;
                V a = *ap;
                if constexpr (VEC == 4) {
                    a.x += G.x * G.x; a.y += G.y * G.y; a.z += G.z * G.z; a.w += G.w * G.w;
                    x.x -= lr * G.x / (sqrtf(a.x) + eps); x.y -= lr * G.y / (sqrtf(a.y) + eps);
                    x.z -= lr * G.z / (sqrtf(a.z) + eps); x.w -= lr * G.w / (sqrtf(a.w) + eps);
                } else {
                    a += G * G; x -= lr * G / (sqrtf(a) + eps);
                }
                *ap = a;
            } else {
                if constexpr (VEC == 4) { x.x -= lr * G.x; x.y -= lr * G.y; x.z -= lr * G.z; x.w -= lr * G.w; }
                else x -= lr * G;
            }
            *xp = x;
        }
        if (gl == 0) cv.cc[slot] += 1;               // Clock(k)
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
constexpr int TRIM_TILE = TRIM_THREADS * TRIM_ITEMS;   // 1024 slots per workgroup

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
// Every thread of the block gets the same answer.  lds: SEL_BINS words + TRIM_WAVES + 1.
__device__ __forceinline__ void sel_replay(const TrimPlan &tp, int upto, uint32_t m, uint64_t &prefix,
                                           uint32_t &remaining, uint32_t *lds_bins, uint32_t *lds_scan)
{
    prefix = 0; remaining = m;
    for (int p = 0; p < upto; ++p) {
        const int width = sel_width(tp, p), bins = 1 << width;
        // exclusive scan of this pass's histogram: bins <= 2048 = 8 per thread
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
            // the digit whose cumulative count first exceeds `remaining - 1`
            if (local[q] && run < remaining && remaining <= run + local[q]) { lds_bins[0] = (uint32_t)b; lds_bins[1] = run; }
            run += local[q];
        }
        __syncthreads();
        const uint32_t digit = lds_bins[0], below = lds_bins[1];
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
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    if (over <= 0) return;
    uint64_t prefix; uint32_t remaining;
    sel_replay(tp, pass, (uint32_t)over, prefix, remaining, bins, scan);
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
    __shared__ uint32_t bins[SEL_BINS];
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    if (over <= 0) return;
    uint64_t tau; uint32_t take_eq;
    sel_replay(tp, tp.passes, (uint32_t)over, tau, take_eq, bins, scan);
    uint32_t eq = 0;
#pragma unroll
    for (int it = 0; it < TRIM_ITEMS; ++it) {
        const uint32_t slot = blockIdx.x * TRIM_TILE + threadIdx.x * TRIM_ITEMS + it;
        if (slot < cv.n_slots && cv.slot_key[slot] != KEY_NONE && policy_key(cv, tp, slot) == tau) ++eq;
    }
    eq = block_sum<TRIM_WAVES>(eq, scan);
    if (threadIdx.x == 0) tp.tile_eq[blockIdx.x] = eq;
}

// Drops the victims of one slot tile: push if the row holds updates, erase the key, free the
// slot.  Leaves the tile's number of free slots for the free-list kernel.
template <int VEC>
__global__ __launch_bounds__(TRIM_THREADS) void trim_evict_kernel(CacheView cv, TrimPlan tp)
{
    __shared__ uint32_t bins[SEL_BINS];
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    __shared__ uint32_t victims[TRIM_TILE];
    __shared__ uint32_t n_victims;
    const uint32_t tile = blockIdx.x;
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    uint64_t tau = 0; uint32_t take_eq = 0;
    uint32_t eq_before = 0;
    if (over > 0) {
        sel_replay(tp, tp.passes, (uint32_t)over, tau, take_eq, bins, scan);
        eq_before = block_sum_array<TRIM_WAVES>(tp.tile_eq, tile, scan);
    }
    if (threadIdx.x == 0) n_victims = 0;
    // local order of the rows equal to tau: slot order
    uint32_t my_eq = 0, free_here = 0;
    bool eqf[TRIM_ITEMS], ltf[TRIM_ITEMS];
#pragma unroll
    for (int it = 0; it < TRIM_ITEMS; ++it) {
        const uint32_t slot = tile * TRIM_TILE + threadIdx.x * TRIM_ITEMS + it;
        eqf[it] = ltf[it] = false;
        if (slot >= cv.n_slots) continue;
        if (cv.slot_key[slot] == KEY_NONE) { ++free_here; continue; }
        if (over > 0) {
            const uint64_t k = policy_key(cv, tp, slot);
            ltf[it] = k < tau; eqf[it] = k == tau;
            my_eq += eqf[it] ? 1u : 0u;
        }
    }
    uint32_t tot_eq;
    uint32_t eq_rank = eq_before + block_excl_scan<TRIM_WAVES>(my_eq, scan, tot_eq);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < TRIM_ITEMS; ++it) {
        const uint32_t slot = tile * TRIM_TILE + threadIdx.x * TRIM_ITEMS + it;
        bool victim = ltf[it];
        if (eqf[it]) { victim = eq_rank < take_eq; ++eq_rank; }
        if (victim) victims[atomicAdd(&n_victims, 1u)] = slot;
    }
    __syncthreads();
    const uint32_t nv = n_victims;
    const int lanes = cv.geom.lanes;
    const int group = threadIdx.x / lanes, gl = threadIdx.x % lanes, ngroups = TRIM_THREADS / lanes;
    uint32_t dirty = 0;
    for (uint32_t v = group; v < nv; v += ngroups) {
        const uint32_t slot = victims[v];
        const uint32_t key = cv.slot_key[slot];
        const bool has_updates = cv.cc[slot] > cv.cs[slot];
        if (has_updates) push_row<VEC>(cv, key, slot, gl);
        if (gl == 0) {
            dirty += has_updates ? 1u : 0u;
            ht_erase(cv.ht, key);
            tp.ev_ids[atomicAdd(&cv.ds->ev_n, 1u)] = key;
        }
    }
    __syncthreads();
    for (uint32_t v = threadIdx.x; v < nv; v += TRIM_THREADS) cv.slot_key[victims[v]] = KEY_NONE;
    dirty = block_sum<TRIM_WAVES>(dirty, scan);
    free_here = block_sum<TRIM_WAVES>(free_here, scan);
    if (threadIdx.x == 0) {
        tp.tile_free[tile] = free_here + nv;
        if (nv) { atomicAdd(&cv.ds->last.evicted, (unsigned long long)nv); atomicAdd(&cv.ds->total.evicted, (unsigned long long)nv); }
        if (dirty) { atomicAdd(&cv.ds->last.evicted_dirty, (unsigned long long)dirty); atomicAdd(&cv.ds->total.evicted_dirty, (unsigned long long)dirty); }
    }
}

// Lists the free slots in ascending order (only the first max_ids are ever needed) and settles
// the row count after the trim.
__global__ __launch_bounds__(TRIM_THREADS) void trim_free_kernel(CacheView cv, TrimPlan tp)
{
    __shared__ uint32_t scan[TRIM_WAVES + 1];
    const uint32_t tile = blockIdx.x;
    if (tile == 0 && threadIdx.x == 0 && cv.ds->size > (int32_t)cv.capacity) cv.ds->size = (int32_t)cv.capacity;
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
    if (threadIdx.x == 0 && pushed) {
        atomicAdd(&cv.ds->last.flushed, (unsigned long long)pushed);
        atomicAdd(&cv.ds->total.flushed, (unsigned long long)pushed);
    }
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
