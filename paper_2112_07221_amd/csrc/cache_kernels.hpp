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

// Clocks (Section 3.1) and policy counters (Section 4.3) of one cache slot; read and written
// as one 16-byte word where several fields are needed.
struct alignas(16) SlotMeta {
    uint32_t cs;         // start clock c_s
    uint32_t cc;         // local clock c_c
    uint32_t last_use;   // iteration of the last Read that had the key
    uint32_t freq;       // number of Reads that had the key since it was fetched
};
__device__ __forceinline__ uint4 load_meta(const SlotMeta *m, uint32_t slot) { return reinterpret_cast<const uint4 *>(m)[slot]; }
__device__ __forceinline__ void store_meta(SlotMeta *m, uint32_t slot, uint32_t cs, uint32_t cc, uint32_t lu, uint32_t fr)
{
    reinterpret_cast<uint4 *>(m)[slot] = make_uint4(cs, cc, lu, fr);
}

// A global table in pinned host memory is written behind the step: a trim copies the rows it
// evicts (those that hold updates) into a staging buffer in HBM, and the copy over the host link
// travels inside the next Read's fetch kernel, where it shares the link, which is full duplex,
// with the fetches going the other way.  `pend` lets a fetch find a row that is still on its way.
struct HostLink {
    float *rows[2], *acc[2];      // staging, [max_ids][dim] each; trims alternate between the two
    uint32_t *keys[2], *cg[2];    // per staged row: its key and the global clock it will carry
    uint64_t *pend;               // [vocab]: (serial number of the trim << 32) | staging index of the key's staged row,
                                  // or (tag of a list of keys fetched ahead << 32) | place in that list; the tags' top bit tells them apart
    // rows of the coming batch fetched ahead of its Read (Section 4.2), [max_ids] each: the listed keys, where a key's
    // row is staged if its write-back is still to come (else KEY_NONE: it comes from the table), and the rows
    uint32_t *pf_keys, *pf_from;
    float *pf_rows, *pf_acc;
    // (selected, not indexed: indexing kernel arguments at run time would put them in scratch memory)
    __device__ __forceinline__ float *rows_of(int b) const { return b ? rows[1] : rows[0]; }
    __device__ __forceinline__ float *acc_of(int b) const { return b ? acc[1] : acc[0]; }
    __device__ __forceinline__ uint32_t *keys_of(int b) const { return b ? keys[1] : keys[0]; }
    __device__ __forceinline__ uint32_t *cg_of(int b) const { return b ? cg[1] : cg[0]; }
};

// Everything a kernel needs to know about one cache, passed by value.
struct CacheView {
    // global table (Section 3.1): rows, optimizer state, global clock c_g
    float *W, *A;
    uint32_t *Cg;         // the clocks the kernels work on: the caller's array, or its mirror in HBM for a host-backed table
    uint32_t *Cg_host;    // host-backed table: the caller's array, written through; else null
    HostLink hl;
    uint32_t vocab;
    // cache slots
    float *rows, *acc;
    float *rows0, *acc0;  // several workers: every cached row (accumulator) as it was fetched; else null
    // Early push (table in HBM, one worker): the update that fetches a missed key's row (see apply_kernel,
    // fresh rows) writes its result to the global table as well as to the slot, and early_cc[slot] is the
    // c_c at which the two are equal.  A victim whose c_c is still that, and whose global clock is still
    // the c_s it was fetched at (nobody else pushed), is evicted without copying its row: Evict's push
    // has already travelled.  0: not equal at any c_c a row with updates can have.  nullptr: not in use.
    uint32_t *early_cc;
    int many;             // several workers write the global table: Evict pushes what was accumulated since the Fetch (Section 3.1)
    uint32_t freq_cap;    // light-weight LFU (Section 4.3): a row used this often is no longer kept track of; 0: exact policies
    uint32_t *slot_key;
    SlotMeta *meta;       // start clock, local clock, LRU stamp, LFU count: one 16-byte record per slot
    uint32_t n_slots;     // capacity + max_batch_ids
    uint32_t capacity;
    uint32_t max_ids;
    int64_t s;            // staleness bound
    HashTable ht;
    uint32_t *free_list;  // free slots in ascending order (first max_ids of them)
    uint8_t *was_free;    // per slot: free when the current lookup began (its fetches may be filling it now)
    DState *ds;
    Counters *last;       // this call's counters (one of ds->call)
    Counters *next_call;  // the other one: cleared by this call for the next
    RowGeom geom;
    int adagrad;          // element-wise Adagrad: an accumulator row beside every row
    int rowwise;          // row-wise Adagrad: one accumulator per row (acc[slot], A[key]); rows of at most one piece per lane
    int direct;           // no cache: rows/acc alias the global table, a key is its own slot, there are no clocks
};

constexpr int32_t SRC_BACKING = -1;   // gather reads the global row: the key was not cached (or is refetched)
constexpr int32_t SRC_ZERO = -2;      // id outside the vocabulary: the output row is zero

constexpr int PT_THREADS = 1024;                // probe tiles: 1024 sorted positions per workgroup,
constexpr int PT_WAVES = PT_THREADS / WAVE;     // one per thread, so every probe's loads are in flight at once
constexpr int PT_TILE = PT_THREADS;
constexpr int VERIFY_TILE = 1024;                    // positions one workgroup of the id check covers

// Per-call workspaces (sized by max_batch_ids unless noted).  Per-key facts are stored at the
// key's head position in the sorted order.
struct Workspace {
    uint32_t *skey, *perm;        // sorted keys and their original positions
    int32_t *src;                 // per sorted position: slot to gather from, or SRC_*
    int32_t *head_slot;           // at heads: slot of the key (set by fill for a missed key)
    uint8_t *cls;                 // at heads: HIT / STALE / MISS (lookup)
    uint32_t *tile_miss, *tile_stale;     // per probe tile counts
    uint2 *miss_stage, *stale_stage;      // per probe tile: (head position, key) of its missed / stale keys
    uint32_t *bag_of;             // pooled: bag of each original position
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
    int h0_kept;      // the first pass's histogram is kept up to date between trims (by the probe and the eviction), not counted anew
    uint32_t *hist;   // [SEL_MAX_PASSES][SEL_BINS] followed by sup_cnt: zeroed together before the first pass
    uint32_t zero_words;
    uint4 *blk_cnt, *sup_cnt;          // per 1024 slots, and per EV_SUPER such blocks: cached rows with a policy key
                                       // below the threshold (x), equal to it (y), and those of each that hold updates (z, w)
    uint32_t *tile_free;               // free slots per 1024-slot tile
    uint32_t *ev_ids;                  // ids dropped by this trim
    int ev_slot;                       // which of the two evicted-id counts (and staging buffers) this trim appends to
    uint32_t push_seq;                 // host-backed table: serial number of this trim (never 0)
    uint32_t dirty_stamp;              // the tie count runs beside the optimizer step of the Read of this iteration's keys (0: it does not):
                                       // every row that Read touched will hold updates when the step is done, whether its clock has moved yet or not
};

__device__ __forceinline__ uint64_t policy_key(const TrimPlan &tp, const uint4 &meta)
{
    const uint64_t lu = meta.z;
    return tp.lfu ? (((uint64_t)meta.w << tp.bits) | lu) : lu;
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

// LDS of one select stage (a workgroup of TRIM_THREADS threads).
struct TrimLds {
    uint32_t bins[SEL_BINS];
    uint32_t pick[2];
    uint32_t scan[TRIM_WAVES + 1];
};

// Kernels that carry a stage of the next minibatch's sort give it their first workgroups (its
// chain of dependent steps is the longest, so it starts first) and number their own from
// there.  All roles of a kernel share one dynamically sized LDS buffer; the host sizes it for
// the largest role present.
extern __shared__ __align__(16) unsigned char dyn_lds[];
template <typename T> __device__ __forceinline__ T &lds_as() { return *reinterpret_cast<T *>(dyn_lds); }

// Up to two sort stages, of two different announced batches, travel in one kernel.  Returns
// true if this workgroup ran one of them; otherwise bid / nblk number the kernel's own workgroups.
// HIST_ONLY: both are known to be histogram stages (cheap in registers).
template <bool HIST_ONLY = false>
__device__ __forceinline__ bool run_carried(const SortStage &a, const SortStage &b, uint32_t &bid, uint32_t &nblk)
{
    uint32_t *lds = reinterpret_cast<uint32_t *>(dyn_lds);
    if (bid < a.blocks + b.blocks) {
        const bool first = bid < a.blocks;
        const SortStage &st = first ? a : b;
        const uint32_t tile = first ? bid : bid - a.blocks;
        if (HIST_ONLY) { __builtin_amdgcn_s_setprio(3); sort_hist_body(st, tile, lds); }
        else sort_stage_body(st, tile, lds);
        return true;
    }
    bid -= a.blocks + b.blocks; nblk -= a.blocks + b.blocks;
    return false;
}

// One histogram pass of the select over the rows whose key matches the prefix chosen so far.
// Runs in `nblocks` workgroups of TRIM_THREADS threads; `vblock` is this one's index.
// `beside_fill` (the pass runs beside the lookup's fetches): slots that were free when the lookup
// began are skipped - they are being filled right now - and the rows fetched into them, which
// all carry the policy key (freq 1, last_use t_now), are counted from their number `new_rows`.
// `always`: counts even if nothing has to be evicted (the first pass's histogram is kept from
// here on, see h0_shift).
__device__ __forceinline__ void trim_hist_body(const CacheView &cv, const TrimPlan &tp, int pass, uint32_t vblock, uint32_t nblocks, TrimLds &l,
                                               bool beside_fill = false, uint32_t new_rows = 0, uint32_t t_now = 0, bool always = false)
{
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    if (over <= 0 && !always) return;
    uint64_t prefix; uint32_t remaining;
    sel_replay(tp, pass, (uint32_t)over, prefix, remaining, l.pick, l.scan);
    for (int b = threadIdx.x; b < SEL_BINS; b += TRIM_THREADS) l.bins[b] = 0;
    __syncthreads();
    const int shift = sel_shift(tp, pass), width = sel_width(tp, pass);
    const int decided = shift + width;                 // bits above are fixed by the prefix
    if (beside_fill && vblock == 0 && threadIdx.x == 0 && new_rows) {
        const uint64_t k = policy_key(tp, make_uint4(0, 0, t_now, 1));
        if (decided >= 64 || (k >> decided) == (prefix >> decided))
            atomicAdd(&tp.hist[pass * SEL_BINS + ((uint32_t)(k >> shift) & ((1u << width) - 1u))], new_rows);
    }
    for (uint32_t slot = vblock * TRIM_THREADS + threadIdx.x; slot < cv.n_slots; slot += nblocks * TRIM_THREADS) {
        const uint32_t sk = cv.slot_key[slot];
        const uint4 m = load_meta(cv.meta, slot);
        const bool skip = beside_fill ? cv.was_free[slot] != 0 : sk == KEY_NONE;
        if (skip) continue;
        const uint64_t k = policy_key(tp, m);
        if (decided < 64 && (k >> decided) != (prefix >> decided)) continue;
        atomicAdd(&l.bins[(uint32_t)(k >> shift) & ((1u << width) - 1u)], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < SEL_BINS; b += TRIM_THREADS)
        if (l.bins[b]) atomicAdd(&tp.hist[pass * SEL_BINS + b], l.bins[b]);
}

// The first pass's histogram (policy keys of all cached rows by their top digit) need not be
// counted anew for every trim: a Read changes the keys of the rows it finds and adds the rows it
// fetches, a trim removes its victims, nothing else touches policy keys.  So the probe moves the
// rows it touches from their old bin to their new one, and the eviction takes its victims out
// (h0_remove_victims); the select of the next trim starts at its second pass.  The digit layout
// depends on the width of the iteration count: when that grows, the histogram is counted afresh.
__device__ __forceinline__ uint32_t h0_bin(const TrimPlan &tp, uint64_t key)
{
    return (uint32_t)(key >> sel_shift(tp, 0)) & ((1u << sel_width(tp, 0)) - 1u);
}

// All rows in bins below the threshold's first digit were evicted, and of that digit's bin as
// many as the select still had to find there.  One workgroup of TRIM_THREADS threads.
__device__ __forceinline__ void h0_remove_victims(const CacheView &cv, const TrimPlan &tp, uint32_t *lds_pick, uint32_t *lds_scan)
{
    const int32_t over = cv.ds->over;
    if (over <= 0) return;
    uint64_t prefix; uint32_t remaining;
    sel_replay(tp, 1, (uint32_t)over, prefix, remaining, lds_pick, lds_scan);       // (ends with a barrier: every thread has read its bins)
    const uint32_t d0 = h0_bin(tp, prefix);
    for (uint32_t b = threadIdx.x; b < d0; b += TRIM_THREADS) tp.hist[b] = 0;
    if (threadIdx.x == 0) tp.hist[d0] -= remaining;
}

// Sums eight values per thread over the block at once (every thread gets all sums).
// `lds` needs TRIM_WAVES * 8 words.
__device__ __forceinline__ void block_sum8(uint32_t (&v)[8], uint32_t *lds)
{
    const uint32_t lane = lane_id(), w = threadIdx.x / WAVE;
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = wave_sum(v[k]);
    __syncthreads();
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) lds[w * 8 + k] = v[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t t = 0;
#pragma unroll
        for (int ww = 0; ww < TRIM_WAVES; ++ww) t += lds[ww * 8 + k];
        v[k] = t;
    }
}

// Last stage of the select: finds tau (replaying the passes) and counts, per block of EV_SLOTS
// slots (the eviction's workgroups), the cached rows whose policy key lies below tau and those
// whose key equals it, and how many of each hold updates; sup_cnt adds these up per EV_SUPER
// blocks (zero when the select starts).  With these counts the eviction places every victim by
// arithmetic alone (count at the producer, prefix at the consumer).  A workgroup of the count
// covers COUNT_SLOTS slots, a wave of it one block of EV_SLOTS (the replay is paid once per
// workgroup, so the count uses few, the eviction many).
constexpr int EV_ITEMS = 1;
constexpr int EV_SLOTS = TRIM_THREADS * EV_ITEMS;
constexpr int EV_SUPER = 32;
constexpr int COUNT_ITEMS = EV_SLOTS / WAVE;                   // consecutive slots per lane: a wave covers EV_SLOTS
constexpr int COUNT_SLOTS = TRIM_THREADS * COUNT_ITEMS;
static_assert(TRIM_TILE % EV_SLOTS == 0, "eviction workgroups do not straddle free-list tiles");
static_assert(EV_SLOTS % WAVE == 0, "a wave of the count covers one eviction block");

// The slots of a thread: keys (KEY_NONE beyond the end) and metadata.
template <int ITEMS>
__device__ __forceinline__ void load_slots(const CacheView &cv, uint32_t slot0, uint32_t (&key)[ITEMS], uint4 (&meta)[ITEMS])
{
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool in = slot0 + i < cv.n_slots;
        key[i] = in ? cv.slot_key[slot0 + i] : KEY_NONE;
        meta[i] = in ? load_meta(cv.meta, slot0 + i) : make_uint4(0, 0, 0, 0);
    }
}

__device__ __forceinline__ void trim_count_body(const CacheView &cv, const TrimPlan &tp, uint32_t vblock, TrimLds &l)
{
    const int32_t over = cv.ds->size - (int32_t)cv.capacity;
    if (vblock == 0 && threadIdx.x == 0) cv.ds->over = over;
    if (over <= 0) return;
    uint32_t key[COUNT_ITEMS];
    uint4 meta[COUNT_ITEMS];
    load_slots<COUNT_ITEMS>(cv, vblock * COUNT_SLOTS + threadIdx.x * COUNT_ITEMS, key, meta);      // loads first: they overlap the replay
    uint64_t tau; uint32_t take_eq;
    sel_replay(tp, tp.passes, (uint32_t)over, tau, take_eq, l.pick, l.scan);
    uint32_t lt = 0, eq = 0, dlt = 0, deq = 0;
#pragma unroll
    for (int i = 0; i < COUNT_ITEMS; ++i) {
        const bool cached = key[i] != KEY_NONE;
        const uint64_t pk = policy_key(tp, meta[i]);
        const bool dirty = meta[i].y > meta[i].x || (tp.dirty_stamp && meta[i].z == tp.dirty_stamp);
        if (cached && pk < tau) { lt += 1; dlt += dirty; }
        else if (cached && pk == tau) { eq += 1; deq += dirty; }
    }
    // counts of an eviction block stay below 2^16: two to a word
    const uint32_t a = wave_sum(lt | (eq << 16));
    const uint32_t b = wave_sum(dlt | (deq << 16));
    const uint32_t eblk = vblock * TRIM_WAVES + threadIdx.x / WAVE;               // the eviction block this wave covered
    if (lane_id() == 0 && eblk * EV_SLOTS < cv.n_slots) {
        const uint4 c = make_uint4(a & 0xFFFFu, a >> 16, b & 0xFFFFu, b >> 16);
        tp.blk_cnt[eblk] = c;
        uint32_t *sup = reinterpret_cast<uint32_t *>(&tp.sup_cnt[eblk / EV_SUPER]);
        if (c.x) atomicAdd(&sup[0], c.x);
        if (c.y) atomicAdd(&sup[1], c.y);
        if (c.z) atomicAdd(&sup[2], c.z);
        if (c.w) atomicAdd(&sup[3], c.w);
    }
    if (vblock == 0 && threadIdx.x == 0) { cv.ds->sel_tau = tau; cv.ds->sel_take = take_eq; }
}

// Stage `stage` of the select: the histogram passes first, then the count.  Kernels that have
// nothing to do with the trim (the optimizer step) carry a stage in extra workgroups, because
// at minibatch size a kernel boundary costs more than the stage's work.
__device__ __forceinline__ void trim_stage_body(const CacheView &cv, const TrimPlan &tp, int stage, uint32_t vblock, uint32_t nblocks, TrimLds &l)
{
    if (stage < tp.passes) trim_hist_body(cv, tp, stage, vblock, nblocks, l);
    else trim_count_body(cv, tp, vblock, l);
}

__global__ __launch_bounds__(TRIM_THREADS) void trim_stage_kernel(CacheView cv, TrimPlan tp, int stage)
{
    __shared__ TrimLds l;
    trim_stage_body(cv, tp, stage, blockIdx.x, gridDim.x, l);
}

// Lists the free slots of one 1024-slot tile in ascending order behind those of the earlier
// tiles (only the first max_ids are ever needed).  tile_free holds the free count of every
// tile, left by the last trim; the idle twin of that array is cleared for the next trim.
// Workgroup of PT_THREADS threads, one slot each.
__device__ __forceinline__ void free_list_body(const CacheView &cv, const uint32_t *tile_free, uint32_t *tile_free_idle, uint32_t ev_idle,
                                               uint32_t tile, uint32_t *lds)
{
    if (threadIdx.x == 0) tile_free_idle[tile] = 0;
    if (tile == 0 && threadIdx.x == 0) cv.ds->ev_n[ev_idle] = 0;      // (push_n is written by every eviction, and a write-back on its way may still read it)
    const uint32_t slot = tile * PT_TILE + threadIdx.x;
    const bool fr = slot < cv.n_slots && cv.slot_key[slot] == KEY_NONE;
    if (slot < cv.n_slots) cv.was_free[slot] = fr ? 1 : 0;
    const uint32_t before = block_sum_array<PT_WAVES>(tile_free, tile, lds);
    if (before >= cv.max_ids) return;
    uint32_t tot;
    const uint32_t pos = before + block_excl_scan<PT_WAVES>(fr ? 1u : 0u, lds, tot);
    if (fr && pos < cv.max_ids) cv.free_list[pos] = slot;
}

// Find for every sorted position; at the head of every run of equal keys also CheckValid and
// the policy's use count.  LOOKUP: classifies HIT / STALE / MISS, stages missed and stale keys
// per tile for the fill kernel and tells the gather where each position's row comes from.
// Otherwise (update that sorted its own ids): only resolves slots and flags keys not cached.
// Compares one tile of a sorted order with the ids it was built from (PT_THREADS threads).
__device__ __forceinline__ void check_order_body(const CacheView &cv, const Workspace &ws, const int64_t *__restrict__ ids, uint32_t n, uint32_t tile)
{
    const uint32_t j = tile * PT_TILE + threadIdx.x;
    bool changed = false;
    if (j < n) {
        const int64_t id = ids[ws.perm[j]];
        const uint32_t expect = (id < 0 || id >= (int64_t)cv.vocab) ? cv.vocab : (uint32_t)id;
        changed = expect != ws.skey[j];
    }
    if (__any(changed) && lane_id() == 0) atomicOr(&cv.ds->err, ERRBIT_STATE);
}

template <bool LOOKUP>
__global__ __launch_bounds__(PT_THREADS) void probe_kernel(CacheView cv, Workspace ws, uint32_t n, uint32_t t_now, uint32_t ptiles,
                                                           const uint32_t *tile_free, uint32_t *tile_free_idle, uint32_t ev_idle,
                                                           uint32_t *zero_from, uint32_t zero_words, TrimPlan tp,
                                                           const int64_t *__restrict__ check_ids, int pf_idle = -1,
                                                           uint32_t *__restrict__ inv = nullptr)
{
    __shared__ uint32_t lds[PT_WAVES + 1];
    __shared__ uint32_t h0_delta[LOOKUP ? SEL_BINS : 1];       // rows entering (+) and leaving (-) each bin of the kept histogram
    const uint32_t check_blocks = LOOKUP && check_ids ? ptiles : 0u;
    if (blockIdx.x >= ptiles && blockIdx.x < ptiles + check_blocks) {
        // An order that was sorted ahead of this call (an announced batch) is checked against the ids
        // as they are now: the announcement promised they would not change.  Workgroups of their own,
        // on compute units the probe leaves idle.
        check_order_body(cv, ws, check_ids, n, blockIdx.x - ptiles);
        return;
    }
    if (blockIdx.x >= ptiles) {          // extra workgroups of a lookup: the free list for the fill kernel
        // ... and clean select histograms for the trim that follows this lookup
        const uint32_t first = ptiles + check_blocks;
        for (uint32_t i = (blockIdx.x - first) * PT_THREADS + threadIdx.x; i < zero_words; i += (gridDim.x - first) * PT_THREADS) zero_from[i] = 0;
        free_list_body(cv, tile_free, tile_free_idle, ev_idle, blockIdx.x - first, lds);
        return;
    }
    const uint32_t tile = blockIdx.x;
    const uint32_t vocab = cv.vocab;
    const uint32_t j = tile * PT_TILE + threadIdx.x;
    DState *ds = cv.ds;
    if (LOOKUP && inv && j < n) inv[ws.perm[j]] = j;         // pooled lookup: the sorted position of every original position
    const bool keep_h0 = LOOKUP && tp.h0_kept;
    if (keep_h0) {
        for (int b = threadIdx.x; b < SEL_BINS; b += PT_THREADS) h0_delta[b] = 0;
        __syncthreads();
    }

    if (tile == 0 && threadIdx.x == 0) {                      // this call's bookkeeping
        Counters z{};
        *cv.next_call = z;
        cv.last->n = n;
        atomicAdd(&ds->total.n, (unsigned long long)n);
        if (LOOKUP) ds->t = t_now;
        if (LOOKUP && pf_idle >= 0) ds->pf_n[pf_idle] = 0;    // the list of keys to fetch ahead that this lookup's second kernel may fill
    }
    // Find runs once per key, not once per position: by the head of every run of equal keys, and by
    // each wave's first lane (its run may have begun in the wave before); the other positions of a
    // run take where their row comes from from the nearest such lane below them.
    bool head = false, miss = false, stale = false, hit = false, absent = false, bad = false, finder = false;
    int32_t my_src = SRC_ZERO;
    if (j < n) {
        const uint32_t key = ws.skey[j];
        if (key == vocab) {                                   // id outside the vocabulary
            bad = true;
            if (LOOKUP) ws.src[j] = SRC_ZERO;
            ws.head_slot[j] = SLOT_NONE;
            if (j == 0) ds->n_valid = 0;                      // not one valid id in the call
        } else {
            head = j == 0 || ws.skey[j - 1] != key;
            if (j + 1 == n || ws.skey[j + 1] == vocab) ds->n_valid = j + 1;    // one writer: the last valid position
            finder = head || (LOOKUP && lane_id() == 0);
            if (finder) {
                const uint32_t cg = LOOKUP ? cv.Cg[key] : 0u;        // in flight together with the probe's loads
                const int32_t slot = ht_find(cv.ht, key);
                int32_t src = slot == SLOT_NONE ? SRC_BACKING : slot;
                bool valid = true;
                uint4 m = make_uint4(0, 0, 0, 0);
                if (LOOKUP && slot != SLOT_NONE) {
                    m = load_meta(cv.meta, (uint32_t)slot);
                    const uint32_t cs = m.x, cc = m.y;
                    valid = check_valid(cs, cc, cg, cv.s);
                    // A stale row that holds no updates of its own is refetched: its value is the
                    // global row.  (One with updates is pushed first, so its own value stays current.)
                    if (!valid && !(cc > cs)) src = SRC_BACKING;
                }
                my_src = src;
                if (head) {
                    ws.head_slot[j] = slot;
                    if (LOOKUP) {
                        if (slot == SLOT_NONE) miss = true;
                        else {
                            hit = valid; stale = !valid;
                            const bool upkeep = !(cv.freq_cap && m.w >= cv.freq_cap);        // (light-weight LFU: frequent enough, left alone)
                            if (upkeep) store_meta(cv.meta, (uint32_t)slot, m.x, m.y, t_now, m.w + 1);   // one use per key per Read
                            if (keep_h0 && upkeep) {
                                const uint32_t b_old = h0_bin(tp, policy_key(tp, m)), b_new = h0_bin(tp, policy_key(tp, make_uint4(0, 0, t_now, m.w + 1)));
                                if (b_old != b_new) { atomicSub(&h0_delta[b_old], 1u); atomicAdd(&h0_delta[b_new], 1u); }
                            }
                        }
                        ws.cls[j] = (uint8_t)(miss ? CLS_MISS : (stale ? CLS_STALE : CLS_HIT));
                    } else {
                        absent = slot == SLOT_NONE;
                    }
                }
            }
        }
    }
    if (LOOKUP) {
        const uint64_t below = __ballot(finder) & (~0ull >> (63u - lane_id()));
        const int from = below ? 63 - __builtin_clzll(below) : 0;
        const int32_t src = __shfl(my_src, from, WAVE);           // (a valid key has a finder at or below its lane: sorted keys, the invalid ones last)
        if (j < n && !bad) ws.src[j] = src;
    }

    if (__any(bad) && lane_id() == 0) atomicOr(&ds->err, ERRBIT_RANGE);
    if (LOOKUP) {
        // stage this tile's missed and stale keys, in key order, for the fill kernel
        // (a tile has 1024 positions: two counts to a word, one pass of barriers for each pair)
        uint32_t tot_ms;
        const uint32_t ms = block_excl_scan<PT_WAVES>((miss ? 1u : 0u) | (stale ? 1u << 16 : 0u), lds, tot_ms);
        const uint32_t mo = ms & 0xFFFFu, so = ms >> 16, tot_miss = tot_ms & 0xFFFFu, tot_stale = tot_ms >> 16;
        if (miss) ws.miss_stage[tile * PT_TILE + mo] = make_uint2(j, ws.skey[j]);
        if (stale) ws.stale_stage[tile * PT_TILE + so] = make_uint2(j, ws.skey[j]);
        const uint32_t tot_hh = block_sum<PT_WAVES>((hit ? 1u : 0u) | (head ? 1u << 16 : 0u), lds);
        const uint32_t tot_hit = tot_hh & 0xFFFFu, tot_heads = tot_hh >> 16;
        if (threadIdx.x == 0) {
            ws.tile_miss[tile] = tot_miss;
            ws.tile_stale[tile] = tot_stale;
            count2(&cv.last->hit, &ds->total.hit, tot_hit);
            count2(&cv.last->stale, &ds->total.stale, tot_stale);
            count2(&cv.last->miss, &ds->total.miss, tot_miss);
            count2(&cv.last->unique, &ds->total.unique, tot_heads);
            if (tot_miss) atomicAdd(&ds->size, (int32_t)tot_miss);
            if (keep_h0 && tot_miss) atomicAdd(&h0_delta[h0_bin(tp, policy_key(tp, make_uint4(0, 0, t_now, 1)))], tot_miss);   // the rows being fetched
        }
        if (keep_h0) {
            __syncthreads();
            for (int b = threadIdx.x; b < SEL_BINS; b += PT_THREADS)
                if (h0_delta[b]) atomicAdd(&tp.hist[b], h0_delta[b]);          // (differences, modulo 2^32)
        }
    } else {
        if (__any(absent) && lane_id() == 0) atomicOr(&ds->err, ERRBIT_STATE);
        const uint32_t tot_heads = block_sum<PT_WAVES>(head ? 1u : 0u, lds);
        if (threadIdx.x == 0) count2(&cv.last->unique, &ds->total.unique, tot_heads);
    }
}

// No cache (the paper's baseline "Hybrid (w/o Cache)", Section 5): Read and Write go straight to
// the global table.  The sorted order is used as it is; a key stands for its own row.
template <bool LOOKUP>
__global__ __launch_bounds__(PT_THREADS) void direct_probe_kernel(CacheView cv, Workspace ws, uint32_t n, uint32_t t_now, uint32_t ptiles,
                                                                  const int64_t *__restrict__ check_ids, uint32_t *__restrict__ inv = nullptr)
{
    __shared__ uint32_t lds[PT_WAVES + 1];
    if (blockIdx.x >= ptiles) { check_order_body(cv, ws, check_ids, n, blockIdx.x - ptiles); return; }     // (an order sorted ahead, see probe_kernel)
    const uint32_t j = blockIdx.x * PT_TILE + threadIdx.x;
    if (LOOKUP && inv && j < n) inv[ws.perm[j]] = j;         // pooled lookup (see probe_kernel)
    const uint32_t vocab = cv.vocab;
    DState *ds = cv.ds;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        Counters z{};
        *cv.next_call = z;
        cv.last->n = n;
        atomicAdd(&ds->total.n, (unsigned long long)n);
        if (LOOKUP) ds->t = t_now;
    }
    bool head = false, bad = false;
    if (j < n) {
        const uint32_t key = ws.skey[j];
        if (key == vocab) {
            bad = true;
            if (LOOKUP) ws.src[j] = SRC_ZERO;
            ws.head_slot[j] = SLOT_NONE;
            if (j == 0) ds->n_valid = 0;
        } else {
            head = j == 0 || ws.skey[j - 1] != key;
            if (j + 1 == n || ws.skey[j + 1] == vocab) ds->n_valid = j + 1;
            if (LOOKUP) ws.src[j] = (int32_t)key;
            ws.head_slot[j] = (int32_t)key;
            if (LOOKUP && head) ws.cls[j] = (uint8_t)CLS_MISS;        // every key comes from the global table
        }
    }
    if (__any(bad) && lane_id() == 0) atomicOr(&ds->err, ERRBIT_RANGE);
    const uint32_t tot_heads = block_sum<PT_WAVES>(head ? 1u : 0u, lds);
    if (threadIdx.x == 0) count2(&cv.last->unique, &ds->total.unique, tot_heads);
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
    if (cv.rowwise && gl == 0) cv.A[key] = cv.acc[slot];
    if (gl == 0) {
        const uint32_t cc = cv.meta[slot].cc;
        if (cc > cv.Cg[key]) { cv.Cg[key] = cc; if (cv.Cg_host) cv.Cg_host[key] = cc; }
    }
}

// Element-wise w + (x - b): what the server holds after a worker that fetched b and now holds x has pushed.
__device__ __forceinline__ float delta_add(float w, float x, float b) { return w + (x - b); }
__device__ __forceinline__ float4 delta_add(float4 w, float4 x, float4 b)
{
    return make_float4(w.x + (x.x - b.x), w.y + (x.y - b.y), w.z + (x.z - b.z), w.w + (x.w - b.w));
}

// Several workers (Section 3.1, Evict as the paper words it): the worker pushes what it accumulated on
// the row since its Fetch and the server adds it to the global row, c_g = max(c_g, c_c).  With
// `refetch` the cached row then becomes the global row again (the Fetch that follows an Evict(key)
// in Algorithm 2; a row without updates of its own is only fetched); without, the replica keeps its
// view (flush).  Either way it counts its changes anew from here.  Called by a whole row group.
template <int VEC>
__device__ __forceinline__ void sync_row_many(const CacheView &cv, uint32_t key, uint32_t slot, int gl, bool has_updates, bool refetch)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    for (int pass = 0; pass < (cv.adagrad ? 2 : 1); ++pass) {
        V *glob = reinterpret_cast<V *>((pass ? cv.A : cv.W) + (size_t)key * g.dim);
        V *mine = reinterpret_cast<V *>((pass ? cv.acc : cv.rows) + (size_t)slot * g.dim);
        V *base = reinterpret_cast<V *>((pass ? cv.acc0 : cv.rows0) + (size_t)slot * g.dim);
        for (int c = gl; c < g.chunks; c += g.lanes) {
            V w = glob[c];
            const V x = mine[c];
            if (has_updates) { w = delta_add(w, x, base[c]); glob[c] = w; }
            if (refetch) { mine[c] = w; base[c] = w; }
            else base[c] = x;
        }
    }
    if (gl == 0 && has_updates) {
        const uint32_t cc = cv.meta[slot].cc;
        if (cc > cv.Cg[key]) cv.Cg[key] = cc;
    }
}

// Fetch's pull for one row: copy the global row (and the accumulator) into the slot.
template <int VEC>
__device__ __forceinline__ void pull_row(const CacheView &cv, uint32_t key, uint32_t slot, int gl)
{
    const RowGeom g = cv.geom;
    row_copy<VEC>(cv.rows + (size_t)slot * g.dim, cv.W + (size_t)key * g.dim, g.chunks, g.lanes, gl);
    if (cv.adagrad)
        row_copy<VEC>(cv.acc + (size_t)slot * g.dim, cv.A + (size_t)key * g.dim, g.chunks, g.lanes, gl);
    if (cv.rowwise && gl == 0) cv.acc[slot] = cv.A[key];
}

// The same from explicit sources (a staged row).
template <int VEC>
__device__ __forceinline__ void pull_row_from(const CacheView &cv, const float *row, const float *acc, uint32_t slot, int gl)
{
    const RowGeom g = cv.geom;
    row_copy<VEC>(cv.rows + (size_t)slot * g.dim, row, g.chunks, g.lanes, gl);
    if (cv.adagrad) row_copy<VEC>(cv.acc + (size_t)slot * g.dim, acc, g.chunks, g.lanes, gl);
}

// Host-backed table: writes the rows staged by trim `buf` to the global table, with their clocks.
// Runs in `nblocks` workgroups of 256 threads; `vblock` is this one's index.
// LINK_ROWS rows per row group are on their way at a time: a transfer over the host link takes
// microseconds, and what keeps the link full is the number of rows in flight, not the number of
// workgroups (few workgroups, because a compute unit that waits for the host serves its other
// waves' memory requests behind those that wait).
constexpr int LINK_ROWS = 4;
template <int VEC>
__device__ __forceinline__ void deferred_push_body(const CacheView &cv, int buf, uint32_t vblock, uint32_t nblocks)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    const uint32_t n = cv.ds->push_n[buf];
    const uint32_t gid = (vblock * 256u + threadIdx.x) / g.lanes, ngroups = nblocks * 256u / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    for (uint32_t r0 = gid * LINK_ROWS; r0 < n; r0 += ngroups * LINK_ROWS) {
        uint32_t key[LINK_ROWS], at[LINK_ROWS];
#pragma unroll
        for (int k = 0; k < LINK_ROWS; ++k) {
            at[k] = r0 + k < n ? r0 + k : r0;
            key[k] = cv.hl.keys_of(buf)[at[k]];
            if (r0 + k >= n) key[k] = KEY_NONE;          // (KEY_NONE within the list: a tied victim without updates)
        }
        for (int pass = 0; pass < (cv.adagrad ? 2 : 1); ++pass) {
            const float *from = pass ? cv.hl.acc_of(buf) : cv.hl.rows_of(buf);
            float *to = pass ? cv.A : cv.W;
            static_assert(LINK_ROWS == 4, "the copy below is written out for four rows");
            for (int c = gl; c < g.chunks; c += g.lanes) {
                // (named values, not an array: with an array the compiler kept the rows in scratch
                // memory and waited for each store to the host before the next)
                const V v0 = reinterpret_cast<const V *>(from + (size_t)at[0] * g.dim)[c];
                const V v1 = reinterpret_cast<const V *>(from + (size_t)at[1] * g.dim)[c];
                const V v2 = reinterpret_cast<const V *>(from + (size_t)at[2] * g.dim)[c];
                const V v3 = reinterpret_cast<const V *>(from + (size_t)at[3] * g.dim)[c];
                if (key[0] != KEY_NONE) reinterpret_cast<V *>(to + (size_t)key[0] * g.dim)[c] = v0;
                if (key[1] != KEY_NONE) reinterpret_cast<V *>(to + (size_t)key[1] * g.dim)[c] = v1;
                if (key[2] != KEY_NONE) reinterpret_cast<V *>(to + (size_t)key[2] * g.dim)[c] = v2;
                if (key[3] != KEY_NONE) reinterpret_cast<V *>(to + (size_t)key[3] * g.dim)[c] = v3;
            }
        }
        if (gl == 0) {
#pragma unroll
            for (int k = 0; k < LINK_ROWS; ++k)
                if (key[k] != KEY_NONE) cv.Cg_host[key[k]] = cv.hl.cg_of(buf)[at[k]];
        }
    }
}

template <int VEC>
__global__ __launch_bounds__(256) void deferred_push_kernel(CacheView cv, int buf)
{
    deferred_push_body<VEC>(cv, buf, blockIdx.x, gridDim.x);
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

// Fetch of the missed keys, Evict + Fetch of the stale ones (Algorithm 2), and Get, one row
// group per item.  The i-th missed key in ascending key order takes the i-th free slot in
// ascending slot order.  The gather reads a missed key's row from the global table (the same
// values the fetch copies), so it does not wait for the fetch: the first `fill_blocks`
// workgroups fetch, the others gather, side by side.
// POOLED: out[b] = sum of the bag's rows in bag order; else out[perm[j]] = row of position j.
constexpr int GATHER_ROWS = 8;
constexpr int POOL_ROWS = 8;
constexpr int FILL_ROWS = 2;              // missed keys a row group fetches at a time
// A row chunk as the compiler's own vector type (arrays of these stay in registers where arrays
// of the HIP struct type of the same size did not).
typedef float raw_float4 __attribute__((ext_vector_type(4)));
template <int VEC> struct RawVecT { using type = float; };
template <> struct RawVecT<4> { using type = raw_float4; };

// Optional time stamps inside the two heavy kernels, one record of TRACE_WORDS words per workgroup
// (het_profile_trace): [0] start, [5] the last wave's end, [6] role.
// apply_kernel: roles 1 carried sort stage, 2 select stage, 3 id check, 4 tile of the update; for
// role 4 also [1] tile and segments listed, [2] short segments done, [3] long segments done,
// [4] past the barrier before the border runs.
// fill_gather_kernel: roles 1 carried sort stage, 2 fetch, 3 the fetched keys' bookkeeping,
// 4 select stage, 5 gather, 6 host link (write-back, list of rows to fetch ahead).
// Clock: wall_clock64(), 100 MHz.
constexpr int TRACE_WORDS = 8;
struct KernelTrace {
    unsigned long long *rec;     // nullptr: off
    uint32_t cap;                // workgroups the buffer has room for
    __device__ __forceinline__ void stamp(int i) const { if (rec && threadIdx.x == 0 && blockIdx.x < cap) rec[(size_t)blockIdx.x * TRACE_WORDS + i] = wall_clock64(); }
    __device__ __forceinline__ void end() const { if (rec && lane_id() == 0 && blockIdx.x < cap) atomicMax(&rec[(size_t)blockIdx.x * TRACE_WORDS + 5], (unsigned long long)wall_clock64()); }   // (the last wave to leave)
    __device__ __forceinline__ void role(int r) const { if (rec && threadIdx.x == 0 && blockIdx.x < cap) rec[(size_t)blockIdx.x * TRACE_WORDS + 6] = (unsigned long long)r; }
};

// Fetch's pull for FILL_ROWS rows at once (all loads first).  Called by a whole row group.
template <int VEC, bool WITH_ACC>
__device__ __forceinline__ void fetch_rows(const CacheView &cv, const float *const (&srow)[FILL_ROWS], const float *const (&sacc)[FILL_ROWS],
                                           const uint32_t (&slot)[FILL_ROWS], int nin, int gl)
{
    using V = typename RawVecT<VEC>::type;
    const RowGeom g = cv.geom;
    for (int c = gl; c < g.chunks; c += g.lanes) {
        V v[FILL_ROWS], a[FILL_ROWS];
#pragma unroll
        for (int r = 0; r < FILL_ROWS; ++r) {
            v[r] = reinterpret_cast<const V *>(srow[r])[c];
            if constexpr (WITH_ACC) a[r] = reinterpret_cast<const V *>(sacc[r])[c];
        }
#pragma unroll
        for (int r = 0; r < FILL_ROWS; ++r) {
            if (r < nin) {
                reinterpret_cast<V *>(cv.rows + (size_t)slot[r] * g.dim)[c] = v[r];
                if constexpr (WITH_ACC) reinterpret_cast<V *>(cv.acc + (size_t)slot[r] * g.dim)[c] = a[r];
                if (cv.many) {                       // several workers: the row as fetched
                    reinterpret_cast<V *>(cv.rows0 + (size_t)slot[r] * g.dim)[c] = v[r];
                    if constexpr (WITH_ACC) reinterpret_cast<V *>(cv.acc0 + (size_t)slot[r] * g.dim)[c] = a[r];
                }
            }
        }
    }
}

// Host-backed table: the rows the next Read will miss are fetched while the Write in between runs
// (Section 4.2: the next minibatch's indices are known in advance; Section 4.1: communication is
// invoked asynchronously and overlaps computation).  The second kernel of a lookup lists the keys of
// the announced batch that are not cached (nothing is inserted before that batch's own lookup, and a
// key evicted in between is found through `pend`); a kernel on a stream of its own then brings their
// rows from the table into HBM, beside the last trim's write-back going the other way; the next
// lookup's fetch kernel takes them from there.
struct Ahead {
    const uint32_t *skey;   // the announced batch's sorted keys (listing role), or null
    uint32_t n;             // their number
    uint32_t blocks;        // workgroups of the listing role in this launch
    uint32_t list_tag;      // tag the listing role gives the keys it lists (top bit set)
    int list_slot;          // which of ds->pf_n counts them
    uint32_t pending_seq;   // serial number of the trim whose staged rows are still to be written back (0: none)
    uint32_t use_tag;       // fetch role: tag of the rows that were fetched ahead for THIS lookup (0: none)
};

// Lists the keys of an announced batch that are not cached.  Workgroups of 256 threads, one sorted position each.
__device__ __forceinline__ void ahead_list_body(const CacheView &cv, const Ahead &ah, uint32_t vblock)
{
    const uint32_t j = vblock * 256u + threadIdx.x;
    bool want = false;
    uint32_t key = KEY_NONE, from = KEY_NONE;
    if (j < ah.n) {
        key = ah.skey[j];
        const bool head = key != cv.vocab && (j == 0 || ah.skey[j - 1] != key);
        if (head && ht_find(cv.ht, key) == SLOT_NONE) {
            want = true;
            // a row the last trim evicted, whose write-back is still to come: the staged copy is the row
            const uint64_t pe = cv.hl.pend[key];
            if (ah.pending_seq && (uint32_t)(pe >> 32) == ah.pending_seq) from = (uint32_t)pe;
        }
    }
    const uint64_t m = __ballot(want);
    if (!m) return;
    uint32_t base = 0;
    const uint32_t first = (uint32_t)__builtin_ctzll(m);
    if (lane_id() == first) base = atomicAdd(&cv.ds->pf_n[ah.list_slot], (uint32_t)__popcll(m));     // (the order of the list does not matter)
    base = __shfl(base, (int)first, WAVE);
    if (want) {
        const uint32_t at = base + mask_rank(m);
        cv.hl.pf_keys[at] = key;
        cv.hl.pf_from[at] = from;
        cv.hl.pend[key] = ((uint64_t)ah.list_tag << 32) | at;
    }
}

// On the stream beside the main one: the first half of the workgroups write the rows a trim staged
// back to the table (push_buf < 0: nothing to write), the second half bring the listed rows in.
template <int VEC>
__global__ __launch_bounds__(256) void link_kernel(CacheView cv, int push_buf, int list_slot, int staged_buf, uint32_t push_blocks)
{
    const uint32_t half = push_blocks;
    if (blockIdx.x < half) { if (push_buf >= 0) deferred_push_body<VEC>(cv, push_buf, blockIdx.x, half); return; }
    if (list_slot < 0) return;
    const RowGeom g = cv.geom;
    const uint32_t n = cv.ds->pf_n[list_slot];
    const uint32_t gid = ((blockIdx.x - half) * 256u + threadIdx.x) / g.lanes, ngroups = (gridDim.x - half) * 256u / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    using V = typename VecT<VEC>::type;
    for (uint32_t r0 = gid * LINK_ROWS; r0 < n; r0 += ngroups * LINK_ROWS) {
        uint32_t at[LINK_ROWS], key[LINK_ROWS], from[LINK_ROWS];
#pragma unroll
        for (int k = 0; k < LINK_ROWS; ++k) {
            at[k] = r0 + k < n ? r0 + k : r0;            // (past the end: the first row again, to the same place)
            key[k] = cv.hl.pf_keys[at[k]]; from[k] = cv.hl.pf_from[at[k]];
        }
        for (int pass = 0; pass < (cv.adagrad ? 2 : 1); ++pass) {
            const float *table = pass ? cv.A : cv.W, *stage = pass ? cv.hl.acc_of(staged_buf) : cv.hl.rows_of(staged_buf);
            float *to = pass ? cv.hl.pf_acc : cv.hl.pf_rows;
            for (int c = gl; c < g.chunks; c += g.lanes) {
                V v[LINK_ROWS];
#pragma unroll
                for (int k = 0; k < LINK_ROWS; ++k) {
                    const float *row = from[k] != KEY_NONE ? stage + (size_t)from[k] * g.dim : table + (size_t)key[k] * g.dim;
                    v[k] = reinterpret_cast<const V *>(row)[c];
                }
#pragma unroll
                for (int k = 0; k < LINK_ROWS; ++k) reinterpret_cast<V *>(to + (size_t)at[k] * g.dim)[c] = v[k];
            }
        }
    }
}

// Get for bags (sum pooling): one row group adds up one bag at a time, in bag order, in fp64, rounded
// once (a bag may hold hundreds of rows).  Where the rows are is found for as many ids of the bag
// as the group has lanes at once, one id per lane (its sorted position, then source and key there:
// two steps for the whole stretch, not two per POOL_ROWS rows), and handed from lane to lane
// for the row loads; the next stretch is asked for behind the first rows of the present one.
// A row's address carries "does not count" (an id outside the vocabulary) in its lowest bit.
template <int VEC>
__device__ __forceinline__ void pooled_gather_body(const CacheView &cv, const Workspace &ws, uint32_t n, float *__restrict__ out,
                                                   const int64_t *__restrict__ offsets, uint32_t n_bags, const uint32_t *__restrict__ inv,
                                                   uint32_t gid, uint32_t ngroups)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    const int gl = threadIdx.x % g.lanes;
    const int first_lane = (int)(threadIdx.x % WAVE) - gl;
    auto where = [&](uint32_t jj, bool in) -> unsigned long long {
        const int32_t sr = ws.src[jj];
        const uint32_t ky = ws.skey[jj];
        const float *row = sr == SRC_BACKING ? cv.W + (size_t)ky * g.dim : cv.rows + (size_t)(uint32_t)(sr < 0 ? 0 : sr) * g.dim;
        return (unsigned long long)(uintptr_t)row | (in && sr != SRC_ZERO ? 0ull : 1ull);
    };
    for (uint32_t b = gid; b < n_bags; b += ngroups) {
        int64_t lo = offsets[b], hi = offsets[b + 1];
        lo = lo < 0 ? 0 : lo; hi = hi > (int64_t)n ? (int64_t)n : hi;
        for (int c0 = 0; c0 < g.chunks; c0 += g.lanes) {
            const bool mine = c0 + gl < g.chunks;
            const int c = mine ? c0 + gl : 0;    // (a lane beyond the row reads its first piece and stores nothing: every lane hands addresses on)
            double sum[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum[e] = 0.0;
            if (lo < hi) {
                int64_t i0 = lo;
                unsigned long long cur = where(inv[i0 + gl < hi ? i0 + gl : hi - 1], i0 + gl < hi);
                while (i0 < hi) {
                    const int cnt = hi - i0 < (int64_t)g.lanes ? (int)(hi - i0) : g.lanes;
                    const int64_t i1 = i0 + g.lanes;
                    const bool more = i1 < hi;
                    const uint32_t jj1 = more ? inv[i1 + gl < hi ? i1 + gl : hi - 1] : 0u;
                    unsigned long long nxt = 0ull;
                    for (int r0 = 0; r0 < cnt; r0 += POOL_ROWS) {
                        V v[POOL_ROWS];
                        bool counts[POOL_ROWS];
#pragma unroll
                        for (int r = 0; r < POOL_ROWS; ++r) {
                            const int rr = r0 + r < cnt ? r0 + r : cnt - 1;
                            const unsigned long long p = __shfl(cur, first_lane + rr, WAVE);
                            counts[r] = r0 + r < cnt && !(p & 1ull);
                            v[r] = reinterpret_cast<const V *>((uintptr_t)(p & ~1ull))[c];
                        }
                        if (r0 == 0 && more) nxt = where(jj1, i1 + gl < hi);
#pragma unroll
                        for (int r = 0; r < POOL_ROWS; ++r) {
                            const float *vf = reinterpret_cast<const float *>(&v[r]);
#pragma unroll
                            for (int e = 0; e < VEC; ++e) sum[e] += counts[r] ? (double)vf[e] : 0.0;
                        }
                    }
                    cur = nxt; i0 = i1;
                }
            }
            V res;
            float *rf = reinterpret_cast<float *>(&res);
#pragma unroll
            for (int e = 0; e < VEC; ++e) rf[e] = (float)sum[e];
            if (mine) reinterpret_cast<V *>(out + (size_t)b * g.dim)[c] = res;
        }
    }
}

struct FillLds {
    uint32_t pre_miss[MAX_PROBE_TILES], pre_stale[MAX_PROBE_TILES];
    uint32_t scan[4 + 1];
};
// RIDE: 0 carries no sort stage, 1 a histogram stage (cheap in registers: the gather keeps its
// occupancy), 2 any stage.
// TRACE: time stamps (het_profile_trace); a kernel of its own, because the stamps' arguments cost the
// other one scalar registers it has no room for.
template <int VEC, bool POOLED, int RIDE, bool TRACE>
__global__ __launch_bounds__(256) void fill_gather_kernel(CacheView cv, Workspace ws, uint32_t n, uint32_t t_now, uint32_t ptiles, uint32_t fill_blocks,
                                                          TrimPlan tp, uint32_t hist_blocks, float *__restrict__ out, const int64_t *__restrict__ offsets, uint32_t n_bags,
                                                          const uint32_t *__restrict__ inv, SortStage ride, SortStage ride2,
                                                          uint32_t push_blocks, int push_buf, uint32_t push_seq, int hist_pass, Ahead ah,
                                                          KernelTrace tr_arg, int fetch_mode)
{
    using V = typename VecT<VEC>::type;
    uint32_t bid = blockIdx.x, nblk = gridDim.x;
    const KernelTrace tr = TRACE ? tr_arg : KernelTrace{nullptr, 0u};
    tr.stamp(0);
    if (RIDE == 1 && run_carried<true>(ride, ride2, bid, nblk)) { tr.role(1); tr.end(); return; }
    if (RIDE == 2 && run_carried<false>(ride, ride2, bid, nblk)) { tr.role(1); tr.end(); return; }
    if (bid < push_blocks) { deferred_push_body<VEC>(cv, push_buf, bid, push_blocks); tr.role(6); tr.end(); return; }    // host-backed table: the last trim's write-back
    bid -= push_blocks; nblk -= push_blocks;
    if (bid < ah.blocks) { ahead_list_body(cv, ah, bid); tr.role(6); tr.end(); return; }                                 // host-backed table: what to fetch ahead for the coming batch
    bid -= ah.blocks; nblk -= ah.blocks;
    const RowGeom g = cv.geom;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t groups_per_block = 256u / g.lanes;
    if (POOLED) {
        // Get for bags.  These workgroups live longest (a row group adds up a whole bag), so they take
        // the first places; all the other roles' workgroups follow.
        const uint32_t others = fill_blocks + (fill_blocks && fetch_mode != 2 ? ptiles : 0u) + hist_blocks;
        const uint32_t bag_blocks = nblk - others;
        if (bid < bag_blocks) {
            if (fill_blocks == 0 && bid == 0 && threadIdx.x == 0) cv.ds->n_unique = (uint32_t)cv.last->unique;   // (no fetch workgroup does)
            pooled_gather_body<VEC>(cv, ws, n, out, offsets, n_bags, inv, bid * groups_per_block + threadIdx.x / g.lanes, bag_blocks * groups_per_block);
            tr.role(5); tr.end();
            return;
        }
        bid -= bag_blocks; nblk -= bag_blocks;
    }
    // fetch_mode 0: everything.  1: the missed keys' rows are left to the update that follows (it reads
    // them from the global table and writes them to their slots with its step applied: they are
    // neither written nor read once more); all else as usual.  2: only those rows (a call came
    // between that is not that update).
    const uint32_t ins_blocks = fill_blocks && fetch_mode != 2 ? ptiles : 0u;
    if (bid < fill_blocks) {
        FillLds &fl = lds_as<FillLds>();
        const uint32_t tot_miss = tile_prefix_to_lds<4>(ws.tile_miss, ptiles, fl.pre_miss, fl.scan);
        const uint32_t tot_stale = tile_prefix_to_lds<4>(ws.tile_stale, ptiles, fl.pre_stale, fl.scan);
        const uint32_t gid = bid * groups_per_block + threadIdx.x / g.lanes;
        const uint32_t ngroups = fill_blocks * groups_per_block;
        if (bid == 0 && threadIdx.x == 0 && fetch_mode != 2) cv.ds->n_unique = (uint32_t)cv.last->unique;   // for an update that reuses this order
        // Fetch(k) into a new slot, FILL_ROWS keys per row group at a time: where each row comes from
        // and goes to is asked for all of them first, then the rows (few workgroups with several
        // rows in flight each leave the chip to the other roles of this kernel from the start)
        for (uint32_t m0 = gid; m0 < tot_miss && fetch_mode != 1; m0 += ngroups * FILL_ROWS) {
            const float *srow[FILL_ROWS], *sacc[FILL_ROWS];
            uint32_t slot[FILL_ROWS], keyr[FILL_ROWS];
#pragma unroll
            for (int r = 0; r < FILL_ROWS; ++r) {
                const uint32_t m = m0 + r * ngroups < tot_miss ? m0 + r * ngroups : m0;     // (beyond the end: the first row again, not stored)
                const uint32_t tl = tile_of(fl.pre_miss, ptiles, m);
                const uint32_t key = ws.miss_stage[tl * PT_TILE + (m - fl.pre_miss[tl])].y;
                keyr[r] = key;
                slot[r] = cv.free_list[m];
                // host-backed table: a row the last trim evicted may still be on its way to the table
                // (its write-back travels in this very kernel); then the staged copy is the global row
                // or it was fetched ahead into HBM for this very lookup
                const bool link = cv.Cg_host && (push_seq || ah.use_tag);
                const uint64_t pe = link ? cv.hl.pend[key] : 0ull;
                const uint32_t tag = (uint32_t)(pe >> 32);
                const bool staged = link && push_seq && tag == push_seq;
                const bool ahead = link && ah.use_tag && tag == ah.use_tag;
                const size_t at = (size_t)(uint32_t)pe * g.dim;
                srow[r] = staged ? cv.hl.rows_of(push_buf) + at : (ahead ? cv.hl.pf_rows + at : cv.W + (size_t)key * g.dim);
                sacc[r] = staged ? cv.hl.acc_of(push_buf) + at : (ahead ? cv.hl.pf_acc + at : cv.A + (size_t)key * g.dim);
            }
            int nin = 0;                         // rows of this batch that exist (the first ones)
#pragma unroll
            for (int r = 0; r < FILL_ROWS; ++r) nin += m0 + r * ngroups < tot_miss ? 1 : 0;
            if (cv.adagrad) fetch_rows<VEC, true>(cv, srow, sacc, slot, nin, gl);
            else fetch_rows<VEC, false>(cv, srow, sacc, slot, nin, gl);
            if (fetch_mode == 2 && cv.early_cc && gl == 0) {        // the update that would have pushed early is not coming
#pragma unroll
                for (int r = 0; r < FILL_ROWS; ++r)
                    if (r < nin) cv.early_cc[slot[r]] = 0u;
            }
            if (cv.rowwise && gl == 0) {             // (one accumulator per row; such a table is in HBM)
#pragma unroll
                for (int r = 0; r < FILL_ROWS; ++r)
                    if (r < nin) cv.acc[slot[r]] = cv.A[keyr[r]];
            }
        }                                        // (clocks, key and index entry: the workgroups below)
        for (uint32_t m = gid; m < tot_stale && fetch_mode != 2; m += ngroups) {                // Evict(k); Fetch(k) in place
            const uint32_t tl = tile_of(fl.pre_stale, ptiles, m);
            const uint2 jk = ws.stale_stage[tl * PT_TILE + (m - fl.pre_stale[tl])];
            const uint32_t key = jk.y;
            const uint32_t slot = (uint32_t)ws.head_slot[jk.x];
            const bool has_updates = cv.meta[slot].cc > cv.meta[slot].cs;
            if (cv.many) sync_row_many<VEC>(cv, key, slot, gl, has_updates, true);
            else if (has_updates) push_row<VEC>(cv, key, slot, gl);          // now the global row equals the cached one
            else pull_row<VEC>(cv, key, slot, gl);
            if (gl == 0) {
                const uint32_t cg = cv.Cg[key];
                cv.meta[slot].cs = cg; cv.meta[slot].cc = cg;
                if (has_updates) count2(&cv.last->stale_dirty, &cv.ds->total.stale_dirty, 1u);
                if (cv.Cg_host && !has_updates) for (uint32_t jj = jk.x; jj < n && ws.skey[jj] == key; ++jj) ws.src[jj] = (int32_t)slot;
            }
        }
        tr.role(2); tr.end();
        return;
    }

    // Fetch's bookkeeping, one thread per missed key and one workgroup per probe tile, beside the row
    // copies above (done by the same lanes it would stand behind them: two more dependent steps)
    if (bid < fill_blocks + ins_blocks) {
        const uint32_t tl = bid - fill_blocks;
        const uint32_t here = ws.tile_miss[tl];
        const uint32_t before = block_sum_array<4>(ws.tile_miss, tl, lds_as<FillLds>().scan);
        for (uint32_t ml = threadIdx.x; ml < here; ml += 256u) {
            const uint2 jk = ws.miss_stage[tl * PT_TILE + ml];
            const uint32_t slot = cv.free_list[before + ml];
            const uint32_t j = jk.x, key = jk.y;
            const uint32_t cg = cv.Cg[key];
            store_meta(cv.meta, slot, cg, cg, t_now, 1u);                    // c_s = c_c = c_g; first use
            if (cv.early_cc) cv.early_cc[slot] = fetch_mode == 1 ? cg + 1u : 0u;    // (the update that fetches the row will make it c_g + 1)
            cv.slot_key[slot] = key;
            ws.head_slot[j] = (int32_t)slot;
            if (!ht_insert(cv.ht, key, slot)) atomicOr(&cv.ds->err, ERRBIT_INTERNAL);
            // host-backed table: the gather runs after this kernel and reads the cached copy
            if (cv.Cg_host) for (uint32_t jj = j; jj < n && ws.skey[jj] == key; ++jj) ws.src[jj] = (int32_t)slot;
        }
        tr.role(3); tr.end();
        return;
    }
    bid -= ins_blocks; nblk -= ins_blocks;
    if (bid < fill_blocks + hist_blocks) {
        // a pass of the coming trim's select (the first, or the second if the first pass's histogram
        // is kept), over the rows cached before this lookup plus the rows being fetched right now
        // (counted, not read)
        TrimLds &tl = lds_as<TrimLds>();
        const uint32_t new_rows = block_sum_array<TRIM_WAVES>(ws.tile_miss, ptiles, tl.scan);
        trim_hist_body(cv, tp, hist_pass, bid - fill_blocks, hist_blocks, tl, true, new_rows, t_now, hist_pass == 0);
        tr.role(4); tr.end();
        return;
    }
    if (POOLED) return;                  // (never reached: the bags' workgroups came first)
    const uint32_t first_gather = fill_blocks + hist_blocks;
    if (fill_blocks == 0 && bid == 0 && threadIdx.x == 0) cv.ds->n_unique = (uint32_t)cv.last->unique;   // (no fetch workgroup did)
    const uint32_t gid = (bid - first_gather) * groups_per_block + threadIdx.x / g.lanes;
    const uint32_t ngroups = (nblk - first_gather) * groups_per_block;
    {
        // Get, GATHER_ROWS positions per row group at a time: where each row comes from is asked
        // for all of them first, then the rows themselves, so that a group has several rows in
        // flight (one row per group at a time leaves the memory system idle most of the time)
        for (uint32_t j0 = gid * GATHER_ROWS; j0 < n; j0 += ngroups * GATHER_ROWS) {
            int32_t sr[GATHER_ROWS];
            uint32_t pm[GATHER_ROWS], ky[GATHER_ROWS];
#pragma unroll
            for (int r = 0; r < GATHER_ROWS; ++r) {
                const uint32_t j = j0 + r;
                const bool in = j < n;
                sr[r] = in ? ws.src[j] : SRC_ZERO;
                pm[r] = in ? ws.perm[j] : 0u;
                ky[r] = in ? ws.skey[j] : 0u;
            }
            const float *row[GATHER_ROWS];
#pragma unroll
            for (int r = 0; r < GATHER_ROWS; ++r)     // (an id outside the vocabulary reads some row and drops it: no branch between the loads)
                row[r] = sr[r] == SRC_BACKING ? cv.W + (size_t)ky[r] * g.dim : cv.rows + (size_t)(uint32_t)(sr[r] < 0 ? 0 : sr[r]) * g.dim;
            for (int c = gl; c < g.chunks; c += g.lanes) {
                V v[GATHER_ROWS];
#pragma unroll
                for (int r = 0; r < GATHER_ROWS; ++r) v[r] = reinterpret_cast<const V *>(row[r])[c];
#pragma unroll
                for (int r = 0; r < GATHER_ROWS; ++r) {
                    if (sr[r] == SRC_ZERO) v[r] = V{};
                    if (j0 + r < n) reinterpret_cast<V *>(out + (size_t)pm[r] * g.dim)[c] = v[r];
                }
            }
        }
    }
    tr.role(5); tr.end();
}

// Pooled update: the bag of every original position (its gradient row).
__global__ __launch_bounds__(256) void pooled_index_kernel(Workspace ws, uint32_t n, const int64_t *__restrict__ offsets, uint32_t n_bags)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) {
        uint32_t lo = 0, hi = n_bags;            // largest b with offsets[b] <= i
        while (hi - lo > 1) { const uint32_t mid = (lo + hi) / 2; if (offsets[mid] <= (int64_t)i) lo = mid; else hi = mid; }
        ws.bag_of[i] = lo;
    }
}

// Hardware square root and reciprocal (about one unit in the last place each): the Adagrad
// step lr * G / (sqrt(a) + eps) tolerates that a hundred times over, and the correctly rounded
// sequences cost more instructions than everything else in the kernel.
__device__ __forceinline__ float fast_sqrt(float v) { return __builtin_amdgcn_sqrtf(v); }
__device__ __forceinline__ float fast_rcp(float v) { return __builtin_amdgcn_rcpf(v); }

// The optimizer step on one cached row for chunk c of the row, and nothing else.
// Row-wise Adagrad's denominator for the row in `slot`: the row group adds up the squares of the
// gradient's pieces (every lane of the group calls, lanes beyond the row with zeros; the row has one
// piece per lane), the accumulator takes their mean, and the group's first lane stores it.
template <int VEC>
__device__ __forceinline__ float rowwise_rcp(const CacheView &cv, uint32_t slot, const float (&G)[VEC], float eps)
{
    double ss = 0.0;
#pragma unroll
    for (int k = 0; k < VEC; ++k) ss += (double)G[k] * (double)G[k];
    for (int o = cv.geom.lanes / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o, WAVE);     // (the same tree in every lane: the same sum)
    const float a = cv.acc[slot] + (float)(ss / (double)cv.geom.dim);
    if (threadIdx.x % cv.geom.lanes == 0) cv.acc[slot] = a;
    return fast_rcp(fast_sqrt(a) + eps);
}

// `from_key` other than KEY_NONE: the row has not been fetched yet (see apply_kernel, "fresh"): it is
// read from the global table at that key and written to the slot (EARLY: and to the global table).
template <int VEC, bool EARLY = false>
__device__ __forceinline__ void apply_step(const CacheView &cv, uint32_t slot, int c, const double *g64, float lr, float eps, bool act = true,
                                           uint32_t from_key = KEY_NONE)
{
    using V = typename VecT<VEC>::type;
    float G[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) G[k] = act ? (float)g64[k] : 0.f;           // the fp64 sum is rounded to fp32 once
    float row_rcp = 0.f;
    if (cv.rowwise) row_rcp = rowwise_rcp<VEC>(cv, slot, G, eps);
    if (!act) return;
    const bool fresh = from_key != KEY_NONE;
    V *xp = reinterpret_cast<V *>(cv.rows + (size_t)slot * cv.geom.dim) + c;
    V xv = fresh ? reinterpret_cast<const V *>(cv.W + (size_t)from_key * cv.geom.dim)[c] : *xp;
    float *x = reinterpret_cast<float *>(&xv);
    if (cv.rowwise) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) x[k] -= lr * G[k] * row_rcp;
    } else if (cv.adagrad) {
        V *ap = reinterpret_cast<V *>(cv.acc + (size_t)slot * cv.geom.dim) + c;
        V av = fresh ? reinterpret_cast<const V *>(cv.A + (size_t)from_key * cv.geom.dim)[c] : *ap;
        float *a = reinterpret_cast<float *>(&av);
#pragma unroll
        for (int k = 0; k < VEC; ++k) { a[k] += G[k] * G[k]; x[k] -= lr * G[k] * fast_rcp(fast_sqrt(a[k]) + eps); }
        *ap = av;
        if (EARLY && fresh) reinterpret_cast<V *>(cv.A + (size_t)from_key * cv.geom.dim)[c] = av;
    } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k) x[k] -= lr * G[k];
    }
    *xp = xv;
    if (EARLY && fresh) reinterpret_cast<V *>(cv.W + (size_t)from_key * cv.geom.dim)[c] = xv;     // early push
}

// Update + Clock (Algorithm 3) in one kernel.  A workgroup takes a tile of AP_TILE consecutive
// sorted positions, brings their keys, gradient rows' numbers and slots into LDS and lists the
// tile's segments (stretches of equal keys; a run of equal keys is one segment unless it crosses a
// tile border).  Work then goes by segment, not by position:
//   - a segment of up to AP_SOLO positions is summed by one row group, a few gradient rows (ap_batch) in
//     flight at a time, in order of position, in fp64 (the kernel is bound by reading the
//     gradients; summing wide makes a long run of a popular key lose no digits), rounded once;
//   - a longer one by all row groups of the workgroup together: contiguous shares, added in group
//     order through LDS.
// A segment that is a whole run gets the optimizer step and its clock at once: no partial sum ever
// leaves the workgroup.  Only a run that crosses a tile border (at most two per tile) leaves one
// fp64 partial sum per tile it touches in `ApplyBorders::part`, and the tile that arrives last at
// the run's counter adds them up in tile order and applies the step: which tile is last varies,
// the order of the additions does not.  Nobody waits for anybody.
// fresh_rows: the lookup whose order this update reuses left the fetch of its missed keys' rows to
// this kernel (table in HBM, one worker): where a run's key was a miss, the row and accumulator are
// read from the global table instead of the slot; the step's result goes to the slot as always.
// Fetch and Update of Algorithms 2 and 3 in one read and one write of the row.
// VERIFY: the ids must be the ones the sorted order was built from (an update that reuses the
// preceding lookup's order); extra workgroups compare them and flag any difference.
// MAXC: row pieces per lane (dim / VEC / lanes, rounded up).
constexpr int AP_THREADS = 256;
// Gradient rows in flight per row group, and waves per SIMD the kernel is held to (rows of one piece
// per lane).  Tiles of 64 positions: seven waves (72 registers), so that all tiles of a batch of
// config 2's or 4's size are resident from the start, with four rows in flight (three where the
// kernel also pushes early: two more row addresses to keep).  Tiles of 128 positions (rows of more
// than 128 floats): six waves and six rows (four with the early push); seven waves were slower there.
__host__ __device__ constexpr int ap_batch(int ap_tile, bool early) { return ap_tile == 64 ? (early ? 3 : 4) : (early ? 4 : 6); }
__host__ __device__ constexpr int ap_waves(int ap_tile) { return ap_tile == 64 ? 7 : 6; }
constexpr int AP_SOLO = 32;
// Positions per tile (template parameter AP_TILE): 64 where a workgroup has eight row groups or
// more (rows up to 128 floats), 128 for wider rows, whose fewer row groups would otherwise stand
// idle beside the popular keys' long segments and pay for twice as many border crossings.
__host__ __device__ constexpr int ap_tile_for(int lanes) { return lanes <= 32 ? 64 : 128; }

template <int VEC, int AP_TILE> struct ApplyLds {
    static_assert(AP_TILE + 2 <= AP_THREADS && AP_TILE % WAVE == 0, "one thread per position of the tile, two more for the keys outside it");
    double share[AP_THREADS * VEC];      // the row groups' shares of a long segment
    uint32_t key[AP_TILE + 2];           // [0]: key before the tile, [1 + i]: position i, [AP_TILE + 1]: key behind the tile
    uint32_t grow[AP_TILE];              // gradient row of each position
    int32_t slot[AP_TILE];               // slot of the key, valid at run heads
    uint32_t seg_start[AP_TILE + 1];     // first position (within the tile) of every segment, then the tile's count
    uint32_t wave_heads[AP_TILE / WAVE];
    uint64_t fresh[AP_TILE / WAVE];      // per position: a run head whose key missed in the lookup and whose row is fetched here
};

// How many of the conditions cond(1), cond(2), ... hold before the first that does not; found by
// a whole wave, 64 at a time.  cond must be false from some index on.
template <typename F>
__device__ __forceinline__ uint32_t wave_count_leading(F cond)
{
    uint32_t base = 0;
    for (;;) {
        const uint64_t m = __ballot(cond(base + lane_id() + 1));
        if (~m) return base + (uint32_t)__builtin_ctzll(~m);
        base += WAVE;
    }
}

// Adds the gradient rows of tile positions [lo, hi) for row piece cidx to acc64, in order, in fp64.
// If `with_row`, the cached row (and accumulator) of `slot` is requested together with the first
// batch of gradients.
template <int VEC, int BATCH>
__device__ __forceinline__ void add_positions(const CacheView &cv, const float *__restrict__ grads, const uint32_t *grow, uint32_t lo, uint32_t hi,
                                              int cidx, bool act, double (&acc64)[VEC], bool with_row, uint32_t slot,
                                              typename VecT<VEC>::type &xr, typename VecT<VEC>::type &ar, uint32_t from_key = KEY_NONE)
{
    using V = typename VecT<VEC>::type;
    const int dim = cv.geom.dim;
    for (uint32_t b0 = lo; b0 < hi; b0 += BATCH) {
        V v[BATCH];
#pragma unroll
        for (int r = 0; r < BATCH; ++r) {
            v[r] = V{};
            if (act && b0 + r < hi) v[r] = reinterpret_cast<const V *>(grads + (size_t)grow[b0 + r] * dim)[cidx];
        }
        if (with_row && b0 == lo && act) {
            const bool fresh = from_key != KEY_NONE;          // not fetched yet: the global row
            xr = reinterpret_cast<const V *>(fresh ? cv.W + (size_t)from_key * dim : cv.rows + (size_t)slot * dim)[cidx];
            if (cv.adagrad) ar = reinterpret_cast<const V *>(fresh ? cv.A + (size_t)from_key * dim : cv.acc + (size_t)slot * dim)[cidx];
        }
#pragma unroll
        for (int r = 0; r < BATCH; ++r) {
            const float *vf = reinterpret_cast<const float *>(&v[r]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc64[e] += (double)vf[e];          // zero where there is no position
        }
    }
}

template <int VEC, int BATCH>
__device__ __forceinline__ void sum_positions(const CacheView &cv, const float *__restrict__ grads, const uint32_t *grow, uint32_t lo, uint32_t hi,
                                              int cidx, bool act, double (&acc64)[VEC], bool with_row, uint32_t slot,
                                              typename VecT<VEC>::type &xr, typename VecT<VEC>::type &ar, uint32_t from_key = KEY_NONE)
{
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc64[e] = 0.0;
    add_positions<VEC, BATCH>(cv, grads, grow, lo, hi, cidx, act, acc64, with_row, slot, xr, ar, from_key);
}

struct SegWork {
    uint32_t a, b;             // positions [a, b) of the tile
    int32_t slot;
    uint32_t from_key;         // KEY_NONE, or the key whose row has not been fetched yet (fresh)
    bool is_front, is_back;    // the run began in an earlier tile / goes on in a later one
};

// The optimizer step from a row already in registers.
template <int VEC, bool EARLY = false>
__device__ __forceinline__ void apply_loaded(const CacheView &cv, uint32_t slot, int cidx, const double *g64, float lr, float eps,
                                             typename VecT<VEC>::type xv, typename VecT<VEC>::type av, bool act, uint32_t from_key = KEY_NONE)
{
    using V = typename VecT<VEC>::type;
    float *x = reinterpret_cast<float *>(&xv), *a = reinterpret_cast<float *>(&av);
    float Gs[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) Gs[e] = act ? (float)g64[e] : 0.f;          // the fp64 sum is rounded once
    float row_rcp = 0.f;
    if (cv.rowwise) row_rcp = rowwise_rcp<VEC>(cv, slot, Gs, eps);            // (every lane of the row group)
    if (!act) return;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const float G = Gs[e];
        if (cv.rowwise) x[e] -= lr * G * row_rcp;
        else if (cv.adagrad) { a[e] += G * G; x[e] -= lr * G * fast_rcp(fast_sqrt(a[e]) + eps); }
        else x[e] -= lr * G;
    }
    reinterpret_cast<V *>(cv.rows + (size_t)slot * cv.geom.dim)[cidx] = xv;
    if (cv.adagrad) reinterpret_cast<V *>(cv.acc + (size_t)slot * cv.geom.dim)[cidx] = av;
    if (EARLY && from_key != KEY_NONE) {                // early push: a row fetched by this update goes to the global table as well
        reinterpret_cast<V *>(cv.W + (size_t)from_key * cv.geom.dim)[cidx] = xv;
        if (cv.adagrad) reinterpret_cast<V *>(cv.A + (size_t)from_key * cv.geom.dim)[cidx] = av;
    }
}

// What the tiles of one run tell each other inside the kernel goes through loads, stores and
// read-modify-writes of device scope, which are coherent over the whole GPU by themselves (its
// L2 caches are per XCD and ordinary stores may stay in one of them until the kernel ends).  So no
// cache has to be written back or invalidated as a device-scope fence would do, thousands of
// times per kernel: a tile waits for its own stores to be acknowledged, and only then counts
// itself as arrived.
__device__ __forceinline__ void st_device(double *p, double v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ double ld_device(const double *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_device(int32_t *p, int32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int32_t ld_device(const int32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_device(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_device(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void stores_acknowledged() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

struct ApplyBorders {
    double *part;          // [tiles][2][dim]: sum of the segment that came in through the tile's front border / that leaves through its back border
    int32_t *slot;         // [tiles]: slot of the run that leaves through the tile's back border (it starts in this tile)
    uint32_t *from_key;    // [tiles]: that run's key if its row has not been fetched yet, else KEY_NONE
    uint32_t *arrived;     // [tiles]: how many tiles of the run that starts in this tile have stored their sums (zero between kernels)
    // A run over more than AP_GROUP tiles is summed in two levels (see apply_kernel).  A group is named like
    // a sum in `part`, by its first tile and the border through which the run leaves or enters that tile (a
    // run's first group starts at the run's first tile, back border; a tile may end one long run and start
    // another).  The groups' sums lie behind the tiles' sums in `part` ([tiles][2][dim] more), their counters
    // behind the runs' counters in `arrived` ([tiles][2] more): no further kernel arguments.
};
constexpr uint32_t AP_GROUP = 16;

template <int VEC, int MAXC, bool VERIFY, int AP_TILE, bool EARLY>
__global__ __launch_bounds__(AP_THREADS) __attribute__((amdgpu_waves_per_eu(MAXC == 1 ? ap_waves(AP_TILE) : 1))) void apply_kernel(CacheView cv, Workspace ws, ApplyBorders bd, const int64_t *__restrict__ ids,
                                                           const float *__restrict__ grads, const uint32_t *__restrict__ grad_row,
                                                           float lr, float eps, uint32_t n_ids, uint32_t work_blocks, TrimPlan tp, int stage,
                                                           SortStage ride, SortStage ride2, KernelTrace tr, int fresh_rows)
{
    using V = typename VecT<VEC>::type;
    constexpr int BATCH = ap_batch(AP_TILE, EARLY);
    // The tiles' workgroups live longest, so they take the first places; the carried stages, the select
    // stage and the id check follow in the places they leave (the other way round the step was 1 to 2 %
    // longer on every config).
    uint32_t bid = blockIdx.x < work_blocks ? blockIdx.x + (gridDim.x - work_blocks) : blockIdx.x - work_blocks, nblk = gridDim.x;
    tr.stamp(0);
    if (run_carried(ride, ride2, bid, nblk)) { tr.role(1); tr.end(); return; }
    const uint32_t verify_blocks = VERIFY ? (n_ids + VERIFY_TILE - 1) / VERIFY_TILE : 0u;
    const uint32_t stage_blocks = nblk - work_blocks - verify_blocks;
    if (bid < stage_blocks) {            // extra workgroups: a stage of the coming trim's select
        trim_stage_body(cv, tp, stage, bid, stage_blocks, lds_as<TrimLds>());
        tr.role(2); tr.end();
        return;
    }
    bid -= stage_blocks;
    if (VERIFY && bid < verify_blocks) {
        // The ids must be the ones the sorted order was built from: every position's id against the
        // sorted key, by workgroups of their own.  A difference is flagged; the update goes on.
        const uint32_t nvv = cv.ds->n_valid;
        bool bad = false;
#pragma unroll
        for (int i = 0; i < VERIFY_TILE / AP_THREADS; ++i) {
            const uint32_t j = bid * VERIFY_TILE + i * AP_THREADS + threadIdx.x;
            if (j < nvv) bad |= ids[ws.perm[j]] != (int64_t)ws.skey[j];
        }
        if (__any(bad) && lane_id() == 0) atomicOr(&cv.ds->err, ERRBIT_STATE);
        tr.role(3); tr.end();
        return;
    }
    bid -= verify_blocks;
    tr.role(4);
    const RowGeom g = cv.geom;
    const uint32_t group = threadIdx.x / g.lanes, ngroups = AP_THREADS / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    const uint32_t nv = cv.ds->n_valid;
    if (VERIFY && bid == 0 && threadIdx.x == 0) {
        // this call did not sort: its per-call counters start here, with the lookup's key count
        DState *ds = cv.ds;
        Counters z{};
        *cv.next_call = z;
        cv.last->n = n_ids; cv.last->unique = ds->n_unique;
        atomicAdd(&ds->total.n, (unsigned long long)n_ids);
        atomicAdd(&ds->total.unique, (unsigned long long)ds->n_unique);
        if (nv < n_ids) atomicOr(&ds->err, ERRBIT_RANGE);      // the order holds ids outside the vocabulary
    }
    ApplyLds<VEC, AP_TILE> &l = lds_as<ApplyLds<VEC, AP_TILE>>();
    const uint32_t T = bid, j0 = T * AP_TILE;
    const uint32_t *skey = ws.skey;
    {   // the tile: one position per thread, and the keys just outside it
        const uint32_t i = threadIdx.x;
        if (i < AP_TILE) {
            const uint32_t j = j0 + i;
            const bool in = j < n_ids;
            const uint32_t k = in ? skey[j] : KEY_NONE;
            uint32_t pm = in ? ws.perm[j] : 0u;
            const int32_t hs = in ? ws.head_slot[j] : SLOT_NONE;
            // fresh_rows: the lookup left the fetch of its missed keys' rows to this kernel
            const bool fresh = fresh_rows && in && ws.cls[j] == (uint8_t)CLS_MISS && (j == 0 || skey[j - 1] != k);
            if (grad_row && in) pm = grad_row[pm];
            l.key[1 + i] = j < nv ? k : KEY_NONE;
            l.grow[i] = pm;
            l.slot[i] = hs;
            const uint64_t fm = __ballot(fresh);
            if (lane_id() == 0) l.fresh[i / WAVE] = fm;
        } else if (i == AP_TILE) {
            l.key[0] = j0 > 0 && j0 < n_ids ? skey[j0 - 1] : KEY_NONE;
        } else if (i == AP_TILE + 1) {
            const uint32_t jn = j0 + AP_TILE;
            const uint32_t k = jn < n_ids ? skey[jn] : KEY_NONE;
            l.key[AP_TILE + 1] = jn < nv ? k : KEY_NONE;
        }
    }
    if (j0 >= nv) return;                                  // (uniform: nothing valid in this tile)
    const uint32_t cnt = min((uint32_t)AP_TILE, nv - j0);
    __syncthreads();
    {   // the segments, in order
        const uint32_t i = threadIdx.x;
        const bool head = i < cnt && (i == 0 || l.key[i] != l.key[1 + i]);
        const uint64_t m = __ballot(head);
        const uint32_t w = i / WAVE;
        if (i < AP_TILE && lane_id() == 0) l.wave_heads[w] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int ww = 0; ww < AP_TILE / WAVE; ++ww) { const uint32_t c = l.wave_heads[ww]; before += (uint32_t)ww < w ? c : 0u; total += c; }
        if (head) l.seg_start[before + mask_rank(m)] = i;
        if (i == 0) l.seg_start[total] = cnt;
        __syncthreads();
    }
    uint32_t nseg = 0;
#pragma unroll
    for (int ww = 0; ww < AP_TILE / WAVE; ++ww) nseg += l.wave_heads[ww];
    const bool front_open = l.key[0] != KEY_NONE && l.key[0] == l.key[1];                   // the first segment's run began in an earlier tile
    const bool back_open = cnt == AP_TILE && l.key[AP_TILE + 1] != KEY_NONE && l.key[AP_TILE + 1] == l.key[AP_TILE];   // the last one's goes on
    const size_t pstride = (size_t)g.dim;
    // Which tiles the runs that cross this tile's borders touch is asked now, by the two waves that
    // will finish them (see below), so that the answer is there when the sums are.
    const uint32_t wave = threadIdx.x / WAVE;
    const bool through = front_open && back_open && nseg == 1;
    const bool do_front = wave == 0 && front_open, do_back = wave == 1 && back_open && !through;
    uint32_t T0 = T, T1 = T;
    if (do_front || do_back) {
        const uint32_t key = do_front ? l.key[1] : l.key[AP_TILE];
        if (do_front)            // tiles before this one that the run also entered through their front border
            T0 = T - 1 - wave_count_leading([&](uint32_t i) { return i < T && skey[(size_t)(T - i) * AP_TILE - 1] == key; });
        if (do_back || through)  // tiles behind this one that the run also leaves through their back border
            T1 = T + 1 + wave_count_leading([&](uint32_t i) { const uint64_t je = ((uint64_t)T + i + 1) * AP_TILE; return je < nv && skey[je] == key; });
    }
    tr.stamp(1);
    // (does any segment need the whole workgroup?  every thread looks at one)
    const bool any_long = __syncthreads_or(threadIdx.x < nseg && l.seg_start[threadIdx.x + 1] - l.seg_start[threadIdx.x] > AP_SOLO) != 0;

    // segments of up to AP_SOLO positions: one row group each
    auto seg_work = [&](uint32_t sg) {
        SegWork w;
        w.a = l.seg_start[sg]; w.b = l.seg_start[sg + 1];
        w.is_front = sg == 0 && front_open; w.is_back = sg + 1 == nseg && back_open;
        w.slot = w.is_front ? SLOT_NONE : l.slot[w.a];
        w.from_key = !w.is_front && ((l.fresh[w.a / WAVE] >> (w.a % WAVE)) & 1ull) ? l.key[1 + w.a] : KEY_NONE;
        return w;
    };
    // what is left to do once the segment's sum for row piece cidx is there
    auto finish_piece = [&](const SegWork &w, int cidx, bool act, const double (&acc64)[VEC], V xr, V ar) {
        const bool closed = !w.is_front && !w.is_back;
        if (closed) {
            if (w.slot != SLOT_NONE) apply_loaded<VEC, EARLY>(cv, (uint32_t)w.slot, cidx, acc64, lr, eps, xr, ar, act, w.from_key);
        } else if (act) {
            double *mine = bd.part + ((size_t)T * 2 + (w.is_front ? 0 : 1)) * pstride + (size_t)cidx * VEC;
#pragma unroll
            for (int e = 0; e < VEC; ++e) st_device(mine + e, acc64[e]);
        }
    };
    auto finish_segment = [&](const SegWork &w) {
        if (gl == 0) {
            if (w.is_back && !w.is_front) { st_device(&bd.slot[T], w.slot); st_device(&bd.from_key[T], w.from_key); }
            // Clock(k): once per key per Write; a run that goes on in later tiles takes it where it starts
            if (!w.is_front && w.slot != SLOT_NONE && !cv.direct) atomicAdd(&cv.meta[w.slot].cc, 1u);
        }
        if (w.is_front || w.is_back) stores_acknowledged();   // the partial sum, before this tile is counted as arrived
    };
    {
        for (uint32_t sg = group; sg < nseg; sg += ngroups) {
            const SegWork w = seg_work(sg);
            if (w.b - w.a > AP_SOLO) continue;
            const bool step = !w.is_front && !w.is_back && w.slot != SLOT_NONE;
#pragma unroll
            for (int q = 0; q < MAXC; ++q) {
                const int cidx = gl + q * g.lanes;
                const bool act = cidx < g.chunks;
                double acc64[VEC];
                V xr{}, ar{};
                sum_positions<VEC, BATCH>(cv, grads, l.grow, w.a, w.b, cidx, act, acc64, step, (uint32_t)w.slot, xr, ar, w.from_key);
                finish_piece(w, cidx, act, acc64, xr, ar);
            }
            finish_segment(w);
        }
    }
    tr.stamp(2);
    if (any_long) {
        // longer segments (a popular key): all row groups together, one segment at a time
        for (uint32_t sg = 0; sg < nseg; ++sg) {
            const uint32_t a = l.seg_start[sg], b = l.seg_start[sg + 1];
            if (b - a <= AP_SOLO) continue;
            const bool is_front = sg == 0 && front_open, is_back = sg + 1 == nseg && back_open;
            const int32_t slot = is_front ? SLOT_NONE : l.slot[a];
            const uint32_t from_key = !is_front && ((l.fresh[a / WAVE] >> (a % WAVE)) & 1ull) ? l.key[1 + a] : KEY_NONE;
            const bool closed = !is_front && !is_back;
            const bool step = closed && slot != SLOT_NONE;
            const uint32_t per = (b - a + ngroups - 1) / ngroups;
            const uint32_t lo = min(a + group * per, b), hi = min(lo + per, b);
#pragma unroll
            for (int q = 0; q < MAXC; ++q) {
                const int cidx = gl + q * g.lanes;
                const bool act = cidx < g.chunks;
                double acc64[VEC];
                V xr{}, ar{};
                sum_positions<VEC, BATCH>(cv, grads, l.grow, lo, hi, cidx, act, acc64, step && group == 0, (uint32_t)slot, xr, ar, from_key);
                __syncthreads();                            // (the shares of the piece before have been read)
#pragma unroll
                for (int e = 0; e < VEC; ++e) l.share[threadIdx.x * VEC + e] = acc64[e];
                __syncthreads();
                if (group == 0) {
                    double tot[VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) tot[e] = 0.0;
                    for (uint32_t gi = 0; gi < ngroups; ++gi)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) tot[e] += l.share[(gi * g.lanes + gl) * VEC + e];
                    if (step) apply_loaded<VEC, EARLY>(cv, (uint32_t)slot, cidx, tot, lr, eps, xr, ar, act, from_key);
                    else if (!closed && act) {
                        double *mine = bd.part + ((size_t)T * 2 + (is_front ? 0 : 1)) * pstride + (size_t)cidx * VEC;
#pragma unroll
                        for (int e = 0; e < VEC; ++e) st_device(mine + e, tot[e]);
                    }
                }
            }
            if (threadIdx.x == 0) {
                if (is_back && !is_front) { st_device(&bd.slot[T], slot); st_device(&bd.from_key[T], from_key); }
                if (!is_front && slot != SLOT_NONE && !cv.direct) atomicAdd(&cv.meta[slot].cc, 1u);
            }
            if (!closed && group == 0) stores_acknowledged();
        }
    }
    tr.stamp(3);
    if (!front_open && !back_open) { tr.end(); return; }

    // Runs that cross this tile's borders.  Every tile such a run touches has stored one sum; each
    // counts itself as arrived at the run's first tile, and the one that arrives last adds the
    // sums in tile order and applies the step.  The first wave sees to the run that came in
    // through the front border, the second to the run that leaves through the back border (a tile
    // that lies inside one run has only the former).
    __syncthreads();
    tr.stamp(4);
    if (!do_front && !do_back) { tr.end(); return; }
    const uint32_t m = T1 - T0 + 1;
    // Sum of `count` stored sums, four in flight at a time, in order; where(i) is the i-th one's address for row piece 0.
    auto add_up = [&](uint32_t count, auto where, int cidx, bool act, double (&sum)[VEC]) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum[e] = 0.0;
        for (uint32_t i0 = 0; i0 < count; i0 += 4) {
            double part[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t i = i0 + u;
                const double *pp = where(i < count ? i : 0u) + (size_t)(act ? cidx : 0) * VEC;
#pragma unroll
                for (int e = 0; e < VEC; ++e) part[u][e] = i < count && act ? ld_device(pp + e) : 0.0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < VEC; ++e) sum[e] += part[u][e];
        }
    };
    // the i-th tile of the run: its first tile holds the run's sum at its back border, the others at their front border
    auto tile_sum = [&](uint32_t i) { return bd.part + ((size_t)(T0 + i) * 2 + (i == 0 ? 1 : 0)) * pstride; };
    auto arrive = [&](uint32_t *counter, uint32_t expected) {
        uint32_t last = 0;
        if (lane_id() == 0) {
            // (this tile's sums were acknowledged before)
            last = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1 ? 1u : 0u;
            if (last) *counter = 0;                         // clean for the next kernel
        }
        return __shfl(last, 0, WAVE) != 0;
    };
    // A run over more than AP_GROUP tiles (a very popular key) would keep its last tile adding for as
    // long as the rest of the kernel takes: two levels instead.  The tile that arrives last in its
    // group of AP_GROUP consecutive tiles adds the group's sums in tile order and stores the result;
    // the group that arrives last adds the groups' results in group order.  Still a fixed order.
    const bool grouped = m > AP_GROUP;
    const uint32_t ngroups_run = (m + AP_GROUP - 1) / AP_GROUP;
    if (grouped) {
        const uint32_t first = (T - T0) / AP_GROUP * AP_GROUP;          // the group's first tile, counted from T0
        const uint32_t gs = min(AP_GROUP, m - first);
        const size_t gname = (size_t)(T0 + first) * 2 + (first == 0 ? 1 : 0);
        if (!arrive(&bd.arrived[work_blocks + gname], gs)) { tr.end(); return; }
        if (lane_id() < (uint32_t)g.lanes) {
#pragma unroll
            for (int q = 0; q < MAXC; ++q) {
                const int cidx = gl + q * g.lanes;
                const bool act = cidx < g.chunks;
                if (!act) continue;
                double sum[VEC];
                add_up(gs, [&](uint32_t i) { return tile_sum(first + i); }, cidx, act, sum);
                double *mine = bd.part + ((size_t)work_blocks * 2 + gname) * pstride + (size_t)cidx * VEC;
#pragma unroll
                for (int e = 0; e < VEC; ++e) st_device(mine + e, sum[e]);
            }
        }
        stores_acknowledged();
    }
    if (!arrive(&bd.arrived[T0], grouped ? ngroups_run : m) || lane_id() >= (uint32_t)g.lanes) { tr.end(); return; }
    const int32_t slot = ld_device(&bd.slot[T0]);           // (SLOT_NONE: a key that is not cached, flagged where the order was probed)
    const uint32_t from_key = ld_device(&bd.from_key[T0]);
#pragma unroll
    for (int q = 0; q < MAXC; ++q) {
        const int cidx = gl + q * g.lanes;
        const bool act = cidx < g.chunks;
        if (!act && !cv.rowwise) continue;                  // (row-wise Adagrad: every lane of the group takes part in the row's sum)
        double sum[VEC];
        if (grouped) add_up(ngroups_run, [&](uint32_t i) { return (const double *)bd.part + ((size_t)work_blocks * 2 + (size_t)(T0 + i * AP_GROUP) * 2 + (i == 0 ? 1 : 0)) * pstride; }, cidx, act, sum);
        else add_up(m, [&](uint32_t i) { return (const double *)tile_sum(i); }, cidx, act, sum);
        if (slot != SLOT_NONE) apply_step<VEC, EARLY>(cv, (uint32_t)slot, cidx, sum, lr, eps, act, from_key);
    }
    tr.end();
}

// Drops the victims among 1024 consecutive slots, four per thread: erase the key, free the slot,
// raise c_g; then one row group per victim that holds updates copies its row (and accumulator)
// to the global table: Evict's push (Section 3.1).  Where a victim goes in the evicted-id list
// and (host-backed table) in the staging buffer follows from the select's per-block counts, so
// the kernel has no counter that every workgroup would have to add to: at a few nanoseconds
// per addition to one address, thousands of workgroups made those additions the kernel's
// duration.  The workgroup that holds the last victim among the rows tied at the threshold
// writes the call's counters.
struct EvictLds {
    uint32_t scan[TRIM_WAVES * 8 + 8];
    uint32_t v_slot[EV_SLOTS], v_key[EV_SLOTS], v_cg[EV_SLOTS], v_at[EV_SLOTS];
    uint32_t n_push;
};
// MANY: several workers over the table (the push adds what this worker changed to the server's row:
// three more rows in flight per victim, which the one-worker kernel does not pay registers for).
template <int VEC, bool RIDE, bool MANY>
__global__ __launch_bounds__(TRIM_THREADS) void trim_evict_kernel(CacheView cv, TrimPlan tp, SortStage ride, SortStage ride2)
{
    uint32_t blk = blockIdx.x, nblk_ = gridDim.x;
    if (RIDE && run_carried(ride, ride2, blk, nblk_)) return;
    EvictLds &el = lds_as<EvictLds>();
    uint32_t *scan = el.scan, *v_slot = el.v_slot, *v_key = el.v_key, *v_cg = el.v_cg, *v_at = el.v_at;
    if (blk + 1 == nblk_) { h0_remove_victims(cv, tp, v_slot, scan); return; }      // the last workgroup: keeps the first pass's histogram
    DState *ds = cv.ds;
    const uint32_t slot0 = blk * EV_SLOTS + threadIdx.x * EV_ITEMS;
    // everything this thread may need, requested at once
    const int32_t over = ds->over;                     // snapshot taken by the select
    const uint64_t tau = ds->sel_tau;
    const uint32_t take_eq = ds->sel_take;
    uint32_t key[EV_ITEMS];
    uint4 meta[EV_ITEMS];
    load_slots<EV_ITEMS>(cv, slot0, key, meta);
    // counts over the blocks before this one (whole supers, then the blocks of this super), and over all blocks
    uint32_t c8[8] = {0, 0, 0, 0, 0, 0, 0, 0};         // before: lt, eq, dirty lt, dirty eq;  all: dirty lt
    {
        const uint32_t nblocks = (cv.n_slots + EV_SLOTS - 1) / EV_SLOTS, nsup = (nblocks + EV_SUPER - 1) / EV_SUPER;
        const uint32_t sup = blk / EV_SUPER;
        for (uint32_t i = threadIdx.x; i < nsup; i += TRIM_THREADS) {
            const uint4 v = tp.sup_cnt[i];
            c8[4] += v.z;
            if (i < sup) { c8[0] += v.x; c8[1] += v.y; c8[2] += v.z; c8[3] += v.w; }
        }
        const uint32_t b = sup * EV_SUPER + threadIdx.x;
        if (threadIdx.x < EV_SUPER && b < blk) {
            const uint4 v = tp.blk_cnt[b];
            c8[0] += v.x; c8[1] += v.y; c8[2] += v.z; c8[3] += v.w;
        }
    }
    block_sum8(c8, scan);
    const uint32_t lt_before = c8[0], eq_before = c8[1], dlt_before = c8[2], deq_before = c8[3], dlt_total = c8[4];
    if (threadIdx.x == 0) el.n_push = 0;

    // this thread's four slots: below tau / tied with tau, in slot order
    bool lt[EV_ITEMS], eq[EV_ITEMS];
    uint32_t n_lt = 0, n_eq = 0, n_free = 0;
#pragma unroll
    for (int i = 0; i < EV_ITEMS; ++i) {
        const bool cached = key[i] != KEY_NONE && over > 0;
        const uint64_t pk = policy_key(tp, meta[i]);
        lt[i] = cached && pk < tau; eq[i] = cached && pk == tau;
        n_lt += lt[i]; n_eq += eq[i];
        n_free += (slot0 + i < cv.n_slots && key[i] == KEY_NONE) ? 1u : 0u;
    }
    uint32_t tot1;
    const uint32_t ex1 = block_excl_scan<TRIM_WAVES>(n_lt | (n_eq << 16), scan, tot1);
    uint32_t eq_rank = eq_before + (ex1 >> 16);        // rank of the thread's first tied row among all tied rows
    const uint32_t eq_here = tot1 >> 16;
    bool victim[EV_ITEMS], dirty[EV_ITEMS];
    uint32_t eq_at[EV_ITEMS];
    uint32_t n_vic = 0, n_dlt = 0, n_deq_vic = 0;
#pragma unroll
    for (int i = 0; i < EV_ITEMS; ++i) {
        eq_at[i] = eq_rank;
        victim[i] = lt[i] || (eq[i] && eq_rank < take_eq);
        dirty[i] = victim[i] && meta[i].y > meta[i].x;
        eq_rank += eq[i];
        n_vic += victim[i]; n_dlt += dirty[i] && lt[i]; n_deq_vic += dirty[i] && eq[i];
    }
    uint32_t tot2;
    const uint32_t ex2 = block_excl_scan<TRIM_WAVES>(n_vic | (n_dlt << 16), scan, tot2);
    const uint32_t nv = tot2 & 0xFFFFu;
    // victims in earlier blocks: their rows below tau, and their tied rows up to the cut
    uint32_t ev_at = lt_before + min(eq_before, take_eq) + (ex2 & 0xFFFFu);
    uint32_t dlt_at = dlt_before + (ex2 >> 16);
    const int buf = tp.ev_slot;
#pragma unroll
    for (int i = 0; i < EV_ITEMS; ++i) {
        if (victim[i]) {
        const uint32_t slot = slot0 + i, k = key[i], my_cc = meta[i].y;
        tp.ev_ids[ev_at++] = k;
        const uint32_t cg = dirty[i] ? cv.Cg[k] : 0u;                         // in flight together with the erase's loads
        const uint32_t early = dirty[i] && cv.early_cc ? cv.early_cc[slot] : 0u;
        ht_erase(cv.ht, k);
        cv.slot_key[slot] = KEY_NONE;
        // host-backed table: rows below tau that hold updates are staged in slot order, then one
        // place per tied victim (left empty by those without updates)
        const uint32_t stage_at = lt[i] ? dlt_at : dlt_total + eq_at[i];
        if (dirty[i]) {
            if (my_cc > cg) cv.Cg[k] = my_cc;                                 // c_g = max(c_g, c_c)
            // (pushed early by the update that fetched it, not updated since, and nobody else has pushed: the row is there already)
            const bool travelled = early == my_cc && cg == meta[i].x;
            if (!travelled) {
                const uint32_t at = atomicAdd(&el.n_push, 1u);
                v_slot[at] = slot; v_key[at] = k; v_cg[at] = my_cc > cg ? my_cc : cg; v_at[at] = stage_at;
            }
            dlt_at += lt[i];
        } else if (cv.Cg_host && eq[i]) {
            cv.hl.keys_of(buf)[stage_at] = KEY_NONE;
        }
        }
    }
    uint32_t s2[8] = {n_free, n_deq_vic, 0, 0, 0, 0, 0, 0};
    block_sum8(s2, scan);                              // also makes the push list visible to every thread
    const uint32_t free_here = s2[0], deq_vic_here = s2[1];
    const uint32_t np = el.n_push;
    const int lanes = cv.geom.lanes;
    const int group = threadIdx.x / lanes, gl = threadIdx.x % lanes, ngroups = TRIM_THREADS / lanes;
    const RowGeom g = cv.geom;
    // Evict's push, PUSH_ROWS victims per row group at a time (all their loads before the first
    // store).  Host-backed table: the rows go to the staging buffer instead; the next Read's fetch
    // kernel (or a waiting call) sends them over the host link.
    using V = typename VecT<VEC>::type;
    constexpr int PUSH_ROWS = 4;
    static_assert(PUSH_ROWS == 4, "the copy below is written out for four rows");
    const bool host = cv.Cg_host != nullptr;
    const float *src_x = cv.rows, *src_a = cv.acc;
    float *dst_x = host ? cv.hl.rows_of(buf) : cv.W, *dst_a = host ? cv.hl.acc_of(buf) : cv.A;
    for (uint32_t v0 = group * PUSH_ROWS; v0 < np; v0 += ngroups * PUSH_ROWS) {
        uint32_t from[PUSH_ROWS], to[PUSH_ROWS];
#pragma unroll
        for (int r = 0; r < PUSH_ROWS; ++r) {
            const uint32_t v = min(v0 + r, np - 1);
            from[r] = v_slot[v];
            to[r] = host ? v_at[v] : v_key[v];
            if (host && gl == 0 && v0 + r < np) {
                const uint32_t vk = v_key[v];
                cv.hl.keys_of(buf)[to[r]] = vk;
                cv.hl.cg_of(buf)[to[r]] = v_cg[v];
                cv.hl.pend[vk] = ((uint64_t)tp.push_seq << 32) | (uint64_t)to[r];
            }
        }
        const bool adagrad = cv.adagrad != 0;
        for (int c = gl; c < g.chunks; c += g.lanes) {
            V x0, x1, x2, x3, a0{}, a1{}, a2{}, a3{};
            x0 = reinterpret_cast<const V *>(src_x + (size_t)from[0] * g.dim)[c];
            x1 = reinterpret_cast<const V *>(src_x + (size_t)from[1] * g.dim)[c];
            x2 = reinterpret_cast<const V *>(src_x + (size_t)from[2] * g.dim)[c];
            x3 = reinterpret_cast<const V *>(src_x + (size_t)from[3] * g.dim)[c];
            if (adagrad) {
                a0 = reinterpret_cast<const V *>(src_a + (size_t)from[0] * g.dim)[c];
                a1 = reinterpret_cast<const V *>(src_a + (size_t)from[1] * g.dim)[c];
                a2 = reinterpret_cast<const V *>(src_a + (size_t)from[2] * g.dim)[c];
                a3 = reinterpret_cast<const V *>(src_a + (size_t)from[3] * g.dim)[c];
            }
            if (MANY) {
                // several workers: the server adds what this worker accumulated since its Fetch
                // (rows past the end repeat the last one: only the first of the repeats adds)
                const bool r1 = v0 + 1 < np, r2 = v0 + 2 < np, r3 = v0 + 3 < np;
                const V w0 = reinterpret_cast<const V *>(dst_x + (size_t)to[0] * g.dim)[c], b0 = reinterpret_cast<const V *>(cv.rows0 + (size_t)from[0] * g.dim)[c];
                const V w1 = reinterpret_cast<const V *>(dst_x + (size_t)to[1] * g.dim)[c], b1 = reinterpret_cast<const V *>(cv.rows0 + (size_t)from[1] * g.dim)[c];
                const V w2 = reinterpret_cast<const V *>(dst_x + (size_t)to[2] * g.dim)[c], b2 = reinterpret_cast<const V *>(cv.rows0 + (size_t)from[2] * g.dim)[c];
                const V w3 = reinterpret_cast<const V *>(dst_x + (size_t)to[3] * g.dim)[c], b3 = reinterpret_cast<const V *>(cv.rows0 + (size_t)from[3] * g.dim)[c];
                x0 = delta_add(w0, x0, b0);
                x1 = r1 ? delta_add(w1, x1, b1) : x0; x2 = r2 ? delta_add(w2, x2, b2) : x1; x3 = r3 ? delta_add(w3, x3, b3) : x2;
                if (adagrad) {
                    const V u0 = reinterpret_cast<const V *>(dst_a + (size_t)to[0] * g.dim)[c], d0 = reinterpret_cast<const V *>(cv.acc0 + (size_t)from[0] * g.dim)[c];
                    const V u1 = reinterpret_cast<const V *>(dst_a + (size_t)to[1] * g.dim)[c], d1 = reinterpret_cast<const V *>(cv.acc0 + (size_t)from[1] * g.dim)[c];
                    const V u2 = reinterpret_cast<const V *>(dst_a + (size_t)to[2] * g.dim)[c], d2 = reinterpret_cast<const V *>(cv.acc0 + (size_t)from[2] * g.dim)[c];
                    const V u3 = reinterpret_cast<const V *>(dst_a + (size_t)to[3] * g.dim)[c], d3 = reinterpret_cast<const V *>(cv.acc0 + (size_t)from[3] * g.dim)[c];
                    a0 = delta_add(u0, a0, d0);
                    a1 = r1 ? delta_add(u1, a1, d1) : a0; a2 = r2 ? delta_add(u2, a2, d2) : a1; a3 = r3 ? delta_add(u3, a3, d3) : a2;
                }
            }
            // rows past the end repeat the last one: the same values to the same place
            reinterpret_cast<V *>(dst_x + (size_t)to[0] * g.dim)[c] = x0;
            reinterpret_cast<V *>(dst_x + (size_t)to[1] * g.dim)[c] = x1;
            reinterpret_cast<V *>(dst_x + (size_t)to[2] * g.dim)[c] = x2;
            reinterpret_cast<V *>(dst_x + (size_t)to[3] * g.dim)[c] = x3;
            if (adagrad) {
                reinterpret_cast<V *>(dst_a + (size_t)to[0] * g.dim)[c] = a0;
                reinterpret_cast<V *>(dst_a + (size_t)to[1] * g.dim)[c] = a1;
                reinterpret_cast<V *>(dst_a + (size_t)to[2] * g.dim)[c] = a2;
                reinterpret_cast<V *>(dst_a + (size_t)to[3] * g.dim)[c] = a3;
            }
        }
        if (cv.rowwise && gl == 0) {                 // (one accumulator per row; such a table is in HBM)
#pragma unroll
            for (int r = 0; r < PUSH_ROWS; ++r) cv.A[to[r]] = cv.acc[from[r]];
        }
    }
    if (threadIdx.x == 0) {
        if (free_here + nv) atomicAdd(&tp.tile_free[blk / (TRIM_TILE / EV_SLOTS)], free_here + nv);     // (zero when the trim starts; a few workgroups per tile)
        // the call's counters: written by the block that holds the last tied victim (block 0 if there is none)
        const bool closes = over <= 0 ? blk == 0
                          : (take_eq == 0 ? blk == 0 : (eq_before < take_eq && take_eq <= eq_before + eq_here));
        if (closes) {
            const uint32_t evicted = over > 0 ? (uint32_t)over : 0u;
            const uint32_t evicted_dirty = over > 0 ? dlt_total + deq_before + deq_vic_here : 0u;
            ds->ev_n[buf] = evicted;
            ds->push_n[buf] = over > 0 ? dlt_total + take_eq : 0u;
            if (evicted) {
                ds->size -= (int32_t)evicted;
                cv.last->evicted = evicted; ds->total.evicted += evicted;
                cv.last->evicted_dirty = evicted_dirty; ds->total.evicted_dirty += evicted_dirty;
            }
        }
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
        if (key == KEY_NONE || cv.meta[slot].cc <= cv.meta[slot].cs) continue;
        if (cv.many) sync_row_many<VEC>(cv, key, slot, gl, true, false);
        else push_row<VEC>(cv, key, slot, gl);
        if (gl == 0) { const uint32_t cg = cv.Cg[key]; cv.meta[slot].cs = cg; cv.meta[slot].cc = cg; ++pushed; }
    }
    pushed = block_sum<4>(pushed, lds);
    if (blockIdx.x == 0 && threadIdx.x == 0) { Counters z{}; *cv.next_call = z; }
    if (threadIdx.x == 0) count2(&cv.last->flushed, &cv.ds->total.flushed, pushed);
}

// The server's side of a push by a worker that is not modelled otherwise (Section 3.1, Evict): the
// global row ids[i] takes deltas[i][:] and its clock advances by one.  One row group per id.
template <int VEC>
__global__ __launch_bounds__(256) void foreign_update_kernel(CacheView cv, const int64_t *__restrict__ ids, const float *__restrict__ deltas, uint32_t n)
{
    using V = typename VecT<VEC>::type;
    const RowGeom g = cv.geom;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / g.lanes, ngroups = gridDim.x * 256u / g.lanes;
    const int gl = threadIdx.x % g.lanes;
    for (uint32_t i = gid; i < n; i += ngroups) {
        const int64_t id = ids[i];
        if (id < 0 || id >= (int64_t)cv.vocab) { if (gl == 0) atomicOr(&cv.ds->err, ERRBIT_RANGE); continue; }
        V *w = reinterpret_cast<V *>(cv.W + (size_t)id * g.dim);
        const V *d = reinterpret_cast<const V *>(deltas + (size_t)i * g.dim);
        for (int c = gl; c < g.chunks; c += g.lanes) w[c] = delta_add(w[c], d[c], V{});
        if (gl == 0) cv.Cg[id] += 1;
    }
}

// Initial free list (every slot free) and empty slots / hash table.
__global__ __launch_bounds__(256) void init_cache_kernel(CacheView cv, uint32_t n_entries, uint32_t n_buckets)
{
    const uint32_t i0 = blockIdx.x * 256u + threadIdx.x, stride = gridDim.x * 256u;
    for (uint32_t i = i0; i < cv.n_slots; i += stride) {
        cv.slot_key[i] = KEY_NONE; store_meta(cv.meta, i, 0, 0, 0, 0);
    }
    for (uint32_t i = i0; i < cv.max_ids; i += stride) cv.free_list[i] = i;
    for (uint32_t i = i0; i < n_entries; i += stride) cv.ht.entries[i] = ENTRY_EMPTY;
    for (uint32_t i = i0; i < n_buckets; i += stride) cv.ht.reach[i] = 0;
}

} // namespace het
