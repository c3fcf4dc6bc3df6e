// Dedup of a minibatch's ids: the "unique embedding key set" of Algorithm 1 of the paper.
//
// A stable least-significant-digit radix sort of (id, position) pairs over just the bits the
// vocabulary needs, in one to four passes of up to 8 bits.  The result is
//   skey[j], perm[j]   ids ascending with the original position of each; equal ids keep their
//                      original order, so a key's occurrences come in increasing position.
// A run of equal keys in skey is one unique key; its first position is the key's "head".
// Ids outside [0, vocab) get the key `vocab`, which sorts behind every valid id.
//
// The sort is a sequence of stages, two per pass: a histogram stage counts the pass's digit per
// tile of 1024 keys, a scatter stage moves the keys.  Narrow digits and small tiles keep every
// stage a few microseconds long (the ranking of a key costs one ballot per digit bit, and a
// workgroup ranks its keys one after the other), which is what lets other kernels carry them.  Every workgroup of a scatter stage derives
// its output offsets itself from the per-tile histograms ("count at the producer, prefix at the
// consumer"); no workgroup ever waits for another one, and nothing is counted with global
// atomics (a popular id would make hundreds of them hit one address).
//
// A stage is a device function for workgroups of 256 threads, not a kernel: the sort of the
// NEXT minibatch (Section 4.2: its indices are known in advance) touches no cache state, so
// its stages are carried, one per kernel, in extra workgroups of the kernels of the current
// Read and Write.  At minibatch size those kernels are bound by latency, not by throughput, and
// the sort disappears inside them; a stage nobody carried runs as a kernel of its own.
#pragma once
#include "common.hpp"

namespace het {

constexpr int SORT_THREADS = 256;
constexpr int SORT_WAVES = SORT_THREADS / WAVE;
constexpr int SORT_ITEMS = 4;
constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS;     // keys per workgroup
constexpr int SORT_MIN_BITS = 3;                         // a histogram row is read 8 digits at a time
constexpr int SORT_MAX_BITS = 8;
constexpr int SORT_MAX_BINS = 1 << SORT_MAX_BITS;
constexpr int SORT_MAX_PASSES = 4;                       // vocab < 2^32
constexpr int SORT_BINS_PER_THREAD = SORT_MAX_BINS / SORT_THREADS;

struct SortPlan {
    uint32_t n;            // keys
    uint32_t vocab;
    uint32_t ntiles;       // ceil(n / SORT_TILE)
    int passes;            // 1..4
    int width;             // bits per digit (3..8)
    uint32_t *hist;        // [ntiles][bins / 2]: the current pass's digit counts per tile, two 16-bit counts per word
};

// One stage of a sort, as handed to the kernel that runs it.
struct SortStage {
    SortPlan sp;
    const int64_t *ids;                    // the caller's ids (read by stage 0 only)
    const uint32_t *keys_in, *idx_in;      // input of the pass (idx_in unused in pass 0: the payload is the position)
    uint32_t *keys_out, *idx_out;          // output of the pass; the first stage writes the converted ids to keys_out
    int stage;                             // 2p: histogram of pass p;  2p + 1: scatter of pass p
    uint32_t blocks;                       // workgroups the stage needs (sp.ntiles), 0: no stage
};

__host__ __device__ inline uint32_t sort_stage_lds_bytes(int width, int stage)
{
    const uint32_t bins = 1u << width;
    return (stage & 1) ? (SORT_WAVES + 1) * bins * 4u + 64u : bins * 4u;
}

__device__ __forceinline__ uint32_t id_to_key(int64_t id, uint32_t vocab)
{
    return (id >= 0 && id < (int64_t)vocab) ? (uint32_t)id : vocab;
}

// Position of item `it` of this thread inside its tile: a wave owns SORT_ITEMS * 64 consecutive
// keys and walks them 64 at a time, so (wave, item, lane) order is position order.
__device__ __forceinline__ uint32_t sort_pos(uint32_t tile, int it)
{
    const uint32_t w = threadIdx.x / WAVE;
    return tile * SORT_TILE + w * (WAVE * SORT_ITEMS) + it * WAVE + lane_id();
}

// Histogram stage of pass p for one tile.  Pass 0 reads the ids and leaves them as 32-bit keys
// (keys_out) for its scatter stage.  lds: bins words.
__device__ __forceinline__ void sort_hist_body(const SortStage &s, uint32_t tile, uint32_t *lds)
{
    const SortPlan &sp = s.sp;
    const int pass = s.stage >> 1;
    const uint32_t bins = 1u << sp.width, mask = bins - 1u, shift = (uint32_t)(pass * sp.width);
    // all of the tile's keys are requested before the first is used (the pass is uniform: no
    // branch per key)
    uint32_t key[SORT_ITEMS];
    if (pass == 0) {
        int64_t id[SORT_ITEMS];
#pragma unroll
        for (int it = 0; it < SORT_ITEMS; ++it) { const uint32_t i = sort_pos(tile, it); id[it] = i < sp.n ? s.ids[i] : 0; }
#pragma unroll
        for (int it = 0; it < SORT_ITEMS; ++it) key[it] = id_to_key(id[it], sp.vocab);
    } else {
#pragma unroll
        for (int it = 0; it < SORT_ITEMS; ++it) { const uint32_t i = sort_pos(tile, it); key[it] = i < sp.n ? s.keys_in[i] : 0u; }
    }
    for (uint32_t b = threadIdx.x; b < bins; b += SORT_THREADS) lds[b] = 0;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t i = sort_pos(tile, it);
        if (i < sp.n) {
            atomicAdd(&lds[(key[it] >> shift) & mask], 1u);
            if (pass == 0) s.keys_out[i] = key[it];
        }
    }
    __syncthreads();
    for (uint32_t w = threadIdx.x; w < bins / 2; w += SORT_THREADS)
        sp.hist[(size_t)tile * (bins / 2) + w] = lds[2 * w] | (lds[2 * w + 1] << 16);     // a tile has 1024 keys: counts fit 16 bits
}

// Scatter stage of pass p for one tile: stable.  lds: (SORT_WAVES + 1) * bins words + 16.
__device__ __forceinline__ void sort_scatter_body(const SortStage &s, uint32_t tile, uint32_t *lds)
{
    const SortPlan &sp = s.sp;
    const int pass = s.stage >> 1;
    const int width = sp.width;
    const uint32_t bins = 1u << width, mask = bins - 1u, shift = (uint32_t)(pass * width);
    const uint32_t w = threadIdx.x / WAVE;
    uint32_t *wave_hist = lds;                         // [SORT_WAVES][bins]
    uint32_t *tile_base = lds + SORT_WAVES * bins;     // [bins]
    uint32_t *scan_lds = tile_base + bins;             // [SORT_WAVES + 1]

    uint32_t key[SORT_ITEMS], pay[SORT_ITEMS], lrank[SORT_ITEMS];
    // Output offset of each digit for this tile: keys of smaller digits anywhere, plus keys of
    // the same digit in earlier tiles.  A thread adds up eight consecutive digits (one 16-byte
    // load per tile, many loads in flight) over every TLN-th tile; LDS merges the tile lanes.
    {
        uint32_t *tot = wave_hist, *bef = wave_hist + bins;      // borrowed until the ranking starts
        for (uint32_t b = threadIdx.x; b < 2 * bins; b += SORT_THREADS) wave_hist[b] = 0;
        __syncthreads();
        const uint4 *h4 = reinterpret_cast<const uint4 *>(sp.hist);
        const uint32_t octs = bins / 8;                                  // width >= 3
        const uint32_t tln = octs >= SORT_THREADS ? 1u : SORT_THREADS / octs;
        for (uint32_t item = threadIdx.x; item < octs * tln; item += SORT_THREADS) {
            const uint32_t bo = item % octs, tl = item / octs;
            uint32_t t8[8], f8[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { t8[e] = 0; f8[e] = 0; }
            // four tiles at a time (more would cost the carrying kernels occupancy), every load issued before the first add
            for (uint32_t t0 = tl; t0 < sp.ntiles; t0 += 4 * tln) {
                uint4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t t = t0 + u * tln;
                    v[u] = t < sp.ntiles ? h4[(size_t)t * octs + bo] : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t t = t0 + u * tln;
                    const uint32_t c[8] = {v[u].x & 0xFFFFu, v[u].x >> 16, v[u].y & 0xFFFFu, v[u].y >> 16,
                                           v[u].z & 0xFFFFu, v[u].z >> 16, v[u].w & 0xFFFFu, v[u].w >> 16};
                    const bool earlier = t < tile;
#pragma unroll
                    for (int e = 0; e < 8; ++e) { t8[e] += c[e]; f8[e] += earlier ? c[e] : 0u; }
                }
            }
            const uint32_t b = bo * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (tln == 1) { tot[b + e] = t8[e]; bef[b + e] = f8[e]; }
                else { if (t8[e]) atomicAdd(&tot[b + e], t8[e]); if (f8[e]) atomicAdd(&bef[b + e], f8[e]); }
            }
        }
        // The keys (and payload) of this tile are requested here: the offsets' registers are free
        // again, and the loads are on their way while the digits are scanned.  (Held across the
        // whole offset computation they would cost the carrying kernel part of its occupancy.)
#pragma unroll
        for (int it = 0; it < SORT_ITEMS; ++it) {
            const uint32_t i = sort_pos(tile, it);
            key[it] = i < sp.n ? s.keys_in[i] : 0u;
        }
        if (pass == 0) {
#pragma unroll
            for (int it = 0; it < SORT_ITEMS; ++it) pay[it] = sort_pos(tile, it);
        } else {
#pragma unroll
            for (int it = 0; it < SORT_ITEMS; ++it) { const uint32_t i = sort_pos(tile, it); pay[it] = i < sp.n ? s.idx_in[i] : 0u; }
        }
        __syncthreads();
        // exclusive scan over the digits; thread t owns SORT_BINS_PER_THREAD consecutive digits
        const uint32_t b0 = threadIdx.x * SORT_BINS_PER_THREAD;
        uint32_t tq[SORT_BINS_PER_THREAD], fq[SORT_BINS_PER_THREAD], mine = 0;
#pragma unroll
        for (int q = 0; q < SORT_BINS_PER_THREAD; ++q) {
            tq[q] = b0 + q < bins ? tot[b0 + q] : 0u;
            fq[q] = b0 + q < bins ? bef[b0 + q] : 0u;
            mine += tq[q];
        }
        uint32_t total;
        uint32_t run = block_excl_scan<SORT_WAVES>(mine, scan_lds, total);
#pragma unroll
        for (int q = 0; q < SORT_BINS_PER_THREAD; ++q) {
            if (b0 + q < bins) tile_base[b0 + q] = run + fq[q];
            run += tq[q];
        }
        __syncthreads();
        for (uint32_t b = threadIdx.x; b < SORT_WAVES * bins; b += SORT_THREADS) wave_hist[b] = 0;
    }
    __syncthreads();

    // rank of every key among the keys of the same digit before it in the tile: within the wave
    // by ballots over the digit's bits, across the wave's earlier items by a running count
    // First all the ballots (registers only), then the running counts (LDS only): interleaved,
    // every item would wait for both in turn.
    uint32_t lead[SORT_ITEMS];          // for the first lane of each group of equal digits: the group's size
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t i = sort_pos(tile, it);
        const bool valid = i < sp.n;
        const uint32_t d = (key[it] >> shift) & mask;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < SORT_MAX_BITS; ++b) {
            if (b < width) {
                const uint64_t bal = __ballot((d >> b) & 1u);
                const uint32_t flip = ((d >> b) & 1u) - 1u;               // all ones where the lane's bit is clear
                const uint32_t lo = (uint32_t)bal ^ flip, hi = (uint32_t)(bal >> 32) ^ flip;
                peers &= ((uint64_t)hi << 32) | lo;
            }
        }
        const uint32_t r = mask_rank(peers);
        lrank[it] = r;
        lead[it] = (valid && r == 0) ? (uint32_t)__popcll(peers) : 0u;
    }
    volatile uint32_t *my_hist = wave_hist + w * bins;
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t d = (key[it] >> shift) & mask;
        const uint32_t before = my_hist[d];
        lrank[it] += before;
        __builtin_amdgcn_wave_barrier();
        if (lead[it]) my_hist[d] = before + lead[it];
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < bins; b += SORT_THREADS) {
        uint32_t run = tile_base[b];
#pragma unroll
        for (int ww = 0; ww < SORT_WAVES; ++ww) {
            const uint32_t c = wave_hist[ww * bins + b];
            wave_hist[ww * bins + b] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t i = sort_pos(tile, it);
        if (i < sp.n) {
            const uint32_t d = (key[it] >> shift) & mask;
            const uint32_t pos = wave_hist[w * bins + d] + lrank[it];
            s.keys_out[pos] = key[it];
            s.idx_out[pos] = pay[it];
        }
    }
}

// Runs stage s for tile `tile`; `lds` must hold sort_stage_lds_bytes(width, stage) bytes.
__device__ __forceinline__ void sort_stage_body(const SortStage &s, uint32_t tile, uint32_t *lds)
{
    // few workgroups with a long chain of dependent steps, among the many of the carrying kernel:
    // their waves go first when a SIMD has to choose
    __builtin_amdgcn_s_setprio(3);
    if (s.stage & 1) sort_scatter_body(s, tile, lds);
    else sort_hist_body(s, tile, lds);
}

// A stage nobody carried.
__global__ __launch_bounds__(SORT_THREADS) void sort_stage_kernel(SortStage s)
{
    extern __shared__ __align__(16) uint32_t sort_dyn_lds[];
    sort_stage_body(s, blockIdx.x, sort_dyn_lds);
}

// First position of `key` in the sorted keys: lower bound over skey[0 .. hi).
__device__ __forceinline__ uint32_t run_head(const uint32_t *skey, uint32_t hi, uint32_t key)
{
    uint32_t lo = 0;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (skey[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// One past the last position of `key`: upper bound over skey[lo .. n).
__device__ __forceinline__ uint32_t run_end(const uint32_t *skey, uint32_t lo, uint32_t n, uint32_t key)
{
    uint32_t hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (skey[mid] <= key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// One past the last position of the run of `key` that is known to hold position lo - 1, found by
// a row group of `lanes` lanes together: every lane looks at one position per round, the
// spacing grows sixteenfold (by `lanes`) while all of them still hold the key and shrinks again
// once they do not, so a run of a few hundred positions takes three rounds of one load each where
// a binary search over the whole batch takes seventeen.  Called by every lane of the wave (a
// group that has nothing to look for passes active = false); lanes is a power of two <= 64.
__device__ __forceinline__ uint32_t group_run_end(const uint32_t *skey, uint32_t lo, uint32_t n, uint32_t key, bool active, int lanes)
{
    const uint32_t lane = lane_id(), gl = lane % (uint32_t)lanes;
    const uint32_t shift = lane - gl;                                   // first lane of this group in the wave
    const uint64_t gmask = lanes == 64 ? ~0ull : (((1ull << lanes) - 1ull) << shift);
    uint32_t base = lo, step = 1;                                       // positions below base hold the key
    bool going = active && lo < n;
    while (__any(going)) {
        const uint64_t idx = (uint64_t)base + (uint64_t)gl * step + (step - 1);      // the last position of the lane's stretch
        const bool hit = going && idx < n && skey[idx] == key;
        const uint32_t cnt = (uint32_t)__popcll(__ballot(hit) & gmask);   // hits are the first lanes: the keys are sorted
        if (going) {
            base += cnt * step;
            if (cnt == (uint32_t)lanes && (uint64_t)base < n) step *= (uint32_t)lanes;        // all hold it: look further out
            else if (step == 1 || (uint64_t)base >= n) going = false;                        // the end is exactly here
            else step = step / (uint32_t)lanes > 0 ? step / (uint32_t)lanes : 1;             // it ends inside the next stretch: look closer
        }
    }
    return base < n ? base : n;
}

} // namespace het
