// Dedup of a minibatch's ids: the "unique embedding key set" of Algorithm 1 of the paper.
//
// A stable least-significant-digit radix sort of (id, position) pairs over just the bits the
// vocabulary needs, in one to three passes of up to 11 bits.  The result is
//   skey[j], perm[j]   ids ascending with the original position of each; equal ids keep their
//                      original order, so a key's occurrences come in increasing position.
// A run of equal keys in skey is one unique key; its first position is the key's "head".
// Ids outside [0, vocab) get the key `vocab`, which sorts behind every valid id.
//
// Kernel count is what matters at minibatch sizes (a launch costs more than moving 100k
// keys), so a pass is a single kernel: every workgroup owns a tile of keys and derives its
// output offsets itself from the per-tile digit histograms ("count at the producer, prefix at
// the consumer").  The histograms of the first pass are counted from the ids; while a pass
// scatters a key it already counts it for the next pass, in the tile where it lands.  No
// workgroup ever waits for another one.
#pragma once
#include "common.hpp"

namespace het {

constexpr int SORT_THREADS = 512;
constexpr int SORT_WAVES = SORT_THREADS / WAVE;
constexpr int SORT_MAX_BITS = 11;
constexpr int SORT_MAX_BINS = 1 << SORT_MAX_BITS;
constexpr int SORT_MAX_PASSES = 3;                       // vocab < 2^32
constexpr int SORT_BINS_PER_THREAD = SORT_MAX_BINS / SORT_THREADS;

struct SortPlan {
    uint32_t n;            // keys
    uint32_t vocab;
    uint32_t tile;         // keys per workgroup = SORT_THREADS * items
    uint32_t ntiles;
    int passes;            // 1..3
    int width;             // bits per digit (<= 11)
    uint32_t *hist[SORT_MAX_PASSES];   // per pass: [ntiles][1 << width]
};

__device__ __forceinline__ uint32_t id_to_key(int64_t id, uint32_t vocab)
{
    return (id >= 0 && id < (int64_t)vocab) ? (uint32_t)id : vocab;
}

// Position of item `it` of this thread inside its tile: a wave owns ITEMS*64 consecutive keys
// and walks them 64 at a time, so (wave, item, lane) order is position order.
template <int ITEMS>
__device__ __forceinline__ uint32_t sort_pos(uint32_t tile_index, int it)
{
    const uint32_t w = threadIdx.x / WAVE;
    return tile_index * (SORT_THREADS * ITEMS) + w * (WAVE * ITEMS) + it * WAVE + lane_id();
}

// First kernel of a sort: digit histogram of pass 0 per tile, straight from the ids; flags ids
// outside the vocabulary; clears the histograms the later passes count into.  It touches no
// cache state, so the sort of the next minibatch may run beside the current update.
template <int ITEMS>
__global__ __launch_bounds__(SORT_THREADS) void dedup_hist_kernel(const int64_t *__restrict__ ids, SortPlan sp, DState *ds)
{
    __shared__ uint32_t hist[SORT_MAX_BINS];
    const uint32_t tile = blockIdx.x;
    const uint32_t bins = 1u << sp.width, mask = bins - 1u;
    for (uint32_t b = threadIdx.x; b < bins; b += SORT_THREADS) hist[b] = 0;
    for (int p = 1; p < sp.passes; ++p)
        for (uint32_t i = tile * SORT_THREADS + threadIdx.x; i < sp.ntiles * bins; i += gridDim.x * SORT_THREADS) sp.hist[p][i] = 0;
    __syncthreads();
    bool bad = false;
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const uint32_t i = sort_pos<ITEMS>(tile, it);
        if (i < sp.n) {
            const uint32_t key = id_to_key(ids[i], sp.vocab);
            bad |= key == sp.vocab;
            atomicAdd(&hist[key & mask], 1u);
        }
    }
    if (__any(bad) && lane_id() == 0) atomicOr(&ds->err, ERRBIT_RANGE);
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < bins; b += SORT_THREADS) sp.hist[0][tile * bins + b] = hist[b];
}

// One stable scatter pass.  FIRST reads the ids (positions are the payload); later passes
// read the previous pass's keys and payload.
template <int ITEMS, bool FIRST>
__global__ __launch_bounds__(SORT_THREADS) void sort_pass_kernel(const int64_t *__restrict__ ids, const uint32_t *__restrict__ keys_in,
                                                                 const uint32_t *__restrict__ idx_in, uint32_t *__restrict__ keys_out,
                                                                 uint32_t *__restrict__ idx_out, SortPlan sp, int pass)
{
    __shared__ uint32_t wave_hist[SORT_WAVES][SORT_MAX_BINS];
    __shared__ uint32_t tile_base[SORT_MAX_BINS];
    __shared__ uint32_t scan_lds[SORT_WAVES + 1];
    const uint32_t tile = blockIdx.x, w = threadIdx.x / WAVE;
    const int width = sp.width;
    const uint32_t bins = 1u << width, mask = bins - 1u;
    const uint32_t shift = (uint32_t)(pass * width);
    const bool last = pass + 1 == sp.passes;

    // the keys (and payload) of this tile: issued first, they arrive while the offsets are computed
    uint32_t key[ITEMS], pay[ITEMS], lrank[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const uint32_t i = sort_pos<ITEMS>(tile, it);
        const bool valid = i < sp.n;
        key[it] = valid ? (FIRST ? id_to_key(ids[i], sp.vocab) : keys_in[i]) : 0u;
        pay[it] = FIRST ? i : (valid ? idx_in[i] : 0u);
    }
    for (uint32_t b = threadIdx.x; b < SORT_WAVES * SORT_MAX_BINS; b += SORT_THREADS) (&wave_hist[0][0])[b] = 0;

    // Output offset of each digit for this tile: keys of smaller digits anywhere, plus keys of
    // the same digit in earlier tiles.  A thread adds up four consecutive digits (one 16-byte
    // load per tile, many loads in flight) over every TLN-th tile; LDS merges the tile lanes.
    {
        uint32_t *tot = &wave_hist[0][0], *bef = &wave_hist[1][0];      // borrowed until the ranking starts
        for (uint32_t b = threadIdx.x; b < bins; b += SORT_THREADS) { tot[b] = 0; bef[b] = 0; }
        __syncthreads();
        const uint4 *h4 = reinterpret_cast<const uint4 *>(sp.hist[pass]);
        const uint32_t quads = bins / 4;                                 // width >= 2
        const uint32_t tln = quads >= SORT_THREADS ? 1u : SORT_THREADS / quads;
        for (uint32_t item = threadIdx.x; item < quads * tln; item += SORT_THREADS) {
            const uint32_t bq = item % quads, tl = item / quads;
            uint4 t4 = make_uint4(0, 0, 0, 0), f4 = make_uint4(0, 0, 0, 0);
            // sixteen tiles at a time, every load issued before the first add
            for (uint32_t t0 = tl; t0 < sp.ntiles; t0 += 16 * tln) {
                uint4 v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const uint32_t t = t0 + u * tln;
                    v[u] = t < sp.ntiles ? h4[(size_t)t * quads + bq] : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const uint32_t t = t0 + u * tln;
                    t4.x += v[u].x; t4.y += v[u].y; t4.z += v[u].z; t4.w += v[u].w;
                    if (t < tile) { f4.x += v[u].x; f4.y += v[u].y; f4.z += v[u].z; f4.w += v[u].w; }
                }
            }
            const uint32_t b = bq * 4;
            if (tln == 1) {
                tot[b] = t4.x; tot[b + 1] = t4.y; tot[b + 2] = t4.z; tot[b + 3] = t4.w;
                bef[b] = f4.x; bef[b + 1] = f4.y; bef[b + 2] = f4.z; bef[b + 3] = f4.w;
            } else {
                atomicAdd(&tot[b], t4.x); atomicAdd(&tot[b + 1], t4.y); atomicAdd(&tot[b + 2], t4.z); atomicAdd(&tot[b + 3], t4.w);
                atomicAdd(&bef[b], f4.x); atomicAdd(&bef[b + 1], f4.y); atomicAdd(&bef[b + 2], f4.z); atomicAdd(&bef[b + 3], f4.w);
            }
        }
        __syncthreads();
        // exclusive scan over the digits; thread t owns SORT_BINS_PER_THREAD consecutive digits
        const uint32_t b0 = threadIdx.x * SORT_BINS_PER_THREAD;
        uint32_t t8[SORT_BINS_PER_THREAD], f8[SORT_BINS_PER_THREAD], mine = 0;
#pragma unroll
        for (int q = 0; q < SORT_BINS_PER_THREAD; ++q) {
            t8[q] = b0 + q < bins ? tot[b0 + q] : 0u;
            f8[q] = b0 + q < bins ? bef[b0 + q] : 0u;
            mine += t8[q];
        }
        uint32_t total;
        uint32_t run = block_excl_scan<SORT_WAVES>(mine, scan_lds, total);
#pragma unroll
        for (int q = 0; q < SORT_BINS_PER_THREAD; ++q) {
            if (b0 + q < bins) tile_base[b0 + q] = run + f8[q];
            run += t8[q];
        }
        __syncthreads();
        for (uint32_t b = threadIdx.x; b < 2 * SORT_MAX_BINS; b += SORT_THREADS) (&wave_hist[0][0])[b] = 0;
    }
    __syncthreads();

    volatile uint32_t *my_hist = wave_hist[w];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const uint32_t i = sort_pos<ITEMS>(tile, it);
        const bool valid = i < sp.n;
        const uint32_t d = (key[it] >> shift) & mask;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < SORT_MAX_BITS; ++b) {
            if (b < width) {
                const bool bit = (d >> b) & 1u;
                const uint64_t bal = __ballot(bit);
                peers &= bit ? bal : ~bal;
            }
        }
        const uint32_t r = mask_rank(peers);
        const uint32_t before = my_hist[d];
        lrank[it] = before + r;
        __builtin_amdgcn_wave_barrier();
        if (valid && r == 0) my_hist[d] = before + (uint32_t)__popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < bins; b += SORT_THREADS) {
        uint32_t run = tile_base[b];
#pragma unroll
        for (int ww = 0; ww < SORT_WAVES; ++ww) {
            const uint32_t c = wave_hist[ww][b];
            wave_hist[ww][b] = run;
            run += c;
        }
    }
    __syncthreads();
    uint32_t *next = last ? nullptr : sp.hist[pass + 1];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const uint32_t i = sort_pos<ITEMS>(tile, it);
        if (i < sp.n) {
            const uint32_t d = (key[it] >> shift) & mask;
            const uint32_t pos = wave_hist[w][d] + lrank[it];
            keys_out[pos] = key[it];
            idx_out[pos] = pay[it];
            if (next) atomicAdd(&next[(size_t)(pos / sp.tile) * bins + ((key[it] >> (shift + width)) & mask)], 1u);
        }
    }
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

} // namespace het
