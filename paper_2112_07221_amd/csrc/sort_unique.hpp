// Dedup of a minibatch's ids: the "unique embedding key set" of Algorithm 1 of the paper.
//
// A stable least-significant-digit radix sort of (id, position) pairs, 8 bits per pass, over
// just the bits the vocabulary needs, followed by head-flag ranking.  The result is:
//   skey[j], perm[j]   ids ascending, with the original position of each (ties keep the
//                      original order, so a key's occurrences come in increasing position);
//   rank[j]            index of position j's key in the sorted unique key list;
//   ukey[r], seg[r]    the unique keys and where each key's run starts in the sorted order.
// Ids outside [0, vocab) are given the key `vocab`, which sorts behind every valid id, and are
// left out of the unique list.
#pragma once
#include "common.hpp"

namespace het {

constexpr int SORT_THREADS = 256;
constexpr int SORT_WAVES = SORT_THREADS / WAVE;
constexpr int SORT_ITEMS = 8;
constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS;   // 2048 keys per workgroup
constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;

// Position of item `it` of this thread inside its tile: a wave owns 512 consecutive keys and
// walks them 64 at a time, so (wave, item, lane) order is position order.
__device__ __forceinline__ uint32_t sort_pos(uint32_t tile, int it)
{
    const uint32_t w = threadIdx.x / WAVE;
    return tile * SORT_TILE + w * (WAVE * SORT_ITEMS) + it * WAVE + lane_id();
}

constexpr int CALL_BUMP_ITERATION = 1;   // this call is a Read: advance the iteration counter
constexpr int CALL_RESET_LAST = 2;       // start the per-call counters from zero

// Per-tile digit histogram.  FIRST: also turns the int64 ids into 32-bit sort keys, flags ids
// outside the vocabulary and resets the per-call counters (block 0).
template <bool FIRST>
__global__ __launch_bounds__(SORT_THREADS) void sort_count_kernel(
    const int64_t *__restrict__ ids, const uint32_t *__restrict__ keys_in,
    uint32_t *__restrict__ keys0, uint32_t n, uint32_t vocab, uint32_t shift,
    uint32_t *__restrict__ tile_hist, uint32_t ntiles, DState *ds, int call_flags)
{
    __shared__ uint32_t hist[RADIX];
    const uint32_t tile = blockIdx.x;
    for (int b = threadIdx.x; b < RADIX; b += SORT_THREADS) hist[b] = 0;
    __syncthreads();
    bool bad = false;
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t i = sort_pos(tile, it);
        if (i < n) {
            uint32_t key;
            if (FIRST) {
                const int64_t id = ids[i];
                const bool ok = id >= 0 && id < (int64_t)vocab;
                key = ok ? (uint32_t)id : vocab;
                bad |= !ok;
                keys0[i] = key;
            } else {
                key = keys_in[i];
            }
            atomicAdd(&hist[(key >> shift) & (RADIX - 1)], 1u);
        }
    }
    if (FIRST) {
        if (__any(bad) && lane_id() == 0) atomicOr(&ds->err, ERRBIT_RANGE);
        if (tile == 0 && threadIdx.x == 0) {
            if (call_flags & CALL_BUMP_ITERATION) ds->t += 1;
            if (call_flags & CALL_RESET_LAST) { Counters z{}; ds->last = z; }
            ds->last.n = n;
            atomicAdd(&ds->total.n, (unsigned long long)n);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < RADIX; b += SORT_THREADS) tile_hist[b * ntiles + tile] = hist[b];
}

// Exclusive scan, in place, of the RADIX x ntiles histogram laid out digit-major: entry
// (digit, tile) becomes the first output position of that digit's keys from that tile.
constexpr int SCAN_THREADS = 1024;
__global__ __launch_bounds__(SCAN_THREADS) void sort_scan_kernel(uint32_t *__restrict__ tile_hist, uint32_t total)
{
    __shared__ uint32_t lds[SCAN_THREADS / WAVE + 1];
    const uint32_t per = (total + SCAN_THREADS - 1) / SCAN_THREADS;
    const uint32_t lo = min(threadIdx.x * per, total), hi = min(lo + per, total);
    uint32_t s = 0;
    for (uint32_t i = lo; i < hi; ++i) s += tile_hist[i];
    uint32_t tot;
    uint32_t run = block_excl_scan<SCAN_THREADS / WAVE>(s, lds, tot);
    for (uint32_t i = lo; i < hi; ++i) { const uint32_t c = tile_hist[i]; tile_hist[i] = run; run += c; }
}

// Stable scatter of one pass.  Ranking inside the tile: each wave ranks 64 keys at a time with
// eight ballots (lanes holding the same digit find each other), keeps a running per-wave digit
// count in LDS, and the per-wave counts are then turned into offsets in wave order.
template <bool FIRST>
__global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(
    const uint32_t *__restrict__ keys_in, const uint32_t *__restrict__ idx_in,
    uint32_t *__restrict__ keys_out, uint32_t *__restrict__ idx_out, uint32_t n, uint32_t shift,
    const uint32_t *__restrict__ tile_off, uint32_t ntiles)
{
    __shared__ uint32_t wave_hist[SORT_WAVES][RADIX];
    const uint32_t tile = blockIdx.x, w = threadIdx.x / WAVE;
    for (int b = threadIdx.x; b < SORT_WAVES * RADIX; b += SORT_THREADS) (&wave_hist[0][0])[b] = 0;
    __syncthreads();

    uint32_t key[SORT_ITEMS], lrank[SORT_ITEMS];
    volatile uint32_t *my_hist = wave_hist[w];
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t i = sort_pos(tile, it);
        const bool valid = i < n;
        key[it] = valid ? keys_in[i] : 0u;
        const uint32_t d = (key[it] >> shift) & (RADIX - 1);
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
        const uint32_t r = mask_rank(peers);
        const uint32_t before = my_hist[d];
        lrank[it] = before + r;
        __builtin_amdgcn_wave_barrier();
        if (valid && r == 0) my_hist[d] = before + (uint32_t)__popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    for (int b = threadIdx.x; b < RADIX; b += SORT_THREADS) {
        uint32_t run = tile_off[b * ntiles + tile];
#pragma unroll
        for (int ww = 0; ww < SORT_WAVES; ++ww) {
            const uint32_t c = wave_hist[ww][b];
            wave_hist[ww][b] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < SORT_ITEMS; ++it) {
        const uint32_t i = sort_pos(tile, it);
        if (i < n) {
            const uint32_t d = (key[it] >> shift) & (RADIX - 1);
            const uint32_t pos = wave_hist[w][d] + lrank[it];
            keys_out[pos] = key[it];
            idx_out[pos] = FIRST ? i : idx_in[i];
        }
    }
}

// ---- unique: head flags over the sorted keys -------------------------------------------------
constexpr int UQ_THREADS = 256;
constexpr int UQ_WAVES = UQ_THREADS / WAVE;
constexpr int UQ_ITEMS = 4;
constexpr int UQ_TILE = UQ_THREADS * UQ_ITEMS;   // 1024 sorted positions per workgroup

__device__ __forceinline__ bool is_head(const uint32_t *skey, uint32_t j, uint32_t n, uint32_t vocab)
{
    if (j >= n) return false;
    const uint32_t k = skey[j];
    return k != vocab && (j == 0 || skey[j - 1] != k);
}

// tile_heads[tile] = number of distinct valid keys that start inside the tile.
__global__ __launch_bounds__(UQ_THREADS) void unique_count_kernel(
    const uint32_t *__restrict__ skey, uint32_t n, uint32_t vocab, uint32_t *__restrict__ tile_heads)
{
    __shared__ uint32_t lds[UQ_WAVES];
    const uint32_t base = blockIdx.x * UQ_TILE + threadIdx.x * UQ_ITEMS;
    uint32_t c = 0;
#pragma unroll
    for (int it = 0; it < UQ_ITEMS; ++it) c += is_head(skey, base + it, n, vocab) ? 1u : 0u;
    c = block_sum<UQ_WAVES>(c, lds);
    if (threadIdx.x == 0) tile_heads[blockIdx.x] = c;
}

} // namespace het
