// Open-addressing id -> slot table in HBM: the cache's Find (Algorithm 2 of the paper).
//
// The table is an array of buckets of 16 entries; an entry is 64 bits (id in the high word,
// slot in the low word, all ones = empty), so one bucket is one 128-byte line and a probe is
// normally a single line read.  A key lives in its home bucket, or, if that bucket was full
// when it arrived, in one of the following buckets (linear probing over buckets).  `reach[h]`
// records the largest distance any key homed at bucket h was ever displaced; a probe looks at
// buckets h .. h + reach[h] and nothing else.  Because a search always inspects whole buckets,
// deleting an entry is just writing "empty": no tombstones, no rehash.
//
// Phases never mix: probes, inserts and erases run in different kernels, so an insert only
// races with other inserts (settled by a 64-bit compare-and-swap on the entry).  Which entry
// of which bucket a key lands in depends on that race; the id -> slot mapping does not.
#pragma once
#include "common.hpp"

namespace het {

constexpr int BUCKET_ENTRIES = 16;
constexpr uint64_t ENTRY_EMPTY = ~0ull;

struct HashTable {
    uint64_t *entries;    // [n_buckets * BUCKET_ENTRIES]
    uint32_t *reach;      // [n_buckets]
    uint32_t bucket_mask; // n_buckets - 1 (power of two)
    uint32_t shift;       // 32 - log2(n_buckets)
};

__device__ __forceinline__ uint32_t ht_home(const HashTable &ht, uint32_t key)
{
    return ht.shift >= 32 ? 0u : ((key * 0x9E3779B1u) >> ht.shift) & ht.bucket_mask;
}

__device__ __forceinline__ uint64_t ht_pack(uint32_t key, uint32_t slot)
{
    return ((uint64_t)key << 32) | slot;
}

// Looks for `key` in bucket b: all eight 16-byte loads are issued before the first compare.
__device__ __forceinline__ int32_t ht_scan_bucket(const HashTable &ht, uint32_t b, uint32_t key, uint32_t *entry_index)
{
    const uint4 *line = reinterpret_cast<const uint4 *>(ht.entries + (size_t)b * BUCKET_ENTRIES);
    uint4 v[BUCKET_ENTRIES / 2];
#pragma unroll
    for (int q = 0; q < BUCKET_ENTRIES / 2; ++q) v[q] = line[q];      // two entries each: (slot, key), (slot, key)
    int32_t slot = SLOT_NONE;
    uint32_t at = 0;
#pragma unroll
    for (int q = 0; q < BUCKET_ENTRIES / 2; ++q) {
        if (v[q].y == key) { slot = (int32_t)v[q].x; at = 2 * q; }
        if (v[q].w == key) { slot = (int32_t)v[q].z; at = 2 * q + 1; }
    }
    if (entry_index && slot != SLOT_NONE) *entry_index = b * BUCKET_ENTRIES + at;
    return slot;
}

// Slot of `key`, or SLOT_NONE.  If entry_index is given it receives the entry's position.
__device__ __forceinline__ int32_t ht_find(const HashTable &ht, uint32_t key, uint32_t *entry_index = nullptr)
{
    const uint32_t h = ht_home(ht, key);
    const uint32_t reach = ht.reach[h];                  // in flight together with the home bucket
    int32_t slot = ht_scan_bucket(ht, h, key, entry_index);
    for (uint32_t d = 1; slot == SLOT_NONE && d <= reach; ++d) slot = ht_scan_bucket(ht, (h + d) & ht.bucket_mask, key, entry_index);
    return slot;
}

// Inserts a key known to be absent.  Returns false only if every bucket is full.
__device__ __forceinline__ bool ht_insert(const HashTable &ht, uint32_t key, uint32_t slot)
{
    const uint32_t h = ht_home(ht, key);
    const uint64_t e = ht_pack(key, slot);
    for (uint32_t d = 0; d <= ht.bucket_mask; ++d) {
        const uint32_t b = (h + d) & ht.bucket_mask;
        unsigned long long *line = reinterpret_cast<unsigned long long *>(ht.entries + (size_t)b * BUCKET_ENTRIES);
        // one look at the whole bucket, then claim empty entries in order until one claim holds
        const uint4 *line4 = reinterpret_cast<const uint4 *>(line);
        uint4 v[BUCKET_ENTRIES / 2];
#pragma unroll
        for (int q = 0; q < BUCKET_ENTRIES / 2; ++q) v[q] = line4[q];
        uint32_t empties = 0;
#pragma unroll
        for (int q = 0; q < BUCKET_ENTRIES / 2; ++q) {
            if ((v[q].x & v[q].y) == 0xFFFFFFFFu) empties |= 1u << (2 * q);
            if ((v[q].z & v[q].w) == 0xFFFFFFFFu) empties |= 1u << (2 * q + 1);
        }
        while (empties) {
            const int q = __ffs(empties) - 1;
            empties &= empties - 1;
            if (atomicCAS(&line[q], (unsigned long long)ENTRY_EMPTY, (unsigned long long)e) == ENTRY_EMPTY) {
                if (d) atomicMax(&ht.reach[h], d);
                return true;
            }
        }
    }
    return false;
}

__device__ __forceinline__ void ht_erase(const HashTable &ht, uint32_t key)
{
    uint32_t idx;
    if (ht_find(ht, key, &idx) != SLOT_NONE) ht.entries[idx] = ENTRY_EMPTY;
}

} // namespace het
