// Shared device-side definitions of the embedding-cache kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace het {

constexpr int WAVE = 64;
constexpr uint32_t KEY_NONE = 0xFFFFFFFFu;   // free slot / no key
constexpr int32_t SLOT_NONE = -1;

constexpr uint32_t ERRBIT_RANGE = 1u;        // an id outside [0, vocab)
constexpr uint32_t ERRBIT_STATE = 2u;        // update of a key that is not cached
constexpr uint32_t ERRBIT_INTERNAL = 4u;     // hash table could not place a key (never expected)

constexpr int CLS_HIT = 0, CLS_STALE = 1, CLS_MISS = 2;

// Counters of one call, mirrored by het_counters in the public header.
struct Counters {
    unsigned long long n, unique, hit, stale, miss, evicted, evicted_dirty, stale_dirty, flushed;
};

// Small block of device-resident scalars that the kernels of one call hand to each other, so
// that no count has to travel to the host between kernels.
struct DState {
    uint32_t t;          // iteration = number of non-empty lookups; the LRU time stamp
    int32_t size;        // cached rows
    uint32_t n_unique;   // distinct valid ids of the current call
    uint32_t n_valid;    // ids of the current call that lie in [0, vocab)
    uint32_t err;        // sticky ERRBIT_*
    uint32_t ev_n[2];    // ids recorded by a trim; trims alternate, the lookup in between clears the idle count
    uint32_t sel_take;   // trim: how many of the rows whose policy key equals sel_tau are evicted (in slot order)
    unsigned long long sel_tau;   // trim: policy key of the last row to evict
    int32_t over;        // trim: rows above capacity when the select ran (what the eviction removes)
    int32_t pad1;
    uint32_t push_n[2];  // host-backed table: rows a trim staged for write-back; trims alternate like ev_n
    uint32_t pf_n[2];    // host-backed table: keys of a coming batch listed for fetching ahead; the lists alternate
    Counters call[2];    // per-call counters: calls alternate between the two, the idle one is cleared meanwhile
    Counters total;
};

__device__ __forceinline__ uint32_t lane_id()
{
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Number of set bits of a 64-lane mask below the calling lane.
__device__ __forceinline__ uint32_t mask_rank(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        uint32_t u = __shfl_up(v, o, WAVE);
        if (lane >= (uint32_t)o) v += u;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// Exclusive scan of one value per thread over a block of NW waves; `total` gets the block sum.
// `lds` needs NW + 1 words.  Contains block barriers: call from all threads.
template <int NW>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *lds, uint32_t &total)
{
    const uint32_t lane = lane_id(), w = threadIdx.x / WAVE;
    uint32_t inc = wave_incl_scan(v);
    __syncthreads();                       // lds may still be read from a previous use
    if (lane == WAVE - 1) lds[w] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int i = 0; i < NW; ++i) { uint32_t c = lds[i]; lds[i] = run; run += c; }
        lds[NW] = run;
    }
    __syncthreads();
    total = lds[NW];
    return lds[w] + inc - v;
}

// Sum over the block of one value per thread (all threads get it).  `lds` needs NW words.
template <int NW>
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *lds)
{
    const uint32_t lane = lane_id(), w = threadIdx.x / WAVE;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) lds[w] = v;
    __syncthreads();
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) s += lds[i];
    return s;
}

// Sum of a[0 .. count) computed by the whole block (every thread gets it).  Loads go out eight
// at a time per thread before anything is added.
template <int NW>
__device__ __forceinline__ uint32_t block_sum_array(const uint32_t *a, uint32_t count, uint32_t *lds)
{
    uint32_t v = 0;
    for (uint32_t i0 = threadIdx.x; i0 < count; i0 += 8 * NW * WAVE) {
        uint32_t x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { const uint32_t i = i0 + u * NW * WAVE; x[u] = i < count ? a[i] : 0u; }
#pragma unroll
        for (int u = 0; u < 8; ++u) v += x[u];
    }
    return block_sum<NW>(v, lds);
}

// Row geometry: a row of `dim` floats is handled by a group of `lanes` consecutive lanes
// (power of two, at most 64), each moving VEC floats per step.
struct RowGeom {
    int dim;      // floats per row
    int vec;      // 4 if dim % 4 == 0, else 1
    int lanes;    // lanes per row group
    int chunks;   // dim / vec
};

template <int VEC> struct VecT;
template <> struct VecT<4> { using type = float4; };
template <> struct VecT<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void row_copy(float *dst, const float *src, int chunks, int lanes, int gl)
{
    using V = typename VecT<VEC>::type;
    const V *s = reinterpret_cast<const V *>(src);
    V *d = reinterpret_cast<V *>(dst);
    for (int c = gl; c < chunks; c += lanes) d[c] = s[c];
}

template <int VEC>
__device__ __forceinline__ void row_zero(float *dst, int chunks, int lanes, int gl)
{
    using V = typename VecT<VEC>::type;
    V *d = reinterpret_cast<V *>(dst);
    V z{};
    for (int c = gl; c < chunks; c += lanes) d[c] = z;
}

} // namespace het
