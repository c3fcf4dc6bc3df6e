// Reference points for the roofline: kernels that have the memory access pattern of the path's
// two heavy steps and nothing else (no index, no clocks, no sums), so that a measured kernel can
// be set against what the machine delivers for that pattern at that size, not only against the
// streaming peak.  Used by het_profile_rows; not part of the path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace het {

constexpr int PAT_ROWS = 8;          // rows a row group of the gather has on their way at a time
constexpr int PAT_UPDATE_ROWS = 2;   // rows of x (and a, and their gradients) a row group of the update has on their way at a time

// dst[i] = src[idx[i]] for n rows of `dim` floats (dim a multiple of 4): the gather's pattern
// (idx == nullptr: dst[i] = src[i], a streaming copy of the same size).
__global__ __launch_bounds__(256) void pattern_gather_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                             const uint32_t *__restrict__ idx, uint32_t n, int dim)
{
    const int chunks = dim / 4, lanes = chunks < 64 ? chunks : 64;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / lanes, ngroups = gridDim.x * 256u / lanes;
    const int gl = threadIdx.x % lanes;
    if (threadIdx.x / lanes >= 256u / lanes) return;
    for (uint32_t i0 = gid * PAT_ROWS; i0 < n; i0 += ngroups * PAT_ROWS) {
        uint32_t from[PAT_ROWS];
#pragma unroll
        for (int r = 0; r < PAT_ROWS; ++r) { const uint32_t i = i0 + r < n ? i0 + r : n - 1; from[r] = idx ? idx[i] : i; }
        for (int c = gl; c < chunks; c += lanes) {
            float4 v[PAT_ROWS];
#pragma unroll
            for (int r = 0; r < PAT_ROWS; ++r) v[r] = reinterpret_cast<const float4 *>(src + (size_t)from[r] * dim)[c];
#pragma unroll
            for (int r = 0; r < PAT_ROWS; ++r)
                if (i0 + r < n) reinterpret_cast<float4 *>(dst + (size_t)(i0 + r) * dim)[c] = v[r];
        }
    }
}

// x[idx[i]] and a[idx[i]] read, changed and written back, for n distinct rows: the pattern of
// the optimizer step on cached rows (a == nullptr: one array).  With PER > 0 every row also reads
// PER rows of g, numbers gidx[i * PER ...]: the gradients of the key's lookups, which lie
// anywhere in the batch.
template <int PER>
__global__ __launch_bounds__(256) void pattern_update_kernel(float *__restrict__ x, float *__restrict__ a,
                                                             const uint32_t *__restrict__ idx, uint32_t n, int dim,
                                                             const float *__restrict__ g, const uint32_t *__restrict__ gidx)
{
    const int chunks = dim / 4, lanes = chunks < 64 ? chunks : 64;
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) / lanes, ngroups = gridDim.x * 256u / lanes;
    const int gl = threadIdx.x % lanes;
    if (threadIdx.x / lanes >= 256u / lanes) return;
    constexpr int R = PAT_UPDATE_ROWS;
    for (uint32_t i0 = gid * R; i0 < n; i0 += ngroups * R) {
        uint32_t at[R], gat[R][PER > 0 ? PER : 1];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t i = i0 + r < n ? i0 + r : n - 1;
            at[r] = idx[i];
#pragma unroll
            for (int k = 0; k < PER; ++k) gat[r][k] = gidx[(size_t)i * PER + k];
        }
        for (int c = gl; c < chunks; c += lanes) {
            float4 xv[R], av[R], gv[R][PER > 0 ? PER : 1];
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int k = 0; k < PER; ++k) gv[r][k] = reinterpret_cast<const float4 *>(g + (size_t)gat[r][k] * dim)[c];
                xv[r] = reinterpret_cast<const float4 *>(x + (size_t)at[r] * dim)[c];
                av[r] = a ? reinterpret_cast<const float4 *>(a + (size_t)at[r] * dim)[c] : float4{};
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (i0 + r >= n) continue;
                float4 d{1.f, 1.f, 1.f, 1.f};
#pragma unroll
                for (int k = 0; k < PER; ++k) { d.x += gv[r][k].x; d.y += gv[r][k].y; d.z += gv[r][k].z; d.w += gv[r][k].w; }
                av[r].x += d.x; av[r].y += d.y; av[r].z += d.z; av[r].w += d.w;
                xv[r].x -= av[r].x; xv[r].y -= av[r].y; xv[r].z -= av[r].z; xv[r].w -= av[r].w;
                reinterpret_cast<float4 *>(x + (size_t)at[r] * dim)[c] = xv[r];
                if (a) reinterpret_cast<float4 *>(a + (size_t)at[r] * dim)[c] = av[r];
            }
        }
    }
}

} // namespace het
