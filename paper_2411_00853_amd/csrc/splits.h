// Adding up the K-range partial sums a GEMM leaves behind (fixed order: range 0, 1, 2, ...).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

namespace specv {

// Sum of the K ranges' partial sums at p, ranges in index order.  The loads of a batch of ranges
// are issued together (indices past the end clamped, values dropped) so the memory latency is paid
// once per batch; the batch is 2, 4 or 8 wide depending on the (uniform) number of ranges.
template <int W>
__device__ __forceinline__ float4 sum_splits4_w(const float* p, int n_split, size_t stride)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < n_split; s0 += W) {
        float4 a[W];
#pragma unroll
        for (int i = 0; i < W; ++i) a[i] = *reinterpret_cast<const float4*>(p + (size_t)min(s0 + i, n_split - 1) * stride);
#pragma unroll
        for (int i = 0; i < W; ++i) {
            const bool ok = s0 + i < n_split;
            v.x += ok ? a[i].x : 0.f; v.y += ok ? a[i].y : 0.f; v.z += ok ? a[i].z : 0.f; v.w += ok ? a[i].w : 0.f;
        }
    }
    return v;
}

__device__ __forceinline__ float4 sum_splits4(const float* p, int n_split, size_t stride)
{
    if (n_split == 1) return *reinterpret_cast<const float4*>(p);
    if (n_split <= 2) return sum_splits4_w<2>(p, n_split, stride);
    if (n_split <= 4) return sum_splits4_w<4>(p, n_split, stride);
    return sum_splits4_w<8>(p, n_split, stride);
}

template <int W>
__device__ __forceinline__ float sum_splits_w(const float* p, int n_split, size_t stride)
{
    float v = 0.f;
    for (int s0 = 0; s0 < n_split; s0 += W) {
        float a[W];
#pragma unroll
        for (int i = 0; i < W; ++i) a[i] = p[(size_t)min(s0 + i, n_split - 1) * stride];
#pragma unroll
        for (int i = 0; i < W; ++i) v += (s0 + i < n_split) ? a[i] : 0.f;
    }
    return v;
}

__device__ __forceinline__ float sum_splits(const float* p, int n_split, size_t stride)
{
    if (n_split == 1) return p[0];
    if (n_split <= 2) return sum_splits_w<2>(p, n_split, stride);
    if (n_split <= 4) return sum_splits_w<4>(p, n_split, stride);
    return sum_splits_w<8>(p, n_split, stride);
}

// Many sums at once: N float4 columns of one row, all loads of a batch of (up to) W ranges issued
// before the first addition (calling sum_splits4 N times makes N dependent round trips: the
// compiler keeps each call's loads next to its additions).  Ranges are added in index order.
template <int N, int W = 4>
__device__ __forceinline__ void sum_splits4_many(const float* const (&p)[N], int n_split, size_t stride, float4 (&out)[N])
{
#pragma unroll
    for (int x = 0; x < N; ++x) out[x] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < n_split; s0 += W) {
        float4 a[N][W];
#pragma unroll
        for (int x = 0; x < N; ++x)
#pragma unroll
            for (int i = 0; i < W; ++i)
                a[x][i] = *reinterpret_cast<const float4*>(p[x] + (size_t)min(s0 + i, n_split - 1) * stride);
#pragma unroll
        for (int x = 0; x < N; ++x)
#pragma unroll
            for (int i = 0; i < W; ++i) {
                const bool ok = s0 + i < n_split;
                out[x].x += ok ? a[x][i].x : 0.f; out[x].y += ok ? a[x][i].y : 0.f;
                out[x].z += ok ? a[x][i].z : 0.f; out[x].w += ok ? a[x][i].w : 0.f;
            }
    }
}

}  // namespace specv
