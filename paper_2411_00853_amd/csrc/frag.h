// Activation operand fragments.  The kernels that produce a GEMM's input (embedding, residual
// add, attention merge, SiLU gating) write it straight in the order the matrix instruction wants,
// as bf16 head (+ bf16 remainder) planes, so the GEMM stages its X operand with plain 16-byte
// copies: no conversion, no transposition, no bank conflicts.
//
// Layout of an X fragment buffer for M rows (MT = row tiles of the GEMM variant) and K columns:
//   uint4 index ((kb * planes + plane) * MT + mt) * 64 + lane,  kb = k / 32
//   lane = 16 * g + r holds X[16 * mt + r][32 * kb + 8 * g .. + 7]  (8 bf16 = 16 bytes)
// i.e. one 32-column block of all rows and planes is one contiguous run of planes * MT KiB.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union Frag {
    uint4 u;
    bf16x8 v;
    uint16_t h[8];
};

// 8 fp32 values -> bf16 head (round to nearest even) and bf16 remainder of what the head lost
__device__ __forceinline__ void split8(const float (&x)[8], uint4& hi, uint4& lo)
{
    Frag h, l;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 hb = static_cast<__bf16>(x[e]);
        h.v[e] = hb;
        l.v[e] = static_cast<__bf16>(x[e] - static_cast<float>(hb));
    }
    hi = h.u;
    lo = l.u;
}

// write the 8 values X[m][8*k8 .. 8*k8+7] into a fragment buffer
__device__ __forceinline__ void store_x_unit(uint4* xf, int mt_count, int planes, int m, int k8, const float (&x)[8])
{
    uint4 hi, lo;
    split8(x, hi, lo);
    const int kb = k8 >> 2, lane = (k8 & 3) * 16 + (m & 15);
    const size_t base = ((size_t)kb * planes * mt_count + (m >> 4)) * 64 + lane;
    xf[base] = hi;
    if (planes == 2) xf[base + (size_t)mt_count * 64] = lo;
}

// A buffer holds K/32 blocks plus XFRAG_PAD_KB blocks that stay zero (the GEMM's last chunk of a
// K range may overhang the end).
constexpr int XFRAG_PAD_KB = 4;
__host__ __device__ inline size_t xfrag_uint4s(int mt_count, int planes, int K)
{
    return (size_t)(K / 32 + XFRAG_PAD_KB) * planes * mt_count * 64;
}

// 1 / rms of a row from its partial sums of squares (eps inside the root); ssq == NULL -> 1
// The partial sums are fetched eight at a time with clamped indices (surplus values dropped), so that
// all loads of a batch are in flight together: a plain loop over a run-time count waits for every
// load in turn, and this sits on the critical path of kernels that are nothing but latency.
__device__ __forceinline__ float row_inv_rms(const float* ssq, int n_ssq, int m, int d, float eps)
{
    if (!ssq) return 1.f;
    float ss = 0.f;
    const float* p = ssq + (size_t)m * n_ssq;
    for (int i0 = 0; i0 < n_ssq; i0 += 8) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = p[min(i0 + i, n_ssq - 1)];
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += (i0 + i < n_ssq) ? v[i] : 0.f;
    }
    return 1.0f / sqrtf(ss / (float)d + eps);
}

}  // namespace specv
