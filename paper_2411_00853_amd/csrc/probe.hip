// Small standalone kernels: a streaming copy / read of known size (the yardstick for bandwidth
// and for scaling the HBM byte counters) and a one-tile check of the matrix-instruction layout.
#include "common.h"

namespace specv {
namespace {

__global__ void __launch_bounds__(256) copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + k * 256 < n16) v[k] = src[i + k * 256];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + k * 256 < n16) dst[i + k * 256] = v[k];
    }
}

__global__ void __launch_bounds__(256) read_kernel(const float4* __restrict__ src, size_t n16, float* out)
{
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
        float4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = (i + k * 256 < n16) ? src[i + k * 256] : make_float4(0, 0, 0, 0);
#pragma unroll
        for (int k = 0; k < 4; ++k) acc += (v[k].x + v[k].y) + (v[k].z + v[k].w);
    }
    // keep the loads alive; one value per lane slot, no atomics
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// A[16][32], B[32][16] row-major bf16 -> D[16][16] fp32, one wavefront.
// Assumed layout of v_mfma_f32_16x16x32_bf16: lane l supplies A[l%16][8*(l/16)+e] and
// B[8*(l/16)+e][l%16], e = 0..7, and receives D[4*(l/16)+i][l%16], i = 0..3.
__global__ void __launch_bounds__(64) mfma_tile_kernel(const __bf16* __restrict__ a, const __bf16* __restrict__ b,
                                                       float* __restrict__ d)
{
    const int l = threadIdx.x, r = l & 15, g = l >> 4;
    bf16x8 av, bv;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        av[e] = a[r * 32 + 8 * g + e];
        bv[e] = b[(8 * g + e) * 16 + r];
    }
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) d[(4 * g + i) * 16 + r] = acc[i];
}

}  // namespace
}  // namespace specv

using namespace specv;

extern "C" int spec_k_copy(const void* src, void* dst, size_t n_bytes, void* stream)
{
    if (!src || !dst || n_bytes == 0 || (n_bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
        return fail(SPEC_ERR_INVALID_ARG, "spec_k_copy: pointers and size must be non-null multiples of 16");
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + 1023) / 1024;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                       (uint4*)dst, n16);
    SPECV_LAUNCH_CHECK("copy_kernel");
    return SPEC_OK;
}

extern "C" int spec_k_read(const void* src, size_t n_bytes, float* out, void* stream)
{
    if (!src || !out || n_bytes == 0 || (n_bytes & 15) || ((uintptr_t)src & 15))
        return fail(SPEC_ERR_INVALID_ARG, "spec_k_read: pointer and size must be non-null multiples of 16");
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + 1023) / 1024;
    if (blocks > 256 * 16) blocks = 256 * 16;   // out must hold 256*16*256 floats
    hipLaunchKernelGGL(read_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const float4*)src,
                       n16, out);
    SPECV_LAUNCH_CHECK("read_kernel");
    return SPEC_OK;
}

extern "C" int spec_k_mfma_tile(const void* a_bf16, const void* b_bf16, float* d, void* stream)
{
    if (!a_bf16 || !b_bf16 || !d) return fail(SPEC_ERR_INVALID_ARG, "spec_k_mfma_tile: null pointer");
    hipLaunchKernelGGL(mfma_tile_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (const __bf16*)a_bf16,
                       (const __bf16*)b_bf16, d);
    SPECV_LAUNCH_CHECK("mfma_tile_kernel");
    return SPEC_OK;
}
