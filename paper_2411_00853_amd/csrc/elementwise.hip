// The small kernels between the GEMMs and attention.  Each one also adds up the K-range partial
// sums of the GEMM before it (fixed order), so the projections never need a separate reduction
// pass: embedding + RMSNorm, residual add + RMSNorm, SiLU gating, rotary embedding + KV append.
#include "cache_layout.h"
#include "common.h"

namespace specv {
namespace {

constexpr int TPB = 256;

__device__ __forceinline__ double block_sum(double v, double* sh)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const double r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ float sum_splits(const float* p, int n_split, size_t stride)
{
    float v = p[0];
    for (int s = 1; s < n_split; ++s) v += p[(size_t)s * stride];
    return v;
}

// x[m] = E[token_m];  h[m] = x / sqrt(mean(x^2) + eps) * gain
template <typename T>
__global__ void __launch_bounds__(TPB) embed_rmsnorm_kernel(const T* __restrict__ E, const int32_t* __restrict__ row_tok,
                                                            const float* __restrict__ gain, float eps, int d,
                                                            float* __restrict__ x, float* __restrict__ h)
{
    __shared__ double sh[4];
    const int m = blockIdx.x;
    const T* e = E + (size_t)row_tok[m] * d;
    double ss = 0.0;
    for (int i = threadIdx.x; i < d; i += TPB) {
        const float v = static_cast<float>(e[i]);
        x[(size_t)m * d + i] = v;
        ss += (double)v * v;
    }
    ss = block_sum(ss, sh);
    const float inv = (float)(1.0 / sqrt(ss / d + (double)eps));
    for (int i = threadIdx.x; i < d; i += TPB) h[(size_t)m * d + i] = x[(size_t)m * d + i] * inv * gain[i];
}

// x[m] += sum of partial ranges;  h[m] = rmsnorm(x[m]) * gain
__global__ void __launch_bounds__(TPB) resid_rmsnorm_kernel(const float* __restrict__ partial, int n_split,
                                                            size_t split_stride, int ld, const float* __restrict__ gain,
                                                            float eps, int d, float* __restrict__ x,
                                                            float* __restrict__ h)
{
    __shared__ double sh[4];
    const int m = blockIdx.x;
    double ss = 0.0;
    for (int i = threadIdx.x; i < d; i += TPB) {
        const float v = x[(size_t)m * d + i] + sum_splits(partial + (size_t)m * ld + i, n_split, split_stride);
        x[(size_t)m * d + i] = v;
        ss += (double)v * v;
    }
    ss = block_sum(ss, sh);
    const float inv = (float)(1.0 / sqrt(ss / d + (double)eps));
    for (int i = threadIdx.x; i < d; i += TPB) h[(size_t)m * d + i] = x[(size_t)m * d + i] * inv * gain[i];
}

// act[m][f] = silu(gate) * up.  Interleaved: the GEMM's columns come in 16-wide tiles alternating
// gate and up (see spec_pack_weight); otherwise gate columns [0,F) then up columns [F,2F).
__global__ void __launch_bounds__(TPB) silu_mul_kernel(const float* __restrict__ partial, int n_split, size_t split_stride,
                                                       int ld, int M, int F, int interleaved, float* __restrict__ act)
{
    const size_t total = (size_t)M * F;
    for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < total; i += (size_t)gridDim.x * TPB) {
        const int m = (int)(i / F), f = (int)(i % F);
        const int cg = interleaved ? ((f >> 4) << 5) + (f & 15) : f;
        const int cu = interleaved ? cg + 16 : F + f;
        const float g = sum_splits(partial + (size_t)m * ld + cg, n_split, split_stride);
        const float u = sum_splits(partial + (size_t)m * ld + cu, n_split, split_stride);
        act[i] = g / (1.f + expf(-g)) * u;
    }
}

// One workgroup per row: sum the q|k|v partial ranges, rotate q and k at the row's absolute
// position (pairs (i, i+hd/2), angle from the table), write q, and put k and v -- rounded to the
// cache's storage type -- into the row's slot at that position.
template <bool BF16>
__global__ void __launch_bounds__(TPB) rope_append_kernel(const float* __restrict__ partial, int n_split,
                                                          size_t split_stride, int ld, StepTables t, CacheGeom g,
                                                          int n_q_heads, int layer, const float* __restrict__ cos_sin,
                                                          void* cache, float* __restrict__ q_out)
{
    const int m = blockIdx.x;
    const int pos = t.row_pos[m];
    const int hd = g.head_dim, half = hd >> 1;
    const int dq = n_q_heads * hd, dkv = g.n_kv_heads * hd;
    const float* row = partial + (size_t)m * ld;
    if (pos < 0) {   // row of a skipped sequence: defined output, no cache write
        for (int i = threadIdx.x; i < dq; i += TPB) q_out[(size_t)m * dq + i] = 0.f;
        return;
    }
    const int slot = t.seq_slot[t.row_seq[m]];
    const float* cs = cos_sin + (size_t)pos * hd;   // [half][2]
    // rotation pairs of q and k
    const int n_pairs = (n_q_heads + g.n_kv_heads) * half;
    for (int p = threadIdx.x; p < n_pairs; p += TPB) {
        const int head = p / half, i = p % half;
        const int col = head * hd + i;   // q heads then k heads are contiguous in the GEMM output
        const float a = sum_splits(row + col, n_split, split_stride);
        const float b = sum_splits(row + col + half, n_split, split_stride);
        const float c = cs[2 * i], s = cs[2 * i + 1];
        const float ra = a * c - b * s, rb = a * s + b * c;
        if (head < n_q_heads) {
            q_out[(size_t)m * dq + col] = ra;
            q_out[(size_t)m * dq + col + half] = rb;
        } else {
            const int kh = head - n_q_heads;
            const size_t base = cache_head_base(g, layer, slot, kh);
            if constexpr (BF16) {
                __bf16* c16 = static_cast<__bf16*>(cache);
                c16[base + tiled_k_offset(hd, pos, i)] = static_cast<__bf16>(ra);
                c16[base + tiled_k_offset(hd, pos, i + half)] = static_cast<__bf16>(rb);
            } else {
                float* c32 = static_cast<float*>(cache);
                c32[base + plain_offset(g, 0, pos, i)] = ra;
                c32[base + plain_offset(g, 0, pos, i + half)] = rb;
            }
        }
    }
    for (int e = threadIdx.x; e < dkv; e += TPB) {
        const int kh = e / hd, i = e % hd;
        const float v = sum_splits(row + dq + dkv + e, n_split, split_stride);
        const size_t base = cache_head_base(g, layer, slot, kh);
        if constexpr (BF16)
            static_cast<__bf16*>(cache)[base + tiled_v_offset(hd, pos, i)] = static_cast<__bf16>(v);
        else
            static_cast<float*>(cache)[base + plain_offset(g, 1, pos, i)] = v;
    }
}

__global__ void __launch_bounds__(TPB) reduce_splits_kernel(const float* __restrict__ partial, int n_split,
                                                            size_t split_stride, int M, int N, int ld,
                                                            float* __restrict__ out)
{
    const size_t total = (size_t)M * N;
    for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < total; i += (size_t)gridDim.x * TPB) {
        const int m = (int)(i / N), n = (int)(i % N);
        out[i] = sum_splits(partial + (size_t)m * ld + n, n_split, split_stride);
    }
}

// plain tensor [layer][k|v][head][n_pos][hd]  <->  cache positions [pos0, pos0+n_pos) of one slot
template <bool BF16, bool TO_CACHE>
__global__ void __launch_bounds__(TPB) kv_copy_kernel(CacheGeom g, void* cache, int slot, int pos0, int n_pos, void* plain)
{
    const int hd = g.head_dim;
    const size_t total = (size_t)g.n_layers * 2 * g.n_kv_heads * n_pos * hd;
    for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < total; i += (size_t)gridDim.x * TPB) {
        size_t r = i;
        const int dim = (int)(r % hd); r /= hd;
        const int p = (int)(r % n_pos); r /= n_pos;
        const int head = (int)(r % g.n_kv_heads); r /= g.n_kv_heads;
        const int kv = (int)(r % 2);
        const int layer = (int)(r / 2);
        const size_t base = cache_head_base(g, layer, slot, head);
        size_t off;
        if constexpr (BF16)
            off = base + (kv ? tiled_v_offset(hd, pos0 + p, dim) : tiled_k_offset(hd, pos0 + p, dim));
        else
            off = base + plain_offset(g, kv, pos0 + p, dim);
        if constexpr (BF16) {
            uint16_t* c = static_cast<uint16_t*>(cache);
            uint16_t* q = static_cast<uint16_t*>(plain);
            if (TO_CACHE) c[off] = q[i]; else q[i] = c[off];
        } else {
            float* c = static_cast<float*>(cache);
            float* q = static_cast<float*>(plain);
            if (TO_CACHE) c[off] = q[i]; else q[i] = c[off];
        }
    }
}

unsigned blocks_for(size_t total)
{
    size_t b = (total + TPB - 1) / TPB;
    return (unsigned)(b > 8192 ? 8192 : (b ? b : 1));
}

}  // namespace

CacheGeom make_cache_geom(const spec_model_cfg& c)
{
    CacheGeom g{};
    g.dtype = c.dtype;
    g.n_layers = c.n_layers;
    g.n_slots = c.max_batch;
    g.n_kv_heads = c.n_kv_heads;
    g.head_dim = c.head_dim;
    if (c.dtype == SPEC_DTYPE_BF16) {
        g.t_pad = (c.max_kv_len + 31) / 32 * 32;
        g.head_stride = (size_t)2 * g.t_pad * c.head_dim;
        g.slot_stride = (size_t)c.n_kv_heads * g.head_stride;
    } else {
        g.t_pad = c.max_kv_len;
        g.head_stride = (size_t)g.t_pad * c.head_dim;
        g.slot_stride = (size_t)2 * c.n_kv_heads * g.head_stride;
    }
    g.layer_stride = (size_t)c.max_batch * g.slot_stride;
    return g;
}

int launch_embed_rmsnorm(int dtype, const void* tok_embed, const int32_t* row_tok, const float* gain, float eps, int M,
                         int d, float* x, float* h, hipStream_t s)
{
    if (dtype == SPEC_DTYPE_BF16)
        hipLaunchKernelGGL(embed_rmsnorm_kernel<__bf16>, dim3(M), dim3(TPB), 0, s, (const __bf16*)tok_embed, row_tok, gain,
                           eps, d, x, h);
    else
        hipLaunchKernelGGL(embed_rmsnorm_kernel<float>, dim3(M), dim3(TPB), 0, s, (const float*)tok_embed, row_tok, gain,
                           eps, d, x, h);
    SPECV_LAUNCH_CHECK("embed_rmsnorm_kernel");
    return SPEC_OK;
}

int launch_resid_rmsnorm(const float* partial, int n_split, size_t split_stride, int ld, const float* gain, float eps,
                         int M, int d, float* x, float* h, hipStream_t s)
{
    hipLaunchKernelGGL(resid_rmsnorm_kernel, dim3(M), dim3(TPB), 0, s, partial, n_split, split_stride, ld, gain, eps, d,
                       x, h);
    SPECV_LAUNCH_CHECK("resid_rmsnorm_kernel");
    return SPEC_OK;
}

int launch_silu_mul(const float* partial, int n_split, size_t split_stride, int ld, int M, int F, bool interleaved,
                    float* act, hipStream_t s)
{
    hipLaunchKernelGGL(silu_mul_kernel, dim3(blocks_for((size_t)M * F)), dim3(TPB), 0, s, partial, n_split,
                       split_stride, ld, M, F, interleaved ? 1 : 0, act);
    SPECV_LAUNCH_CHECK("silu_mul_kernel");
    return SPEC_OK;
}

int launch_rope_append(const float* partial, int n_split, size_t split_stride, int ld, const StepTables& t, int M,
                       const CacheGeom& g, int n_q_heads, int layer, const float* cos_sin, void* cache, float* q_out,
                       hipStream_t s)
{
    if (g.dtype == SPEC_DTYPE_BF16)
        hipLaunchKernelGGL(rope_append_kernel<true>, dim3(M), dim3(TPB), 0, s, partial, n_split, split_stride, ld, t, g,
                           n_q_heads, layer, cos_sin, cache, q_out);
    else
        hipLaunchKernelGGL(rope_append_kernel<false>, dim3(M), dim3(TPB), 0, s, partial, n_split, split_stride, ld, t, g,
                           n_q_heads, layer, cos_sin, cache, q_out);
    SPECV_LAUNCH_CHECK("rope_append_kernel");
    return SPEC_OK;
}

int launch_reduce_splits(const float* partial, int n_split, size_t split_stride, int M, int N, int ld, float* out,
                         hipStream_t s)
{
    hipLaunchKernelGGL(reduce_splits_kernel, dim3(blocks_for((size_t)M * N)), dim3(TPB), 0, s, partial, n_split,
                       split_stride, M, N, ld, out);
    SPECV_LAUNCH_CHECK("reduce_splits_kernel");
    return SPEC_OK;
}

int launch_kv_copy(const CacheGeom& g, void* cache, int slot, int pos0, int n_pos, void* plain, bool to_cache,
                   hipStream_t s)
{
    const size_t total = (size_t)g.n_layers * 2 * g.n_kv_heads * n_pos * g.head_dim;
    const dim3 grid(blocks_for(total));
    if (g.dtype == SPEC_DTYPE_BF16) {
        if (to_cache) hipLaunchKernelGGL((kv_copy_kernel<true, true>), grid, dim3(TPB), 0, s, g, cache, slot, pos0, n_pos, plain);
        else hipLaunchKernelGGL((kv_copy_kernel<true, false>), grid, dim3(TPB), 0, s, g, cache, slot, pos0, n_pos, plain);
    } else {
        if (to_cache) hipLaunchKernelGGL((kv_copy_kernel<false, true>), grid, dim3(TPB), 0, s, g, cache, slot, pos0, n_pos, plain);
        else hipLaunchKernelGGL((kv_copy_kernel<false, false>), grid, dim3(TPB), 0, s, g, cache, slot, pos0, n_pos, plain);
    }
    SPECV_LAUNCH_CHECK("kv_copy_kernel");
    return SPEC_OK;
}

}  // namespace specv
