// The small kernels between the GEMMs and attention.  Each one also adds up the K-range partial
// sums of the GEMM before it (fixed order), so the projections never need a separate reduction
// pass: embedding + RMSNorm, residual add + RMSNorm, SiLU gating, rotary embedding + KV append.
#include "cache_layout.h"
#include "common.h"
#include "frag.h"
#include "splits.h"

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

// Emit 8 consecutive values of a row as the next GEMM's operand: x * gain, as fragments (bf16 path)
// and/or plain fp32 (fp32 path, where the normalisation is applied separately).
__device__ __forceinline__ void emit_operand(const XOut& xo, int m, int k8, int d, const float (&v)[8],
                                             const float* __restrict__ gain)
{
    if (xo.frags) {
        float g[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = v[e] * (gain ? gain[k8 * 8 + e] : 1.f);
        store_x_unit(static_cast<uint4*>(xo.frags), xo.mt, xo.planes, m, k8, g);
    }
    if (xo.plain) {
#pragma unroll
        for (int e = 0; e < 8; ++e) xo.plain[(size_t)m * d + k8 * 8 + e] = v[e];
    }
}

constexpr int UNIT_TPB = SSQ_CHUNK / 8;   // one thread per 8 columns of a chunk

// One workgroup per (row, SSQ_CHUNK columns): x = E[token] (or x += partial sums); ssq[m][chunk] =
// sum x^2 over the chunk; x * gain goes out as the next GEMM's operand.  d is a multiple of 8.
template <typename T, bool EMBED>
__global__ void __launch_bounds__(UNIT_TPB) resid_kernel(const T* __restrict__ E, const int32_t* __restrict__ row_tok,
                                                         const float* __restrict__ partial, int n_split,
                                                         size_t split_stride, int ld, int d, float* __restrict__ x,
                                                         float* __restrict__ ssq, const float* __restrict__ gain,
                                                         XOut xo)
{
    __shared__ double sh[2];
    const int m = blockIdx.x, chunk = blockIdx.y;
    const int k8 = chunk * UNIT_TPB + threadIdx.x;
    double ss = 0.0;
    if (k8 * 8 < d) {
        float v[8];
        float* xp = x + (size_t)m * d + k8 * 8;
        if constexpr (EMBED) {
            const T* e = E + (size_t)row_tok[m] * d + k8 * 8;
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = static_cast<float>(e[i]);
        } else {
            const float4 a = *reinterpret_cast<const float4*>(xp), b = *reinterpret_cast<const float4*>(xp + 4);
            const float* pp = partial + (size_t)m * ld + k8 * 8;
            const float* cols[2] = {pp, pp + 4};
            float4 sums[2];
            sum_splits4_many<2, 8>(cols, n_split, split_stride, sums);   // up to 8 ranges in one round trip
            const float4 pa = sums[0], pb = sums[1];
            v[0] = a.x + pa.x; v[1] = a.y + pa.y; v[2] = a.z + pa.z; v[3] = a.w + pa.w;
            v[4] = b.x + pb.x; v[5] = b.y + pb.y; v[6] = b.z + pb.z; v[7] = b.w + pb.w;
        }
        *reinterpret_cast<float4*>(xp) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(xp + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += (double)v[i] * v[i];
        emit_operand(xo, m, k8, d, v, gain);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) ssq[(size_t)m * gridDim.y + chunk] = (float)(sh[0] + sh[1]);
}

// h = x / sqrt(mean(x^2) + eps) * gain from the partial sums of squares
__global__ void __launch_bounds__(TPB) rmsnorm_apply_kernel(const float* __restrict__ x, const float* __restrict__ ssq,
                                                            int n_ssq, const float* __restrict__ gain, float eps, int d,
                                                            float* __restrict__ h)
{
    const int m = blockIdx.x;
    float ss = 0.f;
    for (int i = 0; i < n_ssq; ++i) ss += ssq[(size_t)m * n_ssq + i];
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += TPB) h[(size_t)m * d + i] = x[(size_t)m * d + i] * inv * gain[i];
}

// act[m][f] = silu(gate) * up for 8 consecutive f per thread, gate and up first scaled by the row's
// 1/rms (the FFN norm's scale, see NormScale).  Interleaved: the GEMM's columns come in 16-wide
// tiles alternating gate and up (see spec_pack_weight); otherwise gate columns [0,F) then up
// columns [F,2F).  The result goes out as the down projection's operand.  F is a multiple of 8.
__global__ void __launch_bounds__(TPB) silu_mul_kernel(const float* __restrict__ partial, int n_split, size_t split_stride,
                                                       int ld, int M, int F, int interleaved, NormScale ns, XOut xo)
{
    const int units = F / 8;
    for (int i = blockIdx.x * TPB + threadIdx.x; i < M * units; i += gridDim.x * TPB) {
        const int m = i / units, k8 = i % units, f = k8 * 8;
        const int cg = interleaved ? ((f >> 4) << 5) + (f & 15) : f;
        const int cu = interleaved ? cg + 16 : F + f;
        const float r = row_inv_rms(ns.ssq, ns.n_ssq, m, ns.d, ns.eps);
        const float* pg = partial + (size_t)m * ld + cg;
        const float* pu = partial + (size_t)m * ld + cu;
        const float* cols[4] = {pg, pg + 4, pu, pu + 4};
        float4 sums[4];
        sum_splits4_many(cols, n_split, split_stride, sums);   // one memory round trip for all four
        const float4 g0 = sums[0], g1 = sums[1], u0 = sums[2], u1 = sums[3];
        const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float ge = g[e] * r;
            v[e] = ge / (1.f + expf(-ge)) * (u[e] * r);
        }
        emit_operand(xo, m, k8, F, v, nullptr);
    }
}

// One 64-lane workgroup per (row, head of the q|k|v projection): sum the partial ranges, rotate
// q and k heads at the row's absolute position (pairs (i, i+hd/2), angle from the table), write q,
// and put k and v -- rounded to the cache's storage type -- into the row's slot at that position.
template <bool BF16>
__global__ void __launch_bounds__(64) rope_append_kernel(const float* __restrict__ partial, int n_split,
                                                         size_t split_stride, int ld, StepTables t, CacheGeom g,
                                                         int n_q_heads, int layer, const float* __restrict__ cos_sin,
                                                         NormScale ns, void* cache, float* __restrict__ q_out)
{
    const int m = blockIdx.x, head = blockIdx.y;
    const int pos = t.row_pos[m];
    const int rope_pos = t.tree ? t.row_rope[m] : pos;   // loaded alongside pos, not after the branch below
    const int hd = g.head_dim, half = hd >> 1;
    const int dq = n_q_heads * hd;
    const float* row = partial + (size_t)m * ld + head * hd;
    if (pos < 0) {   // row of a skipped sequence: defined output, no cache write
        if (head < n_q_heads)
            for (int i = threadIdx.x; i < hd; i += 64) q_out[(size_t)m * dq + head * hd + i] = 0.f;
        return;
    }
    const int slot = t.seq_slot[t.row_seq[m]];
    const float rs = row_inv_rms(ns.ssq, ns.n_ssq, m, ns.d, ns.eps);   // the attention norm's row scale
    if (head < n_q_heads + g.n_kv_heads) {
        const float* cs = cos_sin + (size_t)rope_pos * hd;   // [half][2]; depth in the window, not the slot
        for (int i = threadIdx.x; i < half; i += 64) {
            const float a = sum_splits(row + i, n_split, split_stride) * rs;
            const float b = sum_splits(row + i + half, n_split, split_stride) * rs;
            const float c = cs[2 * i], s = cs[2 * i + 1];
            const float ra = a * c - b * s, rb = a * s + b * c;
            if (head < n_q_heads) {
                q_out[(size_t)m * dq + head * hd + i] = ra;
                q_out[(size_t)m * dq + head * hd + i + half] = rb;
            } else {
                if constexpr (BF16) {
                    __bf16* c16 = static_cast<__bf16*>(cache);
                    const size_t blk = cache_block_base(g, layer, slot, head - n_q_heads, pos >> 5);
                    c16[blk + tiled_k_within(hd, pos & 31, i)] = static_cast<__bf16>(ra);
                    c16[blk + tiled_k_within(hd, pos & 31, i + half)] = static_cast<__bf16>(rb);
                } else {
                    const size_t base = cache_head_base(g, layer, slot, head - n_q_heads);
                    float* c32 = static_cast<float*>(cache);
                    c32[base + plain_offset(g, 0, pos, i)] = ra;
                    c32[base + plain_offset(g, 0, pos, i + half)] = rb;
                }
            }
        }
    } else {
        const int hv = head - n_q_heads - g.n_kv_heads;
        const size_t base = BF16 ? cache_block_base(g, layer, slot, hv, pos >> 5) : cache_head_base(g, layer, slot, hv);
        for (int i = threadIdx.x; i < hd; i += 64) {
            const float v = sum_splits(row + i, n_split, split_stride) * rs;
            if constexpr (BF16)
                static_cast<__bf16*>(cache)[base + tiled_v_within(hd, pos & 31, i)] = static_cast<__bf16>(v);
            else
                static_cast<float*>(cache)[base + plain_offset(g, 1, pos, i)] = v;
        }
    }
}

__global__ void __launch_bounds__(TPB) reduce_splits_kernel(const float* __restrict__ partial, int n_split,
                                                            size_t split_stride, int M, int N, int ld, NormScale ns,
                                                            float* __restrict__ out)
{
    const size_t total = (size_t)M * N;
    for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < total; i += (size_t)gridDim.x * TPB) {
        const int m = (int)(i / N), n = (int)(i % N);
        out[i] = sum_splits(partial + (size_t)m * ld + n, n_split, split_stride)
                 * row_inv_rms(ns.ssq, ns.n_ssq, m, ns.d, ns.eps);
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
        size_t off;
        if constexpr (BF16)
            off = cache_block_base(g, layer, slot, head, (pos0 + p) >> 5)
                  + (kv ? tiled_v_within(hd, (pos0 + p) & 31, dim) : tiled_k_within(hd, (pos0 + p) & 31, dim));
        else
            off = cache_head_base(g, layer, slot, head) + plain_offset(g, kv, pos0 + p, dim);
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
        g.head_stride = (size_t)64 * c.head_dim;
        g.blk_stride = (size_t)c.n_kv_heads * g.head_stride;
        g.slot_stride = (size_t)(g.t_pad / 32) * g.blk_stride;
    } else {
        g.t_pad = c.max_kv_len;
        g.head_stride = (size_t)g.t_pad * c.head_dim;
        g.slot_stride = (size_t)2 * c.n_kv_heads * g.head_stride;
    }
    g.layer_stride = (size_t)c.max_batch * g.slot_stride;
    return g;
}

int launch_embed(int dtype, const void* tok_embed, const int32_t* row_tok, int M, int d, float* x, float* ssq,
                 const float* gain, const XOut& xo, hipStream_t s)
{
    if (d % 8) return fail(SPEC_ERR_SHAPE, "d_model must be a multiple of 8");
    const dim3 grid(M, ssq_chunks(d));
    if (dtype == SPEC_DTYPE_BF16)
        hipLaunchKernelGGL((resid_kernel<__bf16, true>), grid, dim3(UNIT_TPB), 0, s, (const __bf16*)tok_embed, row_tok,
                           nullptr, 0, 0, 0, d, x, ssq, gain, xo);
    else
        hipLaunchKernelGGL((resid_kernel<float, true>), grid, dim3(UNIT_TPB), 0, s, (const float*)tok_embed, row_tok,
                           nullptr, 0, 0, 0, d, x, ssq, gain, xo);
    SPECV_LAUNCH_CHECK("resid_kernel<embed>");
    return SPEC_OK;
}

int launch_resid(const float* partial, int n_split, size_t split_stride, int ld, int M, int d, float* x, float* ssq,
                 const float* gain, const XOut& xo, hipStream_t s)
{
    if (d % 8 || ld % 4 || split_stride % 4) return fail(SPEC_ERR_SHAPE, "residual rows must be multiples of 8 wide");
    const dim3 grid(M, ssq_chunks(d));
    hipLaunchKernelGGL((resid_kernel<float, false>), grid, dim3(UNIT_TPB), 0, s, nullptr, nullptr, partial, n_split,
                       split_stride, ld, d, x, ssq, gain, xo);
    SPECV_LAUNCH_CHECK("resid_kernel");
    return SPEC_OK;
}

int launch_rmsnorm_apply(const float* x, const float* ssq, const float* gain, float eps, int M, int d, float* h,
                         hipStream_t s)
{
    hipLaunchKernelGGL(rmsnorm_apply_kernel, dim3(M), dim3(TPB), 0, s, x, ssq, ssq_chunks(d), gain, eps, d, h);
    SPECV_LAUNCH_CHECK("rmsnorm_apply_kernel");
    return SPEC_OK;
}

int launch_silu_mul(const float* partial, int n_split, size_t split_stride, int ld, int M, int F, bool interleaved,
                    const NormScale& ns, const XOut& xo, hipStream_t s)
{
    if (F % 8 || ld % 4 || split_stride % 4) return fail(SPEC_ERR_SHAPE, "d_ffn must be a multiple of 8");
    hipLaunchKernelGGL(silu_mul_kernel, dim3(blocks_for((size_t)M * F / 8)), dim3(TPB), 0, s, partial, n_split,
                       split_stride, ld, M, F, interleaved ? 1 : 0, ns, xo);
    SPECV_LAUNCH_CHECK("silu_mul_kernel");
    return SPEC_OK;
}

int launch_rope_append(const float* partial, int n_split, size_t split_stride, int ld, const StepTables& t, int M,
                       const CacheGeom& g, int n_q_heads, int layer, const float* cos_sin, const NormScale& ns,
                       void* cache, float* q_out, hipStream_t s)
{
    const dim3 grid(M, n_q_heads + 2 * g.n_kv_heads);
    if (g.dtype == SPEC_DTYPE_BF16)
        hipLaunchKernelGGL(rope_append_kernel<true>, grid, dim3(64), 0, s, partial, n_split, split_stride, ld, t, g,
                           n_q_heads, layer, cos_sin, ns, cache, q_out);
    else
        hipLaunchKernelGGL(rope_append_kernel<false>, grid, dim3(64), 0, s, partial, n_split, split_stride, ld, t, g,
                           n_q_heads, layer, cos_sin, ns, cache, q_out);
    SPECV_LAUNCH_CHECK("rope_append_kernel");
    return SPEC_OK;
}

int launch_reduce_splits(const float* partial, int n_split, size_t split_stride, int M, int N, int ld,
                         const float* ssq, int n_ssq, int d, float eps, float* out, hipStream_t s)
{
    NormScale ns{ssq, n_ssq, d, eps};
    hipLaunchKernelGGL(reduce_splits_kernel, dim3(blocks_for((size_t)M * N)), dim3(TPB), 0, s, partial, n_split,
                       split_stride, M, N, ld, ns, out);
    SPECV_LAUNCH_CHECK("reduce_splits_kernel");
    return SPEC_OK;
}

// After a tree was verified: the kept nodes' keys and values move from their window slots to the
// positions right behind the root, in path order.  Sources increase along a path and are never
// below their destination, and each thread moves the same dims in every step, so moving in place,
// one path node after the other, never overwrites an entry that is still needed.
template <bool BF16>
__global__ void __launch_bounds__(64) kv_compact_kernel(CacheGeom g, void* cache, StepTables t, int Kmax,
                                                        const int32_t* __restrict__ n_accepted,
                                                        const int32_t* __restrict__ path)
{
    const int b = blockIdx.x;
    if (!t.seq_ok[b]) return;
    const int a = n_accepted[b];
    const int n = t.seq_n[b], hd = g.head_dim;
    const int layer = blockIdx.y / g.n_kv_heads, head = blockIdx.y % g.n_kv_heads;
    const int slot = t.seq_slot[b];
    const size_t base = cache_head_base(g, layer, slot, head);   // fp32 only
    for (int k = 1; k <= a; ++k) {
        const int node = path[b * Kmax + k - 1];
        if (node < 0 || node >= Kmax) return;   // cannot happen: the walk writes a valid indices first
        const int src = n + node + 1, dst = n + k;
        if (src == dst) continue;
        for (int i = threadIdx.x; i < hd; i += 64) {
            if constexpr (BF16) {
                uint16_t* c = static_cast<uint16_t*>(cache);
                const size_t sb = cache_block_base(g, layer, slot, head, src >> 5);
                const size_t db = cache_block_base(g, layer, slot, head, dst >> 5);
                c[db + tiled_k_within(hd, dst & 31, i)] = c[sb + tiled_k_within(hd, src & 31, i)];
                c[db + tiled_v_within(hd, dst & 31, i)] = c[sb + tiled_v_within(hd, src & 31, i)];
            } else {
                float* c = static_cast<float*>(cache);
                c[base + plain_offset(g, 0, dst, i)] = c[base + plain_offset(g, 0, src, i)];
                c[base + plain_offset(g, 1, dst, i)] = c[base + plain_offset(g, 1, src, i)];
            }
        }
    }
}

int launch_kv_compact(const CacheGeom& g, void* cache, const StepTables& t, int B, int Kmax, const int32_t* n_accepted,
                      const int32_t* path, hipStream_t s)
{
    const dim3 grid(B, g.n_layers * g.n_kv_heads);
    if (g.dtype == SPEC_DTYPE_BF16)
        hipLaunchKernelGGL(kv_compact_kernel<true>, grid, dim3(64), 0, s, g, cache, t, Kmax, n_accepted, path);
    else
        hipLaunchKernelGGL(kv_compact_kernel<false>, grid, dim3(64), 0, s, g, cache, t, Kmax, n_accepted, path);
    SPECV_LAUNCH_CHECK("kv_compact_kernel");
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
