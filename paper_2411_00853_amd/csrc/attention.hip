// Windowed-causal attention of the verify step: the K+1 query tokens of a sequence (times the
// query heads that share a kv head) attend over the sequence's cached positions plus the window
// tokens up to and including themselves.  All queries of a (sequence, kv head) share ONE streamed
// pass over that head's keys and values -- this is why scoring K drafts costs about as much as one
// token (the paper's observation behind speculative sampling) -- so the kernel is bound by reading
// the cache from HBM once, and is organised around that stream:
//
//  * The cache is stored in operand order (cache_layout.h): every 16-byte lane load of a key or
//    value operand is part of a contiguous 1 KiB wavefront read, and a 32-position block (keys then
//    values) is one contiguous 64*hd*2-byte run.  The next block is in flight while the current
//    one is processed (two register buffers per wavefront).
//  * Scores are computed transposed (S^T = K * Q^T) so that the exponentiated scores leave the
//    matrix instruction in exactly the register order the second product (O^T = V^T * P^T) wants:
//    no LDS round trip, no cross-lane movement except the 2-step maximum over a query's 4 lanes.
//  * Online softmax in fp32 (base 2), one running maximum and sum per query, per wavefront.
//  * The position range is cut into chunks across wavefronts to fill the machine; chunk results
//    (unnormalised output, maximum, sum) are merged by a second small kernel in a fixed order.
//  * Queries and probabilities enter the bf16 matrix instruction as head + remainder pairs; at a
//    handful of query rows the matrix cores are far from busy, and this keeps the only bf16
//    rounding in the path the one that the cache's storage type imposes.
#include "attention_kernel.h"

namespace specv {
namespace {

// out[m][hq][:] = sum_c w_c o_c / sum_c w_c l_c with w_c = 2^(m_c - max m), chunks in index order.
// One thread per 8 consecutive dims of a (row, query head); the result goes out as the output
// projection's operand fragments.
__global__ void __launch_bounds__(64) attn_merge_kernel(StepTables t, LookaheadPack ks, int n_kv_heads, int n_q_heads,
                                                        int hd, int max_chunks, int r_cap,
                                                        const float* __restrict__ part_o,
                                                        const float* __restrict__ part_ml, XOut xo)
{
    const int per_head = hd / 8;
    const int m = blockIdx.x;
    const int unit = blockIdx.y * 64 + threadIdx.x;       // 8-dim unit within the row
    const int hq = unit / per_head, d8 = unit % per_head;
    if (hq >= n_q_heads) return;
    const int b = t.row_seq[m];
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (t.seq_ok[b]) {
        const int group = n_q_heads / n_kv_heads;
        const int j = m - t.seq_row0[b];
        const int r = j * group + hq % group;
        const int total = t.seq_n[b] + ks.k[b] + 1;
        const int ck = seq_chunk_keys(total, max_chunks);
        const int n_chunks = (total + ck - 1) / ck;
        const size_t item0 = ((size_t)b * n_kv_heads + hq / group) * max_chunks;
        // Chunks are taken eight at a time, every load of a batch issued before the first use
        // (indices past the end clamped, their terms dropped), so that a batch costs one memory round
        // trip; a loop that loads, tests and then loads again per chunk pays two per chunk.  The
        // arithmetic is the plain definition: global max first, then the weighted sums in chunk order.
        constexpr int MB = 8;
        auto ml_at = [&](int c) {
            return *reinterpret_cast<const float2*>(part_ml + ((item0 + min(c, n_chunks - 1)) * r_cap + r) * 2);
        };
        float2 ml0[MB];
        float4 oa[MB], ob[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            ml0[i] = ml_at(i);
            const float* po = part_o + ((item0 + min(i, n_chunks - 1)) * r_cap + r) * hd + d8 * 8;
            oa[i] = *reinterpret_cast<const float4*>(po);
            ob[i] = *reinterpret_cast<const float4*>(po + 4);
        }
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < MB; ++i) mx = fmaxf(mx, i < n_chunks ? ml0[i].x : -INFINITY);
        for (int c0 = MB; c0 < n_chunks; c0 += MB) {
            float2 t2[MB];
#pragma unroll
            for (int i = 0; i < MB; ++i) t2[i] = ml_at(c0 + i);
#pragma unroll
            for (int i = 0; i < MB; ++i) mx = fmaxf(mx, c0 + i < n_chunks ? t2[i].x : -INFINITY);
        }
        float den = 0.f;
        auto add = [&](bool use, float2 ml, const float4& a, const float4& bq) {
            // a chunk entirely after this query's position has max -inf and takes no part
            const bool on = use && ml.x != -INFINITY;
            const float w = on ? exp2f(ml.x - mx) : 0.f;
            den += on ? w * ml.y : 0.f;
            v[0] += on ? w * a.x : 0.f; v[1] += on ? w * a.y : 0.f; v[2] += on ? w * a.z : 0.f; v[3] += on ? w * a.w : 0.f;
            v[4] += on ? w * bq.x : 0.f; v[5] += on ? w * bq.y : 0.f; v[6] += on ? w * bq.z : 0.f; v[7] += on ? w * bq.w : 0.f;
        };
#pragma unroll
        for (int i = 0; i < MB; ++i) add(i < n_chunks, ml0[i], oa[i], ob[i]);
        for (int c0 = MB; c0 < n_chunks; c0 += MB) {
            float2 t2[MB];
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                t2[i] = ml_at(c0 + i);
                const float* po = part_o + ((item0 + min(c0 + i, n_chunks - 1)) * r_cap + r) * hd + d8 * 8;
                oa[i] = *reinterpret_cast<const float4*>(po);
                ob[i] = *reinterpret_cast<const float4*>(po + 4);
            }
#pragma unroll
            for (int i = 0; i < MB; ++i) add(c0 + i < n_chunks, t2[i], oa[i], ob[i]);
        }
        const float inv = 1.0f / den;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= inv;
    }
    store_x_unit(static_cast<uint4*>(xo.frags), xo.mt, xo.planes, m, unit, v);
}

// Plain fp32 attention for fp32 caches: one workgroup per (row, query head).
__global__ void __launch_bounds__(256) attn_f32_kernel(StepTables t, CacheGeom g, int n_q_heads, int layer,
                                                       const float* __restrict__ cache, const float* __restrict__ q,
                                                       float scale, float* __restrict__ out)
{
    extern __shared__ float sh[];   // [hd] query, [n_keys] scores
    __shared__ float red[4];
    const int m = blockIdx.x, hq = blockIdx.y;
    const int hd = g.head_dim;
    const int pos = t.row_pos[m];
    float* dst = out + ((size_t)m * n_q_heads + hq) * hd;
    if (pos < 0) {
        for (int i = threadIdx.x; i < hd; i += 256) dst[i] = 0.f;
        return;
    }
    const int n_keys = pos + 1;
    const int n_cached = t.seq_n[t.row_seq[m]];
    const uint32_t wmask = t.tree ? t.row_mask[m] : 0xffffffffu;   // chains: n_keys = pos + 1 is the whole rule
    const int slot = t.seq_slot[t.row_seq[m]];
    const int hkv = hq / (n_q_heads / g.n_kv_heads);
    const float* kbase = cache + cache_head_base(g, layer, slot, hkv) + plain_offset(g, 0, 0, 0);
    const float* vbase = cache + cache_head_base(g, layer, slot, hkv) + plain_offset(g, 1, 0, 0);
    float* qs = sh;
    float* sc = sh + hd;
    for (int i = threadIdx.x; i < hd; i += 256) qs[i] = q[((size_t)m * n_q_heads + hq) * hd + i];
    __syncthreads();
    float mx = -INFINITY;
    for (int k = threadIdx.x; k < n_keys; k += 256) {
        float a = 0.f;
        for (int e = 0; e < hd; ++e) a = fmaf(qs[e], kbase[(size_t)k * hd + e], a);
        a *= scale;
        if (k >= n_cached && !((wmask >> (k - n_cached)) & 1u)) a = -INFINITY;   // window slot not on this row's path
        sc[k] = a;
        mx = fmaxf(mx, a);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float z = 0.f;
    for (int k = threadIdx.x; k < n_keys; k += 256) {
        const float p = expf(sc[k] - mx);
        sc[k] = p;
        z += p;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) z += __shfl_xor(z, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = z;
    __syncthreads();
    z = (red[0] + red[1]) + (red[2] + red[3]);
    for (int e = threadIdx.x; e < hd; e += 256) {
        float a = 0.f;
        for (int k = 0; k < n_keys; ++k) a = fmaf(sc[k], vbase[(size_t)k * hd + e], a);
        dst[e] = a / z;
    }
}

}  // namespace

static int g_items_per_cu = 0;   // wavefront work items per compute unit to aim for; 0 = default
void set_attn_items_per_cu(int n) { g_items_per_cu = n; }
static int g_max_chunks = 16;   // most chunks per (sequence, kv head)
static bool g_max_chunks_set = false;
void set_attn_max_chunks(int n)
{
    g_max_chunks_set = n >= 1 && n <= 16;
    g_max_chunks = g_max_chunks_set ? n : 16;
}
static int g_merge_min_pairs = 0;   // fewest (sequence, kv head) pairs for merging inside the workgroup; 0 = default
void set_attn_merge_min_pairs(int n) { g_merge_min_pairs = n; }
static int g_small_positions = 2816;   // cache capacity per sequence up to which the small-launch plan applies
void set_attn_small_positions(int n) { g_small_positions = n >= 0 ? n : 2816; }

AttnPlan plan_attention(int max_kv_len, int batch, int n_kv_heads, int cu_count, bool paged)
{
    // One wavefront per (sequence, kv head, position chunk).  Measured on MI355X: a few long
    // streams beat many short ones (each wavefront keeps 32 KiB in flight and HBM likes long
    // sequential runs), so aim for two wavefronts per compute unit when every sequence is at full
    // length.  Chunks are whole 32-position cache blocks.
    AttnPlan p{};
    const long want_items = (long)(g_items_per_cu > 0 ? g_items_per_cu : 2) * cu_count;
    const long per = (long)batch * n_kv_heads;
    long chunks = want_items / per;
    if (chunks < 1) chunks = 1;
    // Never a single chunk for a long cache: the wavefront whose chunk holds the window first puts the
    // window's keys and values together (4-8 us), and with two chunks per pair the other half of the
    // wavefronts stream meanwhile (plan_launch makes the one exception, where two chunks would not all
    // be resident).
    if (chunks < 2 && max_kv_len >= 1024) chunks = 2;
    if (chunks > g_max_chunks) chunks = g_max_chunks;   // (16 unless set: the merge walks a row's chunks one after the other)
    // a paged wavefront keeps the page numbers of at most 64 blocks, whatever that makes of the chunk count
    if (paged && chunks < (max_kv_len + 2047) / 2048) chunks = (max_kv_len + 2047) / 2048;
    long keys = (max_kv_len + chunks - 1) / chunks;
    keys = (keys + 31) / 32 * 32;
    p.chunk_keys = (int)keys;
    p.max_chunks = (max_kv_len + p.chunk_keys - 1) / p.chunk_keys;
    return p;
}

// A wavefront holds at most 64 query rows (four row tiles) of one kv head: (query heads per kv head) x
// (window length).  When a step's longest window gives more, the query heads of a kv head are dealt to
// kv_share work items of group / kv_share heads each -- to the kernel they look like kv heads of their
// own that happen to read the same cache head, which is then streamed kv_share times.  The smallest
// divisor of the group that brings the rows down to 64 (a window has at most 16 rows, so one exists).
static int attn_kv_share(int group, int window)
{
    for (int s = 1; s < group; ++s)
        if (group % s == 0 && (group / s) * window <= 64) return s;
    return group;
}

size_t attn_partial_floats(int max_kv_len, int max_batch, int n_kv_heads, int group, int max_window, int hd,
                           int cu_count, bool paged)
{
    size_t worst = 0;
    for (int share = 1; share <= group; ++share) {
        if (group % share) continue;
        for (int b = 1; b <= max_batch; ++b) {
            const AttnPlan p = plan_attention(max_kv_len, b, n_kv_heads * share, cu_count, paged);
            const size_t e = (size_t)b * n_kv_heads * p.max_chunks * group * max_window * hd;
            if (e > worst) worst = e;
        }
    }
    return worst;
}


// wavefronts per workgroup for a launch with max_chunks chunks per (sequence, kv head): 1, 2, 4 or 8,
// or 0 when the chunks go to memory and attn_merge_kernel merges them
// (a workgroup sits on ONE compute unit: with few (sequence, kv head) pairs and many chunks each,
// merging inside the workgroup would leave most of the chip idle -- measured slower for the draft
// model's 64 pairs x 8 chunks -- so it needs at least half as many workgroups as compute units)
// (any_pairs: a small launch, see plan_launch, merges in the workgroup however few pairs it has)
static int merge_width(int hd, int rt, int max_chunks, int n_pairs, int cu_count, bool any_pairs)
{
    const int cw = max_chunks <= 1 ? 1 : max_chunks <= 2 ? 2 : max_chunks <= 4 ? 4 : max_chunks <= 8 ? 8 : 0;
    const int need = g_merge_min_pairs > 0 ? g_merge_min_pairs : cu_count / 2;
    return cw > 0 && merge_fits(hd, rt, cw) && (any_pairs || n_pairs >= need) ? cw : 0;
}

// What a launch does with its (sequence, kv head) pairs: how many work items share a cache head
// (attn_kv_share, at least what the row limit asks for) and how the positions are cut.
// Small launches -- at most an eighth as many pairs as compute units and short caches -- are bound by
// latency, not by the stream: there a kv
// head's query heads are spread over more work items while those still fit on half the compute units
// (duplicate reads hit L2), each item is cut into at most four chunks, and the four wavefronts merge
// inside their workgroup -- one kernel where there were three (rotary/append, chunks, merge).
// Measured at the 1B-shape (8 kv heads x 4 query heads), per step: batch 1 at 1024 positions 1.017 ->
// 0.948 ms, at 2048 1.071 -> 1.012, at 2560 1.061 -> 1.045, at 3072 1.065 -> 1.077, at 4096 1.083 ->
// 1.134 (one block in flight per wavefront: chunks of a thousand positions are latency-bound);
// batch 4 at 3072 1.214 -> 1.193, batch 8 at 2304 1.320 -> 1.279, batch 12 at 2048 1.758 -> 1.696.
// The same model as the draft of a decoding round at batch 8 (one or two rows per sequence, 2300
// positions) loses 1.8 % per round with it, so the plan stops at 32 pairs (batch 4 of this shape).
// Hence a limit on the cache capacity per sequence (counted in positions of 64-dim heads: a 128-dim
// head moves twice the bytes per position).  Only with several query heads per kv head: the work items
// of one kv head then read the same blocks and most of the traffic stays in L2; with one head per kv
// head every workgroup streams from HBM through a single compute unit, and the plan loses (7B-shape,
// 32 x 128-dim kv heads, batch 1 at 1024 positions: 3.35 -> 3.44 ms, at 2048 3.47 -> 3.73, batch 3 4.04 -> 4.07).
struct AttnLaunchPlan {
    int share;
    AttnPlan p;
    bool small;
};
static AttnLaunchPlan plan_launch(const CacheGeom& g, bool paged, int n_q_heads, int kmax, int B, int max_kv_len,
                                  int cu_count)
{
    AttnLaunchPlan lp{};
    const int group = n_q_heads / g.n_kv_heads;
    lp.share = attn_kv_share(group, kmax + 1);
    lp.small = group >= 2 && B * g.n_kv_heads * 8 <= cu_count && (long)max_kv_len * g.head_dim <= 64L * g_small_positions
               && !g_max_chunks_set && g_merge_min_pairs == 0 && g_items_per_cu == 0;
    if (lp.small)
        for (int s = lp.share + 1; s <= group; ++s)
            if (group % s == 0 && B * g.n_kv_heads * s <= cu_count / 2) lp.share = s;
    lp.p = plan_attention(max_kv_len, B, g.n_kv_heads * lp.share, cu_count, paged);
    // The variant that puts queries, keys and values together itself needs, at 128-dim heads, more than
    // half a SIMD's registers (the prologue parks values in the accumulation registers): one wavefront
    // per SIMD, 4 per compute unit.  Where two chunks per pair overflow those slots and one chunk per pair
    // fits them, one chunk, all wavefronts resident at once, is faster (7B-shape, 2048 positions,
    // attention per layer: batch 20 161 -> 140 us, batch 24 176 -> 163, batch 28 and 32 -2 %; 32 sequences
    // of 512..4096 positions 8.74 -> 8.55 ms per step; from batch 40 on, where neither fits, two chunks win).
    {
        const long pairs = (long)B * g.n_kv_heads * lp.share, slots = 4L * cu_count;
        const int rt1 = ((kmax + 1) * (group / lp.share) + 15) / 16;
        if (g.head_dim == 128 && rt1 == 1 && lp.p.max_chunks == 2 && lp.p.chunk_keys >= 192 && !lp.small && !paged
            && !g_max_chunks_set && g_items_per_cu == 0 && pairs <= slots && 2 * pairs > slots) {
            lp.p.chunk_keys = (max_kv_len + 31) / 32 * 32;
            lp.p.max_chunks = 1;
        }
    }
    // (a paged wavefront holds the page numbers of at most 64 blocks: no chunk beyond 2048 positions)
    const int few = std::max(4, paged ? (max_kv_len + 2047) / 2048 : 1);
    if (lp.small && lp.p.max_chunks > few) {
        lp.p.chunk_keys = ((max_kv_len + few - 1) / few + 31) / 32 * 32;
        lp.p.max_chunks = (max_kv_len + lp.p.chunk_keys - 1) / lp.p.chunk_keys;
    }
    // Two blocks: measured over 0..128 positions, 7B-shape paged step 5.04 -> 4.95 ms, decoding round 6.69 -> 6.62 ms,
    // contiguous 7B-shape, tree and long-context steps 0.2-0.7 % shorter, nothing longer (32 and 96 positions were
    // slower than none: the main loop takes two blocks per trip).
    lp.p.lag_keys = 64;
    return lp;
}


AttnDescription describe_attention(const CacheGeom& g, bool paged, int n_q_heads, int kmax, int B, int max_kv_len,
                                   int max_window, int cu_count)
{
    AttnDescription d{};
    const AttnLaunchPlan lp = plan_launch(g, paged, n_q_heads, kmax, B, max_kv_len, cu_count);
    const int group = n_q_heads / (g.n_kv_heads * lp.share);
    d.share = lp.share;
    d.small = lp.small ? 1 : 0;
    d.max_chunks = lp.p.max_chunks;
    d.chunk_keys = lp.p.chunk_keys;
    d.row_tiles = ((kmax + 1) * group + 15) / 16;
    d.wavefronts = d.row_tiles >= 1 && d.row_tiles <= 4
                       ? merge_width(g.head_dim, d.row_tiles, lp.p.max_chunks, B * g.n_kv_heads * lp.share, cu_count, lp.small)
                       : 0;
    d.fused = fused_fits(g.head_dim, d.row_tiles) && lp.p.chunk_keys >= 192 ? 1 : 0;
    d.partial_floats = (size_t)B * g.n_kv_heads * lp.share * lp.p.max_chunks * group * max_window * g.head_dim;
    return d;
}

bool attention_takes_qkv(const CacheGeom& g, int n_q_heads, const LookaheadPack& ks, int B, int max_kv_len, int cu_count)
{
    if (g.dtype != SPEC_DTYPE_BF16) return false;
    int kmax = 0;
    for (int b = 0; b < B; ++b) kmax = ks.k[b] > kmax ? ks.k[b] : kmax;
    const AttnLaunchPlan lp = plan_launch(g, g.table != nullptr, n_q_heads, kmax, B, max_kv_len, cu_count);
    const int rt = ((kmax + 1) * (n_q_heads / g.n_kv_heads / lp.share) + 15) / 16;
    if (!fused_fits(g.head_dim, rt)) return false;
    // Every wavefront of a (sequence, kv head) puts the queries together again: with short chunks
    // (few sequences, many chunks each) that costs more than the separate kernel it replaces
    // (measured: batch 1 at 1B-shape, 128-position chunks, 2 % slower; 256-position chunks faster).
    return lp.p.chunk_keys >= 192;
}

int launch_attention(int max_kv_len, int cu_count, const StepTables& t, const LookaheadPack& ks, int B, int M, const CacheGeom& g,
                     int n_q_heads, int layer, const void* cache, const float* q, float* part_o, float* part_ml,
                     size_t part_cap, const XOut& xo, int max_window, Profiler* prof, hipStream_t s, const QkvSrc* qkv,
                     void* cache_w)
{
    QkvSrc src{};
    if (qkv) src = *qkv;
    const int hd = g.head_dim;
    const float scale = 1.0f / sqrtf((float)hd);
    if (g.dtype != SPEC_DTYPE_BF16) {
        // scores for one row live in LDS: positions * 4 bytes
        const size_t lds = (size_t)(hd + g.t_pad) * sizeof(float);
        if (lds > 60 * 1024) return fail(SPEC_ERR_SHAPE, "fp32 attention supports max_kv_len up to ~15000");
        ProfScope ps(prof, SPEC_PROF_ATTENTION, s);
        hipLaunchKernelGGL(attn_f32_kernel, dim3(M, n_q_heads), dim3(256), lds, s, t, g, n_q_heads, layer,
                           (const float*)cache, q, scale, xo.plain);
        SPECV_LAUNCH_CHECK("attn_f32_kernel");
        return SPEC_OK;
    }
    int kmax = 0;
    for (int b = 0; b < B; ++b) kmax = ks.k[b] > kmax ? ks.k[b] : kmax;
    const AttnLaunchPlan lp = plan_launch(g, g.table != nullptr, n_q_heads, kmax, B, max_kv_len, cu_count);
    const int share = lp.share;
    const int n_items_kv = g.n_kv_heads * share;          // (sequence, kv head) work items per sequence
    const AttnPlan p = lp.p;
    if (g.table && p.chunk_keys > 2048)
        return fail(SPEC_ERR_SHAPE, "paged attention handles chunks of up to 2048 positions, this plan has %d", p.chunk_keys);
    const int group = n_q_heads / n_items_kv;             // query heads of one work item
    const int r_cap = group * max_window;
    const size_t part_need = (size_t)B * n_items_kv * p.max_chunks * r_cap * hd;
    if (part_need > part_cap)
        return fail(SPEC_ERR_SHAPE, "this step's attention plan (%d chunks per sequence and kv head) needs %zu floats of "
                    "chunk results, the handle holds %zu: set the attention tuning knobs before spec_verify_init",
                    p.max_chunks, part_need, part_cap);
    const int rt = ((kmax + 1) * group + 15) / 16;
    const dim3 grid((unsigned)B * n_items_kv * p.max_chunks), wg_grid((unsigned)B * n_items_kv);
    const float sl2 = scale * 1.4426950408889634f;
    if (hd != 64 && hd != 128) return fail(SPEC_ERR_SHAPE, "bf16 attention needs head_dim 64 or 128");
    const int cw = rt >= 1 && rt <= 4 ? merge_width(hd, rt, p.max_chunks, B * n_items_kv, cu_count, lp.small) : 0;
    int rc;
    {
        ProfScope ps(prof, SPEC_PROF_ATTENTION, s);
        // several work items per cache head: its second reader should find it in the caches
        if (share > 1)
            rc = launch_chunks_reuse(hd, rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, share, layer, cache, q, p, r_cap, sl2,
                                     part_o, part_ml, src, cache_w, xo);
        else if (hd == 128)
            rc = launch_chunks<128, true>(rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, share, layer, cache, q, p, r_cap, sl2,
                                          part_o, part_ml, src, cache_w, xo);
        else
            rc = launch_chunks<64, true>(rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, share, layer, cache, q, p, r_cap, sl2,
                                         part_o, part_ml, src, cache_w, xo);
    }
    if (rc) return rc;
    if (cw > 0) return SPEC_OK;   // the workgroups merged their chunks themselves
    ProfScope ps(prof, SPEC_PROF_ATTN_MERGE, s);
    hipLaunchKernelGGL(attn_merge_kernel, dim3(M, (n_q_heads * hd / 8 + 63) / 64), dim3(64), 0, s, t, ks, n_items_kv,
                       n_q_heads, hd, p.max_chunks, r_cap, part_o, part_ml, xo);
    SPECV_LAUNCH_CHECK("attn_merge_kernel");
    return SPEC_OK;
}

}  // namespace specv
