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
#include "cache_layout.h"
#include "common.h"
#include "frag.h"
#include "splits.h"

namespace specv {
namespace {

__device__ __forceinline__ void split_frag(const float (&x)[8], Frag& hi, Frag& lo)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 hb = static_cast<__bf16>(x[e]);
        hi.v[e] = hb;
        lo.v[e] = static_cast<__bf16>(x[e] - static_cast<float>(hb));
    }
}

// A sequence's positions are cut into max_chunks equal runs of whole 32-position blocks (at least
// 128 positions each), from its own current length: the launch is sized for the longest sequence
// the cache can hold, but a shorter one still spreads over all of its wavefronts.
__device__ __forceinline__ int seq_chunk_keys(int total, int max_chunks)
{
    const int per = (total + max_chunks - 1) / max_chunks;
    return max((per + 31) & ~31, 128);
}

// PAGED: the blocks of a slot are looked up in the page table.  A wavefront keeps the page numbers
// of its chunk's (at most 64) blocks one per lane and broadcasts the one it needs, so the address
// of a prefetch never waits for memory.
// FUSED: the kernel takes the QKV projection's partial sums instead of finished queries: every
// wavefront adds up, scales and rotates the queries it needs, and the wavefront whose chunk holds
// window positions does the same for the window's keys and values of its kv head, stores them in
// the cache (for later steps) and only then starts to stream -- so no separate rotary/append kernel
// runs between the projection and the attention.
// CW > 0: one workgroup of CW wavefronts per (sequence, kv head), wavefront c taking chunk c; the
// chunk results meet in LDS and the workgroup itself writes the merged, normalised output as the
// output projection's operand fragments (same arithmetic and order as attn_merge_kernel): no second
// kernel, no round trip of the chunk results through memory.  CW == 0: one wavefront per workgroup,
// chunk results to part_o / part_ml for attn_merge_kernel (more chunks than a workgroup can hold).
template <int HD, int RT, bool PAGED, bool FUSED, int CW>
__global__ void __launch_bounds__(CW > 0 ? 64 * CW : 64)
    attn_chunk_kernel(StepTables t, LookaheadPack ks, CacheGeom g, int n_q_heads, int kv_share, int layer,
                      const uint4* cache, const float* __restrict__ q, int max_chunks, int r_cap, float scale_log2e,
                      float* __restrict__ part_o, float* __restrict__ part_ml, QkvSrc src, uint16_t* cache_w, XOut xo)
{
    constexpr int STEPS = HD / 32;     // 32-dim steps of the score product
    constexpr int DT = HD / 16;        // 16-dim tiles of the output
    const int lane = threadIdx.x & 63, c16 = lane & 15, gq = lane >> 4;
    const int item = CW > 0 ? blockIdx.x * max_chunks + (threadIdx.x >> 6) : blockIdx.x;   // ((b, hkv), chunk)
    const int chunk = CW > 0 ? (int)(threadIdx.x >> 6) : item % max_chunks;
    // kv_share > 1: the query heads of one kv head are dealt to kv_share work items ("hkv" counts those,
    // "group" is the heads of one item), which all stream the keys and values of cache head hkc
    const int n_items_kv = g.n_kv_heads * kv_share;
    const int hkv = (CW > 0 ? blockIdx.x : item / max_chunks) % n_items_kv;
    const int b = (CW > 0 ? blockIdx.x : item / max_chunks) / n_items_kv;
    const int hkc = hkv / kv_share;
    const int K = ks.k[b];
    const int group = n_q_heads / n_items_kv;
    const int rows = (K + 1) * group;
    const int row0 = t.seq_row0[b];
    if (!t.seq_ok[b]) {
        if constexpr (CW > 0) {   // rows of a skipped sequence: zero operand rows, as the merge kernel writes them
            const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int u = threadIdx.x; u < rows * (HD / 8); u += 64 * CW) {
                const int r = u / (HD / 8), d8 = u % (HD / 8);
                store_x_unit(static_cast<uint4*>(xo.frags), xo.mt, xo.planes, row0 + r / group,
                             (hkv * group + r % group) * (HD / 8) + d8, z);
            }
        }
        return;
    }
    const int n = t.seq_n[b];
    const int total = n + K + 1;
    const int ck = seq_chunk_keys(total, max_chunks);
    const int key0 = chunk * ck;
    const bool active = chunk < max_chunks && key0 < total;
    if constexpr (CW == 0) {
        if (!active) return;
    }
    const int dq = n_q_heads * HD;
    floatx4 acc[RT][DT];
    float m_run[RT], l_run[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m_run[rt] = -INFINITY;
        l_run[rt] = 0.f;
#pragma unroll
        for (int d = 0; d < DT; ++d) acc[rt][d] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    if (active) {
    const int key1 = min(key0 + ck, total);

    const int blk0 = key0 >> 5, blk1 = (key1 + 31) >> 5;
    const uint4* head;
    int my_page = 0;
    if constexpr (PAGED) {
        head = cache + ((size_t)layer * g.n_kv_heads + hkc) * (64 * HD) / 8;   // offset inside a page
        const int p = g.table[(size_t)t.seq_slot[b] * g.blocks_per_slot + min(blk0 + lane, blk1 - 1)];
        my_page = p < 0 ? 0 : p;
    } else {
        head = cache + cache_head_base(g, layer, t.seq_slot[b], hkc) / 8;
    }
    const size_t blk_u4 = g.blk_stride / 8;   // from one block of this head to the next (contiguous cache)

    uint4 ka[2][STEPS], va[DT], kb[2][STEPS], vb[DT];
    // unconditional loads (a block index past the chunk re-reads the chunk's last block): with no
    // branch around them the compiler counts outstanding loads exactly and the prefetch stays in flight
    auto load_block = [&](int blk, uint4(&kk)[2][STEPS], uint4(&vv)[DT]) {
        const int bb = min(blk, blk1 - 1);
        const uint4* p;
        if constexpr (PAGED)
            p = head + (size_t)__builtin_amdgcn_readlane(my_page, bb - blk0) * (g.page_stride / 8) + lane;
        else
            p = head + (size_t)bb * blk_u4 + lane;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int s = 0; s < STEPS; ++s) kk[sub][s] = p[sub * (2 * HD) + s * 64];
#pragma unroll
        for (int d = 0; d < DT; ++d) vv[d] = p[4 * HD + d * 64];
    };
    load_block(blk0, ka, va);   // the stream starts before anything else is fetched

    // queries, pre-scaled by log2(e)/sqrt(hd), as bf16 head + remainder operand fragments
    Frag qh[RT][STEPS], ql[RT][STEPS];
    int n_vis[RT];           // cached positions below this are visible to the query (0 for padding rows)
    uint32_t wmask[RT];      // window slots (positions n + i) the query attends to
    // Where this lane's share of a row tile's queries starts in the partial sums: 8 dims of every
    // 32-dim step, i.e. 2 * STEPS float4 columns.
    auto q_columns = [&](int rt, const float** cols, float& rs) {
        const int r = rt * 16 + c16;
        const bool real = r < rows;
        const int j = real ? r / group : 0, hl = real ? r % group : 0;
        const int m = row0 + j;
        rs = row_inv_rms(src.ns.ssq, src.ns.n_ssq, m, src.ns.d, src.ns.eps);
        const float* pq = src.partial + (size_t)m * src.ld + (hkv * group + hl) * HD + 8 * gq;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            cols[2 * s] = pq + 32 * s;
            cols[2 * s + 1] = pq + 32 * s + 4;
        }
    };
    // Scale, rotate and split them: dims d and d + HD/2 (a rotary pair) sit in steps s and
    // s + STEPS/2 of the same lane.
    auto q_finish = [&](int rt, const float4* sums, float rs, int j, float sc) {
        float raw[STEPS][8];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const float4 a = sums[2 * s], b = sums[2 * s + 1];
            raw[s][0] = a.x * rs; raw[s][1] = a.y * rs; raw[s][2] = a.z * rs; raw[s][3] = a.w * rs;
            raw[s][4] = b.x * rs; raw[s][5] = b.y * rs; raw[s][6] = b.z * rs; raw[s][7] = b.w * rs;
        }
        const int rpos = t.tree ? t.row_rope[row0 + j] : n + j;
        const float* cs = src.cos_sin + (size_t)rpos * HD + 2 * (8 * gq);   // [HD/2][2] per position
#pragma unroll
        for (int s = 0; s < STEPS / 2; ++s) {
            float x0[8], x1[8];
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const float4 c2 = *reinterpret_cast<const float4*>(cs + 2 * (32 * s) + 4 * e4);   // cos,sin of 2 dims
                const float ca[2] = {c2.x, c2.z}, sa[2] = {c2.y, c2.w};
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const int e = 2 * e4 + h2;
                    const float a = raw[s][e], bq = raw[s + STEPS / 2][e];
                    x0[e] = (a * ca[h2] - bq * sa[h2]) * sc;
                    x1[e] = (a * sa[h2] + bq * ca[h2]) * sc;
                }
            }
            split_frag(x0, qh[rt][s], ql[rt][s]);
            split_frag(x1, qh[rt][s + STEPS / 2], ql[rt][s + STEPS / 2]);
        }
    };
    // 64-dim heads: the partial sums of two row tiles are requested together (the same number of
    // loads in flight as one tile of a 128-dim head)
    constexpr int RB = (FUSED && HD == 64 && RT >= 2) ? 2 : 1;
    float4 pre[RB > 1 ? RT + 1 : 1][2 * STEPS];   // sums fetched ahead (batched variant only)
    float pre_rs[RB > 1 ? RT + 1 : 1];
    if constexpr (RB > 1) {
#pragma unroll
        for (int rt0 = 0; rt0 < RT; rt0 += 2) {
            const float* cols[2][2 * STEPS];
            q_columns(rt0, cols[0], pre_rs[rt0]);
            q_columns(min(rt0 + 1, RT - 1), cols[1], pre_rs[rt0 + 1]);
            const float* flat[4 * STEPS];
            float4 fsum[4 * STEPS];
#pragma unroll
            for (int x = 0; x < 4 * STEPS; ++x) flat[x] = cols[x / (2 * STEPS)][x % (2 * STEPS)];
            sum_splits4_many(flat, src.n_split, src.stride, fsum);
#pragma unroll
            for (int x = 0; x < 4 * STEPS; ++x) pre[rt0 + x / (2 * STEPS)][x % (2 * STEPS)] = fsum[x];
        }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int r = rt * 16 + c16;
        const bool real = r < rows;
        const int j = real ? r / group : 0, hl = real ? r % group : 0;
        n_vis[rt] = real ? n : 0;
        wmask[rt] = !real ? 0u : (t.tree ? t.row_mask[row0 + j] : (2u << j) - 1u);
        const float sc = real ? scale_log2e : 0.f;   // rows past the window contribute zeros
        if constexpr (FUSED && RB > 1) {
            q_finish(rt, pre[rt], pre_rs[rt], j, sc);
        } else if constexpr (FUSED) {
            const float* cols[2 * STEPS];
            float rs;
            q_columns(rt, cols, rs);
            float4 sums[2 * STEPS];
            sum_splits4_many(cols, src.n_split, src.stride, sums);
            q_finish(rt, sums, rs, j, sc);
        } else {
            const float4* qsrc = reinterpret_cast<const float4*>(q + (size_t)(row0 + j) * dq + (hkv * group + hl) * HD + 8 * gq);
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float4 a = qsrc[8 * s], b = qsrc[8 * s + 1];
                const float x[8] = {a.x * sc, a.y * sc, a.z * sc, a.w * sc, b.x * sc, b.y * sc, b.z * sc, b.w * sc};
                split_frag(x, qh[rt][s], ql[rt][s]);
            }
        }
    }

    auto process = [&](int blk, const uint4(&kk)[2][STEPS], uint4(&vv)[DT]) {
        const int kbase = blk * 32;
        const bool tail = kbase + 32 > n || kbase >= key1;   // reaches the window / the end: mask per element
        if (tail) {
            // values of positions that do not exist yet may hold anything: zero them
#pragma unroll
            for (int d = 0; d < DT; ++d) {
                Frag f;
                f.u = vv[d];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = kbase + (e < 4 ? 4 * gq + e : 16 + 4 * gq + e - 4);
                    if (key >= total) f.h[e] = 0;
                }
                vv[d] = f.u;
            }
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            floatx4 st[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                st[sub] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    Frag kf;
                    kf.u = kk[sub][s];
                    st[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qh[rt][s].v, st[sub], 0, 0, 0);
                    st[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, ql[rt][s].v, st[sub], 0, 0, 0);
                }
            }
            float sv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) sv[e] = st[e >> 2][e & 3];
            if (tail) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = kbase + (e < 4 ? 4 * gq + e : 16 + 4 * gq + e - 4);
                    const int w = key - n;   // window slot, if >= 0
                    const bool vis = key < n_vis[rt] || (w >= 0 && w < 32 && ((wmask[rt] >> w) & 1u));
                    if (!vis || kbase >= key1) sv[e] = -INFINITY;
                }
            }
            float mx = sv[0];
#pragma unroll
            for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // The reference exponent m_run of a row only moves when a score exceeds it by more than
            // 8 (weights stay below 2^8, far inside fp32 and the two-plane split): after the first
            // blocks that is rare, and a trip in which no row of the wavefront moves skips the
            // rescaling of the accumulators -- 32 multiplications and as many register moves each way,
            // about as many issue cycles as the block's matrix products.  Sums and outputs stay
            // relative to m_run, which is all the merge needs.
            const bool move = mx > m_run[rt] + 8.f;
            if (__builtin_amdgcn_ballot_w64(move) != 0) {
                const float m_to = move ? mx : m_run[rt];
                const float m_fin = (m_to == -INFINITY) ? 0.f : m_to;
                const float alpha = move ? __builtin_amdgcn_exp2f(m_run[rt] - m_fin) : 1.f;
                m_run[rt] = m_to;
                l_run[rt] *= alpha;
#pragma unroll
                for (int d = 0; d < DT; ++d) {
                    acc[rt][d][0] *= alpha; acc[rt][d][1] *= alpha; acc[rt][d][2] *= alpha; acc[rt][d][3] *= alpha;
                }
            }
            const float m_use = (m_run[rt] == -INFINITY) ? 0.f : m_run[rt];
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                sv[e] = __builtin_amdgcn_exp2f(sv[e] - m_use);   // arguments <= 8; far below -126 the result is 0
                ps += sv[e];
            }
            l_run[rt] += ps;
            Frag ph, pl;
            split_frag(sv, ph, pl);
#pragma unroll
            for (int d = 0; d < DT; ++d) {
                Frag vf;
                vf.u = vv[d];
                floatx4 a = acc[rt][d];
                a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, ph.v, a, 0, 0, 0);
                a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pl.v, a, 0, 0, 0);
                acc[rt][d] = a;
            }
        }
    };

    // Two blocks per trip, no branch inside: a block index past the chunk holds only positions
    // >= total, which the tail masking turns into zero weight, so an odd block count just ends with
    // one idle half trip.
    if constexpr (FUSED) {
        // The window's keys (rotated) and values of this kv head that fall into this chunk.  HD/8
        // lanes share a position (each 4 rotary pairs of the key and 8 dims of the value), so a
        // wavefront covers 8 positions per trip in rounds of 64 / (HD/8); each round's loads are issued
        // together.  (Putting both rounds of a 128-dim head in flight at once costs registers the main
        // loop needs: measured slower.)
        const int w0 = max(key0, n), w1 = key1;   // positions [w0, w1) are window slots of this chunk
        if (w0 < w1) {
            constexpr int HALF = HD / 2, LP = HD / 8, PPR = 64 / LP, NR = 8 / PPR;
            const int u = lane / LP, tq = lane % LP;
            const int slot = t.seq_slot[b];
            const int kcol = n_q_heads * HD + hkc * HD, vcol = (n_q_heads + g.n_kv_heads) * HD + hkc * HD;
            for (int p0 = w0; p0 < w1; p0 += 8) {
                float kr[NR][8], vr[NR][8];
                int posr[NR];
#pragma unroll
                for (int h = 0; h < NR; ++h) {
                    const int pc = min(p0 + PPR * h + u, w1 - 1);   // clamped: the loads are unconditional
                    posr[h] = pc;
                    const int m = row0 + (pc - n);
                    const float rs = row_inv_rms(src.ns.ssq, src.ns.n_ssq, m, src.ns.d, src.ns.eps);
                    const float* prow = src.partial + (size_t)m * src.ld;
                    const int rpos = t.tree ? t.row_rope[m] : pc;
                    const float* cols[4] = {prow + kcol + 4 * tq, prow + kcol + HALF + 4 * tq, prow + vcol + 8 * tq,
                                            prow + vcol + 8 * tq + 4};
                    float4 kv4[4];
                    sum_splits4_many(cols, src.n_split, src.stride, kv4);
                    const float a[4] = {kv4[0].x, kv4[0].y, kv4[0].z, kv4[0].w};
                    const float bk[4] = {kv4[1].x, kv4[1].y, kv4[1].z, kv4[1].w};
                    const float* cs = src.cos_sin + (size_t)rpos * HD + 2 * (4 * tq);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float c = cs[2 * e], sn = cs[2 * e + 1];
                        const float x = a[e] * rs, y = bk[e] * rs;
                        kr[h][e] = x * c - y * sn;
                        kr[h][4 + e] = x * sn + y * c;
                    }
                    const float4 A = kv4[2], B = kv4[3];
                    vr[h][0] = A.x * rs; vr[h][1] = A.y * rs; vr[h][2] = A.z * rs; vr[h][3] = A.w * rs;
                    vr[h][4] = B.x * rs; vr[h][5] = B.y * rs; vr[h][6] = B.z * rs; vr[h][7] = B.w * rs;
                }
#pragma unroll
                for (int h = 0; h < NR; ++h) {
                    if (p0 + PPR * h + u < w1) {
                        const size_t blk = cache_block_base(g, layer, slot, hkc, posr[h] >> 5);
                        const int t32 = posr[h] & 31;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            cache_w[blk + tiled_k_within(HD, t32, 4 * tq + e)] =
                                __builtin_bit_cast(uint16_t, static_cast<__bf16>(kr[h][e]));
                            cache_w[blk + tiled_k_within(HD, t32, 4 * tq + e + HALF)] =
                                __builtin_bit_cast(uint16_t, static_cast<__bf16>(kr[h][4 + e]));
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            cache_w[blk + tiled_v_within(HD, t32, 8 * tq + e)] =
                                __builtin_bit_cast(uint16_t, static_cast<__bf16>(vr[h][e]));
                    }
                }
            }
            // the stores must have landed before this wavefront reads the blocks they belong to; only
            // the first block was requested before them
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            if (blk0 >= (w0 >> 5)) load_block(blk0, ka, va);
        }
    }
    for (int blk = blk0; blk < blk1; blk += 2) {
        load_block(blk + 1, kb, vb);
        process(blk, ka, va);
        load_block(blk + 2, ka, va);
        process(blk + 1, kb, vb);
    }
    }   // active

    if constexpr (CW == 0) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float l = l_run[rt];
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const int r = rt * 16 + c16;
            if (r < rows) {
                float* o = part_o + ((size_t)item * r_cap + r) * HD + 4 * gq;
#pragma unroll
                for (int d = 0; d < DT; ++d)
                    *reinterpret_cast<float4*>(o + 16 * d) = make_float4(acc[rt][d][0], acc[rt][d][1], acc[rt][d][2], acc[rt][d][3]);
                if (gq == 0) {
                    part_ml[((size_t)item * r_cap + r) * 2 + 0] = m_run[rt];
                    part_ml[((size_t)item * r_cap + r) * 2 + 1] = l;
                }
            }
        }
    } else {
        // chunk results of the CW wavefronts -> LDS -> merged rows as operand fragments
        __shared__ float s_o[CW][RT * 16][HD];
        __shared__ float s_m[CW][RT * 16], s_l[CW][RT * 16];
        static_assert(CW == 0 || sizeof(float) * CW * RT * 16 * (HD + 2) <= 64 * 1024, "chunk results fit in LDS");
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float l = l_run[rt];
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const int r = rt * 16 + c16;
#pragma unroll
            for (int d = 0; d < DT; ++d)
                *reinterpret_cast<float4*>(&s_o[chunk][r][16 * d + 4 * gq]) =
                    make_float4(acc[rt][d][0], acc[rt][d][1], acc[rt][d][2], acc[rt][d][3]);
            if (gq == 0) {
                s_m[chunk][r] = m_run[rt];
                s_l[chunk][r] = l;
            }
        }
        __syncthreads();
        // out = sum_c w_c o_c / sum_c w_c l_c with w_c = 2^(m_c - max m), chunks in index order
        for (int u = threadIdx.x; u < rows * (HD / 8); u += 64 * CW) {
            const int r = u / (HD / 8), d8 = u % (HD / 8);
            float mx = -INFINITY;
#pragma unroll
            for (int c = 0; c < CW; ++c) mx = fmaxf(mx, s_m[c][r]);
            float den = 0.f;
            float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                const float mc = s_m[c][r];
                const bool on = mc != -INFINITY;   // a chunk entirely after this query's position (or empty)
                const float w = on ? exp2f(mc - mx) : 0.f;
                den += on ? w * s_l[c][r] : 0.f;
                const float4 a = *reinterpret_cast<const float4*>(&s_o[c][r][8 * d8]);
                const float4 bq = *reinterpret_cast<const float4*>(&s_o[c][r][8 * d8 + 4]);
                v[0] += on ? w * a.x : 0.f; v[1] += on ? w * a.y : 0.f; v[2] += on ? w * a.z : 0.f; v[3] += on ? w * a.w : 0.f;
                v[4] += on ? w * bq.x : 0.f; v[5] += on ? w * bq.y : 0.f; v[6] += on ? w * bq.z : 0.f; v[7] += on ? w * bq.w : 0.f;
            }
            const float inv = 1.0f / den;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] *= inv;
            store_x_unit(static_cast<uint4*>(xo.frags), xo.mt, xo.planes, row0 + r / group,
                         (hkv * group + r % group) * (HD / 8) + d8, v);
        }
    }
}

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

// The variants with 128-dim heads and three or four row tiles have no registers left for the fused
// prologue (they would spill); those shapes keep the separate rotary/append kernel.
constexpr bool fused_fits(int hd, int rt) { return !(hd == 128 && rt >= 3); }

// Workgroups of cw wavefronts can merge their chunk results themselves when those fit in 64 KiB of
// LDS, and with 8 wavefronts only where two of them fit on a SIMD (64-dim heads, one row tile).
constexpr bool merge_fits(int hd, int rt, int cw)
{
    return cw * rt * 16 * (hd + 2) * 4 <= 64 * 1024 && (cw < 8 || (hd == 64 && rt == 1));
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
    return lp;
}

template <int HD>
static int launch_chunks(int rt, int cw, dim3 grid, dim3 wg_grid, hipStream_t s, const StepTables& t, const LookaheadPack& ks,
                         const CacheGeom& g, int n_q_heads, int kv_share, int layer, const void* cache, const float* q,
                         const AttnPlan& p, int r_cap, float sl2, float* part_o, float* part_ml, const QkvSrc& src,
                         void* cache_w, const XOut& xo)
{
#define SPECV_ATTN_CW(RT, PG, FU, CW_)                                                                         \
    hipLaunchKernelGGL((attn_chunk_kernel<HD, RT, PG, FU, CW_>), CW_ > 0 ? wg_grid : grid, dim3(CW_ > 0 ? 64 * CW_ : 64), \
                       0, s, t, ks, g, n_q_heads, kv_share, layer, (const uint4*)cache, q, p.max_chunks, r_cap, sl2, part_o, \
                       part_ml, src, (uint16_t*)cache_w, xo)
#define SPECV_ATTN_GO(RT, PG, FU)                                                                              \
    do {                                                                                                         \
        if (cw == 1) SPECV_ATTN_CW(RT, PG, FU, 1);                                                               \
        else if (cw == 2) { if constexpr (merge_fits(HD, RT, 2)) SPECV_ATTN_CW(RT, PG, FU, 2); }                 \
        else if (cw == 4) { if constexpr (merge_fits(HD, RT, 4)) SPECV_ATTN_CW(RT, PG, FU, 4); }                 \
        else if (cw == 8) { if constexpr (merge_fits(HD, RT, 8)) SPECV_ATTN_CW(RT, PG, FU, 8); }                 \
        else SPECV_ATTN_CW(RT, PG, FU, 0);                                                                       \
    } while (0)
#define SPECV_ATTN(RT)                                                                                           \
    do {                                                                                                         \
        if (src.partial) {                                                                                       \
            if constexpr (fused_fits(HD, RT)) {                                                                  \
                if (g.table) SPECV_ATTN_GO(RT, true, true);                                                      \
                else SPECV_ATTN_GO(RT, false, true);                                                             \
            } else {                                                                                             \
                return fail(SPEC_ERR_SHAPE, "attention variant cannot take unfinished queries");                 \
            }                                                                                                    \
        } else if (g.table) SPECV_ATTN_GO(RT, true, false);                                                      \
        else SPECV_ATTN_GO(RT, false, false);                                                                    \
    } while (0)
    switch (rt) {
    case 1: SPECV_ATTN(1); break;
    case 2: SPECV_ATTN(2); break;
    case 3: SPECV_ATTN(3); break;
    case 4: SPECV_ATTN(4); break;
    default: return fail(SPEC_ERR_SHAPE, "attention supports at most 64 query rows per kv head");
    }
#undef SPECV_ATTN
#undef SPECV_ATTN_GO
#undef SPECV_ATTN_CW
    SPECV_LAUNCH_CHECK("attn_chunk_kernel");
    return SPEC_OK;
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
        if (hd == 128)
            rc = launch_chunks<128>(rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, share, layer, cache, q, p, r_cap, sl2, part_o,
                                    part_ml, src, cache_w, xo);
        else
            rc = launch_chunks<64>(rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, share, layer, cache, q, p, r_cap, sl2, part_o,
                                   part_ml, src, cache_w, xo);
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
