// The chunk kernel of the windowed-causal attention and its launch table, shared by the two
// translation units that instantiate it: attention.hip (keys and values fetched with streaming loads:
// every byte is read once per launch) and attention_reuse.hip (ordinary loads, for launches in which
// several work items stream the same cache head).  See attention.hip for the design.
#pragma once

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
// STREAM: the keys and values are fetched with non-temporal loads.  A launch reads every byte of them
// exactly once, and marked that way they pass the caches without displacing what is reused (7B-shape:
// 58.7 -> 54.2 us per launch, Dyn 8.5 -> 7.9 ms of attention per step).  Launches in which several
// work items stream the same cache head take the other variant: there the second reader is served
// from the memory-side cache, and streaming loads cost the 1B-shape step 5 % of its attention time.
typedef unsigned int kv_u32x4 __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ uint4 kv_load(const uint4* p)
{
    if constexpr (STREAM) {
        const kv_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const kv_u32x4*>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    } else {
        return *p;
    }
}

template <int HD, int RT, bool PAGED, bool FUSED, int CW, bool STREAM>
__global__ void __launch_bounds__(CW > 0 ? 64 * CW : 64)
    attn_chunk_kernel(StepTables t, LookaheadPack ks, CacheGeom g, int n_q_heads, int kv_share, int layer,
                      const uint4* cache, const float* __restrict__ q, int max_chunks, int lag_keys, int r_cap, float scale_log2e,
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
    // Equal chunks, except that the chunks before the last are lag_keys longer when the last one stays
    // long enough: its wavefront first puts the window's keys and values together (FUSED), and with a
    // shorter run to stream afterwards it ends with the others instead of after them.
    int ck = seq_chunk_keys(total, max_chunks);
    if (lag_keys > 0) {
        const int n_used = (total + ck - 1) / ck;
        if (n_used >= 2 && total - (n_used - 1) * (ck + lag_keys) >= 2 * lag_keys + 64 && (!PAGED || ck + lag_keys <= 2048))
            ck += lag_keys;
    }
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
            for (int s = 0; s < STEPS; ++s) kk[sub][s] = kv_load<STREAM>(p + sub * (2 * HD) + s * 64);
#pragma unroll
        for (int d = 0; d < DT; ++d) vv[d] = kv_load<STREAM>(p + 4 * HD + d * 64);
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

// The variants with 128-dim heads and three or four row tiles have no registers left for the fused
// prologue (they would spill); those shapes keep the separate rotary/append kernel.
constexpr bool fused_fits(int hd, int rt) { return !(hd == 128 && rt >= 3); }

// Workgroups of cw wavefronts can merge their chunk results themselves when those fit in 64 KiB of
// LDS, and with 8 wavefronts only where two of them fit on a SIMD (64-dim heads, one row tile).
constexpr bool merge_fits(int hd, int rt, int cw)
{
    return cw * rt * 16 * (hd + 2) * 4 <= 64 * 1024 && (cw < 8 || (hd == 64 && rt == 1));
}

template <int HD, bool STREAM>
static int launch_chunks(int rt, int cw, dim3 grid, dim3 wg_grid, hipStream_t s, const StepTables& t, const LookaheadPack& ks,
                         const CacheGeom& g, int n_q_heads, int kv_share, int layer, const void* cache, const float* q,
                         const AttnPlan& p, int r_cap, float sl2, float* part_o, float* part_ml, const QkvSrc& src,
                         void* cache_w, const XOut& xo)
{
    const int lag_keys = src.partial ? p.lag_keys : 0;   // only the fused prologue delays a wavefront
#define SPECV_ATTN_CW(RT, PG, FU, CW_)                                                                         \
    hipLaunchKernelGGL((attn_chunk_kernel<HD, RT, PG, FU, CW_, STREAM>), CW_ > 0 ? wg_grid : grid, dim3(CW_ > 0 ? 64 * CW_ : 64), \
                       0, s, t, ks, g, n_q_heads, kv_share, layer, (const uint4*)cache, q, p.max_chunks, lag_keys, r_cap, sl2, part_o, \
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

}  // namespace

// launch_chunks<HD, false>, compiled in attention_reuse.hip
int launch_chunks_reuse(int hd, int rt, int cw, dim3 grid, dim3 wg_grid, hipStream_t s, const StepTables& t,
                        const LookaheadPack& ks, const CacheGeom& g, int n_q_heads, int kv_share, int layer, const void* cache,
                        const float* q, const AttnPlan& p, int r_cap, float sl2, float* part_o, float* part_ml,
                        const QkvSrc& src, void* cache_w, const XOut& xo);

}  // namespace specv
