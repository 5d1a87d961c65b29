// The decoder's projections: Y[M][N] = X[M][K] * W[N][K]^T with a handful of rows (M = number of
// window tokens in flight) against large bf16 weight matrices.  This is a real dense contraction,
// so it runs on the matrix cores (v_mfma_f32_16x16x32_bf16), but at these M it is bound by
// streaming W from HBM exactly once, and the kernel is organised around that stream:
//
//  * W is stored in tile order (spec_pack_weight): the 16x32 operand tile a wavefront needs is one
//    contiguous 1 KiB block, and the tiles a wavefront walks along K follow each other in memory,
//    so every lane issues plain 16-byte loads that coalesce perfectly and each wave streams a
//    contiguous region.  The loads for the next K chunk are in flight while the current one is
//    multiplied (two register buffers), and nothing but W goes through that pipe.
//  * X (a few hundred KiB, L2 resident) arrives already as bf16 operand fragments (frag.h), written
//    that way by the kernel that produced it, and is staged through LDS once per workgroup and K
//    chunk with plain 16-byte copies, shared by the four wavefronts, double buffered.  With two
//    planes each activation is a bf16 head plus a bf16 remainder (two matrix instructions): the
//    matrix cores have ample slack at these shapes, and activation rounding drops to ~2^-17.
//  * RMSNorm costs nothing here: the producer multiplies by the gain, and the row's 1/rms factors
//    out of the dot product, so the consumer of the GEMM's result applies it as a row scale.
//  * K is cut into ranges across workgroups so that the grid fills all 256 compute units even when
//    N is small; range sums are left in a partial buffer in a fixed order and added up by the
//    consumer kernel (no floating-point atomics: bit-reproducible).
#include "common.h"
#include "frag.h"

namespace specv {
namespace {

// Workgroup index -> (K range, column block).  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2; ranges are assigned so that all workgroups of one K range run on one XCD and the
// slice of X they share stays in that L2.  n_split is a power of two.
__device__ __forceinline__ void map_block(int i, int n_split, int* s, int* nb)
{
    const int x = i & 7, j = i >> 3;
    if (n_split >= 8) {
        const int hi = n_split >> 3;
        *s = x + 8 * (j % hi);
        *nb = j / hi;
    } else {
        const int per = 8 / n_split;
        *s = x % n_split;
        *nb = j * per + x / n_split;
    }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int WPACK_KG = 4;   // K blocks per group of the packed weight order

// All global loads below are unconditional (addresses clamped into range, W zeroed by selects past
// the K range): with no branch around a load the compiler can count outstanding loads exactly, so
// a wait for X never turns into a wait for the whole W stream.
// RS = 2 (many row tiles): eight wavefronts per workgroup, two row halves x four column groups.
// A wavefront then holds the accumulators of MTW = ceil(MT/2) row tiles only, which fits two
// wavefronts per SIMD: the matrix instruction issues faster with a second wavefront to alternate
// with (measured: one 16x16x32 product per 19-20 cycles and SIMD instead of 22-26), and the
// other wavefront's products cover this one's waits.
// EPI = 1 (gate/up projection with a single K range, NT == 2, columns packed so that a gate tile and
// its up tile are neighbours): instead of leaving sums for another kernel, the workgroup applies the
// row scale of the preceding norm, computes silu(gate) * up and writes the result as operand
// fragments of the down projection.  One kernel and one round of partial sums less per layer.
// CG: wavefronts (column groups of NT tiles) per workgroup, 4 unless the launch picks fewer.  With a
// single K range every workgroup streams all of X through its compute unit next to its share of W;
// three wavefronts per workgroup put the 7B-shape gate/up projection on 230 compute units instead of
// 172, and the same stream ran in 32.5 instead of 37.8 us (stand-alone, epilogue removed; without
// any X traffic both take 30 us): what a compute unit can pull from L2 per unit of time, X included,
// is the limit there, not HBM.
struct SwigluOut {
    const float* ssq;   // NormScale of the rows (sums of squares in n_ssq chunks)
    int n_ssq, d;
    float eps;
    uint4* frags;       // fragment buffer of the down projection's operand
    int mt, planes;
};

template <int MT, int NT, int KC, int PLANES, int RS = 1, int EPI = 0, int CG = 4>
__global__ void __launch_bounds__(64 * CG * RS) gemm_skinny_kernel(const u32x4* __restrict__ Xf, const u32x4* __restrict__ Wp,
                                                          float* __restrict__ partial, int M, int n_tiles,
                                                          int kb_total, int kb_per_split, int n_split, int n_blocks,
                                                          SwigluOut so)
{
    constexpr int CHUNK_U4 = KC * PLANES * MT * 64;     // 16-byte units per X chunk (contiguous in Xf)
    constexpr int TPBK = 64 * CG * RS;                    // threads per workgroup: CG column groups x RS row halves
    constexpr int UPT = (CHUNK_U4 + TPBK - 1) / TPBK;     // per thread
    __shared__ u32x4 xs[2][CHUNK_U4];                   // two chunk buffers

    int split, nblk;
    map_block(blockIdx.x, n_split, &split, &nblk);
    if (nblk >= n_blocks) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int MTW = (MT + RS - 1) / RS;               // row tiles of one wavefront
    const int a0 = (wave % RS) * MTW;                       // its first row tile
    const int tile0 = (nblk * CG + wave / RS) * NT;
    const int kb0 = split * kb_per_split;
    const int kb1 = min(kb0 + kb_per_split, kb_total);

    floatx4 acc[MTW][NT];
#pragma unroll
    for (int a = 0; a < MTW; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i) acc[a][i] = floatx4{0.f, 0.f, 0.f, 0.f};

    u32x4 wa[KC][NT], wb[KC][NT];
    u32x4 xr[UPT];
    int xoff[UPT];
#pragma unroll
    for (int u = 0; u < UPT; ++u) xoff[u] = min(u * TPBK + (int)threadIdx.x, CHUNK_U4 - 1);   // surplus threads repeat

    // W tile order: [K group of 4 blocks][column tile][block in group][lane] -- the chunk a workgroup
    // reads in one step (its 4*NT tiles, KC blocks) is one contiguous run, and workgroups of
    // neighbouring column blocks read neighbouring runs
    const u32x4* wbase[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) wbase[i] = Wp + (size_t)min(tile0 + i, n_tiles - 1) * (WPACK_KG * 64) + lane;
    const size_t group_stride = (size_t)n_tiles * (WPACK_KG * 64);

    // Up to four row tiles the weights are fetched with streaming (non-temporal) loads: each is read once
    // per launch by one wavefront, and marked that way the stream leaves the caches to what is reused (the
    // X fragments, the partial sums, a small model's keys and values).  Measured, same box: 7B-shape step
    // 4.934 -> 4.877 ms, 1B-shape 0.947 -> 0.890 ms (its 34 MB of keys and values stay in the memory-side
    // cache from step to step).  From five row tiles on it is a wash (72 rows +0.4 %, 88-96 rows -0.5 %),
    // and where two wavefronts of a workgroup fetch the same tile (RS = 2) the second would miss: 157 rows
    // +6..10 % GEMM time.  Those keep ordinary loads.
    constexpr bool W_STREAM = RS == 1 && MT <= 4;
    // Loads past the end of the range are redirected to its last block (a cache hit, no new HBM
    // traffic); the products of such blocks are suppressed by mask_w.
    auto load_w = [&](int kbase, u32x4(&dst)[KC][NT]) {
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            const int kb = min(kbase + c, kb1 - 1);
            const size_t off = (size_t)(kb / WPACK_KG) * group_stride + (kb % WPACK_KG) * 64;
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                if constexpr (W_STREAM) dst[c][i] = __builtin_nontemporal_load(&wbase[i][off]);
                else dst[c][i] = wbase[i][off];
            }
        }
    };
    auto mask_w = [&](int kbase, u32x4(&w)[KC][NT]) {   // K blocks past the range contribute nothing
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            const bool ok = kbase + c < kb1;
#pragma unroll
            for (int i = 0; i < NT; ++i) w[c][i] = ok ? w[c][i] : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto load_x = [&](int kbase) {
        // fragment buffers carry XFRAG_PAD_KB zeroed blocks past kb_total, so the last chunk of the
        // last range may overhang
        const u32x4* src = Xf + (size_t)min(kbase, kb1 - 1) * (PLANES * MT * 64);
#pragma unroll
        for (int u = 0; u < UPT; ++u) xr[u] = src[xoff[u]];
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int u = 0; u < UPT; ++u) xs[buf][xoff[u]] = xr[u];
    };
    // fragment of the wavefront's a-th row tile (RS = 2 and odd MT: the second half's last tile does
    // not exist; it re-reads the tile before it and its results are dropped)
    auto x_frag = [&](int buf, int c, int plane, int a) {
        const int row_tile = RS == 1 ? a : min(a0 + a, MT - 1);
        return __builtin_bit_cast(bf16x8, xs[buf][((c * PLANES + plane) * MT + row_tile) * 64 + lane]);
    };
    auto compute = [&](const u32x4(&w)[KC][NT], int buf) {
        if constexpr (MT >= 3) {
            // One wavefront per SIMD: nothing else fills the matrix pipeline while this wave waits
            // for an LDS read, so the fragments of row tile t+1 are requested before the products of
            // tile t are issued, and the instruction order is pinned (2 LDS reads, then the 2*NT
            // products of the previous reads); left to itself the scheduler reads, waits, multiplies.
            bf16x8 xh = x_frag(buf, 0, 0, 0), xl = xh;
            if constexpr (PLANES == 2) xl = x_frag(buf, 0, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, PLANES, 0);            // LDS reads of tile 0
#pragma unroll
            for (int t = 0; t < KC * MTW; ++t) {
                const int c = t / MTW, a = t % MTW;
                bf16x8 nh = xh, nl = xl;
                if (t + 1 < KC * MTW) {
                    nh = x_frag(buf, (t + 1) / MTW, 0, (t + 1) % MTW);
                    nl = nh;
                    if constexpr (PLANES == 2) nl = x_frag(buf, (t + 1) / MTW, 1, (t + 1) % MTW);
                }
#pragma unroll
                for (int i = 0; i < NT; ++i)
                    acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xh, __builtin_bit_cast(bf16x8, w[c][i]), acc[a][i], 0, 0, 0);
                if constexpr (PLANES == 2) {
#pragma unroll
                    for (int i = 0; i < NT; ++i)
                        acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xl, __builtin_bit_cast(bf16x8, w[c][i]), acc[a][i], 0, 0, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, PLANES, 0);        // LDS reads of tile t+1
                __builtin_amdgcn_sched_group_barrier(0x008, PLANES * NT, 0);   // products of tile t
                xh = nh;
                xl = nl;
            }
            return;
        }
#pragma unroll
        for (int c = 0; c < KC; ++c)
#pragma unroll
            for (int a = 0; a < MT; ++a) {
                const bf16x8 xh = x_frag(buf, c, 0, a);
                bf16x8 xl = xh;
                if constexpr (PLANES == 2) xl = x_frag(buf, c, 1, a);
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    const bf16x8 wf = __builtin_bit_cast(bf16x8, w[c][i]);
                    acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xh, wf, acc[a][i], 0, 0, 0);
                    if constexpr (PLANES == 2)
                        acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xl, wf, acc[a][i], 0, 0, 0);
                }
            }
    };

    if constexpr (MT >= 8) {
        // Many row tiles: a chunk's products take about as long as a memory round trip, and with two W
        // buffers the loads of chunk j+2 can only be issued after the products of chunk j (they reuse
        // its registers), so products and waiting alternate instead of overlapping.  A third W buffer
        // lets the loads of chunk j+2 go out BEFORE the products of chunk j, and three X register
        // sets keep the fragments of chunks j+2..j+4 in flight (X is the larger of the two streams
        // here and misses L2 as often as not).  One K block per chunk (KC == 1): no chunk is partial,
        // nothing needs masking; loads past the range are redirected to its last block and their
        // chunks never multiplied.
        static_assert(MT < 8 || KC == 1, "the three-buffer pipeline takes one K block per chunk");
        u32x4 wc[KC][NT];
        u32x4 x0[UPT], x1[UPT], x2[UPT];
        auto load_xs = [&](int kbase, u32x4(&dst)[UPT]) {
            const u32x4* src = Xf + (size_t)min(kbase, kb1 - 1) * (PLANES * MT * 64);
#pragma unroll
            for (int u = 0; u < UPT; ++u) dst[u] = src[xoff[u]];
        };
        auto store_xs = [&](int buf, const u32x4(&from)[UPT]) {
#pragma unroll
            for (int u = 0; u < UPT; ++u) xs[buf][xoff[u]] = from[u];
        };
        const int n_chunks = kb1 - kb0;
        // step j: W of chunk j+2 requested, chunk j multiplied, chunk j+1's X (set xn, fetched three
        // steps ago) put into the other LDS buffer, chunk j+4's X requested into the same set
        auto step = [&](int j, const u32x4(&cur)[KC][NT], u32x4(&ahead)[KC][NT], u32x4(&xn)[UPT]) {
            load_w(kb0 + j + 2, ahead);
            compute(cur, j & 1);
            store_xs((j + 1) & 1, xn);
            load_xs(kb0 + j + 4, xn);
            __syncthreads();
        };
        load_w(kb0, wa);
        __builtin_amdgcn_sched_barrier(0);
        load_xs(kb0, x0);
        load_xs(kb0 + 1, x1);
        load_xs(kb0 + 2, x2);
        load_w(kb0 + 1, wb);
        store_xs(0, x0);
        load_xs(kb0 + 3, x0);
        __syncthreads();
        int j = 0;
        for (; j + 3 <= n_chunks; j += 3) {
            step(j, wa, wc, x1);
            step(j + 1, wb, wa, x2);
            step(j + 2, wc, wb, x0);
        }
        if (j < n_chunks) {
            step(j, wa, wc, x1);
            if (j + 1 < n_chunks) step(j + 1, wb, wa, x2);
        }
    } else {
    // The W stream starts first; afterwards X loads are always issued before the W loads of the same
    // step, so that waiting for X (older) leaves the W loads (younger) in flight.
    load_w(kb0, wa);
    __builtin_amdgcn_sched_barrier(0);   // keep the first W loads ahead of everything else
    load_x(kb0);
    store_x(0);
    load_x(kb0 + KC);
    load_w(kb0 + KC, wb);
    __syncthreads();
    // Chunk j is multiplied from LDS buffer j%2 while chunk j+1's X (already in registers) is copied
    // into the other buffer and the loads of chunk j+2 are issued.  The main loop runs while both of
    // its prefetches are inside the range; the last one to three chunks are finished below without
    // loading anything past the range.  Only the last chunk can be partial (mask_w).
    const int n_chunks = (kb1 - kb0 + KC - 1) / KC;
    int j = 0;
    for (; j + 3 < n_chunks; j += 2) {
        const int kbase = kb0 + j * KC;
        compute(wa, 0);
        store_x(1);
        load_x(kbase + 2 * KC);
        load_w(kbase + 2 * KC, wa);
        __syncthreads();
        compute(wb, 1);
        store_x(0);
        load_x(kbase + 3 * KC);
        load_w(kbase + 3 * KC, wb);
        __syncthreads();
    }
    {
        const int kbase = kb0 + j * KC;
        const int left = n_chunks - j;   // 1, 2 or 3 (0 only for an empty range)
        if (left == 3) {
            compute(wa, 0);
            store_x(1);
            load_x(kbase + 2 * KC);
            load_w(kbase + 2 * KC, wa);
            __syncthreads();
            compute(wb, 1);
            store_x(0);
            __syncthreads();
            mask_w(kbase + 2 * KC, wa);
            compute(wa, 0);
        } else if (left == 2) {
            compute(wa, 0);
            store_x(1);
            __syncthreads();
            mask_w(kbase + KC, wb);
            compute(wb, 1);
        } else if (left == 1) {
            mask_w(kbase, wa);
            compute(wa, 0);
        }
    }
    }   // MT < 8

    const int g = lane >> 4, c = lane & 15;
    if constexpr (EPI == 1) {
        static_assert(EPI == 0 || (NT == 2 && RS == 1), "the SwiGLU epilogue pairs the two column tiles of a wavefront");
        static_assert(EPI == 0 || sizeof(xs) >= CG * MT * 256 * sizeof(float), "tile staging fits the X chunk buffers");
        __shared__ float rsv[MT * 16];
        __syncthreads();                                      // everyone is done with the X chunk buffers
        float* tw = reinterpret_cast<float*>(&xs[0][0]) + wave * (MT * 256);   // [MT*16 rows][16 units]
        for (int m = threadIdx.x; m < MT * 16; m += TPBK)
            rsv[m] = m < M ? row_inv_rms(so.ssq, so.n_ssq, m, so.d, so.eps) : 0.f;
        __syncthreads();
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ml = a * 16 + 4 * g + r;
                const float rs = rsv[ml];
                const float ge = acc[a][0][r] * rs, ue = acc[a][1][r] * rs;
                tw[ml * 16 + c] = ge / (1.f + expf(-ge)) * ue;
            }
        __syncthreads();
        if (tile0 + 1 < n_tiles) {
            const int f0 = (tile0 >> 1) * 16;                 // first FFN unit of this tile pair
            for (int u = lane; u < MT * 32; u += 64) {
                const int row = u >> 1, oct = u & 1;
                if (row < M) {
                    const float4 lo4 = *reinterpret_cast<const float4*>(tw + row * 16 + oct * 8);
                    const float4 hi4 = *reinterpret_cast<const float4*>(tw + row * 16 + oct * 8 + 4);
                    const float v[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
                    store_x_unit(so.frags, so.mt, so.planes, row, (f0 >> 3) + oct, v);
                }
            }
        }
        return;
    }
    const int n_pad = n_tiles * 16;
    float* out = partial + (size_t)split * M * n_pad;
#pragma unroll
    for (int a = 0; a < MTW; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int tile = tile0 + i;
            if (tile < n_tiles && a0 + a < MT) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = (a0 + a) * 16 + 4 * g + r;
                    if (m < M) out[(size_t)m * n_pad + tile * 16 + c] = acc[a][i][r];
                }
            }
        }
}

// zero a fragment buffer (a kernel rather than a memset node, so that the call can be captured in a graph)
__global__ void __launch_bounds__(256) zero_kernel(uint4* __restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = make_uint4(0, 0, 0, 0);
}

// fp32 row-major X[M][K] (optionally times gain[K]) -> fragment buffer
__global__ void __launch_bounds__(256) pack_x_kernel(const float* __restrict__ X, const float* __restrict__ gain, int M,
                                                     int K, int mt_count, int planes, uint4* __restrict__ xf)
{
    const int units = K / 8;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < M * units; i += gridDim.x * 256) {
        const int m = i / units, k8 = i % units;
        const float4 a = *reinterpret_cast<const float4*>(X + (size_t)m * K + k8 * 8);
        const float4 b = *reinterpret_cast<const float4*>(X + (size_t)m * K + k8 * 8 + 4);
        float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        if (gain)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] *= gain[k8 * 8 + e];
        store_x_unit(xf, mt_count, planes, m, k8, v);
    }
}

// Plain fp32 product for the small fp32 configurations: 16x16 output tile per workgroup, K in
// slabs of 32 through LDS.
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                       float* __restrict__ Y, int M, int N, int K)
{
    __shared__ float xs[16][33], ws[16][33];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
    float acc = 0.f;
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int i = threadIdx.x; i < 16 * 32; i += 256) {
            const int r = i >> 5, c = i & 31;
            xs[r][c] = (m0 + r < M && k0 + c < K) ? X[(size_t)(m0 + r) * K + k0 + c] : 0.f;
            ws[r][c] = (n0 + r < N && k0 + c < K) ? W[(size_t)(n0 + r) * K + k0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 32; ++c) acc = fmaf(xs[ty][c], ws[tx][c], acc);
        __syncthreads();
    }
    if (m0 + ty < M && n0 + tx < N) Y[(size_t)(m0 + ty) * N + n0 + tx] = acc;
}

__global__ void __launch_bounds__(256) pack_weight_kernel(const uint16_t* __restrict__ src, uint4* __restrict__ dst,
                                                          int n_out, int n_in, int n_tiles, int interleave)
{
    const int kb_total = n_in / 32;
    const int kb_pad = (kb_total + WPACK_KG - 1) / WPACK_KG * WPACK_KG;
    const size_t total = (size_t)n_tiles * kb_pad * 64;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        // i = ((group * n_tiles + tile) * WPACK_KG + block in group) * 64 + lane
        const int lane = (int)(i & 63);
        size_t r = i >> 6;
        const int kbi = (int)(r % WPACK_KG); r /= WPACK_KG;
        const int j = (int)(r % n_tiles);
        const int kb = (int)(r / n_tiles) * WPACK_KG + kbi;
        int row = j * 16 + (lane & 15);
        if (interleave) row = ((j & 1) ? n_out / 2 : 0) + (j >> 1) * 16 + (lane & 15);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < n_out && kb < kb_total)
            v = *reinterpret_cast<const uint4*>(src + (size_t)row * n_in + kb * 32 + (lane >> 4) * 8);
        dst[i] = v;
    }
}

template <int MT, int NT, int KC, int RS, int CG>
int launch_groups(const GemmPlan& p, const void* xf, const void* w, int M, int K, int n_tiles, float* partial,
                  hipStream_t s)
{
    const int n_blocks = (n_tiles + CG * NT - 1) / (CG * NT);
    int grid = n_blocks * p.n_split;
    if (p.n_split < 8) grid = (n_blocks + (8 / p.n_split) - 1) / (8 / p.n_split) * 8;
    if (p.planes == 2)
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, KC, 2, RS, 0, CG>), dim3(grid), dim3(64 * CG * RS), 0, s, (const u32x4*)xf,
                           (const u32x4*)w, partial, M, n_tiles, K / 32, p.kb_per_split, p.n_split, n_blocks, SwigluOut{});
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, KC, 1, RS, 0, CG>), dim3(grid), dim3(64 * CG * RS), 0, s, (const u32x4*)xf,
                           (const u32x4*)w, partial, M, n_tiles, K / 32, p.kb_per_split, p.n_split, n_blocks, SwigluOut{});
    SPECV_LAUNCH_CHECK("gemm_skinny_kernel");
    return SPEC_OK;
}

template <int MT, int NT, int KC, int RS = 1>
int launch_variant(const GemmPlan& p, const void* xf, const void* w, int M, int K, int n_tiles, float* partial,
                   hipStream_t s)
{
    if constexpr (RS == 2 || (MT <= 4 && NT == 2)) {
        if (p.cg == 3) return launch_groups<MT, NT, KC, RS, 3>(p, xf, w, M, K, n_tiles, partial, s);
    }
    if constexpr (MT <= 4 && NT == 2) {
        if (p.cg == 2) return launch_groups<MT, NT, KC, RS, 2>(p, xf, w, M, K, n_tiles, partial, s);
    }
    return launch_groups<MT, NT, KC, RS, 4>(p, xf, w, M, K, n_tiles, partial, s);
}

struct Variant {
    int mt, nt, kc;   // row tiles, column tiles per wave, K blocks per LDS chunk
};
// row tiles -> (column tiles per wave, K blocks per LDS chunk); LDS = 2 buffers * planes * mt * kc KiB.
// Up to 4 row tiles there is a second, wider variant (4 column tiles per wave, 2 K blocks per
// chunk) for matrices with many columns.
// From 6 row tiles on the matrix cores and the LDS reads of X start to matter: several column tiles
// per wave (each X fragment read from LDS feeds that many products) keep LDS traffic per W byte down.
// From 8 row tiles on the workgroup has eight wavefronts (two row halves) and the three-buffer
// pipeline of one K block per chunk (see the kernel): both measured slower at 6 row tiles (88
// rows), faster from 8 on (120 rows -6 %, 160 -7 %, 250 and 320 -20 %).  Those variants come in
// even row-tile counts only: the two row halves of a workgroup take ceil(mt/2) tiles each, so an
// odd count costs what the next even one does.
constexpr Variant kVariants[] = {{1, 2, 4}, {2, 2, 4}, {3, 2, 4}, {4, 2, 2}, {5, 4, 2}, {6, 4, 2},
                                 {8, 4, 1}, {10, 4, 1}, {12, 4, 1}, {14, 2, 1}, {16, 2, 1}, {18, 2, 1},
                                 {20, 2, 1}, {22, 2, 1}};
constexpr int kWideMaxMt = 4;
// column tiles from which the wide variant is taken (up to 4 row tiles) and below which 5-12 row tiles
// take two tiles per wavefront.  The wide variant fills the chip from 340 tiles on, but between that
// and 1000 tiles (the 7B-shape QKV projection: 768) the narrow one does with half the K ranges -- half
// the partial sums for the attention kernel to add up: step 5.088 -> 5.057 ms, decoding round with the
// configuration's draft (QKV of 384 tiles) 7.15 -> 7.07 ms.
constexpr int kWideMinTiles = 340;
constexpr int kWideMinTilesFewRows = 1000;

const Variant* pick_variant(int M)
{
    const int mt = (M + 15) / 16;
    for (const Variant& v : kVariants)
        if (v.mt >= mt) return &v;
    return nullptr;
}

int g_wg_target = 0;   // workgroups per launch to aim for; 0 = two thirds of the compute units
int g_balance_groups = 1;   // many-row launches: four column groups of three tiles instead of three of four

}  // namespace

void set_gemm_wg_target(int t) { g_wg_target = t; }

int gemm_row_tiles(int M)
{
    const Variant* v = pick_variant(M);
    return v ? v->mt : 0;
}

GemmPlan plan_gemm(int M, int N, int K, int cu_count, bool split_x)
{
    GemmPlan p{};
    const Variant* v = pick_variant(M);
    p.mt = v ? v->mt : 0;
    p.nt = v ? v->nt : 1;
    p.planes = split_x ? 2 : 1;
    int kc = v ? v->kc : 4;
    p.n_pad = (N + 15) / 16 * 16;
    const int n_tiles = p.n_pad / 16;
    if (p.mt <= kWideMaxMt && n_tiles >= kWideMinTilesFewRows) {
        p.nt = 4;
        kc = 2;
    }
    // 5 to 12 row tiles and few columns (the 4096-column output and down projections): two column tiles
    // per wavefront instead of four -- twice the column blocks, so half the K ranges fill the chip and
    // half the partial sums are written and read back (16 ranges x 157 rows x 4096 columns were 41 MB
    // against 33.5 MB of weights).  Costs LDS reads per product, gains more: step -3 % at 88 rows,
    // projections and their consumers -0.3 ms of 6.6 at 157 rows.
    if (p.mt >= 5 && p.mt <= 12 && n_tiles < kWideMinTiles) p.nt = 2;
    p.cg = 4;
    p.rs = p.mt >= 8 ? 2 : 1;
    const int kb_total = K / 32;
    // K ranges: a power of two, just enough of them that the launch has about `target` workgroups.
    // Measured on MI355X: every launch pays a few microseconds of ramp-up and tail whatever its
    // size, and long-lived workgroups stream best, so fewer, longer ranges win as long as roughly
    // two thirds of the compute units have a workgroup; more ranges only add partial-sum traffic
    // (M*N*4 bytes each way per range).  At most 16 ranges, each at least two LDS chunks long.
    const int target = g_wg_target > 0 ? g_wg_target : (2 * cu_count) / 3;
    // Ranges are whole K groups of the packed order (below), so cutting a short K too finely leaves
    // ranges with nothing in them -- workgroups that only write zeros for the consumer to add; no
    // doubling that would leave more than one range in eight empty.
    auto ranges_with_work = [&](int n) {
        const int per = ((kb_total + n - 1) / n + WPACK_KG - 1) / WPACK_KG * WPACK_KG;
        return (kb_total + per - 1) / per;
    };
    auto ranges_for = [&](int blocks_x) {
        int n = 1;
        while (n < 16 && blocks_x * n < target && (kb_total + 2 * n - 1) / (2 * n) >= 2 * kc
               && ranges_with_work(2 * n) * 8 >= 2 * n * 7)
            n *= 2;
        return n;
    };
    // Few rows and few columns (up to four row tiles, under 340 column tiles: the 4096-column projections, a small
    // model's QKV): two column groups per workgroup.  Twice the column blocks fill the chip with half the K ranges,
    // i.e. half the partial sums for the launch to write and for its consumer to add up, and two wavefronts per
    // compute unit stream as fast as four (stand-alone read of 33 and 90 MB: 4.7 and 5.8 TB/s either way).  1B-shape
    // step 0.884 -> 0.850 ms (its attention adds up four QKV ranges instead of eight), batch 8 1.242 -> 1.205,
    // decoding round -0.3 %.  Only while a workgroup's K range stays within 2048: a workgroup stages all rows of
    // X over its range, and at 2752 (the 7B-shape down projection in four ranges) the launch was 1.7 us slower,
    // as much as its consumers gained; at 2048 (K = 8192) and below it costs the launch nothing.
    if (p.mt <= 4 && p.nt == 2 && n_tiles < kWideMinTiles) {
        const int n2 = ranges_for((n_tiles + 2 * p.nt - 1) / (2 * p.nt));
        if ((kb_total + n2 - 1) / n2 * 32 <= 2048) p.cg = 2;
    }
    const int wg_x = (n_tiles + p.cg * p.nt - 1) / (p.cg * p.nt);
    const int s = ranges_for(wg_x);
    p.n_split = s;
    // Few rows, two column tiles per wavefront: three column groups per workgroup where four leave more than a
    // fifth of the compute units without a workgroup and three fill them (7B-shape QKV: 192 workgroups of four
    // wavefronts -> 256 of three).  A read stream of that size (100 MB) runs 10 % faster from 256 workgroups than
    // from 192, and since the weights are fetched with streaming loads the GEMM follows: QKV 25.5 -> 22.5 us per
    // launch, 7B-shape step 4.915 -> 4.853 ms, 1B-shape 0.897 -> 0.884, decoding round 6.67 -> 6.58 ms (before the
    // streaming loads the same change gained nothing).  With four tiles per wavefront or five to seven row tiles
    // it is mixed (72 rows -1 %, 88-96 rows +1.3..1.6 % per step) and is not made.
    if (p.mt <= 4 && p.nt == 2) {
        const int wg3 = (n_tiles + 3 * p.nt - 1) / (3 * p.nt) * s;
        if (p.cg == 4 && wg_x * s * 5 < cu_count * 4 && wg3 <= cu_count) p.cg = 3;
    }
    // Many rows (the eight-wavefront variants): the matrix instructions set the pace, so compute units
    // without a workgroup are lost time; three column groups per workgroup instead of four when that
    // brings the launch from under four fifths of the compute units to at most all of them
    // (157 rows: QKV 192 -> 256 workgroups, gate/up 172 -> 230; GEMM time of that step -6 %).
    if (p.mt >= 8 && p.rs == 2) {
        const int wg3 = (n_tiles + 3 * p.nt - 1) / (3 * p.nt) * s;
        if (wg_x * s * 5 < cu_count * 4 && wg3 <= cu_count) {
            // Twelve column tiles per workgroup either way; as four column groups of three tiles the
            // workgroup keeps eight wavefronts, two on every SIMD, where three groups of four tiles
            // put two wavefronts on two SIMDs and one on the others (the loaded ones set the pace).
            if (p.nt == 4 && g_balance_groups) p.nt = 3;
            else p.cg = 3;
        }
    }
    // ranges start on a K group of the packed order so that every chunk is one contiguous run
    p.kb_per_split = ((kb_total + s - 1) / s + WPACK_KG - 1) / WPACK_KG * WPACK_KG;
    return p;
}

size_t gemm_partial_elems(const GemmPlan& p, int M) { return (size_t)p.n_split * M * p.n_pad; }

int launch_gemm_bf16(const GemmPlan& p, const void* x_frags, const void* w_packed, int M, int N, int K, float* partial,
                     hipStream_t s)
{
    if (M < 1 || M > GEMM_MAX_ROWS) return fail(SPEC_ERR_SHAPE, "GEMM supports 1..%d rows, got %d", GEMM_MAX_ROWS, M);
    if (K % 32) return fail(SPEC_ERR_SHAPE, "GEMM needs K %% 32 == 0, got %d", K);
    const int n_tiles = (N + 15) / 16;
#define SPECV_GEMM(MT_, NT_, KC_, ...)                                                                  \
    if (p.mt == MT_ && p.nt == NT_ && p.rs == (1, ##__VA_ARGS__))                                         \
        return launch_variant<MT_, NT_, KC_, ##__VA_ARGS__>(p, x_frags, w_packed, M, K, n_tiles, partial, s)
    SPECV_GEMM(1, 4, 2);
    SPECV_GEMM(2, 4, 2);
    SPECV_GEMM(3, 4, 2);
    SPECV_GEMM(4, 4, 2);
    SPECV_GEMM(1, 2, 4);
    SPECV_GEMM(2, 2, 4);
    SPECV_GEMM(3, 2, 4);
    SPECV_GEMM(4, 2, 2);
    SPECV_GEMM(5, 2, 2);
    SPECV_GEMM(6, 2, 2);
    SPECV_GEMM(5, 4, 2);
    SPECV_GEMM(6, 4, 2);
    SPECV_GEMM(8, 2, 1, 2);
    SPECV_GEMM(10, 2, 1, 2);
    SPECV_GEMM(12, 2, 1, 2);
    SPECV_GEMM(8, 3, 1, 2);
    SPECV_GEMM(10, 3, 1, 2);
    SPECV_GEMM(12, 3, 1, 2);
    SPECV_GEMM(8, 4, 1, 2);
    SPECV_GEMM(10, 4, 1, 2);
    SPECV_GEMM(12, 4, 1, 2);
    SPECV_GEMM(14, 2, 1, 2);
    SPECV_GEMM(16, 2, 1, 2);
    SPECV_GEMM(18, 2, 1, 2);
    SPECV_GEMM(20, 2, 1, 2);
    SPECV_GEMM(22, 2, 1, 2);
#undef SPECV_GEMM
    return fail(SPEC_ERR_SHAPE, "no GEMM variant for %d rows (%d row tiles, %d column tiles per wave)", M, p.mt, p.nt);
}

namespace {
int g_swiglu_min_wgs = 0;   // 0: a third of the compute units
int g_swiglu_cg = 0;        // 0: chosen by swiglu_column_groups; 2, 3, 4: forced (tests)
}
void set_swiglu_min_wgs(int n) { g_swiglu_min_wgs = n; }
void set_swiglu_column_groups(int n) { g_swiglu_cg = n >= 2 && n <= 4 ? n : 0; }

// The gate/up projection can finish SwiGLU itself when it runs as ONE K range of 128-column
// workgroups (narrow variants, up to 4 row tiles) and that still gives enough workgroups.
bool gemm_swiglu_fits(int M, int F, int cu_count)
{
    const int mt = gemm_row_tiles(M);
    if (mt < 1 || mt > 4 || F % 16) return false;   // (6 row tiles measured, with four and with three wavefronts per workgroup: the narrow GEMM loses more than the kernel saved)
    const int wgs = (2 * F / 16 + 7) / 8;
    // measured: 172 workgroups (F = 11008) step -1.9 %, 128 workgroups (F = 8192) -3.5 %
    return wgs >= (g_swiglu_min_wgs > 0 ? g_swiglu_min_wgs : cu_count / 3);
}

template <int MT, int KC, int CG>
static int launch_swiglu_cg(int planes, const void* xf, const void* w, int M, int K, int n_tiles, const SwigluOut& so,
                            hipStream_t s)
{
    const int n_blocks = (n_tiles + 2 * CG - 1) / (2 * CG);
    const int grid = (n_blocks + 7) / 8 * 8;       // map_block deals workgroups to the 8 XCDs
    const int kb = K / 32;
    if (planes == 2)
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, 2, KC, 2, 1, 1, CG>), dim3(grid), dim3(64 * CG), 0, s, (const u32x4*)xf,
                           (const u32x4*)w, nullptr, M, n_tiles, kb, (kb + WPACK_KG - 1) / WPACK_KG * WPACK_KG, 1, n_blocks, so);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, 2, KC, 1, 1, 1, CG>), dim3(grid), dim3(64 * CG), 0, s, (const u32x4*)xf,
                           (const u32x4*)w, nullptr, M, n_tiles, kb, (kb + WPACK_KG - 1) / WPACK_KG * WPACK_KG, 1, n_blocks, so);
    SPECV_LAUNCH_CHECK("gemm_skinny_kernel (SwiGLU)");
    return SPEC_OK;
}

// wavefronts per workgroup of the SwiGLU GEMM: as few as still give no more workgroups than compute
// units (the number of wavefronts in the launch is the same either way, one per pair of column tiles;
// fewer per workgroup spread them, and the X traffic, over more compute units)
static int swiglu_column_groups(int n_tiles, int cu_count)
{
    for (int cg = 2; cg < 4; ++cg)
        if ((n_tiles + 2 * cg - 1) / (2 * cg) <= cu_count) return cg;
    return 4;
}

template <int MT, int KC>
static int launch_swiglu_variant(int planes, const void* xf, const void* w, int M, int K, int n_tiles, const SwigluOut& so,
                                 int cu_count, hipStream_t s)
{
    switch (g_swiglu_cg > 0 ? g_swiglu_cg : swiglu_column_groups(n_tiles, cu_count)) {
    case 2: return launch_swiglu_cg<MT, KC, 2>(planes, xf, w, M, K, n_tiles, so, s);
    case 3: return launch_swiglu_cg<MT, KC, 3>(planes, xf, w, M, K, n_tiles, so, s);
    default: return launch_swiglu_cg<MT, KC, 4>(planes, xf, w, M, K, n_tiles, so, s);
    }
}

int launch_gemm_swiglu(const void* x_frags, int planes, const void* w_gate_up, int M, int F, int K, const float* ssq,
                       int n_ssq, int d, float eps, void* act_frags, int act_mt, int act_planes, int cu_count, hipStream_t s)
{
    if (K % 32 || F % 16) return fail(SPEC_ERR_SHAPE, "SwiGLU GEMM needs K %% 32 == 0 and F %% 16 == 0");
    const SwigluOut so{ssq, n_ssq, d, eps, static_cast<uint4*>(act_frags), act_mt, act_planes};
    const int n_tiles = 2 * F / 16;
    switch (gemm_row_tiles(M)) {
    case 1: return launch_swiglu_variant<1, 4>(planes, x_frags, w_gate_up, M, K, n_tiles, so, cu_count, s);
    case 2: return launch_swiglu_variant<2, 4>(planes, x_frags, w_gate_up, M, K, n_tiles, so, cu_count, s);
    case 3: return launch_swiglu_variant<3, 4>(planes, x_frags, w_gate_up, M, K, n_tiles, so, cu_count, s);
    case 4: return launch_swiglu_variant<4, 2>(planes, x_frags, w_gate_up, M, K, n_tiles, so, cu_count, s);
    default: return fail(SPEC_ERR_SHAPE, "no SwiGLU GEMM variant for %d rows", M);
    }
}

int launch_pack_x(const float* x, const float* gain, int M, int K, int mt_count, int planes, void* x_frags, hipStream_t s)
{
    const int total = M * (K / 8);
    int blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(pack_x_kernel, dim3(blocks), dim3(256), 0, s, x, gain, M, K, mt_count, planes, (uint4*)x_frags);
    SPECV_LAUNCH_CHECK("pack_x_kernel");
    return SPEC_OK;
}

int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* y, hipStream_t s)
{
    dim3 grid((N + 15) / 16, (M + 15) / 16);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, x, w, y, M, N, K);
    SPECV_LAUNCH_CHECK("gemm_f32_kernel");
    return SPEC_OK;
}

}  // namespace specv

using namespace specv;

extern "C" size_t spec_packed_weight_bytes(int32_t n_out, int32_t n_in)
{
    if (n_out <= 0 || n_in <= 0 || n_in % 32) return 0;
    const size_t kb_pad = (size_t)(n_in / 32 + WPACK_KG - 1) / WPACK_KG * WPACK_KG;
    return (size_t)((n_out + 15) / 16) * kb_pad * 1024;
}

extern "C" int spec_pack_weight(const void* src, void* dst, int32_t n_out, int32_t n_in, int32_t interleave_halves,
                                void* stream)
{
    if (!src || !dst || n_out <= 0 || n_in <= 0) return fail(SPEC_ERR_INVALID_ARG, "spec_pack_weight: bad pointer or size");
    if (n_in % 32) return fail(SPEC_ERR_SHAPE, "spec_pack_weight: n_in must be a multiple of 32");
    if (interleave_halves && (n_out % 32)) return fail(SPEC_ERR_SHAPE, "spec_pack_weight: interleaving needs n_out/2 %% 16 == 0");
    if (((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return fail(SPEC_ERR_INVALID_ARG, "spec_pack_weight: 16-byte alignment");
    const int n_tiles = (n_out + 15) / 16;
    const size_t total = spec_packed_weight_bytes(n_out, n_in) / 16;
    size_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t*)src, (uint4*)dst, n_out, n_in, n_tiles, interleave_halves ? 1 : 0);
    SPECV_LAUNCH_CHECK("pack_weight_kernel");
    return SPEC_OK;
}

extern "C" void spec_k_set_gemm_wg_target(int32_t workgroups) { set_gemm_wg_target(workgroups); }
extern "C" void spec_k_set_gemm_balance_groups(int32_t on) { g_balance_groups = on != 0; }
extern "C" void spec_k_set_swiglu_min_wgs(int32_t workgroups) { set_swiglu_min_wgs(workgroups); }
extern "C" void spec_k_set_swiglu_column_groups(int32_t groups) { set_swiglu_column_groups(groups); }
extern "C" void spec_k_set_attn_items_per_cu(int32_t items) { set_attn_items_per_cu(items); }
extern "C" void spec_k_set_attn_merge_min_pairs(int32_t pairs) { set_attn_merge_min_pairs(pairs); }
extern "C" void spec_k_set_attn_max_chunks(int32_t chunks) { set_attn_max_chunks(chunks); }
extern "C" void spec_k_set_attn_small_positions(int32_t positions) { set_attn_small_positions(positions); }

extern "C" size_t spec_k_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M < 1 || M > GEMM_MAX_ROWS || N < 1 || K < 32 || K % 32) return 0;
    GemmPlan p = plan_gemm(M, N, K, 256, true);
    // partial sums of the widest plan (16 ranges) + the X fragment buffer (both planes)
    const size_t part = (size_t)16 * M * p.n_pad * sizeof(float);
    return part + xfrag_uint4s(p.mt, 2, K) * sizeof(uint4) + 256;
}

extern "C" int spec_k_gemm_bf16(const float* x, const void* w_packed, float* y, int32_t M, int32_t N, int32_t K,
                                int32_t split_x, void* workspace, void* stream)
{
    if (!x || !w_packed || !y || !workspace) return fail(SPEC_ERR_INVALID_ARG, "spec_k_gemm_bf16: null pointer");
    if (M < 1 || M > GEMM_MAX_ROWS || N < 1 || K < 32 || K % 32) return fail(SPEC_ERR_SHAPE, "spec_k_gemm_bf16: unsupported shape");
    GemmPlan p = plan_gemm(M, N, K, 256, split_x != 0);
    float* partial = (float*)workspace;
    char* xf = (char*)workspace + (((size_t)16 * M * p.n_pad * sizeof(float) + 255) & ~(size_t)255);
    const size_t n_xf = xfrag_uint4s(p.mt, p.planes, K);
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n_xf + 255) / 256 < 2048 ? (n_xf + 255) / 256 : 2048)), dim3(256), 0,
                       (hipStream_t)stream, (uint4*)xf, n_xf);
    SPECV_LAUNCH_CHECK("zero_kernel");
    int rc = launch_pack_x(x, nullptr, M, K, p.mt, p.planes, xf, (hipStream_t)stream);
    if (rc) return rc;
    rc = launch_gemm_bf16(p, xf, w_packed, M, N, K, partial, (hipStream_t)stream);
    if (rc) return rc;
    return launch_reduce_splits(partial, p.n_split, (size_t)M * p.n_pad, M, N, p.n_pad, nullptr, 0, 0, 0.f, y,
                                (hipStream_t)stream);
}

extern "C" int spec_k_gemm_f32(const float* x, const float* w, float* y, int32_t M, int32_t N, int32_t K, void* stream)
{
    if (!x || !w || !y || M < 1 || N < 1 || K < 1) return fail(SPEC_ERR_INVALID_ARG, "spec_k_gemm_f32: bad argument");
    return launch_gemm_f32(x, w, M, N, K, y, (hipStream_t)stream);
}
