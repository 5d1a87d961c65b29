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
//  * X (a few hundred KiB, L2 resident) is staged through LDS once per workgroup and K chunk, already
//    in operand order, and shared by the four wavefronts.  With split_x each activation is fed as
//    a bf16 head plus a bf16 remainder (two matrix instructions): the matrix cores have ample slack
//    at these shapes, and activation rounding drops to ~2^-17.
//  * K is cut into ranges across workgroups so that the grid fills all 256 compute units even when
//    N is small; range sums are left in a partial buffer in a fixed order and added up by the
//    consumer kernel (no floating-point atomics: bit-reproducible).
#include "common.h"

namespace specv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union Frag {
    uint4 u;
    bf16x8 v;
};

__device__ __forceinline__ void split8(const float4& a, const float4& b, uint4& hi, uint4& lo, bool want_lo)
{
    const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    Frag h, l;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 hb = static_cast<__bf16>(x[e]);          // round to nearest even
        h.v[e] = hb;
        l.v[e] = static_cast<__bf16>(x[e] - static_cast<float>(hb));
    }
    hi = h.u;
    if (want_lo) lo = l.u;
}

template <int MT, int NT, int KC, bool SPLIT>
__global__ void __launch_bounds__(256) gemm_skinny_kernel(const float* __restrict__ X, const uint4* __restrict__ Wp,
                                                          float* __restrict__ partial, int M, int K, int n_tiles,
                                                          int kb_total, int kb_per_split)
{
    constexpr int PLANES = SPLIT ? 2 : 1;
    constexpr int UNITS = MT * 16 * KC * 4;             // 8-element groups of X per chunk
    constexpr int UPT = (UNITS + 255) / 256;            // per thread
    __shared__ uint4 xs[PLANES][MT][KC][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile0 = (blockIdx.x * 4 + wave) * NT;
    const int kb0 = blockIdx.y * kb_per_split;
    const int kb1 = min(kb0 + kb_per_split, kb_total);

    floatx4 acc[MT][NT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i) acc[a][i] = floatx4{0.f, 0.f, 0.f, 0.f};

    uint4 wa[KC][NT], wb[KC][NT];
    float4 xr[UPT][2];

    auto load_w = [&](int kbase, uint4(&dst)[KC][NT]) {
#pragma unroll
        for (int c = 0; c < KC; ++c)
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const int kb = kbase + c, tile = tile0 + i;
                dst[c][i] = (kb < kb1 && tile < n_tiles) ? Wp[((size_t)tile * kb_total + kb) * 64 + lane]
                                                         : make_uint4(0, 0, 0, 0);
            }
    };
    auto load_x = [&](int kbase) {
#pragma unroll
        for (int u = 0; u < UPT; ++u) {
            const int unit = u * 256 + threadIdx.x;
            const int row = unit / (KC * 4), kg = unit % (KC * 4);
            const int kb = kbase + kg / 4;
            xr[u][0] = xr[u][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (unit < UNITS && row < M && kb < kb1) {
                const float4* p = reinterpret_cast<const float4*>(X + (size_t)row * K + kb * 32 + (kg & 3) * 8);
                xr[u][0] = p[0];
                xr[u][1] = p[1];
            }
        }
    };
    auto store_x = [&]() {
#pragma unroll
        for (int u = 0; u < UPT; ++u) {
            const int unit = u * 256 + threadIdx.x;
            if (unit < UNITS) {
                const int row = unit / (KC * 4), kg = unit % (KC * 4);
                uint4 hi, lo;
                split8(xr[u][0], xr[u][1], hi, lo, SPLIT);
                const int l = (kg & 3) * 16 + (row & 15);
                xs[0][row >> 4][kg >> 2][l] = hi;
                if constexpr (SPLIT) xs[PLANES - 1][row >> 4][kg >> 2][l] = lo;
            }
        }
    };
    auto compute = [&](const uint4(&w)[KC][NT]) {
#pragma unroll
        for (int c = 0; c < KC; ++c)
#pragma unroll
            for (int a = 0; a < MT; ++a) {
                Frag xh, xl;
                xh.u = xs[0][a][c][lane];
                if constexpr (SPLIT) xl.u = xs[PLANES - 1][a][c][lane];
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    Frag wf;
                    wf.u = w[c][i];
                    acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xh.v, wf.v, acc[a][i], 0, 0, 0);
                    if constexpr (SPLIT)
                        acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xl.v, wf.v, acc[a][i], 0, 0, 0);
                }
            }
    };

    // Order inside an iteration: X loads (older) first, then the next chunk's W loads, so that
    // waiting for X does not wait for the W stream.
    load_w(kb0, wa);
    for (int kbase = kb0; kbase < kb1; kbase += 2 * KC) {
        load_x(kbase);
        load_w(kbase + KC, wb);
        __syncthreads();            // previous chunk's readers are done with xs
        store_x();
        __syncthreads();
        compute(wa);
        if (kbase + KC < kb1) {
            load_x(kbase + KC);
            load_w(kbase + 2 * KC, wa);
            __syncthreads();
            store_x();
            __syncthreads();
            compute(wb);
        }
    }

    const int n_pad = n_tiles * 16;
    float* out = partial + (size_t)blockIdx.y * M * n_pad;
    const int g = lane >> 4, c = lane & 15;
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int tile = tile0 + i;
            if (tile < n_tiles) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = a * 16 + 4 * g + r;
                    if (m < M) out[(size_t)m * n_pad + tile * 16 + c] = acc[a][i][r];
                }
            }
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
    const size_t total = (size_t)n_tiles * kb_total * 64;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int lane = (int)(i & 63);
        const size_t tk = i >> 6;
        const int kb = (int)(tk % kb_total), j = (int)(tk / kb_total);
        int row = j * 16 + (lane & 15);
        if (interleave) row = ((j & 1) ? n_out / 2 : 0) + (j >> 1) * 16 + (lane & 15);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < n_out) v = *reinterpret_cast<const uint4*>(src + (size_t)row * n_in + kb * 32 + (lane >> 4) * 8);
        dst[i] = v;
    }
}

template <int MT, int NT, int KC>
int launch_variant(const GemmPlan& p, const float* x, const void* w, int M, int K, int n_tiles, bool split,
                   float* partial, hipStream_t s)
{
    dim3 grid((n_tiles + 4 * NT - 1) / (4 * NT), p.n_split);
    if (split)
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, KC, true>), grid, dim3(256), 0, s, x, (const uint4*)w, partial, M,
                           K, n_tiles, K / 32, p.kb_per_split);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, KC, false>), grid, dim3(256), 0, s, x, (const uint4*)w, partial,
                           M, K, n_tiles, K / 32, p.kb_per_split);
    SPECV_LAUNCH_CHECK("gemm_skinny_kernel");
    return SPEC_OK;
}

struct Variant {
    int mt, nt, kc;
};
// row tiles -> (column tiles per wave, K blocks per LDS chunk); LDS = planes * mt * kc KiB
constexpr Variant kVariants[] = {{1, 2, 8}, {2, 2, 8}, {3, 2, 8}, {4, 2, 8}, {6, 1, 4},
                                 {8, 1, 4}, {11, 1, 2}, {16, 1, 2}, {22, 1, 2}};

const Variant* pick_variant(int M)
{
    const int mt = (M + 15) / 16;
    for (const Variant& v : kVariants)
        if (v.mt >= mt) return &v;
    return nullptr;
}

}  // namespace

GemmPlan plan_gemm(int M, int N, int K, int cu_count)
{
    GemmPlan p{};
    const Variant* v = pick_variant(M);
    p.mt = v ? v->mt : 0;
    p.nt = v ? v->nt : 1;
    const int kc = v ? v->kc : 8;
    p.n_pad = (N + 15) / 16 * 16;
    const int n_tiles = p.n_pad / 16;
    const int wg_x = (n_tiles + 4 * p.nt - 1) / (4 * p.nt);
    const int kb_total = K / 32;
    // enough workgroups to keep two per compute unit busy, K ranges a whole number of LDS chunks,
    // and never more than 16 ranges (partial sums cost M*N*4 bytes each way per range)
    int want = (2 * cu_count + wg_x - 1) / wg_x;
    if (want < 1) want = 1;
    if (want > 16) want = 16;
    int per = (kb_total + want - 1) / want;
    per = (per + 2 * kc - 1) / (2 * kc) * (2 * kc);
    if (per > kb_total) per = kb_total;
    p.kb_per_split = per;
    p.n_split = (kb_total + per - 1) / per;
    return p;
}

size_t gemm_partial_elems(const GemmPlan& p, int M) { return (size_t)p.n_split * M * p.n_pad; }

int launch_gemm_bf16(const GemmPlan& p, const float* x, const void* w_packed, int M, int N, int K, bool split_x,
                     float* partial, hipStream_t s)
{
    if (M < 1 || M > 352) return fail(SPEC_ERR_SHAPE, "GEMM supports 1..352 rows, got %d", M);
    if (K % 32) return fail(SPEC_ERR_SHAPE, "GEMM needs K %% 32 == 0, got %d", K);
    const int n_tiles = (N + 15) / 16;
    switch (p.mt) {
    case 1: return launch_variant<1, 2, 8>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 2: return launch_variant<2, 2, 8>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 3: return launch_variant<3, 2, 8>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 4: return launch_variant<4, 2, 8>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 6: return launch_variant<6, 1, 4>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 8: return launch_variant<8, 1, 4>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 11: return launch_variant<11, 1, 2>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 16: return launch_variant<16, 1, 2>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    case 22: return launch_variant<22, 1, 2>(p, x, w_packed, M, K, n_tiles, split_x, partial, s);
    default: return fail(SPEC_ERR_SHAPE, "no GEMM variant for %d rows", M);
    }
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
    return (size_t)((n_out + 15) / 16 * 16) * n_in * 2;
}

extern "C" int spec_pack_weight(const void* src, void* dst, int32_t n_out, int32_t n_in, int32_t interleave_halves,
                                void* stream)
{
    if (!src || !dst || n_out <= 0 || n_in <= 0) return fail(SPEC_ERR_INVALID_ARG, "spec_pack_weight: bad pointer or size");
    if (n_in % 32) return fail(SPEC_ERR_SHAPE, "spec_pack_weight: n_in must be a multiple of 32");
    if (interleave_halves && (n_out % 32)) return fail(SPEC_ERR_SHAPE, "spec_pack_weight: interleaving needs n_out/2 %% 16 == 0");
    if (((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return fail(SPEC_ERR_INVALID_ARG, "spec_pack_weight: 16-byte alignment");
    const int n_tiles = (n_out + 15) / 16;
    const size_t total = (size_t)n_tiles * (n_in / 32) * 64;
    size_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t*)src, (uint4*)dst, n_out, n_in, n_tiles, interleave_halves ? 1 : 0);
    SPECV_LAUNCH_CHECK("pack_weight_kernel");
    return SPEC_OK;
}

extern "C" size_t spec_k_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M < 1 || M > 352 || N < 1 || K < 32) return 0;
    GemmPlan p = plan_gemm(M, N, K, 256);
    return gemm_partial_elems(p, M) * sizeof(float);
}

extern "C" int spec_k_gemm_bf16(const float* x, const void* w_packed, float* y, int32_t M, int32_t N, int32_t K,
                                int32_t split_x, void* workspace, void* stream)
{
    if (!x || !w_packed || !y || !workspace) return fail(SPEC_ERR_INVALID_ARG, "spec_k_gemm_bf16: null pointer");
    if (M < 1 || M > 352 || N < 1 || K < 32 || K % 32) return fail(SPEC_ERR_SHAPE, "spec_k_gemm_bf16: unsupported shape");
    GemmPlan p = plan_gemm(M, N, K, 256);
    int rc = launch_gemm_bf16(p, x, w_packed, M, N, K, split_x != 0, (float*)workspace, (hipStream_t)stream);
    if (rc) return rc;
    return launch_reduce_splits((const float*)workspace, p.n_split, (size_t)M * p.n_pad, M, N, p.n_pad, y,
                                (hipStream_t)stream);
}

extern "C" int spec_k_gemm_f32(const float* x, const float* w, float* y, int32_t M, int32_t N, int32_t K, void* stream)
{
    if (!x || !w || !y || M < 1 || N < 1 || K < 1) return fail(SPEC_ERR_INVALID_ARG, "spec_k_gemm_f32: bad argument");
    return launch_gemm_f32(x, w, M, N, K, y, (hipStream_t)stream);
}
