// Rejection-sampling part of the verify step: softmax statistics of every target and draft row,
// the accept scan, the residual / extra-token draw and the KV length update.
//
// The procedure is the one the paper describes in its section "Speculative Sampling Results"
// (compare the two models' probabilities of each proposed token, keep a prefix, resample the
// first rejected token from a combination of the distributions, draw one more token from the
// target if nothing was rejected), with the cited works' formulas: keep x iff u*q(x) < p(x),
// resample from max(0, p - q).
//
// The vocabulary-wide work is pure streaming, so it is laid out for HBM: every logit is read once
// by the statistics pass (float4 per lane, 64 values per lane in flight); only the one or two
// rows that the final draw needs are read again.  Sums are kept in fp64 and every reduction has a
// fixed order (no floating-point atomics), so results are reproducible bit for bit.
#include "cache_layout.h"
#include "common.h"

#include <cstring>
#include <mutex>

namespace specv {

namespace {

constexpr int TPB = 256;

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------------------------------------
// Row bookkeeping.  One workgroup; thread b owns sequence b.
// ---------------------------------------------------------------------------------------------
// (a workgroup of TPB threads, all of them calling; row0: SPEC_MAX_BATCH + 1 ints of LDS)
__device__ __forceinline__ void prepare_rows(const StepTables& t, const LookaheadPack& ks, int B, int Kmax, int V,
                                             int max_batch, int max_kv_len, int has_cache,
                                             const int32_t* __restrict__ seq_slot,
                                             const int32_t* __restrict__ last_token,
                                             const int32_t* __restrict__ draft_tokens,
                                             const int32_t* __restrict__ kv_len, int32_t* flag, int* row0)
{
    const int b = threadIdx.x;
    if (b == 0) {
        int r = 0, st = 0;
        for (int i = 0; i < B; ++i) {
            row0[i] = r;
            t.seq_row0[i] = r;
            t.seq_stat0[i] = st;
            r += ks.k[i] + 1;
            st += 2 * ks.k[i] + 1;
        }
        row0[B] = r;
        t.seq_row0[B] = r;
        t.seq_stat0[B] = st;
    }
    __syncthreads();
    if (b >= B) return;
    const int K = ks.k[b];
    int ok = 1, err = 0;
    int slot = b, n = 0;
    if (has_cache) {
        slot = seq_slot[b];
        if (slot < 0 || slot >= max_batch) {
            ok = 0;
            err = SPEC_ERR_INVALID_ARG;
            slot = 0;
        } else {
            // two sequences of one step must not share a slot
            for (int i = 0; i < b; ++i)
                if (seq_slot[i] == slot) { ok = 0; err = SPEC_ERR_INVALID_ARG; }
            n = kv_len[slot];
            if (n < 0 || n + K + 1 > max_kv_len) { ok = 0; err = SPEC_ERR_KV_OVERFLOW; }
            else if (ok && !pool_cover(t.pool, slot, n, n + K + 1)) { ok = 0; err = SPEC_ERR_KV_OVERFLOW; }
        }
    }
    int t0 = last_token ? last_token[b] : 0;
    if (t0 < 0 || t0 >= V) { ok = 0; err = SPEC_ERR_TOKEN_RANGE; }
    for (int i = 0; i < K; ++i) {
        int x = draft_tokens[b * Kmax + i];
        if (x < 0 || x >= V) { ok = 0; err = SPEC_ERR_TOKEN_RANGE; }
    }
    if (!ok) atomicCAS(flag, 0, err);
    t.seq_n[b] = ok ? n : 0;
    t.seq_ok[b] = ok;
    t.seq_slot[b] = slot;
    for (int j = 0; j <= K; ++j) {
        int r = row0[b] + j;
        t.row_seq[r] = b;
        t.row_pos[r] = ok ? n + j : -1;
        t.row_rope[r] = ok ? n + j : 0;
        t.row_mask[r] = (2u << j) - 1u;   // causal window: slots 0..j
        int tok = (j == 0) ? t0 : draft_tokens[b * Kmax + j - 1];
        t.row_tok[r] = ok ? tok : 0;
    }
}

__global__ void __launch_bounds__(TPB) prepare_kernel(StepTables t, LookaheadPack ks, int B, int Kmax, int V,
                                                      int max_batch, int max_kv_len, int has_cache,
                                                      const int32_t* __restrict__ seq_slot,
                                                      const int32_t* __restrict__ last_token,
                                                      const int32_t* __restrict__ draft_tokens,
                                                      const int32_t* __restrict__ kv_len, int32_t* flag)
{
    __shared__ int row0[SPEC_MAX_BATCH + 1];
    prepare_rows(t, ks, B, Kmax, V, max_batch, max_kv_len, has_cache, seq_slot, last_token, draft_tokens, kv_len, flag,
                 row0);
}

// A step with more window rows than one decoder pass takes is scored group by group: the row
// bookkeeping above runs once for the whole step (so that what it decides -- skipped sequences, a slot
// named twice, pages taken -- is decided once), and each pass gets the entries of its own sequences
// with rows and sequence numbers counted from the group's start.
__global__ void __launch_bounds__(TPB) slice_tables_kernel(StepTables full, StepTables sub, int b0, int Bg)
{
    const int r0 = full.seq_row0[b0], st0 = full.seq_stat0[b0];
    const int n_rows = full.seq_row0[b0 + Bg] - r0;
    for (int i = threadIdx.x; i <= Bg; i += TPB) {
        sub.seq_row0[i] = full.seq_row0[b0 + i] - r0;
        sub.seq_stat0[i] = full.seq_stat0[b0 + i] - st0;
        if (i < Bg) {
            sub.seq_n[i] = full.seq_n[b0 + i];
            sub.seq_ok[i] = full.seq_ok[b0 + i];
            sub.seq_slot[i] = full.seq_slot[b0 + i];
        }
    }
    for (int r = threadIdx.x; r < n_rows; r += TPB) {
        sub.row_seq[r] = full.row_seq[r0 + r] - b0;
        sub.row_pos[r] = full.row_pos[r0 + r];
        sub.row_tok[r] = full.row_tok[r0 + r];
        sub.row_rope[r] = full.row_rope[r0 + r];
        sub.row_mask[r] = full.row_mask[r0 + r];
    }
}

// ---------------------------------------------------------------------------------------------
// Pass 1: per (row, chunk) maximum and sum of exp((l - max)/T).
// Statistics rows of sequence b: K_b+1 target rows, then K_b draft rows.
// ---------------------------------------------------------------------------------------------
// draft_rows: draft logits rows per sequence in memory (Kmax for a chain of proposals; Kmax+1 for
// a tree, whose root has a row of its own)
// Which rows the pass walks.  STAT_CHAIN / STAT_TREE: sequence b has K_b + 1 target rows and K_b
// (chain) or K_b + 1 (tree) draft rows, found from the lookaheads in the kernel arguments alone, so
// the pass does not depend on the row tables.  STAT_PLAIN: one row per sequence, its logits row taken
// from seq_row0 (a proposing model's draw, whose row is not the one the lookaheads would give).
enum { STAT_CHAIN = 0, STAT_TREE = 1, STAT_PLAIN = 2 };

// The row bookkeeping of a step that runs no decoder pass (logits supplied by the caller), done by the
// statistics pass's first workgroup next to its own chunk instead of by a kernel of its own: the pass
// itself does not read the tables, the kernels after it do.
struct PrepIn {
    int on, Kmax;
    const int32_t* draft_tokens;
    int32_t* flag;
};

// The sequence b that statistics row srow belongs to, the row's number inside the sequence (local), the
// sequence's first target row (r0) and its lookahead (K), from the lookaheads in the kernel arguments.
// Every wavefront finds it for itself: lane i takes sequences i, i + 64, ... (all loads issued together,
// one memory round trip; walking the sequences one after the other costs one round trip each),
// prefix sums across the lanes place each sequence's rows, and the lane whose range holds srow answers.
__device__ __forceinline__ void find_stat_row(const LookaheadPack& ks, int B, int srow, bool tree, int* b_out,
                                              int* local_out, int* r0_out, int* K_out)
{
    constexpr int ROUNDS = SPEC_MAX_BATCH / 64;
    const int lane = threadIdx.x & 63;
    int kk[ROUNDS];
#pragma unroll
    for (int g = 0; g < ROUNDS; ++g) kk[g] = ks.k[min(g * 64 + lane, SPEC_MAX_BATCH - 1)];
    int base_st = 0, base_r = 0, b = 0, st = 0, r0 = 0, K = 0;
#pragma unroll
    for (int g = 0; g < ROUNDS; ++g) {
        const int i = g * 64 + lane;
        const int k = kk[g];
        const int n = i < B ? 2 * k + 1 + (tree ? 1 : 0) : 0, r = i < B ? k + 1 : 0;
        int ps = n, pr = r;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int a = __shfl_up(ps, off), c = __shfl_up(pr, off);
            if (lane >= off) {
                ps += a;
                pr += c;
            }
        }
        const int st_excl = base_st + ps - n;
        const bool hit = n > 0 && st_excl <= srow && srow < st_excl + n;
        const unsigned long long m = __ballot(hit);
        if (m) {
            const int src = __ffsll((long long)m) - 1;
            b = g * 64 + src;
            st = __shfl(st_excl, src);
            r0 = __shfl(base_r + pr - r, src);
            K = __shfl(k, src);
        }
        base_st += __shfl(ps, 63);
        base_r += __shfl(pr, 63);
    }
    *b_out = b;
    *local_out = srow - st;
    *r0_out = r0;
    *K_out = K;
}

template <bool VEC4>
__global__ void __launch_bounds__(TPB) stats_kernel(StepTables t, LookaheadPack ks, int B, int draft_rows, int V,
                                                    int n_chunks, const float* __restrict__ target,
                                                    const float* __restrict__ draft, float inv_T,
                                                    float* __restrict__ part_max, double* __restrict__ part_sum,
                                                    float* __restrict__ copy_out, size_t copy_stride, int layout,
                                                    PrepIn prep)
{
    __shared__ float smax[TPB / 64];
    __shared__ double ssum[TPB / 64];
    __shared__ int prep_row0[SPEC_MAX_BATCH + 1];
    if (prep.on && blockIdx.x == 0)
        prepare_rows(t, ks, B, prep.Kmax, V, SPEC_MAX_BATCH, 0, 0, nullptr, nullptr, prep.draft_tokens, nullptr, prep.flag,
                     prep_row0);
    const int srow = blockIdx.x / n_chunks;
    const int chunk = blockIdx.x % n_chunks;
    const float* row;
    if (layout == STAT_PLAIN) {
        row = target + (size_t)t.seq_row0[srow] * V;
    } else {
        int b, local, r0, K;
        find_stat_row(ks, B, srow, layout == STAT_TREE, &b, &local, &r0, &K);
        row = local <= K ? target + (size_t)(r0 + local) * V : draft + ((size_t)b * draft_rows + (local - K - 1)) * V;
    }
    const int base = chunk * STAT_CHUNK;
    const int lim = min(STAT_CHUNK, V - base);

    constexpr int PER = STAT_CHUNK / TPB;   // 64 values per lane
    float v[PER];
    // copy_out: plain-draw mode (one statistics row per sequence): keep the row for the verifier
    if constexpr (VEC4) {
        const float4* p4 = reinterpret_cast<const float4*>(row + base);
#pragma unroll
        for (int i = 0; i < PER / 4; ++i) {
            int idx = i * TPB + threadIdx.x;
            float4 x = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (idx * 4 < lim) {   // lim is a multiple of 4 when VEC4
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                const f32x4 y = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p4 + idx));
                x = make_float4(y.x, y.y, y.z, y.w);
            }
            v[4 * i + 0] = x.x; v[4 * i + 1] = x.y; v[4 * i + 2] = x.z; v[4 * i + 3] = x.w;
        }
        if (copy_out) {   // whole 16-byte stores (the launcher checked the alignment of the copy as well)
            float4* d4 = reinterpret_cast<float4*>(copy_out + (size_t)srow * copy_stride + base);
#pragma unroll
            for (int i = 0; i < PER / 4; ++i) {
                const int idx = i * TPB + threadIdx.x;
                if (idx * 4 < lim) d4[idx] = make_float4(v[4 * i + 0], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            int idx = i * TPB + threadIdx.x;
            v[i] = idx < lim ? row[base + idx] : -INFINITY;
        }
    }
    if (!VEC4 && copy_out) {
        float* dst = copy_out + (size_t)srow * copy_stride + base;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = i * TPB + (int)threadIdx.x;
            if (idx < lim) dst[idx] = v[i];
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < PER; ++i) m = fmaxf(m, v[i]);
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) smax[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(smax[0], smax[1]), fmaxf(smax[2], smax[3]));
    const float mm = (m == -INFINITY) ? 0.f : m;   // a chunk of -inf logits contributes nothing

    double acc = 0.0;
#pragma unroll
    for (int i = 0; i < PER; ++i) acc += (double)__expf((v[i] - mm) * inv_T);   // exp(-inf) = 0 for padding
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) ssum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        part_max[(size_t)srow * n_chunks + chunk] = m;
        part_sum[(size_t)srow * n_chunks + chunk] = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
    }
}

// Combine the chunk statistics of one row: max of maxima, sums rescaled to it.
__device__ __forceinline__ void combine_row(const float* pm, const double* ps, int n_chunks, double inv_T, float* m_out,
                                            double* z_out)
{
    // chunks eight at a time, the loads of a batch issued together (indices past the end clamped,
    // their terms dropped): a plain loop over a run-time count waits for every load in turn
    float m = -INFINITY;
    for (int c0 = 0; c0 < n_chunks; c0 += 8) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = pm[min(c0 + i, n_chunks - 1)];
#pragma unroll
        for (int i = 0; i < 8; ++i) m = fmaxf(m, v[i]);   // a repeated value does not change the maximum
    }
    double z = 0.0;
    for (int c0 = 0; c0 < n_chunks; c0 += 8) {
        float v[8];
        double sv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            v[i] = pm[min(c0 + i, n_chunks - 1)];
            sv[i] = ps[min(c0 + i, n_chunks - 1)];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (c0 + i < n_chunks) z += sv[i] * exp((double)(v[i] - m) * inv_T);
    }
    *m_out = m;
    *z_out = z;
}

// ---------------------------------------------------------------------------------------------
// Pass 2: accept scan (every workgroup of a sequence repeats it: a handful of scalars) and the
// mass of the final-draw distribution inside this workgroup's chunk of the vocabulary.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) accept_mass_kernel(StepTables t, LookaheadPack ks, int Kmax, int V,
                                                          int n_stat_chunks, int n_res_chunks,
                                                          const float* __restrict__ target,
                                                          const float* __restrict__ draft,
                                                          const int32_t* __restrict__ draft_tokens,
                                                          const float* __restrict__ uniforms, int u_stride,
                                                          float inv_T_f, const float* __restrict__ part_max,
                                                          const double* __restrict__ part_sum, SamplerWorkspace w)
{
    __shared__ float row_m[2 * SPEC_MAX_LOOKAHEAD + 2];
    __shared__ double row_z[2 * SPEC_MAX_LOOKAHEAD + 2];
    __shared__ int s_a;
    __shared__ double ssum[TPB / 64];
    const int b = blockIdx.y;
    const int chunk = blockIdx.x;
    const int K = ks.k[b];
    const double inv_T = (double)inv_T_f;
    const int st0 = t.seq_stat0[b];
    if ((int)threadIdx.x < 2 * K + 1)
        combine_row(part_max + (size_t)(st0 + threadIdx.x) * n_stat_chunks,
                    part_sum + (size_t)(st0 + threadIdx.x) * n_stat_chunks, n_stat_chunks, inv_T,
                    &row_m[threadIdx.x], &row_z[threadIdx.x]);
    __syncthreads();
    const float* trow0 = target + (size_t)t.seq_row0[b] * V;
    const float* drow0 = draft + (size_t)b * Kmax * V;
    if (threadIdx.x < 64) {
        // lane i tests proposal i (all positions at once: the tests are independent, only the first
        // failure matters); padding lanes repeat the last proposal and are masked out
        const int i = min((int)threadIdx.x, max(K - 1, 0));
        bool keep = true;
        if (K > 0) {
            const int x = draft_tokens[b * Kmax + i];
            const bool xin = x >= 0 && x < V;   // out-of-range ids were flagged by prepare; stay in bounds
            const float lp = xin ? trow0[(size_t)i * V + x] : 0.f;
            const float lq = xin ? drow0[(size_t)i * V + x] : 0.f;
            const double ep = exp((double)(lp - row_m[i]) * inv_T);
            const double eq = exp((double)(lq - row_m[K + 1 + i]) * inv_T);
            // keep iff u * q(x) < p(x)  <=>  u * eq * Zp < ep * Zq
            const double u = (double)uniforms[b * u_stride + i];
            keep = u * eq * row_z[i] < ep * row_z[K + 1 + i];
        }
        const unsigned long long failed = __ballot(!keep && (int)threadIdx.x < K);
        if (threadIdx.x == 0) s_a = failed ? __builtin_ctzll(failed) : K;
    }
    __syncthreads();
    const int a = s_a;
    const bool residual = a < K;
    const float* prow = trow0 + (size_t)a * V;            // a == K: the extra-token row
    const float* qrow = drow0 + (size_t)(residual ? a : 0) * V;
    const float mp = row_m[a];
    const double izp = 1.0 / row_z[a];
    const float mq = residual ? row_m[K + 1 + a] : 0.f;
    const double izq = residual ? 1.0 / row_z[K + 1 + a] : 0.0;

    const int base = chunk * RES_CHUNK;
    const int lim = min(RES_CHUNK, V - base);
    // all of a lane's logits are requested before the first is used (indices past the end clamped,
    // their terms dropped): one memory round trip instead of one per element
    constexpr int PER = RES_CHUNK / TPB;
    float lp[PER], lq[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) lp[k] = prow[base + min((int)threadIdx.x + k * TPB, lim - 1)];
    if (residual) {
#pragma unroll
        for (int k = 0; k < PER; ++k) lq[k] = qrow[base + min((int)threadIdx.x + k * TPB, lim - 1)];
    }
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        double pv = (double)__expf((lp[k] - mp) * inv_T_f) * izp;
        if (residual) {
            double qv = (double)__expf((lq[k] - mq) * inv_T_f) * izq;
            pv = pv > qv ? pv - qv : 0.0;
        }
        if ((int)threadIdx.x + k * TPB < lim) acc += pv;
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) ssum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        w.chunk_mass[(size_t)b * n_res_chunks + chunk] = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
        if (chunk == 0) {
            w.accepted[b] = a;
            w.row_max[2 * b] = mp;
            w.row_max[2 * b + 1] = mq;
            w.row_inv_z[2 * b] = izp;
            w.row_inv_z[2 * b + 1] = izq;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Pass 3: locate u*S among the chunk masses, scan that chunk in ascending token id, emit.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) final_draw_kernel(StepTables t, LookaheadPack ks, int Kmax, int V,
                                                         int n_res_chunks, const float* __restrict__ target,
                                                         const float* __restrict__ draft,
                                                         const int32_t* __restrict__ draft_tokens,
                                                         const float* __restrict__ uniforms, int u_stride,
                                                         float inv_T_f, SamplerWorkspace w, int auto_rollback,
                                                         int32_t* kv_len, int32_t* __restrict__ n_accepted,
                                                         int32_t* __restrict__ out_tokens, DrawEmit emit)
{
    __shared__ double r[RES_CHUNK];
    __shared__ double wave_tot[TPB / 64];
    __shared__ int s_chunk, s_tok;
    __shared__ double s_before, s_target;
    const int b = blockIdx.x;
    const int K = ks.k[b];
    if (!t.seq_ok[b]) {
        if (emit.tokens) {   // plain draw: an invalid id makes whoever consumes it skip the sequence too
            if (threadIdx.x == 0) {
                emit.tokens[b * emit.stride + emit.offset] = -1;
                emit.next_token[b] = -1;
            }
            return;
        }
        if (threadIdx.x == 0) n_accepted[b] = -1;
        for (int i = threadIdx.x; i <= Kmax; i += TPB) out_tokens[b * (Kmax + 1) + i] = -1;
        return;
    }
    const int a = w.accepted[b];
    bool residual = a < K;
    // the chunk masses, fetched by as many lanes at once and then walked by one from LDS
    __shared__ double s_mass[TPB];
    const double* mass = w.chunk_mass + (size_t)b * n_res_chunks;
    if (n_res_chunks <= TPB) {
        if ((int)threadIdx.x < n_res_chunks) s_mass[threadIdx.x] = mass[threadIdx.x];
        __syncthreads();
        mass = s_mass;
    }
    if (threadIdx.x == 0) {
        double S = 0.0;
        for (int c = 0; c < n_res_chunks; ++c) S += mass[c];
        // S > 0 always holds for the extra-token row; for a residual it holds in exact arithmetic
        // (a rejection means p(x) < q(x), so p exceeds q elsewhere).  S <= 0 falls back to p_a below.
        s_before = S;
        s_chunk = -1;
        if (S > 0.0) {
            const double target_mass = (double)uniforms[b * u_stride + K] * S;
            double c0 = 0.0;
            int pick = -1, last_pos = -1;
            double last_before = 0.0;
            for (int c = 0; c < n_res_chunks; ++c) {
                if (mass[c] > 0.0) { last_pos = c; last_before = c0; }
                if (c0 + mass[c] > target_mass) { pick = c; break; }
                c0 += mass[c];
            }
            if (pick < 0) { pick = last_pos; c0 = last_before; }
            s_chunk = pick;
            s_before = c0;
            s_target = target_mass;
        }
    }
    __syncthreads();
    const float* prow = target + (size_t)(t.seq_row0[b] + a) * V;
    const float* qrow = draft + ((size_t)b * Kmax + (residual ? a : 0)) * V;
    const float mp = w.row_max[2 * b], mq = w.row_max[2 * b + 1];
    const double izp = w.row_inv_z[2 * b], izq = w.row_inv_z[2 * b + 1];
    int c_lo = s_chunk, c_hi = s_chunk + 1;
    double before = s_before, target_mass = s_target;
    if (s_chunk < 0) {   // degenerate residual: draw from p_a over the whole vocabulary, chunk by chunk
        residual = false;
        c_lo = 0;
        c_hi = n_res_chunks;
        before = 0.0;
        target_mass = (double)uniforms[b * u_stride + K];   // p_a sums to 1
    }
    if (threadIdx.x == 0) s_tok = -1;
    int last_positive = -1;
    constexpr int PER = RES_CHUNK / TPB;   // 16 consecutive ids per lane
    for (int c = c_lo; c < c_hi; ++c) {
        const int base = c * RES_CHUNK;
        const int lim = min(RES_CHUNK, V - base);
        __syncthreads();
        {
            // all loads first (clamped), then the arithmetic: one memory round trip per chunk
            float lp[PER], lq[PER];
#pragma unroll
            for (int k = 0; k < PER; ++k) lp[k] = prow[base + min((int)threadIdx.x + k * TPB, lim - 1)];
            if (residual) {
#pragma unroll
                for (int k = 0; k < PER; ++k) lq[k] = qrow[base + min((int)threadIdx.x + k * TPB, lim - 1)];
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = threadIdx.x + k * TPB;
                double pv = (double)__expf((lp[k] - mp) * inv_T_f) * izp;
                if (residual) {
                    double qv = (double)__expf((lq[k] - mq) * inv_T_f) * izq;
                    pv = pv > qv ? pv - qv : 0.0;
                }
                r[i] = i < lim ? pv : 0.0;
            }
        }
        __syncthreads();
        // lane-local sums of 16 consecutive ids, then an inclusive scan over the 256 lanes
        double loc = 0.0;
        int my_last = -1;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            double x = r[threadIdx.x * PER + i];
            loc += x;
            if (x > 0.0) my_last = base + threadIdx.x * PER + i;
        }
        double inc = loc;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            double up = __shfl_up(inc, o);
            if ((int)(threadIdx.x & 63) >= o) inc += up;
        }
        if ((threadIdx.x & 63) == 63) wave_tot[threadIdx.x >> 6] = inc;
        __syncthreads();
        double off = before;
        for (int wv = 0; wv < (int)(threadIdx.x >> 6); ++wv) off += wave_tot[wv];
        inc += off;
        const double exc = inc - loc;
        // the lane whose range [exc, inc) the target mass falls in walks its ids
        if (inc > target_mass && !(exc > target_mass)) {
            double cdf = exc;
            int tok = -1;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                cdf += r[threadIdx.x * PER + i];
                if (tok < 0 && cdf > target_mass) tok = base + threadIdx.x * PER + i;
            }
            if (tok < 0) tok = my_last;   // rounding between the lane sum and the running sum
            if (tok >= 0) atomicMax(&s_tok, tok);
        }
        // remember the last id with positive mass in case rounding leaves no crossing at all
        int wl = my_last;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) wl = max(wl, __shfl_xor(wl, o));
        last_positive = max(last_positive, wl);
        __syncthreads();
        if (s_tok >= 0) break;
        before += (wave_tot[0] + wave_tot[1]) + (wave_tot[2] + wave_tot[3]);
    }
    __syncthreads();
    // cross-wave maximum of last_positive through LDS (reuse wave_tot storage as ints is not safe; use r)
    int* scratch = reinterpret_cast<int*>(r);
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = last_positive;
    __syncthreads();
    if (threadIdx.x == 0) {
        int y = s_tok;
        if (y < 0) y = max(max(scratch[0], scratch[1]), max(scratch[2], scratch[3]));
        if (y < 0) y = 0;
        if (emit.tokens) {
            emit.tokens[b * emit.stride + emit.offset] = y;
            emit.next_token[b] = y;
            if (emit.kv_len) emit.kv_len[t.seq_slot[b]] = t.seq_n[b] + emit.kv_add;
            return;
        }
        n_accepted[b] = a;
        int32_t* o = out_tokens + b * (Kmax + 1);
        for (int i = 0; i < a; ++i) o[i] = draft_tokens[b * Kmax + i];
        o[a] = y;
        for (int i = a + 1; i <= Kmax; ++i) o[i] = -1;
        if (kv_len) {
            kv_len[t.seq_slot[b]] = t.seq_n[b] + (auto_rollback ? a : K) + 1;
            pool_trim(t.pool, t.seq_slot[b], t.seq_n[b] + (auto_rollback ? a : K) + 1);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Temperature 0.  Pass 1: per (target row, chunk) the maximum and the lowest id that holds it.
// Pass 2 (one wavefront per sequence): combine the chunks of each window row in ascending order,
// compare with the proposals, emit.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) argmax_kernel(int V, int n_chunks, const float* __restrict__ target,
                                                     float* __restrict__ part_max, int32_t* __restrict__ part_idx)
{
    __shared__ float sv[TPB / 64];
    __shared__ int si[TPB / 64];
    const int row = blockIdx.x / n_chunks, chunk = blockIdx.x % n_chunks;
    const float* p = target + (size_t)row * V;
    const int base = chunk * STAT_CHUNK;
    const int lim = min(STAT_CHUNK, V - base);
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < lim; i += TPB) {   // ascending ids per thread: '>' keeps the first maximum
        const float x = p[base + i];
        if (x > best || bi == 0x7fffffff) {
            best = x;
            bi = base + i;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o);
        const int oi = __shfl_xor(bi, o);
        if (ob > best || (ob == best && oi < bi)) {
            best = ob;
            bi = oi;
        }
    }
    if ((threadIdx.x & 63) == 0) {
        sv[threadIdx.x >> 6] = best;
        si[threadIdx.x >> 6] = bi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < TPB / 64; ++w)
            if (sv[w] > best || (sv[w] == best && si[w] < bi)) {
                best = sv[w];
                bi = si[w];
            }
        part_max[(size_t)row * n_chunks + chunk] = best;
        part_idx[(size_t)row * n_chunks + chunk] = bi;
    }
}

__global__ void __launch_bounds__(64) greedy_emit_kernel(StepTables t, LookaheadPack ks, int Kmax, int n_chunks,
                                                         const float* __restrict__ part_max,
                                                         const int32_t* __restrict__ part_idx,
                                                         const int32_t* __restrict__ draft_tokens, int auto_rollback,
                                                         int32_t* kv_len, int32_t* __restrict__ n_accepted,
                                                         int32_t* __restrict__ out_tokens, DrawEmit emit)
{
    const int b = blockIdx.x;
    if (threadIdx.x != 0) return;
    if (emit.tokens) {   // a proposing model's step (every K_b = 0): the most likely token of the sequence's row
        int y = -1;
        if (t.seq_ok[b]) {
            const size_t r = (size_t)t.seq_row0[b] * n_chunks;
            float best = part_max[r];
            y = part_idx[r];
            for (int c = 1; c < n_chunks; ++c)
                if (part_max[r + c] > best) {
                    best = part_max[r + c];
                    y = part_idx[r + c];
                }
            if (emit.kv_len) emit.kv_len[t.seq_slot[b]] = t.seq_n[b] + emit.kv_add;
        }
        emit.tokens[b * emit.stride + emit.offset] = y;
        emit.next_token[b] = y;
        return;
    }
    int32_t* o = out_tokens + b * (Kmax + 1);
    if (!t.seq_ok[b]) {
        n_accepted[b] = -1;
        for (int i = 0; i <= Kmax; ++i) o[i] = -1;
        return;
    }
    const int K = ks.k[b];
    int a = 0;
    for (int j = 0; j <= K; ++j) {
        const size_t r = (size_t)(t.seq_row0[b] + j) * n_chunks;
        float best = part_max[r];
        int bi = part_idx[r];
        for (int c = 1; c < n_chunks; ++c)
            if (part_max[r + c] > best) {   // chunks ascend in id: a later equal maximum does not win
                best = part_max[r + c];
                bi = part_idx[r + c];
            }
        if (j < K && draft_tokens[b * Kmax + j] == bi) {
            o[a++] = bi;
            continue;
        }
        o[a] = bi;
        break;
    }
    for (int i = a + 1; i <= Kmax; ++i) o[i] = -1;
    n_accepted[b] = a;
    if (kv_len) {
        kv_len[t.seq_slot[b]] = t.seq_n[b] + (auto_rollback ? a : K) + 1;
        pool_trim(t.pool, t.seq_slot[b], t.seq_n[b] + (auto_rollback ? a : K) + 1);
    }
}

// Temperature 0 on a tree: from the root, move to the first child (index order) whose token is the
// most likely token of the current node's row; otherwise that token ends the step.
__global__ void __launch_bounds__(64) tree_greedy_kernel(StepTables t, LookaheadPack ks, int Kmax, int n_chunks,
                                                         const float* __restrict__ part_max,
                                                         const int32_t* __restrict__ part_idx,
                                                         const int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ tokens, int auto_rollback,
                                                         int32_t* kv_len, int32_t* __restrict__ n_accepted,
                                                         int32_t* __restrict__ out_tokens, int32_t* __restrict__ path)
{
    const int b = blockIdx.x;
    if (threadIdx.x != 0) return;
    int32_t* o = out_tokens + b * (Kmax + 1);
    int32_t* pth = path + b * Kmax;
    if (!t.seq_ok[b]) {
        n_accepted[b] = -1;
        for (int i = 0; i <= Kmax; ++i) o[i] = -1;
        for (int i = 0; i < Kmax; ++i) pth[i] = -1;
        return;
    }
    const int N = ks.k[b];
    int cur = -1, a = 0;
    for (;;) {
        const size_t r = (size_t)(t.seq_row0[b] + cur + 1) * n_chunks;
        float best = part_max[r];
        int bi = part_idx[r];
        for (int c = 1; c < n_chunks; ++c)
            if (part_max[r + c] > best) {
                best = part_max[r + c];
                bi = part_idx[r + c];
            }
        int next = -1;
        for (int c = cur + 1; c < N; ++c)
            if (parent[b * Kmax + c] == cur && tokens[b * Kmax + c] == bi) { next = c; break; }
        o[a] = bi;
        if (next < 0) break;
        pth[a++] = next;
        cur = next;
    }
    for (int i = a + 1; i <= Kmax; ++i) o[i] = -1;
    for (int i = a; i < Kmax; ++i) pth[i] = -1;
    n_accepted[b] = a;
    if (kv_len) {
        // with auto_rollback the kept path is still to be moved: its pages go back after that
        // (tree_trim_kernel), never here
        kv_len[t.seq_slot[b]] = t.seq_n[b] + (auto_rollback ? a : N) + 1;
        if (!auto_rollback) pool_trim(t.pool, t.seq_slot[b], t.seq_n[b] + N + 1);
    }
}

// ---------------------------------------------------------------------------------------------
// Token trees.  Window slot 0 is the sequence's last token (the root), slot i+1 is node i; the
// nodes come in topological order with parent[i] = -1 (child of the root) or an index < i.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) prepare_tree_kernel(StepTables t, LookaheadPack ks, int B, int Kmax, int V,
                                                           int max_batch, int max_kv_len, int has_cache,
                                                           const int32_t* __restrict__ seq_slot,
                                                           const int32_t* __restrict__ last_token,
                                                           const int32_t* __restrict__ parent,
                                                           const int32_t* __restrict__ tokens,
                                                           const int32_t* __restrict__ kv_len, int32_t* flag)
{
    __shared__ int row0[SPEC_MAX_BATCH + 1];
    const int b = threadIdx.x;
    if (b == 0) {
        int r = 0, st = 0;
        for (int i = 0; i < B; ++i) {
            row0[i] = r;
            t.seq_row0[i] = r;
            t.seq_stat0[i] = st;
            r += ks.k[i] + 1;
            st += 2 * ks.k[i] + 2;   // target and draft row of the root and of every node
        }
        row0[B] = r;
        t.seq_row0[B] = r;
        t.seq_stat0[B] = st;
    }
    __syncthreads();
    if (b >= B) return;
    const int N = ks.k[b];
    int ok = 1, err = 0;
    int slot = b, n = 0;
    if (has_cache) {
        slot = seq_slot[b];
        if (slot < 0 || slot >= max_batch) {
            ok = 0;
            err = SPEC_ERR_INVALID_ARG;
            slot = 0;
        } else {
            for (int i = 0; i < b; ++i)
                if (seq_slot[i] == slot) { ok = 0; err = SPEC_ERR_INVALID_ARG; }
            n = kv_len[slot];
            if (n < 0 || n + N + 1 > max_kv_len) { ok = 0; err = SPEC_ERR_KV_OVERFLOW; }
            else if (ok && !pool_cover(t.pool, slot, n, n + N + 1)) { ok = 0; err = SPEC_ERR_KV_OVERFLOW; }
        }
    }
    const int t0 = last_token ? last_token[b] : 0;
    if (t0 < 0 || t0 >= V) { ok = 0; err = SPEC_ERR_TOKEN_RANGE; }
    for (int i = 0; i < N; ++i) {
        const int x = tokens[b * Kmax + i], p = parent[b * Kmax + i];
        if (x < 0 || x >= V) { ok = 0; err = SPEC_ERR_TOKEN_RANGE; }
        if (p < -1 || p >= i) { ok = 0; err = SPEC_ERR_INVALID_ARG; }
    }
    if (!ok) atomicCAS(flag, 0, err);
    t.seq_n[b] = ok ? n : 0;
    t.seq_ok[b] = ok;
    t.seq_slot[b] = slot;
    // slot j: depth and the set of slots on its path (itself included)
    int depth[SPEC_MAX_LOOKAHEAD + 1];
    uint32_t mask[SPEC_MAX_LOOKAHEAD + 1];
    depth[0] = 0;
    mask[0] = 1u;
    for (int j = 0; j <= N; ++j) {
        if (j > 0) {
            const int ps = ok ? parent[b * Kmax + j - 1] + 1 : 0;   // parent's slot
            depth[j] = depth[ps] + 1;
            mask[j] = mask[ps] | (1u << j);
        }
        const int r = row0[b] + j;
        t.row_seq[r] = b;
        t.row_pos[r] = ok ? n + j : -1;
        t.row_rope[r] = ok ? n + depth[j] : 0;
        t.row_mask[r] = mask[j];
        const int tok = (j == 0) ? t0 : tokens[b * Kmax + j - 1];
        t.row_tok[r] = ok ? tok : 0;
    }
}

constexpr int TREE_TPB = 1024;   // the walk is one workgroup per sequence: make it a big one

struct TreeOut {
    int32_t* n_accepted;   // [B]
    int32_t* out_tokens;   // [B][Kmax+1]
    int32_t* path;         // [B][Kmax] kept node indices root-down, then -1
};

// The walk of one sequence's tree (one workgroup).  At the current node r starts as the target
// distribution p; a child with token x is kept iff u * q(x) < r(x); every rejection replaces r by
// max(0, r - q) renormalised.  r is never materialised: r_k(v) is recomputed from p(v), q(v) and the
// masses S_1..S_k of the earlier levels, so a rejection costs one pass over the two logits rows.
__global__ void __launch_bounds__(TREE_TPB) tree_walk_kernel(StepTables t, LookaheadPack ks, int Kmax, int V,
                                                        int n_stat_chunks, const float* __restrict__ target,
                                                        const float* __restrict__ draft,
                                                        const int32_t* __restrict__ parent,
                                                        const int32_t* __restrict__ tokens,
                                                        const float* __restrict__ uniforms, float inv_T_f,
                                                        const float* __restrict__ part_max,
                                                        const double* __restrict__ part_sum, int auto_rollback,
                                                        int32_t* kv_len, TreeOut out)
{
    constexpr int MAXN = SPEC_MAX_LOOKAHEAD;
    __shared__ float row_m[2 * MAXN + 2];
    __shared__ double row_z[2 * MAXN + 2];
    __shared__ double level_S[MAXN + 1];     // level_S[k]: mass of the unnormalised r_k, k >= 1
    __shared__ double wsum[TREE_TPB / 64];
    __shared__ double r[RES_CHUNK];
    __shared__ int s_tok, s_chunk;
    __shared__ double s_val, s_before, s_target;
    const int b = blockIdx.x;
    const int N = ks.k[b];
    if (!t.seq_ok[b]) {
        if (threadIdx.x == 0) out.n_accepted[b] = -1;
        for (int i = threadIdx.x; i <= Kmax; i += TREE_TPB) out.out_tokens[b * (Kmax + 1) + i] = -1;
        for (int i = threadIdx.x; i < Kmax; i += TREE_TPB) out.path[b * Kmax + i] = -1;
        return;
    }
    const double inv_T = (double)inv_T_f;
    const int st0 = t.seq_stat0[b];
    if ((int)threadIdx.x < 2 * N + 2)
        combine_row(part_max + (size_t)(st0 + threadIdx.x) * n_stat_chunks,
                    part_sum + (size_t)(st0 + threadIdx.x) * n_stat_chunks, n_stat_chunks, inv_T,
                    &row_m[threadIdx.x], &row_z[threadIdx.x]);
    __syncthreads();
    const float* trow0 = target + (size_t)t.seq_row0[b] * V;
    const float* drow0 = draft + (size_t)b * (Kmax + 1) * V;
    const int32_t* par = parent + b * Kmax;
    const int32_t* tok = tokens + b * Kmax;

    int cur = -1, level = 0, a = 0;
    const float* prow = trow0;
    const float* qrow = drow0;
    float mp = row_m[0], mq = row_m[N + 1];
    double izp = 1.0 / row_z[0], izq = 1.0 / row_z[N + 1];
    // r_level(v) from the two rows (level and the masses are uniform over the workgroup)
    auto resid = [&](float lp, float lq, int lev) -> double {
        double pv = (double)__expf((lp - mp) * inv_T_f) * izp;
        if (lev > 0) {
            const double qv = (double)__expf((lq - mq) * inv_T_f) * izq;
            pv = pv > qv ? pv - qv : 0.0;
            for (int k = 1; k < lev; ++k) {
                pv = pv / level_S[k];
                pv = pv > qv ? pv - qv : 0.0;
            }
        }
        return pv;
    };
    auto block_sum = [&](double v) -> double {
        v = wave_sum(v);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
        __syncthreads();
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < TREE_TPB / 64; ++w) tot += wsum[w];   // fixed order
        return tot;
    };

    // What the test of node c needs from memory does not depend on the walk (a node is always tested
    // against its parent's rows): lane c fetches it for all nodes at once, and every thread then
    // takes the same decisions from LDS -- no load and no barrier per tested node.
    __shared__ int s_par[MAXN], s_ntok[MAXN];
    __shared__ double s_ep[MAXN], s_eq[MAXN], s_u[MAXN];
    if ((int)threadIdx.x < N) {
        const int c = threadIdx.x;
        const int pr = par[c] + 1;                 // row of the parent (0: the root)
        const int x = tok[c];
        s_par[c] = par[c];
        s_ntok[c] = x;
        s_u[c] = (double)uniforms[b * (Kmax + 1) + c];
        s_ep[c] = exp((double)(trow0[(size_t)pr * V + x] - row_m[pr]) * inv_T);
        s_eq[c] = exp((double)(drow0[(size_t)pr * V + x] - row_m[N + 1 + pr]) * inv_T);
    }
    __syncthreads();

    for (int c = 0; c < N; ++c) {
        if (s_par[c] != cur) continue;
        bool keep;
        {
            const double u = s_u[c], ep = s_ep[c], eq = s_eq[c];
            if (level == 0) {
                keep = u * eq * row_z[cur + 1] < ep * row_z[N + 1 + cur + 1];   // u q(x) < p(x), division-free
            } else {
                const double qx = eq * izq;
                double rx = ep * izp;
                rx = rx > qx ? rx - qx : 0.0;
                for (int k = 1; k < level; ++k) {
                    rx = rx / level_S[k];
                    rx = rx > qx ? rx - qx : 0.0;
                }
                keep = u * qx * level_S[level] < rx;   // u q(x) < r(x) / S
            }
        }
        if (keep) {
            if (threadIdx.x == 0) {
                out.path[b * Kmax + a] = c;
                out.out_tokens[b * (Kmax + 1) + a] = s_ntok[c];
            }
            ++a;
            cur = c;
            level = 0;
            prow = trow0 + (size_t)(c + 1) * V;
            qrow = drow0 + (size_t)(c + 1) * V;
            mp = row_m[c + 1];
            mq = row_m[N + 1 + c + 1];
            izp = 1.0 / row_z[c + 1];
            izq = 1.0 / row_z[N + 1 + c + 1];
            continue;
        }
        // rejected: mass of max(0, r/S - q)
        double acc = 0.0;
        const double div = level > 0 ? level_S[level] : 1.0;
        for (int v0 = threadIdx.x; v0 < V; v0 += 8 * TREE_TPB) {
            // eight elements per trip, loads first (indices past the end clamped, their terms dropped)
            float lpv[8], lqv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int v = min(v0 + k * TREE_TPB, V - 1);
                lpv[k] = prow[v];
                lqv[k] = qrow[v];
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                double pv = resid(lpv[k], lqv[k], level);
                if (level > 0) pv = pv / div;
                const double qv = (double)__expf((lqv[k] - mq) * inv_T_f) * izq;
                if (v0 + k * TREE_TPB < V) acc += pv > qv ? pv - qv : 0.0;
            }
        }
        const double S_new = block_sum(acc);
        if (S_new > 0.0) {   // <= 0 cannot happen in exact arithmetic; then r stays as it is
            if (threadIdx.x == 0) level_S[level + 1] = S_new;
            ++level;
        }
        __syncthreads();
    }

    // final draw from r_level of the current node: chunk masses, then a scan inside one chunk
    const int n_res_chunks = (V + RES_CHUNK - 1) / RES_CHUNK;
    constexpr int PER = RES_CHUNK / TREE_TPB;
    double total = 0.0;   // meaningful in thread 0
    __shared__ double mass[64];
    for (int c0 = 0; c0 < n_res_chunks; c0 += 64) {
        for (int cc = c0; cc < min(c0 + 64, n_res_chunks); ++cc) {
            const int base = cc * RES_CHUNK;
            const int lim = min(RES_CHUNK, V - base);
            double acc = 0.0;
            {
                float lpv[PER], lqv[PER];
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    const int i = min((int)threadIdx.x + k * TREE_TPB, lim - 1);
                    lpv[k] = prow[base + i];
                    lqv[k] = qrow[base + i];
                }
#pragma unroll
                for (int k = 0; k < PER; ++k)
                    if ((int)threadIdx.x + k * TREE_TPB < lim) acc += resid(lpv[k], lqv[k], level);
            }
            const double m = block_sum(acc);
            if (threadIdx.x == 0) mass[cc - c0] = m;
        }
        __syncthreads();
        if (threadIdx.x == 0)
            for (int cc = c0; cc < min(c0 + 64, n_res_chunks); ++cc) total += mass[cc - c0];
        if (n_res_chunks > 64) __syncthreads();
    }
    // (vocabularies beyond 64 chunks of 4096 would need the masses kept in global memory; the
    // launch wrapper rejects them)
    if (threadIdx.x == 0) {
        const double target_mass = (double)uniforms[b * (Kmax + 1) + N] * total;
        double c0 = 0.0, last_before = 0.0;
        int pick = -1, last_pos = -1;
        for (int cc = 0; cc < n_res_chunks; ++cc) {
            if (mass[cc] > 0.0) { last_pos = cc; last_before = c0; }
            if (c0 + mass[cc] > target_mass) { pick = cc; break; }
            c0 += mass[cc];
        }
        if (pick < 0) { pick = last_pos; c0 = last_before; }
        if (pick < 0) { pick = 0; c0 = 0.0; }
        s_chunk = pick;
        s_before = c0;
        s_target = target_mass;
        s_tok = -1;
    }
    __syncthreads();
    {
        const int base = s_chunk * RES_CHUNK;
        const int lim = min(RES_CHUNK, V - base);
        const double before = s_before, target_mass = s_target;
        {
            float lpv[PER], lqv[PER];
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = min((int)threadIdx.x + k * TREE_TPB, lim - 1);
                lpv[k] = prow[base + i];
                lqv[k] = qrow[base + i];
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int i = threadIdx.x + k * TREE_TPB;
                r[i] = i < lim ? resid(lpv[k], lqv[k], level) : 0.0;
            }
        }
        __syncthreads();
        double loc = 0.0;
        int my_last = -1;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const double x = r[threadIdx.x * PER + i];
            loc += x;
            if (x > 0.0) my_last = base + threadIdx.x * PER + i;
        }
        double inc = loc;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(inc, o);
            if ((int)(threadIdx.x & 63) >= o) inc += up;
        }
        if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
        __syncthreads();
        double off = before;
        for (int wv = 0; wv < (int)(threadIdx.x >> 6); ++wv) off += wsum[wv];
        inc += off;
        const double exc = inc - loc;
        if (inc > target_mass && !(exc > target_mass)) {
            double cdf = exc;
            int y = -1;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                cdf += r[threadIdx.x * PER + i];
                if (y < 0 && cdf > target_mass) y = base + threadIdx.x * PER + i;
            }
            if (y < 0) y = my_last;
            if (y >= 0) atomicMax(&s_tok, y);
        }
        int wl = my_last;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) wl = max(wl, __shfl_xor(wl, o));
        __syncthreads();
        int* scratch = reinterpret_cast<int*>(wsum);
        if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = wl;
        __syncthreads();
        if (threadIdx.x == 0) {
            int y = s_tok;
            if (y < 0)
                for (int w = 0; w < TREE_TPB / 64; ++w) y = max(y, scratch[w]);
            if (y < 0) y = 0;
            out.n_accepted[b] = a;
            int32_t* o = out.out_tokens + b * (Kmax + 1);
            o[a] = y;
            for (int i = a + 1; i <= Kmax; ++i) o[i] = -1;
            for (int i = a; i < Kmax; ++i) out.path[b * Kmax + i] = -1;
            if (kv_len) {
                // with auto_rollback the kept path is still to be moved: its pages go back after
                // that (tree_trim_kernel), never here
                kv_len[t.seq_slot[b]] = t.seq_n[b] + (auto_rollback ? a : N) + 1;
                if (!auto_rollback) pool_trim(t.pool, t.seq_slot[b], t.seq_n[b] + N + 1);
            }
        }
    }
}

// kv_len[slot] = len where 0 <= len <= kv_len[slot]; anything else leaves the slot alone and flags.
__global__ void __launch_bounds__(TPB) rollback_kernel(RollbackPack p, int n, int max_batch, int32_t* kv_len,
                                                       int32_t* flag, PagePool pool)
{
    const int i = threadIdx.x;
    if (i >= n) return;
    const int slot = p.slot[i], len = p.len[i];
    if (slot < 0 || slot >= max_batch) { atomicCAS(flag, 0, (int)SPEC_ERR_INVALID_ARG); return; }
    if (len < 0 || len > kv_len[slot]) { atomicCAS(flag, 0, (int)SPEC_ERR_ROLLBACK); return; }
    kv_len[slot] = len;
    pool_trim(pool, slot, len);
}

// Paged cache, after a tree step's compaction: hand back the pages beyond the new length.  The walk
// cannot do it: a kept node's keys and values may still sit in a block above n + a + 1 until
// kv_compact_kernel has moved them (n = 28, kept node in window slot 4: position 32 is in the
// second block, the new length 30 needs the first only).
__global__ void __launch_bounds__(TPB) tree_trim_kernel(StepTables t, int B, const int32_t* __restrict__ n_accepted)
{
    const int b = threadIdx.x;
    if (b >= B || !t.seq_ok[b]) return;
    const int a = n_accepted[b];
    if (a >= 0) pool_trim(t.pool, t.seq_slot[b], t.seq_n[b] + a + 1);
}

__global__ void pool_cover_kernel(PagePool pool, int slot, int pos0, int pos1, int32_t* flag)
{
    if (threadIdx.x == 0 && blockIdx.x == 0 && !pool_cover(pool, slot, pos0, pos1)) atomicCAS(flag, 0, (int)SPEC_ERR_KV_OVERFLOW);
}

}  // namespace

int launch_prepare(const StepTables& t, const LookaheadPack& ks, int B, int Kmax, int V, int max_batch,
                   int max_kv_len, bool has_cache, const int32_t* seq_slot, const int32_t* last_token,
                   const int32_t* draft_tokens, const int32_t* kv_len, int32_t* flag, hipStream_t s)
{
    hipLaunchKernelGGL(prepare_kernel, dim3(1), dim3(TPB), 0, s, t, ks, B, Kmax, V, max_batch, max_kv_len,
                       has_cache ? 1 : 0, seq_slot, last_token, draft_tokens, kv_len, flag);
    SPECV_LAUNCH_CHECK("prepare_kernel");
    return SPEC_OK;
}

int launch_greedy(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax, int V,
                  int M, const float* target_logits, const int32_t* draft_tokens, int auto_rollback, int32_t* kv_len,
                  int32_t* n_accepted, int32_t* out_tokens, const DrawEmit* emit, Profiler* prof, hipStream_t s)
{
    DrawEmit em{};
    if (emit) em = *emit;
    const int n_chunks = (V + STAT_CHUNK - 1) / STAT_CHUNK;
    {
        ProfScope ps(prof, SPEC_PROF_SAMPLER_STATS, s);
        hipLaunchKernelGGL(argmax_kernel, dim3((unsigned)M * n_chunks), dim3(TPB), 0, s, V, n_chunks, target_logits,
                           w.part_max, w.part_idx);
        SPECV_LAUNCH_CHECK("argmax_kernel");
    }
    ProfScope ps(prof, SPEC_PROF_SAMPLER_DRAW, s);
    hipLaunchKernelGGL(greedy_emit_kernel, dim3(B), dim3(64), 0, s, t, ks, Kmax, n_chunks, w.part_max, w.part_idx,
                       draft_tokens, auto_rollback, kv_len, n_accepted, out_tokens, em);
    SPECV_LAUNCH_CHECK("greedy_emit_kernel");
    return SPEC_OK;
}

int launch_tree_greedy(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax, int V,
                       int M, const float* target_logits, const int32_t* parent, const int32_t* tokens,
                       int auto_rollback, int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens, int32_t* path,
                       Profiler* prof, hipStream_t s)
{
    const int n_chunks = (V + STAT_CHUNK - 1) / STAT_CHUNK;
    {
        ProfScope ps(prof, SPEC_PROF_SAMPLER_STATS, s);
        hipLaunchKernelGGL(argmax_kernel, dim3((unsigned)M * n_chunks), dim3(TPB), 0, s, V, n_chunks, target_logits,
                           w.part_max, w.part_idx);
        SPECV_LAUNCH_CHECK("argmax_kernel");
    }
    ProfScope ps(prof, SPEC_PROF_SAMPLER_DRAW, s);
    hipLaunchKernelGGL(tree_greedy_kernel, dim3(B), dim3(64), 0, s, t, ks, Kmax, n_chunks, w.part_max, w.part_idx,
                       parent, tokens, auto_rollback, kv_len, n_accepted, out_tokens, path);
    SPECV_LAUNCH_CHECK("tree_greedy_kernel");
    return SPEC_OK;
}

int launch_prepare_tree(const StepTables& t, const LookaheadPack& ks, int B, int Kmax, int V, int max_batch,
                        int max_kv_len, bool has_cache, const int32_t* seq_slot, const int32_t* last_token,
                        const int32_t* parent, const int32_t* tokens, const int32_t* kv_len, int32_t* flag,
                        hipStream_t s)
{
    hipLaunchKernelGGL(prepare_tree_kernel, dim3(1), dim3(TPB), 0, s, t, ks, B, Kmax, V, max_batch, max_kv_len,
                       has_cache ? 1 : 0, seq_slot, last_token, parent, tokens, kv_len, flag);
    SPECV_LAUNCH_CHECK("prepare_tree_kernel");
    return SPEC_OK;
}

int launch_tree_sampler(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax,
                        int V, int n_stat_rows, const float* target_logits, const float* draft_logits,
                        const int32_t* parent, const int32_t* tokens, const float* uniforms, float temperature,
                        int auto_rollback, int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens,
                        int32_t* path, Profiler* prof, hipStream_t s)
{
    const int n_stat_chunks = (V + STAT_CHUNK - 1) / STAT_CHUNK;
    if ((V + RES_CHUNK - 1) / RES_CHUNK > 64)
        return fail(SPEC_ERR_SHAPE, "tree verification supports vocabularies up to %d", 64 * RES_CHUNK);
    const float inv_T = 1.0f / temperature;
    const bool vec4 = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(target_logits) & 15) == 0)
                      && ((reinterpret_cast<uintptr_t>(draft_logits) & 15) == 0);
    dim3 g1((unsigned)n_stat_rows * n_stat_chunks);
    {
        ProfScope ps(prof, SPEC_PROF_SAMPLER_STATS, s);
        if (vec4)
            hipLaunchKernelGGL(stats_kernel<true>, g1, dim3(TPB), 0, s, t, ks, B, Kmax + 1, V, n_stat_chunks,
                               target_logits, draft_logits, inv_T, w.part_max, w.part_sum, (float*)nullptr, (size_t)0,
                               (int)STAT_TREE, PrepIn{});
        else
            hipLaunchKernelGGL(stats_kernel<false>, g1, dim3(TPB), 0, s, t, ks, B, Kmax + 1, V, n_stat_chunks,
                               target_logits, draft_logits, inv_T, w.part_max, w.part_sum, (float*)nullptr, (size_t)0,
                               (int)STAT_TREE, PrepIn{});
        SPECV_LAUNCH_CHECK("stats_kernel");
    }
    ProfScope ps(prof, SPEC_PROF_SAMPLER_DRAW, s);
    TreeOut o{n_accepted, out_tokens, path};
    hipLaunchKernelGGL(tree_walk_kernel, dim3(B), dim3(TREE_TPB), 0, s, t, ks, Kmax, V, n_stat_chunks, target_logits,
                       draft_logits, parent, tokens, uniforms, inv_T, w.part_max, w.part_sum, auto_rollback, kv_len, o);
    SPECV_LAUNCH_CHECK("tree_walk_kernel");
    return SPEC_OK;
}

int launch_rollback(const RollbackPack& p, int n, int max_batch, int32_t* kv_len, int32_t* flag, const PagePool& pool,
                    hipStream_t s)
{
    hipLaunchKernelGGL(rollback_kernel, dim3(1), dim3(TPB), 0, s, p, n, max_batch, kv_len, flag, pool);
    SPECV_LAUNCH_CHECK("rollback_kernel");
    return SPEC_OK;
}

int launch_slice_tables(const StepTables& full, const StepTables& sub, int b0, int Bg, hipStream_t s)
{
    hipLaunchKernelGGL(slice_tables_kernel, dim3(1), dim3(TPB), 0, s, full, sub, b0, Bg);
    SPECV_LAUNCH_CHECK("slice_tables_kernel");
    return SPEC_OK;
}

int launch_tree_trim(const StepTables& t, int B, const int32_t* n_accepted, hipStream_t s)
{
    if (!t.pool.table) return SPEC_OK;
    hipLaunchKernelGGL(tree_trim_kernel, dim3(1), dim3(TPB), 0, s, t, B, n_accepted);
    SPECV_LAUNCH_CHECK("tree_trim_kernel");
    return SPEC_OK;
}

int launch_pool_cover(const PagePool& pool, int slot, int pos0, int pos1, int32_t* flag, hipStream_t s)
{
    if (!pool.table) return SPEC_OK;
    hipLaunchKernelGGL(pool_cover_kernel, dim3(1), dim3(64), 0, s, pool, slot, pos0, pos1, flag);
    SPECV_LAUNCH_CHECK("pool_cover_kernel");
    return SPEC_OK;
}

int launch_sampler(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax,
                   int V, int n_stat_rows, const float* target_logits, const float* draft_logits,
                   const int32_t* draft_tokens, const float* uniforms, int u_stride, float temperature,
                   int auto_rollback, int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens,
                   const DrawEmit* emit, Profiler* prof, hipStream_t s, int32_t* prepare_flag)
{
    const int n_stat_chunks = (V + STAT_CHUNK - 1) / STAT_CHUNK;
    const int n_res_chunks = (V + RES_CHUNK - 1) / RES_CHUNK;
    const float inv_T = 1.0f / temperature;
    PrepIn prep{};
    if (prepare_flag) {   // no decoder pass ran: the statistics pass fills the row tables itself
        prep.on = 1;
        prep.Kmax = Kmax;
        prep.draft_tokens = draft_tokens;
        prep.flag = prepare_flag;
    }
    const int layout = emit ? (int)STAT_PLAIN : (int)STAT_CHAIN;
    DrawEmit em{};
    if (emit) {
        if (n_stat_rows != B) return fail(SPEC_ERR_INVALID_ARG, "a plain draw needs every lookahead to be 0");
        em = *emit;
    }
    const bool vec4 = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(target_logits) & 15) == 0)
                      && ((reinterpret_cast<uintptr_t>(draft_logits) & 15) == 0)
                      && ((reinterpret_cast<uintptr_t>(em.logits_copy) & 15) == 0) && (em.copy_stride % 4 == 0);
    dim3 g1((unsigned)n_stat_rows * n_stat_chunks);
    {
    ProfScope ps(prof, SPEC_PROF_SAMPLER_STATS, s);
    if (vec4)
        hipLaunchKernelGGL(stats_kernel<true>, g1, dim3(TPB), 0, s, t, ks, B, Kmax, V, n_stat_chunks,
                           target_logits, draft_logits, inv_T, w.part_max, w.part_sum, em.logits_copy, em.copy_stride,
                           layout, prep);
    else
        hipLaunchKernelGGL(stats_kernel<false>, g1, dim3(TPB), 0, s, t, ks, B, Kmax, V, n_stat_chunks,
                           target_logits, draft_logits, inv_T, w.part_max, w.part_sum, em.logits_copy, em.copy_stride,
                           layout, prep);
    SPECV_LAUNCH_CHECK("stats_kernel");
    }
    ProfScope ps(prof, SPEC_PROF_SAMPLER_DRAW, s);
    hipLaunchKernelGGL(accept_mass_kernel, dim3(n_res_chunks, B), dim3(TPB), 0, s, t, ks, Kmax, V, n_stat_chunks,
                       n_res_chunks, target_logits, draft_logits, draft_tokens, uniforms, u_stride, inv_T, w.part_max,
                       w.part_sum, w);
    SPECV_LAUNCH_CHECK("accept_mass_kernel");
    hipLaunchKernelGGL(final_draw_kernel, dim3(B), dim3(TPB), 0, s, t, ks, Kmax, V, n_res_chunks, target_logits,
                       draft_logits, draft_tokens, uniforms, u_stride, inv_T, w, auto_rollback, kv_len, n_accepted,
                       out_tokens, em);
    SPECV_LAUNCH_CHECK("final_draw_kernel");
    return SPEC_OK;
}

}  // namespace specv

// ---------------------------------------------------------------------------------------------
// The sampling part of the verify step for callers that cannot allocate: no handle, no hipMalloc.
// The row tables and the sampler's workspace (chunk statistics, chunk masses, per-sequence
// scalars, the error flag) live in one device array of fixed size instead of a handle's arena.
// ---------------------------------------------------------------------------------------------
namespace specv {
namespace {

constexpr int NA_MAX_BATCH = SPEC_NOALLOC_MAX_BATCH;
constexpr int NA_MAX_VOCAB = SPEC_NOALLOC_MAX_VOCAB;
constexpr int NA_MAX_ROWS = NA_MAX_BATCH * (SPEC_MAX_LOOKAHEAD + 1);
constexpr int NA_MAX_STAT = NA_MAX_BATCH * (2 * SPEC_MAX_LOOKAHEAD + 1);
constexpr int NA_STAT_CHUNKS = (NA_MAX_VOCAB + STAT_CHUNK - 1) / STAT_CHUNK;
constexpr int NA_RES_CHUNKS = (NA_MAX_VOCAB + RES_CHUNK - 1) / RES_CHUNK;

struct NoAllocScratch {
    double part_sum[(size_t)NA_MAX_STAT * NA_STAT_CHUNKS];
    double chunk_mass[(size_t)NA_MAX_BATCH * NA_RES_CHUNKS];
    double row_inv_z[2 * NA_MAX_BATCH];
    float part_max[(size_t)NA_MAX_STAT * NA_STAT_CHUNKS];
    int32_t part_idx[(size_t)NA_MAX_STAT * NA_STAT_CHUNKS];
    float row_max[2 * NA_MAX_BATCH];
    int32_t accepted[NA_MAX_BATCH];
    int32_t seq_row0[NA_MAX_BATCH + 1], seq_stat0[NA_MAX_BATCH + 1];
    int32_t seq_n[NA_MAX_BATCH], seq_ok[NA_MAX_BATCH], seq_slot[NA_MAX_BATCH];
    int32_t row_seq[NA_MAX_ROWS], row_pos[NA_MAX_ROWS], row_tok[NA_MAX_ROWS], row_rope[NA_MAX_ROWS];
    uint32_t row_mask[NA_MAX_ROWS];
    int32_t flag[4];
};
static_assert(sizeof(NoAllocScratch) <= (size_t)640 * 1024, "the fixed workspace is meant to stay modest");

// Every GPU the library runs on holds its own copy of this array until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress: kernels get the address looked up below.
static __device__ __align__(256) unsigned char scratch[sizeof(NoAllocScratch)];

constexpr int NA_MAX_DEVICES = 64;
NoAllocScratch* g_scratch_ptr[NA_MAX_DEVICES];   // per device; written once, under g_scratch_lock
std::mutex g_scratch_lock;

// Address of the current device's copy of the array (looked up on the first call on that device).
int scratch_of_current_device(NoAllocScratch** out)
{
    int dev = -1;
    SPECV_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= NA_MAX_DEVICES) return fail(SPEC_ERR_DEVICE, "device index %d is not supported", dev);
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        SPECV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SPEC_ERR_DEVICE, "hipGetSymbolAddress returned no address for the fixed workspace");
        g_scratch_ptr[dev] = static_cast<NoAllocScratch*>(p);
    }
    *out = g_scratch_ptr[dev];
    return SPEC_OK;
}

__global__ void fill_i32_kernel(int32_t* __restrict__ p, int n, int32_t v)
{
    if ((int)threadIdx.x < n) p[threadIdx.x] = v;
}

}  // namespace
}  // namespace specv

using namespace specv;

extern "C" int spec_sample_step_noalloc(int32_t vocab, int32_t max_lookahead, const spec_step_args* args,
                                        const spec_step_out* out, void* stream)
{
    if (!args || !out) return fail(SPEC_ERR_INVALID_ARG, "NULL args or out");
    if (vocab < 1 || vocab > NA_MAX_VOCAB)
        return fail(SPEC_ERR_SHAPE, "vocab %d outside 1..%d (the fixed workspace is sized for that)", vocab, NA_MAX_VOCAB);
    if (max_lookahead < 0 || max_lookahead > SPEC_MAX_LOOKAHEAD)
        return fail(SPEC_ERR_SHAPE, "max_lookahead %d outside 0..%d", max_lookahead, SPEC_MAX_LOOKAHEAD);
    const int B = args->batch, Kmax = max_lookahead;
    if (B < 1 || B > NA_MAX_BATCH)
        return fail(SPEC_ERR_SHAPE, "batch %d outside 1..%d (the fixed workspace is sized for that)", B, NA_MAX_BATCH);
    if (!args->target_logits_in) return fail(SPEC_ERR_INVALID_ARG, "target_logits_in is NULL: this entry point runs no decoder pass");
    if (!args->lookahead) return fail(SPEC_ERR_INVALID_ARG, "lookahead is NULL");
    if (!(args->temperature >= 0.f)) return fail(SPEC_ERR_INVALID_ARG, "temperature must be >= 0");
    const bool greedy = args->temperature == 0.f;
    if (!greedy && !args->uniforms) return fail(SPEC_ERR_INVALID_ARG, "uniforms is NULL");
    if (!out->n_accepted || !out->out_tokens) return fail(SPEC_ERR_INVALID_ARG, "n_accepted or out_tokens is NULL");
    LookaheadPack ks;
    memset(&ks, 0, sizeof(ks));
    int M = 0, n_stat = 0, any_draft = 0;
    for (int b = 0; b < B; ++b) {
        const int k = args->lookahead[b];
        if (k < 0 || k > Kmax) return fail(SPEC_ERR_INVALID_ARG, "lookahead[%d] = %d outside 0..%d", b, k, Kmax);
        ks.k[b] = (uint8_t)k;
        M += k + 1;
        n_stat += 2 * k + 1;
        any_draft |= k;
    }
    if (any_draft && (!args->draft_tokens || (!greedy && !args->draft_logits)))
        return fail(SPEC_ERR_INVALID_ARG, "draft_tokens or draft_logits is NULL");
    NoAllocScratch* w = nullptr;
    int rc = scratch_of_current_device(&w);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    // the array keeps the last call's contents: the flag must start at zero (a fill kernel, so that
    // the call can be captured); every other entry that is read was written earlier in this call
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, s, w->flag, 4, 0);
    SPECV_LAUNCH_CHECK("fill_i32_kernel");
    StepTables t{};
    t.seq_row0 = w->seq_row0;
    t.seq_stat0 = w->seq_stat0;
    t.seq_n = w->seq_n;
    t.seq_ok = w->seq_ok;
    t.seq_slot = w->seq_slot;
    t.row_seq = w->row_seq;
    t.row_pos = w->row_pos;
    t.row_tok = w->row_tok;
    t.row_rope = w->row_rope;
    t.row_mask = w->row_mask;
    t.tree = 0;
    SamplerWorkspace sw{};
    sw.part_max = w->part_max;
    sw.part_sum = w->part_sum;
    sw.chunk_mass = w->chunk_mass;
    sw.accepted = w->accepted;
    sw.row_inv_z = w->row_inv_z;
    sw.row_max = w->row_max;
    sw.part_idx = w->part_idx;
    if (greedy) {   // the greedy rule's kernels read the tables from the start
        rc = launch_prepare(t, ks, B, Kmax, vocab, NA_MAX_BATCH, 0, false, nullptr, nullptr, args->draft_tokens, nullptr,
                            w->flag, s);
        if (rc) return rc;
    }
    if (out->logits_out) {
        // a copy node, not an allocation; callers under capture simply pass logits_out = NULL
        SPECV_HIP(hipMemcpyAsync(out->logits_out, args->target_logits_in, (size_t)M * vocab * sizeof(float),
                                 hipMemcpyDeviceToDevice, s));
    }
    if (greedy)
        return launch_greedy(t, sw, ks, B, Kmax, vocab, M, args->target_logits_in, args->draft_tokens, 0, nullptr,
                             out->n_accepted, out->out_tokens, nullptr, nullptr, s);
    return launch_sampler(t, sw, ks, B, Kmax, vocab, n_stat, args->target_logits_in, args->draft_logits,
                          args->draft_tokens, args->uniforms, Kmax + 1, args->temperature, 0, nullptr, out->n_accepted,
                          out->out_tokens, nullptr, nullptr, s, w->flag);
}
