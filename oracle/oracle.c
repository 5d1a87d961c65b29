/*
 * CPU oracle for the speculative-sampling verify step -- see oracle.h.
 * TEST INFRASTRUCTURE ONLY: never part of the product path.
 *
 * Plain C.  Sums run in fp64 in index order; no blocking or reordering of any sum.  The only
 * concession to speed is oracle_verify_rows, which carries several rows through a layer at
 * once (each row's own sums unchanged) and is required by the tests to be bit-identical to
 * the one-token-at-a-time definition.
 */
#include "oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ storage types */

static inline float bf16_widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16 -> fp32, round to nearest, ties to even; NaN stays NaN. */
float oracle_round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        u |= 0x00400000u; /* quiet NaN survives truncation */
        u &= 0xffff0000u;
    } else {
        u += 0x7fffu + ((u >> 16) & 1u);
        u &= 0xffff0000u;
    }
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static inline uint16_t bf16_bits(float rounded)
{
    uint32_t u;
    memcpy(&u, &rounded, 4);
    return (uint16_t)(u >> 16);
}

static inline float load_elem(int dtype, const void* base, int64_t idx)
{
    return dtype == ORACLE_BF16 ? bf16_widen(((const uint16_t*)base)[idx]) : ((const float*)base)[idx];
}

static inline void store_cache(int dtype, void* base, int64_t idx, float v)
{
    if (dtype == ORACLE_BF16)
        ((uint16_t*)base)[idx] = bf16_bits(oracle_round_bf16(v));
    else
        ((float*)base)[idx] = v;
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ building blocks */

/* out = x / sqrt(mean(x^2) + eps) * gain */
void oracle_rmsnorm(int32_t d, const float* x, const float* gain, float eps, float* out)
{
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += (double)x[i] * (double)x[i];
    double inv = 1.0 / sqrt(ss / (double)d + (double)eps);
    for (int i = 0; i < d; ++i) out[i] = (float)((double)x[i] * inv * (double)gain[i]);
}

/* Rotary embedding of one head vector at absolute position pos.  Dimension i (i < hd/2) is
 * paired with i + hd/2; the pair is rotated by the angle pos * theta^(-2i/hd). */
void oracle_rope(int32_t hd, float theta, int32_t pos, float* v)
{
    int half = hd / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)hd);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = (float)(a * c - b * s);
        v[i + half] = (float)(a * s + b * c);
    }
}

/* y[o] = sum_i x[i] * W[o][i] */
void oracle_linear(int32_t dtype, const void* W, int32_t n_out, int32_t n_in, const float* x, float* y)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; ++o) {
        double acc = 0.0;
        int64_t row = (int64_t)o * n_in;
        for (int i = 0; i < n_in; ++i) acc += (double)x[i] * (double)load_elem(dtype, W, row + i);
        y[o] = (float)acc;
    }
}

static inline int64_t cache_index(const oracle_model* m, const oracle_cache* c, int layer, int kv,
                                  int head, int pos)
{
    return (int64_t)layer * c->layer_stride
           + (((int64_t)kv * m->n_kv_heads + head) * m->max_kv_len + pos) * m->head_dim;
}

/* softmax(q.K_t / sqrt(hd) over t in [0,n_pos)) . V, keys and values read from the cache */
void oracle_attend(const oracle_model* m, const oracle_cache* c, int32_t layer, int32_t kv_head,
                   int32_t n_pos, const float* q, float* out)
{
    int hd = m->head_dim;
    double* s = (double*)malloc(sizeof(double) * (size_t)n_pos);
    double scale = 1.0 / sqrt((double)hd);
    double mx = -INFINITY;
    for (int t = 0; t < n_pos; ++t) {
        int64_t k0 = cache_index(m, c, layer, 0, kv_head, t);
        double acc = 0.0;
        for (int e = 0; e < hd; ++e) acc += (double)q[e] * (double)load_elem(m->dtype, c->base, k0 + e);
        s[t] = acc * scale;
        if (s[t] > mx) mx = s[t];
    }
    double Z = 0.0;
    for (int t = 0; t < n_pos; ++t) {
        s[t] = exp(s[t] - mx);
        Z += s[t];
    }
    for (int e = 0; e < hd; ++e) {
        double acc = 0.0;
        for (int t = 0; t < n_pos; ++t) {
            int64_t v0 = cache_index(m, c, layer, 1, kv_head, t);
            acc += s[t] * (double)load_elem(m->dtype, c->base, v0 + e);
        }
        out[e] = (float)(acc / Z);
    }
    free(s);
}

static inline float silu_mul(float g, float u)
{
    double gd = g;
    return (float)(gd / (1.0 + exp(-gd)) * (double)u);
}

/* ------------------------------------------------------------------ single-token decode */

static int check_model(const oracle_model* m)
{
    if (!m || m->n_layers <= 0 || m->d_model <= 0 || m->n_q_heads <= 0 || m->n_kv_heads <= 0
        || m->head_dim <= 0 || (m->head_dim & 1) || m->d_ffn <= 0 || m->vocab <= 0
        || m->n_q_heads % m->n_kv_heads != 0 || (m->dtype != ORACLE_FP32 && m->dtype != ORACLE_BF16)
        || m->max_kv_len <= 0)
        return -1;
    return 0;
}

int oracle_decode_one(const oracle_model* m, const oracle_weights* w, const oracle_cache* c,
                      int32_t pos, int32_t token, float* logits)
{
    if (check_model(m) || pos < 0 || pos >= m->max_kv_len || token < 0 || token >= m->vocab) return -1;
    const int d = m->d_model, hd = m->head_dim, Hq = m->n_q_heads, Hkv = m->n_kv_heads, F = m->d_ffn;
    const int dq = Hq * hd, dkv = Hkv * hd, group = Hq / Hkv;

    float* x = (float*)malloc(sizeof(float) * d);
    float* h = (float*)malloc(sizeof(float) * d);
    float* qkv = (float*)malloc(sizeof(float) * (dq + 2 * dkv));
    float* att = (float*)malloc(sizeof(float) * dq);
    float* y = (float*)malloc(sizeof(float) * d);
    float* gu = (float*)malloc(sizeof(float) * 2 * F);
    float* act = (float*)malloc(sizeof(float) * F);

    for (int i = 0; i < d; ++i) x[i] = load_elem(m->dtype, w->tok_embed, (int64_t)token * d + i);

    for (int l = 0; l < m->n_layers; ++l) {
        /* attention block */
        oracle_rmsnorm(d, x, w->attn_norm[l], m->rms_eps, h);
        oracle_linear(m->dtype, w->w_qkv[l], dq + 2 * dkv, d, h, qkv);
        float* q = qkv;
        float* k = qkv + dq;
        float* v = qkv + dq + dkv;
        for (int hh = 0; hh < Hq; ++hh) oracle_rope(hd, m->rope_theta, pos, q + hh * hd);
        for (int hh = 0; hh < Hkv; ++hh) {
            oracle_rope(hd, m->rope_theta, pos, k + hh * hd);
            int64_t k0 = cache_index(m, c, l, 0, hh, pos), v0 = cache_index(m, c, l, 1, hh, pos);
            for (int e = 0; e < hd; ++e) {
                store_cache(m->dtype, c->base, k0 + e, k[hh * hd + e]);
                store_cache(m->dtype, c->base, v0 + e, v[hh * hd + e]);
            }
        }
#pragma omp parallel for schedule(static)
        for (int hh = 0; hh < Hq; ++hh)
            oracle_attend(m, c, l, hh / group, pos + 1, q + hh * hd, att + hh * hd);
        oracle_linear(m->dtype, w->w_o[l], d, dq, att, y);
        for (int i = 0; i < d; ++i) x[i] = x[i] + y[i];

        /* feed-forward block */
        oracle_rmsnorm(d, x, w->ffn_norm[l], m->rms_eps, h);
        oracle_linear(m->dtype, w->w_gate_up[l], 2 * F, d, h, gu);
        for (int i = 0; i < F; ++i) act[i] = silu_mul(gu[i], gu[F + i]);
        oracle_linear(m->dtype, w->w_down[l], d, F, act, y);
        for (int i = 0; i < d; ++i) x[i] = x[i] + y[i];
    }
    oracle_rmsnorm(d, x, w->final_norm, m->rms_eps, h);
    oracle_linear(m->dtype, w->lm_head, m->vocab, d, h, logits);

    free(x); free(h); free(qkv); free(att); free(y); free(gu); free(act);
    return 0;
}

int oracle_verify_sequential(const oracle_model* m, const oracle_weights* w, const oracle_cache* c,
                             int32_t n, const int32_t* window, int32_t n_window, float* logits)
{
    for (int j = 0; j < n_window; ++j) {
        int rc = oracle_decode_one(m, w, c, n + j, window[j], logits + (int64_t)j * m->vocab);
        if (rc) return rc;
    }
    return 0;
}

/* ------------------------------------------------------------------ all rows per layer */

#define ROW_BLOCK 16

/* Y[r][o] = sum_i X[r][i] * W[o][i] for R rows.  Each (r,o) sum runs over i in index order in
 * fp64 exactly as oracle_linear does; rows are only interleaved, never combined.  (The product
 * of two fp32 values is exact in fp64, so fused and unfused multiply-add agree.) */
/* acc[r] = sum_i xt[i][r] * wrow[i] for the ROW_BLOCK rows of one block: every row's sum runs
 * over i in index order in fp64 exactly as oracle_linear's does; rows are only interleaved,
 * never combined.  (The product of two fp32 values is exact in fp64, so fused and unfused
 * multiply-add agree and the vector width does not matter.) */
__attribute__((target_clones("avx2", "default")))
static void dot_block(const double* xt, const double* wrow, int n_in, double* acc)
{
    double a[ROW_BLOCK];
    for (int r = 0; r < ROW_BLOCK; ++r) a[r] = 0.0;
    for (int i = 0; i < n_in; ++i) {
        double wv = wrow[i];
        for (int r = 0; r < ROW_BLOCK; ++r) a[r] += xt[(size_t)i * ROW_BLOCK + r] * wv;
    }
    for (int r = 0; r < ROW_BLOCK; ++r) acc[r] = a[r];
}

/* Y[r][o] = sum_i X[r][i] * W[o][i] for R rows. */
static void linear_rows(int dtype, const void* W, int n_out, int n_in, const float* X, int R, float* Y)
{
    int nblk = (R + ROW_BLOCK - 1) / ROW_BLOCK;
    /* XT[blk][i][r]: activations transposed per row block, widened to fp64, zero padded */
    double* XT = (double*)calloc((size_t)nblk * n_in * ROW_BLOCK, sizeof(double));
    for (int r = 0; r < R; ++r) {
        double* dst = XT + (size_t)(r / ROW_BLOCK) * n_in * ROW_BLOCK + (r % ROW_BLOCK);
        for (int i = 0; i < n_in; ++i) dst[(size_t)i * ROW_BLOCK] = (double)X[(size_t)r * n_in + i];
    }
#pragma omp parallel
    {
        double* wrow = (double*)malloc(sizeof(double) * n_in);
#pragma omp for schedule(static)
        for (int o = 0; o < n_out; ++o) {
            int64_t row = (int64_t)o * n_in;
            for (int i = 0; i < n_in; ++i) wrow[i] = (double)load_elem(dtype, W, row + i);
            for (int b = 0; b < nblk; ++b) {
                double acc[ROW_BLOCK];
                dot_block(XT + (size_t)b * n_in * ROW_BLOCK, wrow, n_in, acc);
                int lim = R - b * ROW_BLOCK < ROW_BLOCK ? R - b * ROW_BLOCK : ROW_BLOCK;
                for (int r = 0; r < lim; ++r) Y[(size_t)(b * ROW_BLOCK + r) * n_out + o] = (float)acc[r];
            }
        }
        free(wrow);
    }
    free(XT);
}

int oracle_verify_rows(const oracle_model* m, const oracle_weights* w, int32_t n_seq,
                       const oracle_cache* caches, const int32_t* n, const int32_t* n_window,
                       const int32_t* windows, float* logits)
{
    if (check_model(m) || n_seq <= 0) return -1;
    const int d = m->d_model, hd = m->head_dim, Hq = m->n_q_heads, Hkv = m->n_kv_heads, F = m->d_ffn;
    const int dq = Hq * hd, dkv = Hkv * hd, group = Hq / Hkv, nqkv = dq + 2 * dkv;

    int M = 0;
    for (int s = 0; s < n_seq; ++s) {
        if (n_window[s] <= 0 || n[s] < 0 || n[s] + n_window[s] > m->max_kv_len) return -1;
        M += n_window[s];
    }
    int* row_seq = (int*)malloc(sizeof(int) * M);
    int* row_pos = (int*)malloc(sizeof(int) * M);
    for (int s = 0, r = 0; s < n_seq; ++s)
        for (int j = 0; j < n_window[s]; ++j, ++r) {
            row_seq[r] = s;
            row_pos[r] = n[s] + j;
            if (windows[r] < 0 || windows[r] >= m->vocab) { free(row_seq); free(row_pos); return -1; }
        }

    float* x = (float*)malloc(sizeof(float) * (size_t)M * d);
    float* h = (float*)malloc(sizeof(float) * (size_t)M * d);
    float* qkv = (float*)malloc(sizeof(float) * (size_t)M * nqkv);
    float* att = (float*)malloc(sizeof(float) * (size_t)M * dq);
    float* y = (float*)malloc(sizeof(float) * (size_t)M * d);
    float* gu = (float*)malloc(sizeof(float) * (size_t)M * 2 * F);
    float* act = (float*)malloc(sizeof(float) * (size_t)M * F);

    for (int r = 0; r < M; ++r)
        for (int i = 0; i < d; ++i)
            x[(size_t)r * d + i] = load_elem(m->dtype, w->tok_embed, (int64_t)windows[r] * d + i);

    for (int l = 0; l < m->n_layers; ++l) {
        for (int r = 0; r < M; ++r)
            oracle_rmsnorm(d, x + (size_t)r * d, w->attn_norm[l], m->rms_eps, h + (size_t)r * d);
        linear_rows(m->dtype, w->w_qkv[l], nqkv, d, h, M, qkv);
        /* rotate, then put every window token's key and value into its sequence's cache */
        for (int r = 0; r < M; ++r) {
            float* q = qkv + (size_t)r * nqkv;
            float* k = q + dq;
            float* v = k + dkv;
            const oracle_cache* c = &caches[row_seq[r]];
            for (int hh = 0; hh < Hq; ++hh) oracle_rope(hd, m->rope_theta, row_pos[r], q + hh * hd);
            for (int hh = 0; hh < Hkv; ++hh) {
                oracle_rope(hd, m->rope_theta, row_pos[r], k + hh * hd);
                int64_t k0 = cache_index(m, c, l, 0, hh, row_pos[r]);
                int64_t v0 = cache_index(m, c, l, 1, hh, row_pos[r]);
                for (int e = 0; e < hd; ++e) {
                    store_cache(m->dtype, c->base, k0 + e, k[hh * hd + e]);
                    store_cache(m->dtype, c->base, v0 + e, v[hh * hd + e]);
                }
            }
        }
        /* row r sees cache positions [0, pos_r]: the cached prefix plus window tokens up to itself */
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
        for (int r = 0; r < M; ++r)
            for (int hh = 0; hh < Hq; ++hh)
                oracle_attend(m, &caches[row_seq[r]], l, hh / group, row_pos[r] + 1,
                              qkv + (size_t)r * nqkv + hh * hd, att + (size_t)r * dq + hh * hd);
        linear_rows(m->dtype, w->w_o[l], d, dq, att, M, y);
        for (size_t i = 0; i < (size_t)M * d; ++i) x[i] = x[i] + y[i];

        for (int r = 0; r < M; ++r)
            oracle_rmsnorm(d, x + (size_t)r * d, w->ffn_norm[l], m->rms_eps, h + (size_t)r * d);
        linear_rows(m->dtype, w->w_gate_up[l], 2 * F, d, h, M, gu);
        for (int r = 0; r < M; ++r)
            for (int i = 0; i < F; ++i)
                act[(size_t)r * F + i] = silu_mul(gu[(size_t)r * 2 * F + i], gu[(size_t)r * 2 * F + F + i]);
        linear_rows(m->dtype, w->w_down[l], d, F, act, M, y);
        for (size_t i = 0; i < (size_t)M * d; ++i) x[i] = x[i] + y[i];
    }
    for (int r = 0; r < M; ++r)
        oracle_rmsnorm(d, x + (size_t)r * d, w->final_norm, m->rms_eps, h + (size_t)r * d);
    linear_rows(m->dtype, w->lm_head, m->vocab, d, h, M, logits);

    free(x); free(h); free(qkv); free(att); free(y); free(gu); free(act);
    free(row_seq); free(row_pos);
    return 0;
}

/* ------------------------------------------------------------------ rejection sampling */

/* p = softmax(logits / T) in fp64 */
void oracle_softmax(int32_t V, const float* logits, float T, double* p)
{
    double mx = -INFINITY;
    for (int v = 0; v < V; ++v) {
        p[v] = (double)logits[v] / (double)T;
        if (p[v] > mx) mx = p[v];
    }
    double Z = 0.0;
    for (int v = 0; v < V; ++v) {
        p[v] = exp(p[v] - mx);
        Z += p[v];
    }
    for (int v = 0; v < V; ++v) p[v] /= Z;
}

/* r = max(0, p - q), S = sum r */
void oracle_residual(int32_t V, const double* p, const double* q, double* r, double* S)
{
    double s = 0.0;
    for (int v = 0; v < V; ++v) {
        r[v] = p[v] > q[v] ? p[v] - q[v] : 0.0;
        s += r[v];
    }
    *S = s;
}

/* First id (ascending) whose inclusive prefix sum of r exceeds target; if rounding leaves none,
 * the last id with r > 0.  lo/hi receive the prefix sums just before and at the chosen id. */
int32_t oracle_inverse_cdf(int32_t V, const double* r, double target, double* lo, double* hi)
{
    double c = 0.0;
    int last_pos = -1;
    double last_lo = 0.0, last_hi = 0.0;
    for (int v = 0; v < V; ++v) {
        double nc = c + r[v];
        if (r[v] > 0.0) { last_pos = v; last_lo = c; last_hi = nc; }
        if (nc > target) {
            if (lo) *lo = c;
            if (hi) *hi = nc;
            return v;
        }
        c = nc;
    }
    if (lo) *lo = last_lo;
    if (hi) *hi = last_hi;
    return last_pos;
}

int oracle_greedy(int32_t V, int32_t K, const float* target_logits, const int32_t* draft_tokens,
                  int32_t* n_accepted, int32_t* out_tokens, float* min_gap)
{
    if (V <= 0 || K < 0) return -1;
    int a = 0;
    float gap_min = INFINITY;
    for (int i = 0; i <= K; ++i) {
        const float* row = target_logits + (size_t)i * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (row[v] > row[best]) best = v;
        float second = -INFINITY;
        for (int v = 0; v < V; ++v)
            if (v != best && row[v] > second) second = row[v];
        if (V > 1 && row[best] - second < gap_min) gap_min = row[best] - second;
        if (i < K && draft_tokens[i] == best) {
            out_tokens[a++] = best;
            continue;
        }
        out_tokens[a] = best;
        break;
    }
    for (int i = a + 1; i <= K; ++i) out_tokens[i] = -1;
    *n_accepted = a;
    if (min_gap) *min_gap = gap_min;
    return 0;
}

int oracle_tree_greedy(int32_t V, int32_t N, const int32_t* parent, const int32_t* tokens,
                       const float* target_logits, int32_t* n_accepted, int32_t* path, int32_t* out_tokens,
                       float* min_gap)
{
    if (V <= 0 || N < 0) return -1;
    for (int i = 0; i < N; ++i)
        if (parent[i] < -1 || parent[i] >= i || tokens[i] < 0 || tokens[i] >= V) return -1;
    int cur = -1, a = 0;
    float gap_min = INFINITY;
    for (;;) {
        const float* row = target_logits + (size_t)(cur + 1) * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (row[v] > row[best]) best = v;
        float second = -INFINITY;
        for (int v = 0; v < V; ++v)
            if (v != best && row[v] > second) second = row[v];
        if (V > 1 && row[best] - second < gap_min) gap_min = row[best] - second;
        int next = -1;
        for (int c = cur + 1; c < N; ++c)
            if (parent[c] == cur && tokens[c] == best) { next = c; break; }
        if (next < 0) {
            out_tokens[a] = best;
            break;
        }
        path[a] = next;
        out_tokens[a] = best;
        ++a;
        cur = next;
    }
    for (int i = a + 1; i <= N; ++i) out_tokens[i] = -1;
    for (int i = a; i < N; ++i) path[i] = -1;
    *n_accepted = a;
    if (min_gap) *min_gap = gap_min;
    return 0;
}

int oracle_tree_sample(int32_t V, int32_t N, const int32_t* parent, const int32_t* tokens,
                       const float* target_logits, const float* draft_logits, const float* uniforms, float T,
                       int32_t* n_accepted, int32_t* path, int32_t* out_tokens, oracle_tree_diag* diag)
{
    if (V <= 0 || N < 0 || !(T > 0.0f)) return -1;
    for (int i = 0; i < N; ++i)
        if (parent[i] < -1 || parent[i] >= i || tokens[i] < 0 || tokens[i] >= V) return -1;
    double* r = (double*)malloc(sizeof(double) * V);
    double* q = (double*)malloc(sizeof(double) * V);
    double* t = (double*)malloc(sizeof(double) * V);
    if (diag) {
        memset(diag, 0, sizeof(*diag));
        for (int i = 0; i < 16; ++i) diag->accept_ratio[i] = -1.0;
    }
    int cur = -1, a = 0, level = 0;
    double S = 1.0;     /* r is kept unnormalised: the distribution is r / S (S = 1 while r is p itself) */
    for (;;) {
        /* arrive at a node: r = its target distribution, q = the draft's */
        oracle_softmax(V, target_logits + (size_t)(cur + 1) * V, T, r);
        oracle_softmax(V, draft_logits + (size_t)(cur + 1) * V, T, q);
        level = 0;
        S = 1.0;
        int moved = 0;
        for (int c = cur + 1; c < N; ++c) {
            if (parent[c] != cur) continue;
            const int x = tokens[c];
            const double rx = r[x] / S;
            if (diag && c < 16) {
                double ratio = q[x] > 0.0 ? rx / q[x] : (rx > 0.0 ? INFINITY : 0.0);
                diag->accept_ratio[c] = ratio < 1.0 ? ratio : 1.0;
            }
            if ((double)uniforms[c] * q[x] < rx) {
                path[a] = c;
                out_tokens[a] = x;
                ++a;
                cur = c;
                moved = 1;
                break;
            }
            /* rejected: r <- max(0, r/S - q) */
            double S_new = 0.0;
            for (int v = 0; v < V; ++v) {
                const double pv = r[v] / S;
                t[v] = pv > q[v] ? pv - q[v] : 0.0;
                S_new += t[v];
            }
            if (S_new > 0.0) {   /* S_new <= 0 cannot happen in exact arithmetic; then r stays */
                memcpy(r, t, sizeof(double) * V);
                S = S_new;
                ++level;
            }
        }
        if (!moved) break;
    }
    if (level == 0) {
        S = 0.0;
        for (int v = 0; v < V; ++v) S += r[v];
    }
    double target = (double)uniforms[N] * S, lo, hi;
    const int y = oracle_inverse_cdf(V, r, target, &lo, &hi);
    out_tokens[a] = y;
    for (int i = a + 1; i <= N; ++i) out_tokens[i] = -1;
    for (int i = a; i < N; ++i) path[i] = -1;
    *n_accepted = a;
    if (diag) {
        diag->final_S = S;
        diag->final_target = target;
        diag->final_cdf_lo = lo;
        diag->final_cdf_hi = hi;
        diag->final_node = cur;
        diag->final_level = level;
    }
    free(r); free(q); free(t);
    return 0;
}

int oracle_sample(int32_t V, int32_t K, const float* target_logits, const float* draft_logits,
                  const int32_t* draft_tokens, const float* uniforms, float T,
                  int32_t* n_accepted, int32_t* out_tokens, oracle_sample_diag* diag)
{
    if (V <= 0 || K < 0 || !(T > 0.0f)) return -1;
    for (int i = 0; i < K; ++i)
        if (draft_tokens[i] < 0 || draft_tokens[i] >= V) return -1;
    double* p = (double*)malloc(sizeof(double) * V);
    double* q = (double*)malloc(sizeof(double) * V);
    double* r = (double*)malloc(sizeof(double) * V);
    if (diag) memset(diag, 0, sizeof(*diag));

    /* keep drafts while u * q(x) < p(x), i.e. with probability min(1, p(x)/q(x)) */
    int a = K;
    for (int i = 0; i < K; ++i) {
        oracle_softmax(V, target_logits + (size_t)i * V, T, p);
        oracle_softmax(V, draft_logits + (size_t)i * V, T, q);
        int x = draft_tokens[i];
        if (diag && i < 16) {
            double ratio = q[x] > 0.0 ? p[x] / q[x] : (p[x] > 0.0 ? INFINITY : 0.0);
            diag->accept_ratio[i] = ratio < 1.0 ? ratio : 1.0;
        }
        if (!((double)uniforms[i] * q[x] < p[x])) { a = i; break; }
    }

    /* the one final draw: residual at the first rejection, or the target's next-token
     * distribution after the last draft when every draft was kept */
    double S;
    int is_res = 0;
    if (a < K) {
        /* p and q currently hold row a */
        oracle_residual(V, p, q, r, &S);
        is_res = 1;
        if (!(S > 0.0)) { /* cannot happen in exact arithmetic; fall back to p_a */
            memcpy(r, p, sizeof(double) * V);
            S = 0.0;
            for (int v = 0; v < V; ++v) S += r[v];
            is_res = 0;
        }
    } else {
        oracle_softmax(V, target_logits + (size_t)K * V, T, r);
        S = 0.0;
        for (int v = 0; v < V; ++v) S += r[v];
    }
    double target = (double)uniforms[K] * S, lo, hi;
    int y = oracle_inverse_cdf(V, r, target, &lo, &hi);

    for (int i = 0; i < a; ++i) out_tokens[i] = draft_tokens[i];
    out_tokens[a] = y;
    for (int i = a + 1; i <= K; ++i) out_tokens[i] = -1;
    *n_accepted = a;
    if (diag) {
        diag->final_S = S;
        diag->final_target = target;
        diag->final_cdf_lo = lo;
        diag->final_cdf_hi = hi;
        diag->final_row = a;
        diag->final_is_residual = is_res;
    }
    free(p); free(q); free(r);
    return 0;
}
