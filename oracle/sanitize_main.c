/*
 * Sanitizer driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Built together with oracle.c under -fsanitize=address,undefined (see oracle.build_sanitized) and run
 * by tests/test_oracle_sanitized.py: it drives every exported routine of the oracle over small
 * seeded inputs -- fp32 and bf16 models, grouped-query attention, ragged windows, trees, the greedy
 * rule, the degenerate cases (K = 0, empty cache, one-token vocabulary) -- so that an out-of-bounds
 * access, a use of uninitialised or freed memory, a signed overflow or a misaligned access in the
 * checker itself is reported.  It also re-checks three properties the method fixes (scoring a window
 * at once equals decoding its tokens one by one, bit for bit; identical distributions keep every
 * proposal; a chain-shaped tree behaves like the linear procedure) and exits non-zero if one fails.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "oracle.h"

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static double unit(void)
{
    g_state ^= g_state << 13;
    g_state ^= g_state >> 7;
    g_state ^= g_state << 17;
    return (double)(g_state >> 11) / 9007199254740992.0;
}
static float gauss(float std) { return std * (float)(sqrt(-2.0 * log(unit() + 1e-300)) * cos(6.283185307179586 * unit())); }

static uint16_t to_bf16(float x)
{
    float r = oracle_round_bf16(x);
    uint32_t u;
    memcpy(&u, &r, 4);
    return (uint16_t)(u >> 16);
}

static void* matrix(int dtype, size_t n, float std)
{
    if (dtype == ORACLE_FP32) {
        float* p = malloc(n * sizeof(float));
        for (size_t i = 0; i < n; ++i) p[i] = gauss(std);
        return p;
    }
    uint16_t* p = malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) p[i] = to_bf16(gauss(std));
    return p;
}

static int fails = 0;
#define CHECK(cond, what) do { if (!(cond)) { printf("FAILED: %s\n", what); ++fails; } } while (0)

static void forward_cases(int dtype)
{
    enum { L = 2, D = 64, HQ = 4, HKV = 2, HD = 16, F = 96, V = 53, T = 24 };
    oracle_model m = {L, D, HQ, HKV, HD, F, V, dtype, T, 1e-5f, 10000.0f};
    const size_t es = dtype == ORACLE_FP32 ? 4 : 2;
    float* gains[2 * L + 1];
    const void *wqkv[L], *wo[L], *wgu[L], *wd[L];
    const float *an[L], *fn[L];
    for (int i = 0; i < 2 * L + 1; ++i) {
        gains[i] = malloc(D * sizeof(float));
        for (int k = 0; k < D; ++k) gains[i][k] = 1.0f + 0.1f * gauss(1.0f);
    }
    void* owned[4 * L + 2];
    int n_owned = 0;
    for (int l = 0; l < L; ++l) {
        owned[n_owned++] = (void*)(wqkv[l] = matrix(dtype, (size_t)(HQ + 2 * HKV) * HD * D, 0.08f));
        owned[n_owned++] = (void*)(wo[l] = matrix(dtype, (size_t)D * HQ * HD, 0.08f));
        owned[n_owned++] = (void*)(wgu[l] = matrix(dtype, (size_t)2 * F * D, 0.08f));
        owned[n_owned++] = (void*)(wd[l] = matrix(dtype, (size_t)D * F, 0.08f));
        an[l] = gains[2 * l];
        fn[l] = gains[2 * l + 1];
    }
    void* emb = matrix(dtype, (size_t)V * D, 0.08f);
    void* lm = matrix(dtype, (size_t)V * D, 0.08f);
    oracle_weights w = {emb, gains[2 * L], lm, an, wqkv, wo, fn, wgu, wd};
    const size_t plane = (size_t)2 * HKV * T * HD;
    /* three sequences: 9 cached + window of 5, empty cache + window of 3, 13 cached + window of 1 */
    const int n_seq = 3, n0[3] = {9, 0, 13}, nw[3] = {5, 3, 1};
    void *ca[3], *cb[3];
    oracle_cache a[3], b[3];
    int32_t windows[9], prompt[13];
    for (int i = 0; i < 9; ++i) windows[i] = (int32_t)(unit() * V);
    for (int s = 0; s < n_seq; ++s) {
        ca[s] = calloc(L * plane, es);
        cb[s] = calloc(L * plane, es);
        a[s].base = ca[s];
        a[s].layer_stride = (int64_t)plane;
        b[s].base = cb[s];
        b[s].layer_stride = (int64_t)plane;
        float row[V];
        for (int i = 0; i < n0[s]; ++i) {
            prompt[i] = (int32_t)(unit() * V);
            CHECK(oracle_decode_one(&m, &w, &a[s], i, prompt[i], row) == 0, "decode_one");
        }
        memcpy(cb[s], ca[s], L * plane * es);
    }
    float seq_rows[9 * V], at_once[9 * V];
    int r = 0;
    for (int s = 0; s < n_seq; ++s) {
        CHECK(oracle_verify_sequential(&m, &w, &a[s], n0[s], windows + r, nw[s], seq_rows + (size_t)r * V) == 0,
              "verify_sequential");
        r += nw[s];
    }
    CHECK(oracle_verify_rows(&m, &w, n_seq, b, n0, nw, windows, at_once) == 0, "verify_rows");
    CHECK(memcmp(seq_rows, at_once, sizeof(seq_rows)) == 0, "window at once == one token at a time (bit for bit)");
    for (int s = 0; s < n_seq; ++s) CHECK(memcmp(ca[s], cb[s], L * plane * es) == 0, "caches after both routes agree");
    for (int i = 0; i < 9 * V; ++i) CHECK(isfinite(seq_rows[i]), "finite logits");
    /* one head's attention over the whole cache, and the small building blocks */
    float q[HD], o[HD];
    for (int i = 0; i < HD; ++i) q[i] = gauss(1.0f);
    oracle_attend(&m, &a[0], 1, 1, n0[0] + nw[0], q, o);
    oracle_rope(HD, 10000.0f, 7, q);
    float x[D], y[D];
    for (int i = 0; i < D; ++i) x[i] = gauss(1.0f);
    oracle_rmsnorm(D, x, gains[0], 1e-5f, y);
    oracle_linear(dtype, wo[0], D, HQ * HD, x, y);
    /* arguments that must be refused, not read */
    float row[V];
    CHECK(oracle_decode_one(&m, &w, &a[0], T, 1, row) != 0, "position beyond the cache is refused");
    CHECK(oracle_decode_one(&m, &w, &a[0], 0, V, row) != 0, "token outside the vocabulary is refused");
    for (int s = 0; s < n_seq; ++s) {
        free(ca[s]);
        free(cb[s]);
    }
    for (int i = 0; i < n_owned; ++i) free(owned[i]);
    for (int i = 0; i < 2 * L + 1; ++i) free(gains[i]);
    free(emb);
    free(lm);
}

static void sampler_cases(void)
{
    enum { KMAX = 6 };
    const int vocabs[4] = {1, 2, 37, 1031};
    for (int vi = 0; vi < 4; ++vi) {
        const int V = vocabs[vi];
        for (int K = 0; K <= KMAX; K += 3) {
            float* tl = malloc((size_t)(K + 1) * V * sizeof(float));
            float* dl = malloc((size_t)(K + 1) * V * sizeof(float));
            int32_t toks[KMAX + 1], out[KMAX + 1], out2[KMAX + 1], path[KMAX + 1], parent[KMAX + 1], na, na2;
            float us[KMAX + 1];
            for (int i = 0; i < (K + 1) * V; ++i) {
                tl[i] = gauss(1.5f);
                dl[i] = tl[i] + gauss(0.5f);
            }
            for (int i = 0; i <= K; ++i) {
                toks[i] = (int32_t)(unit() * V);
                us[i] = (float)unit();
                parent[i] = i - 1;
            }
            const float temps[2] = {1.0f, 0.6f};
            for (int ti = 0; ti < 2; ++ti) {
                oracle_sample_diag d;
                CHECK(oracle_sample(V, K, tl, dl, toks, us, temps[ti], &na, out, &d) == 0, "sample");
                CHECK(na >= 0 && na <= K && out[na] >= 0 && out[na] < V, "sample: result in range");
                /* identical distributions keep every proposal */
                CHECK(oracle_sample(V, K, tl, tl, toks, us, temps[ti], &na2, out2, NULL) == 0 && na2 == K,
                      "q == p keeps every proposal");
                /* a chain-shaped tree is the linear procedure (its draft rows: row i+1 unused for the last node) */
                oracle_tree_diag td;
                CHECK(oracle_tree_sample(V, K, parent, toks, tl, dl, us, temps[ti], &na2, path, out2, &td) == 0,
                      "tree_sample");
                CHECK(na2 == na && memcmp(out, out2, sizeof(int32_t) * (size_t)(K + 1)) == 0, "chain tree == linear procedure");
            }
            float gap;
            CHECK(oracle_greedy(V, K, tl, toks, &na, out, &gap) == 0, "greedy");
            CHECK(oracle_tree_greedy(V, K, parent, toks, tl, &na2, path, out2, &gap) == 0 && na2 == na, "tree_greedy on a chain");
            /* a bushy tree: every node hangs below the root or below node 0 */
            for (int i = 1; i < K; ++i) parent[i] = (i & 1) ? -1 : 0;
            CHECK(oracle_tree_sample(V, K, parent, toks, tl, dl, us, 1.0f, &na2, path, out2, NULL) == 0, "bushy tree");
            CHECK(oracle_sample(V, K, tl, dl, toks, us, -1.0f, &na, out, NULL) != 0, "negative temperature is refused");
            double* p = malloc(V * sizeof(double));
            double* r = malloc(V * sizeof(double));
            double S, lo, hi;
            oracle_softmax(V, tl, 0.7f, p);
            oracle_residual(V, p, p, r, &S);
            CHECK(S == 0.0, "residual of a distribution with itself is empty");
            const int y = oracle_inverse_cdf(V, p, 0.999999999, &lo, &hi);
            CHECK(y >= 0 && y < V, "inverse CDF at the top of the range");
            free(p);
            free(r);
            free(tl);
            free(dl);
        }
    }
}

int main(void)
{
    forward_cases(ORACLE_FP32);
    forward_cases(ORACLE_BF16);
    sampler_cases();
    printf("oracle sanitizer driver: %d failed checks, %d threads\n", fails, oracle_threads());
    return fails ? 1 : 0;
}
