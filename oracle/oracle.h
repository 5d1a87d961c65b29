/*
 * CPU oracle for the speculative-sampling verify step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the verify step computes, written
 * from the paper's description of speculative sampling (section "Speculative Sampling
 * Results": a draft model proposes several tokens, the target model scores them in one call,
 * a rejection criterion keeps a prefix, the first rejected token is resampled from a
 * combination of the two distributions, and if everything is kept one more token is sampled
 * from the target) together with the formulas of the works it cites for the method:
 * accept with probability min(1, p/q), resample from normalize(max(0, p - q)).
 *
 * It shares no code with the GPU library and must never be linked into, imported by or
 * called from the product path; only tests, the smoke check and the benchmark's CPU-baseline
 * leg use it.
 *
 * Arithmetic: activations are fp32 values; every sum (dot products, norms, softmax
 * normalisers, prefix sums) is accumulated in fp64 in index order and rounded once.  Weights
 * and KV cache are read in their storage type (fp32, or bf16 widened exactly); keys and
 * values are rounded to the storage type (round-to-nearest-even) when they enter the cache
 * and are attended to only through the cache.  The sampler works in fp64 on fp32 logits.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py against closed
 * forms, library routines on special cases, invariants and brute-force enumeration.  The
 * paper prints no worked numeric example for this path, so absolute logit values of the
 * architecture conventions (pre-norm blocks, RMSNorm eps, RoPE base and pairing, SiLU gating)
 * are pinned through a textbook whole-sequence causal evaluation written with library
 * primitives, not through numbers from the paper.
 */
#ifndef SPEC_ORACLE_H
#define SPEC_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_FP32 = 0, ORACLE_BF16 = 1 };

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;        /* storage of matrices, embedding and KV cache */
    int32_t max_kv_len;   /* positions per (layer, k|v, head) plane of the cache */
    float rms_eps, rope_theta;
} oracle_model;

/* Matrices are [out_features][in_features], rows contiguous.  w_qkv rows: all q heads, then
 * all k heads, then all v heads.  w_gate_up rows: d_ffn gate rows then d_ffn up rows.
 * Norm gains are fp32[d_model].  Per-layer members are arrays of n_layers pointers. */
typedef struct {
    const void* tok_embed;      /* [vocab][d_model] */
    const float* final_norm;
    const void* lm_head;        /* [vocab][d_model] */
    const float* const* attn_norm;
    const void* const* w_qkv;   /* [(Hq+2Hkv)*hd][d_model] */
    const void* const* w_o;     /* [d_model][Hq*hd] */
    const float* const* ffn_norm;
    const void* const* w_gate_up; /* [2*d_ffn][d_model] */
    const void* const* w_down;  /* [d_model][d_ffn] */
} oracle_weights;

/* One sequence's cache: element (layer l, kv in {0=k,1=v}, head h, position t, dim e) lives at
 * base + l*layer_stride + ((kv*Hkv + h)*max_kv_len + t)*hd + e   (in elements of dtype). */
typedef struct {
    void* base;
    int64_t layer_stride;
} oracle_cache;

/* Ordinary single-token autoregressive decode: the token at absolute position pos, on top of
 * cache positions [0,pos).  Writes this token's k,v into the cache at pos and the next-token
 * logits (fp32[vocab]).  This is the definition every other forward routine is held to. */
int oracle_decode_one(const oracle_model* m, const oracle_weights* w, const oracle_cache* c,
                      int32_t pos, int32_t token, float* logits);

/* Verify logits by definition: the n_window tokens fed one at a time through
 * oracle_decode_one at positions n, n+1, ...  logits is [n_window][vocab]. */
int oracle_verify_sequential(const oracle_model* m, const oracle_weights* w, const oracle_cache* c,
                             int32_t n, const int32_t* window, int32_t n_window, float* logits);

/* Same result, bit for bit per row, with all rows of all sequences taken through each layer
 * together so every weight is read once.  windows is the concatenation of the sequences'
 * windows; logits is [sum n_window][vocab] in the same order. */
int oracle_verify_rows(const oracle_model* m, const oracle_weights* w, int32_t n_seq,
                       const oracle_cache* caches, const int32_t* n, const int32_t* n_window,
                       const int32_t* windows, float* logits);

/* Diagnostics of one sequence's sampling, for margin-aware comparison. */
typedef struct {
    double accept_ratio[16];  /* min(1, p(x)/q(x)) per tested position (up to 16 kept) */
    double final_S;           /* total mass of the distribution the final token was drawn from */
    double final_target;      /* u * S */
    double final_cdf_lo;      /* inclusive prefix sum before the chosen token */
    double final_cdf_hi;      /* inclusive prefix sum at the chosen token */
    int32_t final_row;        /* target row the final draw used (a, or K if all accepted) */
    int32_t final_is_residual;
} oracle_sample_diag;

/* Rejection sampling for one sequence with lookahead K (0 <= K).
 * target_logits [K+1][vocab], draft_logits [K][vocab], draft_tokens [K], uniforms [K+1] in [0,1).
 * p_j = softmax(target_logits[j]/T), q_i = softmax(draft_logits[i]/T).
 * Draft i is kept iff u_i * q_i(x_i) < p_i(x_i); a = number kept before the first failure.
 * Final token: inverse CDF (ascending token id, first id whose inclusive prefix sum exceeds
 * u_K * S) of max(0, p_a - q_a) if a < K, else of p_K.
 * out_tokens [K+1]: the a kept drafts, the final token, then -1 padding.  diag may be NULL. */
int oracle_sample(int32_t vocab, int32_t K, const float* target_logits, const float* draft_logits,
                  const int32_t* draft_tokens, const float* uniforms, float temperature,
                  int32_t* n_accepted, int32_t* out_tokens, oracle_sample_diag* diag);

/* Greedy verification (temperature 0: both models put all mass on their most likely token, and the
 * rejection rule collapses): draft i is kept iff it equals argmax of target row i; the final token
 * is argmax of row a (first mismatch) or of row K.  argmax takes the lowest id among equal maxima.
 * min_gap (may be NULL) receives the smallest top-1/top-2 logit gap over the rows that decided. */
int oracle_greedy(int32_t vocab, int32_t K, const float* target_logits, const int32_t* draft_tokens,
                  int32_t* n_accepted, int32_t* out_tokens, float* min_gap);

/* Greedy verification of a token tree (temperature 0): from the root, move to the first child (in
 * index order) whose token is the most likely token of the current node's target row; when there is
 * none, that most likely token is the final token.  target_logits [N+1][vocab] (row 0: the root).
 * path [N], out_tokens [N+1] as in oracle_tree_sample. */
int oracle_tree_greedy(int32_t vocab, int32_t N, const int32_t* parent, const int32_t* tokens,
                       const float* target_logits, int32_t* n_accepted, int32_t* path, int32_t* out_tokens,
                       float* min_gap);

/* Diagnostics of one sequence's tree verification. */
typedef struct {
    double accept_ratio[16];  /* per node i < 16: min(1, r(x_i)/q(x_i)) if the node was tested, else -1 */
    double final_S;
    double final_target;
    double final_cdf_lo;
    double final_cdf_hi;
    int32_t final_node;       /* node whose rows the final draw used (-1 = root) */
    int32_t final_level;      /* rejections at that node before the draw (0: its target distribution) */
} oracle_tree_diag;

/* Verification of a token tree (the tree-structured candidates of the paper's section on
 * EAGLE-style decoding; the accept rule is the multi-candidate form of the same rejection sampling:
 * the children of a node are independent draws from the draft distribution at that node).
 * Nodes 0..N-1 in topological order: parent[i] = -1 (child of the root, i.e. of the sequence's last
 * token) or an index < i.  Row 0 of target_logits / draft_logits belongs to the root, row i+1 to
 * node i: the target's and the draft's next-token distributions after the path to that node.
 * Walk from the root: at the current node with target distribution p and draft distribution q, set
 * r = p; try its children in index order: child c with token x is kept iff u_c * q(x) < r(x); a kept
 * child becomes the current node; after a rejection r <- max(0, r - q) / sum(max(0, r - q)).  When no
 * child is left (a leaf, or all rejected) the final token is drawn from r by inverse CDF with
 * u_N (target u_N * S over the unnormalised r, as in oracle_sample).
 * uniforms [N+1]; path [N]: kept node indices root-down; out_tokens [N+1]: their tokens, the final
 * token, then -1. */
int oracle_tree_sample(int32_t vocab, int32_t N, const int32_t* parent, const int32_t* tokens,
                       const float* target_logits, const float* draft_logits, const float* uniforms,
                       float temperature, int32_t* n_accepted, int32_t* path, int32_t* out_tokens,
                       oracle_tree_diag* diag);

/* Building blocks, exported so tests can pin them one by one. */
void oracle_softmax(int32_t vocab, const float* logits, float temperature, double* p);
void oracle_residual(int32_t vocab, const double* p, const double* q, double* r, double* S);
int32_t oracle_inverse_cdf(int32_t vocab, const double* r, double target, double* lo, double* hi);
void oracle_rmsnorm(int32_t d, const float* x, const float* gain, float eps, float* out);
void oracle_rope(int32_t head_dim, float theta, int32_t pos, float* vec);
void oracle_linear(int32_t dtype, const void* W, int32_t n_out, int32_t n_in, const float* x, float* y);
/* one query head over cache positions [0, n_pos): out[head_dim] */
void oracle_attend(const oracle_model* m, const oracle_cache* c, int32_t layer, int32_t kv_head,
                   int32_t n_pos, const float* q, float* out);
float oracle_round_bf16(float x);
int oracle_threads(void);

#ifdef __cplusplus
}
#endif
#endif
