/*
 * spec_verify.h -- C ABI of the speculative-sampling verify step for AMD MI355X (gfx950).
 *
 * One call, spec_verify_step, does what the paper's section "Speculative Sampling Results"
 * describes after the draft model has proposed its tokens: the target decoder scores the whole
 * draft window in a single pass over its KV cache, the target and draft probabilities of each
 * proposed token are compared, a prefix of the proposals is kept, the first rejected position is
 * resampled from a combination of the two distributions, and one more token is sampled from the
 * target when every proposal was kept.  The formulas are those of the works the paper cites for
 * the method: keep proposal x with probability min(1, p(x)/q(x)); resample from
 * normalize(max(0, p - q)).
 *
 * Conventions common to all entry points
 *  - Every function returns SPEC_OK (0) or a negative spec_status.  Nothing throws or aborts
 *    across this boundary.  spec_last_error() returns a thread-local message for the last failure.
 *  - "device" pointers are HIP device memory on the GPU that was current at spec_verify_init;
 *    "host" pointers are ordinary process memory.  The caller owns every buffer it passes
 *    (weights, KV cache, kv_len, step inputs and outputs) and the stream; the library owns only
 *    the handle and the workspace inside it, released by spec_verify_destroy.  The library never
 *    frees, reallocates or keeps host pointers beyond the call.
 *  - Work is enqueued on the given hipStream_t (passed as void*; NULL = the default stream) and
 *    is NOT synchronised: outputs are valid once the caller has synchronised the stream.
 *    Calls on one handle must not overlap in time (they share its workspace).
 *    spec_verify_step, spec_verify_tree_step, spec_kv_rollback and spec_sample_step_noalloc only queue
 *    kernels (and one device-to-device copy when target_logits_in and logits_out are both given): no
 *    allocation, no synchronisation, no memset -- they may be recorded into a HIP graph and replayed;
 *    per-sequence lookaheads and rollback lengths are host values and are frozen into the recording.
 *  - Host-checkable arguments are validated before anything is launched.  Conditions that depend
 *    on device data (kv_len + K + 1 > max_kv_len, token id >= vocab, rollback beyond the current
 *    length) make the affected sequence a no-op (its n_accepted is written as -1), raise a flag
 *    in the handle and are reported by spec_verify_poll.
 */
#ifndef SPEC_VERIFY_H
#define SPEC_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPEC_OK = 0,
    SPEC_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, temperature <= 0, ... */
    SPEC_ERR_SHAPE = -2,         /* model shape the kernels do not support (see spec_model_cfg) */
    SPEC_ERR_KV_OVERFLOW = -3,   /* a sequence would outgrow max_kv_len (reported by poll) */
    SPEC_ERR_ALLOC = -4,         /* workspace allocation failed */
    SPEC_ERR_DEVICE = -5,        /* a HIP call failed; message holds hipGetErrorString */
    SPEC_ERR_TOKEN_RANGE = -6,   /* a token id outside [0, vocab) (reported by poll) */
    SPEC_ERR_ROLLBACK = -7       /* rollback to a length above the current one (reported by poll) */
} spec_status;

typedef struct spec_handle spec_handle;   /* opaque */

#define SPEC_DTYPE_FP32 0   /* weights, embedding and KV cache in fp32 (small configurations) */
#define SPEC_DTYPE_BF16 1   /* weights, embedding and KV cache in bf16; fp32 accumulation */
#define SPEC_MAX_BATCH 256
#define SPEC_MAX_LOOKAHEAD 15
#define SPEC_MAX_STEP_ROWS 352   /* bf16 models: window rows (sum of K_b + 1) one pass of the decoder takes */

/* Decoder-only transformer: pre-norm residual blocks, RMSNorm, rotary position embedding with
 * dimension i paired with i + head_dim/2 and angle pos * rope_theta^(-2i/head_dim), grouped-query
 * attention with score scale 1/sqrt(head_dim), SwiGLU feed-forward, untied LM head, no biases.
 * Requirements: n_q_heads % n_kv_heads == 0; head_dim in {64, 128} for bf16 (any even value for
 * fp32); d_model, n_q_heads*head_dim and d_ffn multiples of 32 for bf16;
 * 1 <= max_batch <= SPEC_MAX_BATCH; 0 <= max_lookahead <= SPEC_MAX_LOOKAHEAD.
 * bf16 models: the projections take at most SPEC_MAX_STEP_ROWS rows per launch.  A step (linear or
 * tree) whose windows add up to more rows is scored in several passes of the decoder over groups of
 * consecutive sequences -- the weights are streamed once per pass, everything else (row bookkeeping,
 * sampling, rollback, results) is as for one pass; the decoding round of spec_decode.h does the same
 * for both of its models. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_batch;       /* sequences per step, and number of KV-cache slots */
    int32_t max_kv_len;      /* positions a slot can hold, window tokens included */
    int32_t max_lookahead;   /* largest K of any sequence */
    int32_t dtype;           /* SPEC_DTYPE_* */
    float rms_eps, rope_theta;
} spec_model_cfg;

/* Target weights, all device pointers.
 * Norm gains: fp32[d_model].  tok_embed: dtype[vocab][d_model], rows contiguous.
 * Projection matrices are logically [out_features][in_features] with
 *   w_qkv     out = all query heads, then all key heads, then all value heads; in = d_model
 *   w_o       out = d_model; in = n_q_heads*head_dim
 *   w_gate_up out = d_ffn gate rows then d_ffn up rows; in = d_model
 *   w_down    out = d_model; in = d_ffn
 *   lm_head   out = vocab; in = d_model
 * fp32: stored exactly so, rows contiguous.
 * bf16: stored in the streaming tile order produced by spec_pack_weight (below): a 64-lane
 *       wavefront fetches each 16x32 MFMA operand tile as one contiguous 1 KiB read, and the
 *       whole matrix is read in long sequential streams. */
typedef struct {
    const float* attn_norm;
    const void* w_qkv;
    const void* w_o;
    const float* ffn_norm;
    const void* w_gate_up;
    const void* w_down;
} spec_layer_weights;

typedef struct {
    const void* tok_embed;
    const float* final_norm;
    const void* lm_head;
    const spec_layer_weights* layers;   /* host array of n_layers entries (copied at init) */
} spec_weights;

/* Size in bytes of the packed form of a bf16 [n_out][n_in] matrix (n_out padded to 16 rows,
 * n_in/32 padded to a multiple of 4 blocks); 0 if n_in is not a multiple of 32. */
size_t spec_packed_weight_bytes(int32_t n_out, int32_t n_in);

/* Repack a row-major bf16 [n_out][n_in] device matrix into the streaming tile order.
 * A tile covers output features 16j..16j+15 and input features 32kb..32kb+31 and is 512
 * consecutive elements (1 KiB): element (lane, e), lane in [0,64), e in [0,8), holds
 * W[16j + lane%16][32kb + 8*(lane/16) + e] -- the register layout of the 16x16x32 bf16 matrix
 * instruction's operand, so a wavefront fetches a tile with one 16-byte load per lane.
 * Tiles are ordered [kb/4][j][kb%4]: the 4 K blocks of one column tile are adjacent, then the next
 * column tile, and only then the next group of 4 K blocks.  The tiles that the compute units read
 * at the same time (neighbouring column tiles, same K blocks) are therefore neighbours in memory
 * and the whole matrix is swept in a few long sequential streams.  Rows beyond n_out and K blocks
 * beyond n_in/32 are zero.
 * With interleave_halves != 0 (used for w_gate_up) tile index j takes its 16 rows from the first
 * half of the matrix when j is even (rows 16*(j/2)..) and from the second half when j is odd, so a
 * gate tile and the matching up tile are neighbours; n_out/2 must be a multiple of 16.
 * n_in must be a multiple of 32.  src and dst must not overlap. */
int spec_pack_weight(const void* src_row_major, void* dst_packed, int32_t n_out, int32_t n_in,
                     int32_t interleave_halves, void* stream);

/* Bytes the caller must provide for the KV cache of cfg (all layers, max_batch slots). */
size_t spec_kv_cache_bytes(const spec_model_cfg* cfg);

/* Create a handle for one target model and its KV cache.  The paper's description of the method
 * (section "Speculative Sampling Results") speaks only of a target model that scores the proposals
 * "in parallel"; it says nothing about a cache, so the state kept here is a reading: per cache slot
 * the keys and values of every token the target has processed, in the storage type of the weights
 * (bf16 models: bf16 cache; fp32 models: fp32 cache), entries rounded to that type before anything
 * attends to them, and a length kv_len per slot that the step advances and rolls back.
 * weights and kv_cache may both be NULL for a sampler-only handle (every step
 * must then supply target_logits_in).  kv_cache: device buffer of at least spec_kv_cache_bytes;
 * its internal tile order is private -- fill and read it with spec_kv_import / spec_kv_export.
 * kv_len: device int32[max_batch], number of valid cached positions per slot; read and updated
 * by the step and by rollback.  Allocates the workspace; does not touch the caller's buffers. */
int spec_verify_init(const spec_model_cfg* cfg, const spec_weights* weights, void* kv_cache,
                     size_t kv_cache_bytes, int32_t* kv_len, spec_handle** out);

void spec_verify_destroy(spec_handle* h);

/* Paged cache (bf16 models): instead of one contiguous run per slot, the 32-position blocks of all
 * sequences live in pages of a shared pool; a page holds one block of every layer and kv head
 * (spec_kv_page_bytes).  The library keeps the block table and the list of free pages on the
 * device: a step takes pages for the positions it appends, and whatever lowers a cache length
 * (auto_rollback, spec_kv_rollback, the decoding round) hands pages that hold no valid position
 * back, so rejected proposals cost no memory and the pool may be smaller than
 * max_batch * max_kv_len positions.  A sequence whose step finds the pool empty is skipped
 * (SPEC_ERR_KV_OVERFLOW from spec_verify_poll).  Everything else behaves as with spec_verify_init;
 * results are bit-identical.  kv_pool: device buffer of kv_pool_bytes (>= one page), caller-owned. */
size_t spec_kv_page_bytes(const spec_model_cfg* cfg);
int spec_verify_init_paged(const spec_model_cfg* cfg, const spec_weights* weights, void* kv_pool,
                           size_t kv_pool_bytes, int32_t* kv_len, spec_handle** out);
/* Free and total pages (host ints); synchronises the stream. */
int spec_kv_pages(spec_handle* h, int32_t* free_pages, int32_t* total_pages, void* stream);

/* Inputs of one step.  B = batch; Kmax = cfg.max_lookahead; V = cfg.vocab.
 * Sequence b scores the window [last_token[b], draft_tokens[b][0..K_b-1]] at positions
 * n_b .. n_b+K_b where n_b = kv_len[seq_slot[b]].  Target row j of a sequence gives the
 * distribution of the token following window token j, so row i tests draft i and row K_b is the
 * distribution of the extra token.
 * Logits rows (draft_logits, target_logits_in; the tree step's likewise) may hold -inf entries:
 * tokens of probability zero, as top-k or nucleus filtering leaves them.  A proposal the target
 * excludes is rejected, excluded tokens are never emitted, and a row may consist of a single finite
 * entry.  Every row needs at least one finite logit; NaN and +inf are not supported (the result for
 * that sequence is then unspecified). */
typedef struct {
    int32_t batch;                 /* 1 .. max_batch */
    const int32_t* lookahead;      /* HOST int32[B]: K_b in 0 .. Kmax */
    const int32_t* seq_slot;       /* device int32[B]: distinct cache slots in [0, max_batch) */
    const int32_t* last_token;     /* device int32[B] */
    const int32_t* draft_tokens;   /* device int32[B][Kmax] (entries >= K_b ignored) */
    const float* draft_logits;     /* device fp32[B][Kmax][V]; q_i = softmax(draft_logits[b][i]/T) */
    const float* uniforms;         /* device fp32[B][Kmax+1] in [0,1): [b][i], i < K_b decides draft
                                      i (kept iff u*q(x) < p(x)); [b][K_b] drives the final draw */
    float temperature;             /* > 0: applied to target and draft logits alike.  0: the greedy rule --
                                      draft i is kept iff it is the most likely token of target row i
                                      (lowest id among equal maxima), the final token is the most likely
                                      token of the first mismatching row or of row K_b; draft_logits and
                                      uniforms are not read */
    const float* target_logits_in; /* optional device fp32[M][V], M = sum(K_b+1), rows ordered by
                                      (sequence, window offset): if non-NULL the decoder pass is
                                      skipped and only the sampling part runs */
    int32_t auto_rollback;         /* 0: leave kv_len[slot] = n_b+K_b+1 (whole window appended);
                                      1: write kv_len[slot] = n_b + n_accepted + 1 */
} spec_step_args;

typedef struct {
    int32_t* n_accepted;           /* device int32[B]: number of drafts kept (-1: sequence skipped) */
    int32_t* out_tokens;           /* device int32[B][Kmax+1]: kept drafts, final token, then -1 */
    float* logits_out;             /* optional device fp32[M][V]: target logits of the window */
} spec_step_out;

/* The verify step.  The final token is drawn by inverse CDF in ascending token id: the first id
 * whose inclusive prefix sum of r exceeds u*sum(r), with r = max(0, p_a - q_a) at the first
 * rejected position a, or r = p_K when all K drafts were kept. */
int spec_verify_step(spec_handle* h, const spec_step_args* args, const spec_step_out* out, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the sampling part of spec_verify_step -- what that call
 * does on a sampler-only handle when target_logits_in is given -- without a handle.  The row tables,
 * chunk statistics, chunk masses and the error flag, which a handle keeps in its workspace, live in
 * one fixed device array inside the library (about 0.55 MiB, held by every GPU the library runs on
 * until the process ends), sized for
 *     batch <= SPEC_NOALLOC_MAX_BATCH, max_lookahead <= SPEC_MAX_LOOKAHEAD, vocab <= SPEC_NOALLOC_MAX_VOCAB;
 * anything larger is refused with SPEC_ERR_SHAPE before a kernel is launched.  The call allocates
 * and frees nothing and synchronises nothing; the first call on a device also looks the array's
 * address up (a host-side query), so make one call on a device before capturing any.
 * args: as for spec_verify_step with target_logits_in REQUIRED (device fp32[M][vocab]); seq_slot,
 * last_token and auto_rollback are ignored (no cache is touched); Kmax in the array shapes is the
 * max_lookahead given here.  out: n_accepted and out_tokens as for spec_verify_step; results are
 * bit-identical to that call's.  Device-side conditions (a draft token id outside [0, vocab)) write
 * n_accepted[b] = -1 and out_tokens[b][*] = -1 for that sequence; there is no poll for this call.
 * All calls on one GPU share the array, which keeps the previous call's contents (the call clears
 * what must start at zero itself): calls that overlap in time on one GPU -- different streams or
 * threads -- race and must be serialised by the caller. */
#define SPEC_NOALLOC_MAX_BATCH 64
#define SPEC_NOALLOC_MAX_VOCAB 262144
int spec_sample_step_noalloc(int32_t vocab, int32_t max_lookahead, const spec_step_args* args,
                             const spec_step_out* out, void* stream);

/* Verification of a token TREE per sequence (the tree-structured candidates of the paper's
 * section on EAGLE-style decoding) instead of a chain.  Sequence b proposes N_b <= Kmax nodes in
 * topological order; parent[b][i] is -1 (child of the root = the sequence's last token) or the
 * index (< i) of another node; the children of one node are independent draws from the draft
 * distribution at that node.  Window slot 0 is the root, slot i+1 node i: the decoder pass scores
 * all N_b+1 tokens at once, every token attending to the cache and to the slots on its own path
 * only, at rotary position n_b + depth.  Target row j / draft row j (draft_logits[b][j]) are the two
 * models' next-token distributions after the path to slot j.
 * The walk starts at the root with r = p (the target row of the current node) and q (its draft
 * row): the node's children are tried in index order; child c with token x is kept iff
 * uniforms[b][c] * q(x) < r(x), and then becomes the current node; every rejection replaces r by
 * max(0, r - q) renormalised.  When the current node has no child left, the final token is drawn
 * from r by inverse CDF (as in spec_verify_step) with uniforms[b][N_b].
 * A chain (parent[i] = i-1) gives exactly spec_verify_step.  temperature 0 selects the greedy walk:
 * move to the first child whose token is the most likely token of the current node's target row,
 * otherwise emit that token (draft_logits and uniforms are not read).
 * With auto_rollback the kept nodes' keys and values are moved to positions n_b+1..n_b+a and
 * kv_len[slot] = n_b + a + 1; without it the window stays as scored and kv_len = n_b + N_b + 1. */
typedef struct {
    int32_t batch;
    const int32_t* n_nodes;        /* HOST int32[B]: N_b in 0 .. Kmax */
    const int32_t* seq_slot;       /* device int32[B] */
    const int32_t* last_token;     /* device int32[B] */
    const int32_t* parent;         /* device int32[B][Kmax] */
    const int32_t* draft_tokens;   /* device int32[B][Kmax] */
    const float* draft_logits;     /* device fp32[B][Kmax+1][V]: row 0 the root's, row i+1 node i's.  All
                                      N_b+1 rows of a sequence must be readable: the statistics pass
                                      streams every one of them (the values of rows whose node has no
                                      children do not influence the result) */
    const float* uniforms;         /* device fp32[B][Kmax+1]: [b][i] tests node i, [b][N_b] the final draw */
    float temperature;
    const float* target_logits_in; /* optional device fp32[M][V], M = sum(N_b+1): skip the decoder pass */
    int32_t auto_rollback;
} spec_tree_args;

typedef struct {
    int32_t* n_accepted;           /* device int32[B]: kept nodes a (-1: sequence skipped) */
    int32_t* out_tokens;           /* device int32[B][Kmax+1]: their tokens, the final token, then -1 */
    int32_t* path;                 /* device int32[B][Kmax]: kept node indices root-down, then -1 */
    float* logits_out;             /* optional device fp32[M][V] */
} spec_tree_out;

int spec_verify_tree_step(spec_handle* h, const spec_tree_args* args, const spec_tree_out* out, void* stream);

/* Drop cached positions: the counterpart of the paper's "no more tokens are accepted" after the
 * first rejection (section "Speculative Sampling Results") -- the rejected proposals were appended
 * to the cache when the window was scored and must not be attended to again.  The paper does not
 * describe a cache; the reading taken is that the valid prefix of a slot is [0, kv_len) and that a
 * step leaves kv_len = n + a + 1 (last token and the a kept proposals; the final token is the next
 * step's input).  spec_verify_step does this itself with auto_rollback; this call is for callers
 * that roll back on their own (auto_rollback = 0, abandoning or rewinding a sequence).
 * Set kv_len[seq_slot[i]] = new_len[i] for i < n (host arrays, n <= SPEC_MAX_BATCH).  The cache is
 * contiguous per slot, so dropping rejected positions moves no data; stale entries are never read
 * and are overwritten by the next append.  new_len must satisfy 0 <= new_len <= kv_len[slot]. */
int spec_kv_rollback(spec_handle* h, const int32_t* seq_slot, const int32_t* new_len, int32_t n,
                     void* stream);

/* Copy positions [pos0, pos0+n_pos) of one slot between the cache and a plain device tensor
 * dtype[n_layers][2 (k,v)][n_kv_heads][n_pos][head_dim].  Does not change kv_len.  n_pos = 0 does
 * nothing (the tensor pointer may then be NULL). */
int spec_kv_import(spec_handle* h, int32_t slot, int32_t pos0, int32_t n_pos, const void* src, void* stream);
int spec_kv_export(spec_handle* h, int32_t slot, int32_t pos0, int32_t n_pos, void* dst, void* stream);

/* Synchronise the stream and return the first device-side error raised since the last poll
 * (SPEC_OK if none); clears the flag. */
int spec_verify_poll(spec_handle* h, void* stream);

const char* spec_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
