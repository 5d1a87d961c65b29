/*
 * spec_decode.h -- the whole speculative decoding round on the GPU, built on spec_verify.h.
 *
 * Section "Speculative Sampling Results" of the paper: a small draft model decodes K tokens in the
 * ordinary autoregressive way, the target model scores them in one pass, a prefix is kept by
 * comparing the two models' probabilities, the first rejected position is resampled (or one extra
 * token drawn), and the loop repeats.  spec_verify_step is the second half of that round; this
 * header adds the first half and the bookkeeping between rounds, so that any number of rounds can be
 * queued on a stream without the host reading anything back.
 *
 * One round, for every sequence b of the batch (L = current length of its text):
 *   1. draft step 0 feeds the last two tokens of the text (positions L-2, L-1) as one causal window
 *      and draws proposal x_1 from softmax(logits of the second row / T) by inverse CDF with
 *      draft_uniforms[b][0]; draft steps i = 1..K-1 feed x_i at position L-1+i and draw x_{i+1} with
 *      draft_uniforms[b][i].  (Feeding two tokens first makes the round uniform: when the previous
 *      round kept all its proposals the draft has not yet seen the last of them; when it has, the
 *      entry is simply computed again.)  The logits row each proposal was drawn from is kept.
 *   2. the target verifies the window [last token, x_1..x_K] exactly as spec_verify_step does, with
 *      verify_uniforms[b][0..K], and rolls its cache length back to L + a  (a = kept proposals).
 *   3. the a kept proposals and the final token are appended to the sequence's output list; the last
 *      two tokens of the text are updated; the draft's cache length is set to L + a - 1.
 *
 * Preconditions when a batch is started (spec_decode_begin): for each sequence the target's cache
 * holds the text without its last token (kv_len = L-1) and the draft's cache the text without its
 * last two tokens (kv_len = L-2), in the same slot number of both handles.  The two handles must
 * have the same vocabulary; both are used only through this decoder while a batch is active.
 *
 * Conventions as in spec_verify.h: device pointers unless marked host, int32 ids, asynchronous on
 * the given stream, negative status + spec_last_error() for host-detectable errors; sequences with
 * bad device data are skipped and reported by spec_verify_poll on the handle concerned.
 */
#ifndef SPEC_DECODE_H
#define SPEC_DECODE_H

#include "spec_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spec_decoder spec_decoder;

typedef struct {
    int32_t max_batch;       /* <= max_batch of both handles */
    int32_t max_new_tokens;  /* capacity of each sequence's output list */
} spec_decode_cfg;

/* draft may be NULL: then only rounds with lookahead 0 are possible (plain autoregressive sampling
 * from the target, one token per round -- the baseline the method is compared with).
 * The handles are borrowed and must outlive the decoder; the decoder owns its device state. */
int spec_decode_init(spec_handle* target, spec_handle* draft, const spec_decode_cfg* cfg, spec_decoder** out);
void spec_decode_destroy(spec_decoder* d);

/* Start `batch` sequences.  seq_slot, prev_token (text[L-2]; ignored without a draft) and last_token
 * (text[L-1]): device int32[batch], copied.  Output lists are emptied.  Sequences whose draft cache
 * length is not the target's minus one are skipped in every round (flag on the draft handle). */
int spec_decode_begin(spec_decoder* d, int32_t batch, const int32_t* seq_slot, const int32_t* prev_token,
                      const int32_t* last_token, void* stream);

typedef struct {
    int32_t lookahead;              /* K of this round for every sequence: 1..target max_lookahead with a
                                       draft, 0 without */
    const float* draft_uniforms;    /* fp32 [batch][Kt], Kt = target max_lookahead; NULL when K = 0 */
    const float* verify_uniforms;   /* fp32 [batch][Kt+1] */
    float temperature;              /* > 0: used by both models.  0: greedy decoding -- every proposal is
                                       the draft's most likely token, the verification is the greedy rule of
                                       spec_verify_step, and neither uniforms array is read (the emitted
                                       text is then the target's greedy text whatever the draft proposes) */
    const int32_t* lookahead_per_seq; /* optional HOST int32[batch]: K_b in 0..lookahead, the proposals of
                                       sequence b that are put to the target (the draft still runs
                                       `lookahead` steps for the whole batch; the rest of a sequence's
                                       proposals are dropped).  NULL: K_b = lookahead for every sequence.
                                       Rows of target_logits and uniforms follow spec_verify_step: sequence b
                                       has K_b + 1 rows, its final draw reads verify_uniforms[b][K_b] */
} spec_round_args;

/* Queue one round.  Launches only; reads nothing back. */
int spec_decode_round(spec_decoder* d, const spec_round_args* args, void* stream);

typedef struct {
    const int32_t* tokens;        /* device [max_batch][max_new_tokens]: generated tokens per sequence */
    const int32_t* n_tokens;      /* device [max_batch]: how many (may exceed max_new_tokens: the excess
                                     was dropped) */
    const int32_t* n_accepted;    /* device [max_batch]: kept proposals of the latest round, -1 = skipped */
    const int32_t* draft_tokens;  /* device [max_batch][Kt]: proposals of the latest round */
    const float* draft_logits;    /* device [max_batch][Kt][vocab]: the rows they were drawn from */
    const float* target_logits;   /* device [batch*(K+1)][vocab]: the latest verification's rows */
    const int32_t* prev_token;    /* device [max_batch]: text[L-2] after the latest round */
    const int32_t* last_token;    /* device [max_batch]: text[L-1] after the latest round */
    const int64_t* counters;      /* device int64[3]: sequence-rounds run, proposals kept, tokens emitted,
                                     summed since spec_decode_begin */
} spec_decode_view;

/* Pointers into the decoder's device state (valid until destroy; contents follow the stream). */
int spec_decode_get_view(spec_decoder* d, spec_decode_view* out);

/* ---- choosing the lookahead -------------------------------------------------------------------
 * The paper's theme is that the amount of speculative work should follow the data.  For the round
 * above that is the choice of K: long windows pay when proposals are usually kept, short ones when
 * they are not.  This controller keeps, per sequence, exponentially forgotten counts of proposals
 * tested and kept, and picks for the next round the K that maximises the predicted tokens per
 * millisecond of the whole batch:
 *     alpha_b = (kept_b + prior_accept * prior_weight) / (tested_b + prior_weight)
 *     tokens(K) = sum_b (1 - alpha_b^(K+1)) / (1 - alpha_b)        (K+1 when alpha_b = 1)
 *     cost(K)   = K * draft_ms + verify_ms + K * verify_ms_per_token
 *     K_next    = the smallest K in [k_min, k_max] with the largest tokens(K) / cost(K)
 * After a round with lookahead K in which sequence b kept a_b proposals, a_b + 1 proposals were
 * tested if a_b < K, else K:   tested_b <- forget * tested_b + min(a_b + 1, K),
 * kept_b <- forget * kept_b + a_b.  Sequences with a_b < 0 (skipped) are left alone.
 * All host-side, double precision, no device access: the caller copies n_accepted back itself.
 * One K per round for the whole batch sets the number of draft steps: those are launched for the batch
 * and cost what the longest window costs; the estimates are kept per sequence because tokens(K) is a
 * sum over sequences with different alpha_b.
 * On top of that K the controller can give every sequence a window of its own (spec_lookahead_next_per_seq,
 * for spec_round_args.lookahead_per_seq): with rate = tokens(K) / cost(K) of the chosen K, proposal k of
 * sequence b is put to the target only while the chance that it is reached and kept, alpha_b^k, is
 * worth the verification row it costs at that rate:
 *     K_b = the largest k in [1, K] with alpha_b^k >= rate * verify_ms_per_token / batch, else 1
 * (the verification's cost per unit of K is shared by the batch's rows; at least one proposal is always
 * tested, or a sequence that fell behind could never show that it has recovered).  With the costs measured on
 * this hardware a row is so cheap next to a draft step that K_b = K almost always: what adapts to the
 * data is the one K; the per-sequence windows are there for cost models where rows are dear. */
typedef struct {
    double draft_ms;             /* cost of one draft decode step for the batch */
    double verify_ms;            /* cost of a verification with an empty window (K = 0) */
    double verify_ms_per_token;  /* added cost per unit of K */
    int32_t k_min, k_max;        /* 1 <= k_min <= k_max <= SPEC_MAX_LOOKAHEAD */
    double forget;               /* in (0, 1]: weight of the past per round */
    double prior_accept;         /* in [0, 1]: acceptance assumed before any evidence */
    double prior_weight;         /* > 0: how many tested proposals the prior counts for */
} spec_lookahead_cfg;

typedef struct spec_lookahead spec_lookahead;

int spec_lookahead_init(const spec_lookahead_cfg* cfg, int32_t batch, spec_lookahead** out);
void spec_lookahead_destroy(spec_lookahead* c);
/* n_accepted: HOST int32[batch] of the round just finished, which ran with lookahead K */
int spec_lookahead_update(spec_lookahead* c, const int32_t* n_accepted, int32_t K);
/* K for the next round (k_min..k_max), or a negative status */
int32_t spec_lookahead_next(const spec_lookahead* c);
/* The same K, and in K_out (HOST int32[batch]) every sequence's own window 1..K (rule above). */
int32_t spec_lookahead_next_per_seq(const spec_lookahead* c, int32_t* K_out);
/* After a round with windows of their own: as spec_lookahead_update with K_b in place of K
 * (K_per_seq: HOST int32[batch], each 0..SPEC_MAX_LOOKAHEAD; a sequence with K_b = 0 tested nothing). */
int spec_lookahead_update_per_seq(spec_lookahead* c, const int32_t* n_accepted, const int32_t* K_per_seq);
/* current estimate alpha_b of one sequence (diagnostics); NaN if out of range */
double spec_lookahead_accept(const spec_lookahead* c, int32_t b);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_DECODE_H */
