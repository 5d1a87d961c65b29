// The speculative decoding round (spec_decode.h): K autoregressive steps of the draft model, the
// target's verification of the proposed window, and the bookkeeping that lets the next round start
// from device state alone.  Host code here only queues kernels; the decoder passes, the sampler and
// the cache layout are those of the verify step.
#include <cstring>

#include "cache_layout.h"
#include "handle.h"
#include "../../include/spec_decode.h"

using namespace specv;

struct spec_decoder {
    spec_handle* target = nullptr;
    spec_handle* draft = nullptr;
    int max_batch = 0, cap = 0;
    int Kt = 0;   // the target's max_lookahead: row length of draft_tokens / draft_logits / uniforms
    int Kd = 0;   // the draft's max_lookahead (>= 1): row length of `win`
    int V = 0;
    int B = 0;    // sequences of the active batch
    Arena arena;
    int32_t* seq_slot = nullptr;
    int32_t* prev_tok = nullptr;       // text[L-2]
    int32_t* last_tok = nullptr;       // text[L-1]
    int32_t* win = nullptr;            // [max_batch][Kd]; [b][0] = text[L-1]: second row of draft step 0
    int32_t* cur_tok = nullptr;        // the draft's latest proposal: input of its next step
    int32_t* seq_live = nullptr;       // 0: sequence failed the start check and is skipped for good
    int32_t* draft_tokens = nullptr;   // [max_batch][Kt]
    float* draft_logits = nullptr;     // [max_batch][Kt][V]
    int32_t* n_accepted = nullptr;
    int32_t* round_out = nullptr;      // [max_batch][Kt+1]
    int32_t* out_tokens = nullptr;     // [max_batch][cap]
    int32_t* n_out = nullptr;
    int64_t* counters = nullptr;       // rounds*sequences, proposals kept, tokens emitted
    int last_rows = 0;
    StepTables draw_first{}, draw_next{};   // row of each sequence the draft draws from (step 0 / later)
};

namespace {

constexpr int TPB = 256;

__global__ void __launch_bounds__(TPB) begin_kernel(int B, int max_batch, const int32_t* __restrict__ seq_slot_in,
                                                    const int32_t* __restrict__ prev_in,
                                                    const int32_t* __restrict__ last_in, int Kd, int32_t* seq_slot,
                                                    int32_t* prev_tok, int32_t* last_tok, int32_t* win,
                                                    int32_t* seq_live, int32_t* n_out, int64_t* counters,
                                                    const int32_t* __restrict__ target_len,
                                                    const int32_t* __restrict__ draft_len, int32_t* draft_flag,
                                                    int32_t* row_first, int32_t* row_next, int32_t* stat0_first,
                                                    int32_t* stat0_next)
{
    const int b = threadIdx.x;
    if (b == 0)
        for (int i = 0; i < 3; ++i) counters[i] = 0;
    if (row_first) {   // one statistics row per sequence; its logits row: 2b+1 (two-token step) or b
        for (int i = b; i <= B; i += TPB) {
            row_first[i] = 2 * i + 1;
            row_next[i] = i;
            stat0_first[i] = i;
            stat0_next[i] = i;
        }
    }
    if (b >= B) return;
    const int slot = seq_slot_in[b];
    seq_slot[b] = slot;
    last_tok[b] = last_in[b];
    prev_tok[b] = prev_in ? prev_in[b] : 0;
    if (win) win[b * Kd] = last_in[b];
    n_out[b] = 0;
    int live = 1;
    if (draft_len) {
        if (slot < 0 || slot >= max_batch) live = 0;   // the verify step flags the slot itself
        else if (draft_len[slot] != target_len[slot] - 1) {
            live = 0;
            atomicCAS(draft_flag, 0, (int)SPEC_ERR_INVALID_ARG);
        }
    }
    seq_live[b] = live;
}

// After the verification: append what the round produced, move the two trailing tokens, set the
// draft's cache length.  A skipped sequence (n_accepted < 0) keeps its state.
__global__ void __launch_bounds__(TPB) advance_kernel(int B, int Kt, int Kd, int cap,
                                                      const int32_t* __restrict__ n_accepted,
                                                      const int32_t* __restrict__ round_out,
                                                      const int32_t* __restrict__ draft_tokens,
                                                      const int32_t* __restrict__ target_seq_n,
                                                      const int32_t* __restrict__ target_seq_slot,
                                                      int32_t* prev_tok, int32_t* last_tok, int32_t* win,
                                                      int32_t* out_tokens, int32_t* n_out, int32_t* draft_len,
                                                      PagePool draft_pool, int64_t* counters)
{
    __shared__ int s_kept[TPB], s_emit[TPB], s_run[TPB];
    const int b = threadIdx.x;
    int kept = 0, emitted = 0, ran = 0;
    if (b < B) {
        const int a = n_accepted[b];
        if (a >= 0) {
            const int32_t* o = round_out + b * (Kt + 1);
            const int t0 = last_tok[b];
            const int n = n_out[b];
            for (int j = 0; j <= a; ++j)
                if (n + j < cap) out_tokens[(size_t)b * cap + n + j] = o[j];
            n_out[b] = n + a + 1;
            prev_tok[b] = a >= 1 ? draft_tokens[b * Kt + a - 1] : t0;
            last_tok[b] = o[a];
            if (win) win[b * Kd] = o[a];
            // the text grew to L + a + 1 tokens; the draft has valid entries for all but its last two
            if (draft_len) {
                draft_len[target_seq_slot[b]] = target_seq_n[b] + a;
                pool_trim(draft_pool, target_seq_slot[b], target_seq_n[b] + a);
            }
            kept = a;
            emitted = a + 1;
            ran = 1;
        }
    }
    s_kept[threadIdx.x] = kept;
    s_emit[threadIdx.x] = emitted;
    s_run[threadIdx.x] = ran;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long k = 0, e = 0, r = 0;
        for (int i = 0; i < B; ++i) {
            k += s_kept[i];
            e += s_emit[i];
            r += s_run[i];
        }
        counters[0] += r;
        counters[1] += k;
        counters[2] += e;
    }
}

// Sequences that failed the start check must not run: give them an invalid input token, which the
// row bookkeeping of the step turns into "skipped".
__global__ void __launch_bounds__(TPB) mask_dead_kernel(int B, const int32_t* __restrict__ seq_live, int32_t* last_tok,
                                                        int32_t* prev_tok)
{
    const int b = threadIdx.x;
    if (b < B && !seq_live[b]) {
        last_tok[b] = -1;
        prev_tok[b] = -1;
    }
}

}  // namespace

extern "C" int spec_decode_init(spec_handle* target, spec_handle* draft, const spec_decode_cfg* cfg, spec_decoder** out)
{
    if (!target || !cfg || !out) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: NULL argument");
    if (!target->has_model) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: the target handle has no model");
    if (cfg->max_batch < 1 || cfg->max_batch > target->cfg.max_batch || cfg->max_batch > TPB)
        return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: max_batch %d outside 1..%d", cfg->max_batch,
                    target->cfg.max_batch);
    if (cfg->max_new_tokens < 1) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: max_new_tokens must be >= 1");
    if (draft) {
        if (!draft->has_model) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: the draft handle has no model");
        if (draft->cfg.vocab != target->cfg.vocab)
            return fail(SPEC_ERR_SHAPE, "spec_decode_init: draft vocabulary %d differs from the target's %d",
                        draft->cfg.vocab, target->cfg.vocab);
        if (draft->cfg.max_batch < cfg->max_batch)
            return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: the draft handle holds fewer than %d sequences",
                        cfg->max_batch);
        if (draft->cfg.max_lookahead < 1)
            return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: the draft handle needs max_lookahead >= 1");
        if (target->cfg.max_lookahead < 1)
            return fail(SPEC_ERR_INVALID_ARG, "spec_decode_init: the target handle needs max_lookahead >= 1");
    }
    spec_decoder* d = new spec_decoder();
    d->target = target;
    d->draft = draft;
    d->max_batch = cfg->max_batch;
    d->cap = cfg->max_new_tokens;
    d->Kt = target->cfg.max_lookahead;
    d->Kd = draft ? draft->cfg.max_lookahead : 0;
    d->V = target->cfg.vocab;
    const int B = d->max_batch;
    int rc = SPEC_OK;
    auto A = [&](auto** p, size_t count) {
        if (rc == SPEC_OK) rc = d->arena.alloc(reinterpret_cast<void**>(p), (count ? count : 1) * sizeof(**p));
    };
    A(&d->seq_slot, B);
    A(&d->prev_tok, B);
    A(&d->last_tok, B);
    A(&d->cur_tok, B);
    A(&d->seq_live, B);
    A(&d->n_accepted, B);
    A(&d->round_out, (size_t)B * (d->Kt + 1));
    A(&d->out_tokens, (size_t)B * d->cap);
    A(&d->n_out, B);
    A(&d->counters, 3);
    if (draft) {
        A(&d->win, (size_t)B * d->Kd);
        A(&d->draft_tokens, (size_t)B * d->Kt);
        A(&d->draft_logits, (size_t)B * d->Kt * d->V);
        A(&d->draw_first.seq_row0, B + 1);
        A(&d->draw_first.seq_stat0, B + 1);
        A(&d->draw_next.seq_row0, B + 1);
        A(&d->draw_next.seq_stat0, B + 1);
        if (rc == SPEC_OK && hipMemset(d->win, 0, (size_t)B * d->Kd * sizeof(int32_t)) != hipSuccess)
            rc = fail(SPEC_ERR_DEVICE, "hipMemset failed");
        if (rc == SPEC_OK && hipMemset(d->draft_tokens, 0, (size_t)B * d->Kt * sizeof(int32_t)) != hipSuccess)
            rc = fail(SPEC_ERR_DEVICE, "hipMemset failed");
        // everything but the row choice comes from the tables the draft's own row bookkeeping fills
        for (StepTables* t : {&d->draw_first, &d->draw_next}) {
            t->seq_n = draft->tables.seq_n;
            t->seq_ok = draft->tables.seq_ok;
            t->seq_slot = draft->tables.seq_slot;
            t->row_seq = draft->tables.row_seq;
            t->row_pos = draft->tables.row_pos;
            t->row_tok = draft->tables.row_tok;
            t->row_rope = draft->tables.row_rope;
            t->row_mask = draft->tables.row_mask;
            t->pool = draft->tables.pool;
        }
    }
    if (rc != SPEC_OK) {
        d->arena.release();
        delete d;
        return rc;
    }
    *out = d;
    return SPEC_OK;
}

extern "C" void spec_decode_destroy(spec_decoder* d)
{
    if (!d) return;
    d->arena.release();
    delete d;
}

extern "C" int spec_decode_begin(spec_decoder* d, int32_t batch, const int32_t* seq_slot, const int32_t* prev_token,
                                 const int32_t* last_token, void* stream)
{
    if (!d || !seq_slot || !last_token) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_begin: NULL argument");
    if (d->draft && !prev_token) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_begin: prev_token is NULL");
    if (batch < 1 || batch > d->max_batch)
        return fail(SPEC_ERR_INVALID_ARG, "spec_decode_begin: batch %d outside 1..%d", batch, d->max_batch);
    d->B = batch;
    d->last_rows = 0;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(begin_kernel, dim3(1), dim3(TPB), 0, s, batch, d->target->cfg.max_batch, seq_slot,
                       prev_token, last_token, d->Kd, d->seq_slot, d->prev_tok, d->last_tok, d->win, d->seq_live,
                       d->n_out, d->counters, d->target->kv_len, d->draft ? d->draft->kv_len : nullptr,
                       d->draft ? d->draft->flag : nullptr, d->draw_first.seq_row0, d->draw_next.seq_row0,
                       d->draw_first.seq_stat0, d->draw_next.seq_stat0);
    SPECV_LAUNCH_CHECK("begin_kernel");
    return SPEC_OK;
}

extern "C" int spec_decode_round(spec_decoder* d, const spec_round_args* args, void* stream)
{
    if (!d || !args) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: NULL argument");
    if (d->B < 1) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: no active batch (call spec_decode_begin)");
    const int B = d->B, K = args->lookahead, Kt = d->Kt, V = d->V;
    if (d->draft) {
        if (K < 1 || K > Kt) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: lookahead %d outside 1..%d", K, Kt);
        if (!args->draft_uniforms && args->temperature != 0.f)
            return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: draft_uniforms is NULL");
    } else if (K != 0) {
        return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: a decoder without a draft model runs lookahead 0 only");
    }
    if (!(args->temperature >= 0.f)) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: temperature must be >= 0");
    if (args->lookahead_per_seq)
        for (int b = 0; b < B; ++b)
            if (args->lookahead_per_seq[b] < 0 || args->lookahead_per_seq[b] > K)
                return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: lookahead_per_seq[%d] = %d outside 0..%d", b,
                            args->lookahead_per_seq[b], K);
    const bool greedy = args->temperature == 0.f;
    if (!greedy && !args->verify_uniforms) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_round: verify_uniforms is NULL");
    hipStream_t s = (hipStream_t)stream;
    spec_handle* tg = d->target;
    spec_handle* dr = d->draft;
    tg->tables.tree = 0;
    if (dr) dr->tables.tree = 0;
    int rc;
    LookaheadPack ks;

    if (dr) {
        hipLaunchKernelGGL(mask_dead_kernel, dim3(1), dim3(TPB), 0, s, B, d->seq_live, d->last_tok, d->prev_tok);
        SPECV_LAUNCH_CHECK("mask_dead_kernel");
        LookaheadPack zero;
        memset(&zero, 0, sizeof(zero));
        for (int i = 0; i < K; ++i) {
            // step 0: window [text[L-2], text[L-1]]; later steps: the previous proposal alone
            memset(&ks, 0, sizeof(ks));
            if (i == 0)
                for (int b = 0; b < B; ++b) ks.k[b] = 1;
            const int rows = (i == 0 ? 2 : 1) * B;
            rc = launch_prepare(dr->tables, ks, B, d->Kd, V, dr->cfg.max_batch, dr->cfg.max_kv_len, true, d->seq_slot,
                                i == 0 ? d->prev_tok : d->cur_tok, d->win, dr->kv_len, dr->flag, s);
            if (rc) return rc;
            rc = forward_run_grouped(dr, ks, B, rows, dr->logits, s);
            if (rc) return rc;
            DrawEmit em{};
            em.tokens = d->draft_tokens;
            em.stride = Kt;
            em.offset = i;
            em.next_token = d->cur_tok;
            em.kv_len = dr->kv_len;
            em.kv_add = i == 0 ? 2 : 1;
            em.logits_copy = d->draft_logits + (size_t)i * V;
            em.copy_stride = (size_t)Kt * V;
            if (greedy)
                rc = launch_greedy(i == 0 ? d->draw_first : d->draw_next, dr->sampler, zero, B, 0, V, rows, dr->logits,
                                   nullptr, 0, nullptr, nullptr, nullptr, &em, &dr->prof, s);
            else
                rc = launch_sampler(i == 0 ? d->draw_first : d->draw_next, dr->sampler, zero, B, 0, V, B, dr->logits,
                                    nullptr, nullptr, args->draft_uniforms + i, Kt, args->temperature, 0, nullptr,
                                    nullptr, nullptr, &em, &dr->prof, s);
            if (rc) return rc;
        }
    }

    memset(&ks, 0, sizeof(ks));
    int M = 0, n_stat = 0;
    for (int b = 0; b < B; ++b) {
        const int kb = args->lookahead_per_seq ? args->lookahead_per_seq[b] : K;
        ks.k[b] = (uint8_t)kb;
        M += kb + 1;
        n_stat += 2 * kb + 1;
    }
    rc = launch_prepare(tg->tables, ks, B, Kt, V, tg->cfg.max_batch, tg->cfg.max_kv_len, true, d->seq_slot, d->last_tok,
                        d->draft_tokens, tg->kv_len, tg->flag, s);
    if (rc) return rc;
    rc = forward_run_grouped(tg, ks, B, M, tg->logits, s);
    if (rc) return rc;
    if (greedy)
        rc = launch_greedy(tg->tables, tg->sampler, ks, B, Kt, V, M, tg->logits, d->draft_tokens, 1, tg->kv_len,
                           d->n_accepted, d->round_out, nullptr, &tg->prof, s);
    else
        rc = launch_sampler(tg->tables, tg->sampler, ks, B, Kt, V, n_stat, tg->logits, d->draft_logits,
                            d->draft_tokens, args->verify_uniforms, Kt + 1, args->temperature, 1, tg->kv_len,
                            d->n_accepted, d->round_out, nullptr, &tg->prof, s);
    if (rc) return rc;
    d->last_rows = M;
    hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(TPB), 0, s, B, Kt, d->Kd, d->cap, d->n_accepted, d->round_out,
                       d->draft_tokens, tg->tables.seq_n, tg->tables.seq_slot, d->prev_tok, d->last_tok, d->win,
                       d->out_tokens, d->n_out, dr ? dr->kv_len : nullptr, dr ? dr->tables.pool : PagePool{}, d->counters);
    SPECV_LAUNCH_CHECK("advance_kernel");
    return SPEC_OK;
}

extern "C" int spec_decode_get_view(spec_decoder* d, spec_decode_view* out)
{
    if (!d || !out) return fail(SPEC_ERR_INVALID_ARG, "spec_decode_get_view: NULL argument");
    out->tokens = d->out_tokens;
    out->n_tokens = d->n_out;
    out->n_accepted = d->n_accepted;
    out->draft_tokens = d->draft_tokens;
    out->draft_logits = d->draft_logits;
    out->target_logits = d->target->logits;
    out->prev_token = d->prev_tok;
    out->last_token = d->last_tok;
    out->counters = d->counters;
    return SPEC_OK;
}
