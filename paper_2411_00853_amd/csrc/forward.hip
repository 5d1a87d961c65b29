// The decoder pass of the verify step: the order in which the kernels run for one window.
// Per layer: RMSNorm -> QKV projection -> rotary + KV append -> windowed-causal attention ->
// output projection (+residual) -> RMSNorm -> gate/up projection -> SiLU gating -> down projection
// (+residual); then the final norm and the LM head.  Every reduction of GEMM K-range partial sums
// is folded into the kernel that consumes the GEMM's result.
#include <cmath>
#include <cstring>
#include <vector>

#include "frag.h"
#include "handle.h"

namespace specv {

namespace {
struct Dims {
    int d, dq, dkv, nqkv, F, V;
};
Dims dims_of(const spec_model_cfg& c)
{
    Dims z;
    z.d = c.d_model;
    z.dq = c.n_q_heads * c.head_dim;
    z.dkv = c.n_kv_heads * c.head_dim;
    z.nqkv = z.dq + 2 * z.dkv;
    z.F = c.d_ffn;
    z.V = c.vocab;
    return z;
}
}  // namespace

int forward_init(spec_handle* h, int max_rows)
{
    const spec_model_cfg& c = h->cfg;
    const Dims z = dims_of(c);
    h->max_rows = max_rows;
    if (!h->geom.table) h->geom = make_cache_geom(c);   // a paged handle set its geometry already
    // The bf16 projections take at most GEMM_MAX_ROWS rows per launch.  A handle whose batch and
    // lookahead limits multiply to more than that is still usable: the limit then applies to the rows
    // of each step (the sum of K_b + 1), which the step checks.
    h->row_cap = c.dtype == SPEC_DTYPE_BF16 ? std::min(max_rows, GEMM_MAX_ROWS) : max_rows;
    const int all_rows = max_rows;   // the logits of a whole step, however many passes it takes
    max_rows = h->row_cap;
    int rc = SPEC_OK;
    Arena& a = h->arena;
    auto A = [&](float** p, size_t count) {
        if (rc == SPEC_OK) rc = a.alloc(reinterpret_cast<void**>(p), count * sizeof(float));
    };
    A(&h->x, (size_t)max_rows * z.d);
    A(&h->hn, (size_t)max_rows * z.d);
    A(&h->ssq, (size_t)max_rows * ssq_chunks(z.d));
    A(&h->q, (size_t)max_rows * z.dq);
    A(&h->att, (size_t)max_rows * z.dq);
    A(&h->act, (size_t)max_rows * z.F);
    A(&h->logits, (size_t)all_rows * z.V);
    A(&h->cos_sin, (size_t)c.max_kv_len * c.head_dim);
    size_t part = 0;
    if (c.dtype == SPEC_DTYPE_BF16) {
        // operand fragments: the widest GEMM input (d_model, q width or d_ffn), both planes, at the
        // row-tile count of the largest step; zeroed once so that padding blocks stay zero
        const int kmax = std::max(std::max(z.d, z.dq), z.F);
        const size_t xf_bytes = xfrag_uint4s(gemm_row_tiles(max_rows), 2, kmax) * sizeof(uint4);
        if (rc == SPEC_OK) rc = a.alloc(&h->xf, xf_bytes);
        if (rc == SPEC_OK && hipMemset(h->xf, 0, xf_bytes) != hipSuccess) rc = fail(SPEC_ERR_DEVICE, "hipMemset failed");
        // the gate/up GEMM reads h->xf while its early workgroups already write the down projection's
        // operand, which therefore has a buffer of its own (rows up to the 4 row tiles that path serves)
        const size_t xa_bytes = xfrag_uint4s(gemm_row_tiles(std::min(max_rows, 64)), 2, z.F) * sizeof(uint4);
        if (rc == SPEC_OK) rc = a.alloc(&h->xf_act, xa_bytes);
        if (rc == SPEC_OK && hipMemset(h->xf_act, 0, xa_bytes) != hipSuccess) rc = fail(SPEC_ERR_DEVICE, "hipMemset failed");
        part = gemm_partial_capacity(c, max_rows, h->cu_count);
        const int group = c.n_q_heads / c.n_kv_heads;
        const size_t po = attn_partial_floats(c.max_kv_len, c.max_batch, c.n_kv_heads, group, c.max_lookahead + 1,
                                              c.head_dim, h->cu_count, h->geom.table != nullptr);
        A(&h->attn_part_o, po);
        A(&h->attn_part_ml, po / c.head_dim * 2);
        h->attn_part_cap = po;
    } else {
        // fp32 path: GEMM results are written whole; one buffer wide enough for any of them
        part = (size_t)max_rows * (size_t)std::max(std::max(z.nqkv, 2 * z.F), z.d);
    }
    A(&h->partial, part);
    h->partial_cap = part;
    if (rc) return rc;

    // rotary table in fp64 on the host: cos, sin of pos * theta^(-2i/hd)
    const int half = c.head_dim / 2;
    std::vector<float> tab((size_t)c.max_kv_len * c.head_dim);
    for (int pos = 0; pos < c.max_kv_len; ++pos)
        for (int i = 0; i < half; ++i) {
            const double ang = (double)pos * std::pow((double)c.rope_theta, -2.0 * i / (double)c.head_dim);
            tab[((size_t)pos * half + i) * 2 + 0] = (float)std::cos(ang);
            tab[((size_t)pos * half + i) * 2 + 1] = (float)std::sin(ang);
        }
    SPECV_HIP(hipMemcpy(h->cos_sin, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice));
    return SPEC_OK;
}

// partial-sum space (floats) for the largest projection at any row count up to max_rows
size_t gemm_partial_capacity(const spec_model_cfg& c, int max_rows, int cu_count)
{
    const Dims z = dims_of(c);
    const int Ns[G_COUNT] = {z.nqkv, z.d, 2 * z.F, z.d, z.V};
    const int Ks[G_COUNT] = {z.d, z.dq, z.d, z.F, z.d};
    size_t part = 0;
    for (int M = 16; M <= (max_rows + 15) / 16 * 16 && M <= GEMM_MAX_ROWS; M += 16)
        for (int i = 0; i < G_COUNT; ++i) {
            const int rows = M < max_rows ? M : max_rows;
            const size_t e = gemm_partial_elems(plan_gemm(rows, Ns[i], Ks[i], cu_count, true), rows);
            if (e > part) part = e;
        }
    return part;
}

void projection_shapes(const spec_model_cfg& c, int* n_out, int* n_in)
{
    const Dims z = dims_of(c);
    const int Ns[G_COUNT] = {z.nqkv, z.d, 2 * z.F, z.d, z.V};
    const int Ks[G_COUNT] = {z.d, z.dq, z.d, z.F, z.d};
    for (int i = 0; i < G_COUNT; ++i) {
        n_out[i] = Ns[i];
        n_in[i] = Ks[i];
    }
}

// Decoder passes of a step of M rows when one pass takes at most cap: groups of consecutive sequences,
// as few groups as filling each to the brim would give (every pass streams all the weights), and among
// the partitions with that many groups the one whose largest group is smallest.  Returns the number of
// passes (0 if max_passes is too few).
int plan_passes(const LookaheadPack& ks, int B, int M, int cap, int* pass_seqs, int* pass_rows, int max_passes)
{
    // groups when each takes sequences while they fit under `limit`
    auto fill = [&](int limit, bool record) {
        int b0 = 0, n = 0;
        while (b0 < B) {
            int Bg = 0, Mg = 0;
            while (b0 + Bg < B && Mg + ks.k[b0 + Bg] + 1 <= limit) {
                Mg += ks.k[b0 + Bg] + 1;
                ++Bg;
            }
            if (Bg == 0) return B + 1;          // a window longer than the limit: no partition
            if (record) {
                if (n == max_passes) return 0;
                pass_seqs[n] = Bg;
                pass_rows[n] = Mg;
            }
            ++n;
            b0 += Bg;
        }
        return n;
    };
    const int fewest = fill(cap, false);
    int limit = (M + fewest - 1) / fewest;       // no partition into `fewest` groups has a smaller largest group
    while (limit < cap && fill(limit, false) > fewest) ++limit;
    return fill(limit, true);
}

int forward_run_grouped(spec_handle* h, const LookaheadPack& ks, int B, int M, float* logits_out, hipStream_t s)
{
    if (M <= h->row_cap) return forward_run(h, h->tables, ks, B, M, logits_out, s);
    if (!h->group_tables.seq_row0) return fail(SPEC_ERR_SHAPE, "%d window rows exceed the %d the handle takes", M, h->row_cap);
    int pass_seqs[SPEC_PLAN_MAX_PASSES], pass_rows[SPEC_PLAN_MAX_PASSES];
    const int n_passes = plan_passes(ks, B, M, h->row_cap, pass_seqs, pass_rows, SPEC_PLAN_MAX_PASSES);
    if (n_passes == 0) return fail(SPEC_ERR_SHAPE, "a step of %d rows needs more than %d decoder passes", M, SPEC_PLAN_MAX_PASSES);
    StepTables sub = h->group_tables;
    sub.pool = h->tables.pool;
    sub.tree = h->tables.tree;
    int b0 = 0, r0 = 0;
    for (int g = 0; g < n_passes; ++g) {
        LookaheadPack kg;
        memset(&kg, 0, sizeof(kg));
        for (int i = 0; i < pass_seqs[g]; ++i) kg.k[i] = ks.k[b0 + i];
        int rc = launch_slice_tables(h->tables, sub, b0, pass_seqs[g], s);
        if (rc) return rc;
        rc = forward_run(h, sub, kg, pass_seqs[g], pass_rows[g], logits_out + (size_t)r0 * h->cfg.vocab, s);
        if (rc) return rc;
        b0 += pass_seqs[g];
        r0 += pass_rows[g];
    }
    return SPEC_OK;
}

int forward_run(spec_handle* h, const StepTables& t, const LookaheadPack& ks, int B, int M, float* logits_out, hipStream_t s)
{
    const spec_model_cfg& c = h->cfg;
    const Dims z = dims_of(c);
    const bool bf16 = c.dtype == SPEC_DTYPE_BF16;
    int rc;
    if (M < 1 || M > h->row_cap) return fail(SPEC_ERR_SHAPE, "%d window rows; the handle takes 1..%d per step", M, h->row_cap);
#define RUN(cls, expr)                          \
    do {                                        \
        {                                       \
            ProfScope ps_(&h->prof, cls, s);    \
            rc = (expr);                        \
        }                                       \
        if (rc) return rc;                      \
    } while (0)

    // bf16 path: every producer writes the next GEMM's operand as fragments of (value * gain); the
    // GEMM leaves K-range partial sums in h->partial, and its consumer adds them up and applies the
    // row's 1/rms where the operand was a normalised residual.  fp32 path: plain rows, normalisation
    // materialised, GEMM results whole.
    struct Out {
        int n_split;
        size_t stride;
        int ld;
    };
    const int n_ssq = ssq_chunks(z.d);
    const int mt = bf16 ? gemm_row_tiles(M) : 0;
    const int planes = h->split_act ? 2 : 1;
    const XOut to_xf{bf16 ? h->xf : nullptr, mt, planes, nullptr};            // operand of QKV / gate-up / LM head
    const XOut to_att{bf16 ? h->xf : nullptr, mt, planes, bf16 ? nullptr : h->att};
    const XOut to_act{bf16 ? h->xf : nullptr, mt, planes, bf16 ? nullptr : h->act};
    const NormScale scaled{bf16 ? h->ssq : nullptr, n_ssq, z.d, c.rms_eps};
    const NormScale unscaled{nullptr, 0, 0, 0.f};
    auto gemm = [&](int cls, const float* plain_in, const float* gain, const void* w, int N, int K, Out* o,
                    const void* in_frags = nullptr) -> int {
        if (bf16) {
            const GemmPlan p = plan_gemm(M, N, K, h->cu_count, h->split_act);
            // the plan follows process-wide tuning knobs; the buffer was sized with those in force at init
            if (gemm_partial_elems(p, M) > h->partial_cap)
                return fail(SPEC_ERR_SHAPE, "this step's GEMM plan (%d K ranges) needs %zu partial sums, the handle holds %zu: "
                            "set the GEMM tuning knobs before spec_verify_init", p.n_split, gemm_partial_elems(p, M),
                            h->partial_cap);
            o->n_split = p.n_split;
            o->ld = p.n_pad;
            o->stride = (size_t)M * p.n_pad;
            ProfScope ps_(&h->prof, cls, s);
            return launch_gemm_bf16(p, in_frags ? in_frags : h->xf, w, M, N, K, h->partial, s);
        }
        o->n_split = 1;
        o->ld = N;
        o->stride = 0;
        if (gain) {
            ProfScope ps_(&h->prof, SPEC_PROF_GLUE, s);
            int r = launch_rmsnorm_apply(plain_in, h->ssq, gain, c.rms_eps, M, z.d, h->hn, s);
            if (r) return r;
            plain_in = h->hn;
        }
        ProfScope ps_(&h->prof, cls, s);
        return launch_gemm_f32(plain_in, (const float*)w, M, N, K, h->partial, s);
    };

    RUN(SPEC_PROF_GLUE, launch_embed(c.dtype, h->tok_embed, t.row_tok, M, z.d, h->x, h->ssq, h->layers[0].attn_norm, to_xf, s));
    Out o;
    const bool swiglu_in_gemm = bf16 && gemm_swiglu_fits(M, z.F, h->cu_count);
    const bool fuse = h->fuse_rope && attention_takes_qkv(h->geom, c.n_q_heads, ks, B, c.max_kv_len, h->cu_count);
    for (int l = 0; l < c.n_layers; ++l) {
        const spec_layer_weights& w = h->layers[l];
        rc = gemm(SPEC_PROF_GEMM_QKV, h->x, w.attn_norm, w.w_qkv, z.nqkv, z.d, &o);
        if (rc) return rc;
        if (fuse) {
            // the attention kernel adds up, scales and rotates q, k, v itself and appends k, v
            const QkvSrc qkv{h->partial, o.n_split, o.stride, o.ld, scaled, h->cos_sin};
            rc = launch_attention(c.max_kv_len, h->cu_count, t, ks, B, M, h->geom, c.n_q_heads, l, h->kv_cache,
                                  h->q, h->attn_part_o, h->attn_part_ml, h->attn_part_cap, to_att, c.max_lookahead + 1, &h->prof, s, &qkv,
                                  h->kv_cache);
        } else {
            RUN(SPEC_PROF_GLUE, launch_rope_append(h->partial, o.n_split, o.stride, o.ld, t, M, h->geom, c.n_q_heads, l,
                                                   h->cos_sin, scaled, h->kv_cache, h->q, s));
            rc = launch_attention(c.max_kv_len, h->cu_count, t, ks, B, M, h->geom, c.n_q_heads, l, h->kv_cache,
                                  h->q, h->attn_part_o, h->attn_part_ml, h->attn_part_cap, to_att, c.max_lookahead + 1, &h->prof, s);
        }
        if (rc) return rc;
        rc = gemm(SPEC_PROF_GEMM_O, h->att, nullptr, w.w_o, z.d, z.dq, &o);
        if (rc) return rc;
        RUN(SPEC_PROF_GLUE, launch_resid(h->partial, o.n_split, o.stride, o.ld, M, z.d, h->x, h->ssq, w.ffn_norm, to_xf, s));
        if (swiglu_in_gemm) {
            // the gate/up GEMM applies the norm's row scale and SwiGLU itself and writes the down
            // projection's operand (into the second fragment buffer: it is still reading the first)
            RUN(SPEC_PROF_GEMM_GATE_UP, launch_gemm_swiglu(h->xf, planes, w.w_gate_up, M, z.F, z.d, h->ssq, n_ssq, z.d, c.rms_eps,
                                                   h->xf_act, mt, planes, h->cu_count, s));
            rc = gemm(SPEC_PROF_GEMM_DOWN, h->act, nullptr, w.w_down, z.d, z.F, &o, h->xf_act);
        } else {
            rc = gemm(SPEC_PROF_GEMM_GATE_UP, h->x, w.ffn_norm, w.w_gate_up, 2 * z.F, z.d, &o);
            if (rc) return rc;
            RUN(SPEC_PROF_GLUE, launch_silu_mul(h->partial, o.n_split, o.stride, o.ld, M, z.F, bf16, scaled, to_act, s));
            rc = gemm(SPEC_PROF_GEMM_DOWN, h->act, nullptr, w.w_down, z.d, z.F, &o);
        }
        if (rc) return rc;
        const float* next_gain = (l + 1 < c.n_layers) ? h->layers[l + 1].attn_norm : h->final_norm;
        RUN(SPEC_PROF_GLUE, launch_resid(h->partial, o.n_split, o.stride, o.ld, M, z.d, h->x, h->ssq, next_gain, to_xf, s));
    }
    if (bf16) {
        rc = gemm(SPEC_PROF_GEMM_LM_HEAD, h->x, h->final_norm, h->lm_head, z.V, z.d, &o);
        if (rc) return rc;
        RUN(SPEC_PROF_GLUE, launch_reduce_splits(h->partial, o.n_split, o.stride, M, z.V, o.ld, h->ssq, n_ssq, z.d, c.rms_eps,
                                 logits_out, s));
    } else {
        RUN(SPEC_PROF_GLUE, launch_rmsnorm_apply(h->x, h->ssq, h->final_norm, c.rms_eps, M, z.d, h->hn, s));
        RUN(SPEC_PROF_GEMM_LM_HEAD, launch_gemm_f32(h->hn, (const float*)h->lm_head, M, z.V, z.d, logits_out, s));
    }
    (void)unscaled;
#undef RUN
    return SPEC_OK;
}

}  // namespace specv
