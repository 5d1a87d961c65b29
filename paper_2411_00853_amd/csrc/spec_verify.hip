// C ABI of the verify step: handle, argument checks, workspace, and the order of kernel launches.
// Every step of the path runs in the kernels of this library; this file only validates, sizes and
// enqueues.
#include "common.h"
#include <vector>

#include "frag.h"
#include "handle.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

namespace specv {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(int status, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

int Arena::alloc(void** out, size_t bytes)
{
    *out = nullptr;
    if (bytes == 0) bytes = 16;
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(SPEC_ERR_ALLOC, "workspace allocation of %zu bytes failed", bytes);
    }
    blocks.push_back(p);
    total += bytes;
    *out = p;
    return SPEC_OK;
}

void Arena::release()
{
    for (void* p : blocks) (void)hipFree(p);
    blocks.clear();
    total = 0;
}

void Profiler::begin(int cls, hipStream_t s)
{
    if (used == cap) {
        const int ncap = cap ? cap * 2 : 1024;
        Rec* n = static_cast<Rec*>(realloc(recs, sizeof(Rec) * ncap));
        if (!n) return;
        recs = n;
        for (int i = cap; i < ncap; ++i) {
            (void)hipEventCreate(&recs[i].start);
            (void)hipEventCreate(&recs[i].stop);
        }
        cap = ncap;
    }
    recs[used].cls = cls;
    (void)hipEventRecord(recs[used].start, s);
}

void Profiler::end(hipStream_t s)
{
    if (used < cap) (void)hipEventRecord(recs[used++].stop, s);
}

static int check_cfg(const spec_model_cfg* c, bool has_model)
{
    if (!c) return fail(SPEC_ERR_INVALID_ARG, "cfg is NULL");
    if (c->vocab <= 0) return fail(SPEC_ERR_INVALID_ARG, "vocab must be positive");
    if (c->max_batch < 1 || c->max_batch > SPEC_MAX_BATCH)
        return fail(SPEC_ERR_INVALID_ARG, "max_batch must be in 1..%d", SPEC_MAX_BATCH);
    if (c->max_lookahead < 0 || c->max_lookahead > SPEC_MAX_LOOKAHEAD)
        return fail(SPEC_ERR_INVALID_ARG, "max_lookahead must be in 0..%d", SPEC_MAX_LOOKAHEAD);
    if (!has_model) return SPEC_OK;
    if (c->dtype != SPEC_DTYPE_FP32 && c->dtype != SPEC_DTYPE_BF16)
        return fail(SPEC_ERR_INVALID_ARG, "dtype must be SPEC_DTYPE_FP32 or SPEC_DTYPE_BF16");
    if (c->n_layers <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0
        || c->d_ffn <= 0 || c->max_kv_len <= 0)
        return fail(SPEC_ERR_INVALID_ARG, "model dimensions must be positive");
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f))
        return fail(SPEC_ERR_INVALID_ARG, "rms_eps must be >= 0 and rope_theta > 0");
    if (c->n_q_heads % c->n_kv_heads) return fail(SPEC_ERR_SHAPE, "n_q_heads must be a multiple of n_kv_heads");
    if (c->head_dim & 1) return fail(SPEC_ERR_SHAPE, "head_dim must be even");
    if (c->max_kv_len < c->max_lookahead + 1)
        return fail(SPEC_ERR_SHAPE, "max_kv_len must hold at least one window");
    if (c->dtype == SPEC_DTYPE_BF16) {
        if (c->head_dim != 64 && c->head_dim != 128) return fail(SPEC_ERR_SHAPE, "bf16 needs head_dim 64 or 128");
        if (c->d_model % 32 || (c->n_q_heads * c->head_dim) % 32 || c->d_ffn % 32)
            return fail(SPEC_ERR_SHAPE, "bf16 needs d_model, n_q_heads*head_dim and d_ffn multiples of 32");
    } else {
        if (c->head_dim > 256) return fail(SPEC_ERR_SHAPE, "fp32 needs head_dim <= 256");
    }
    return SPEC_OK;
}

}  // namespace specv

using namespace specv;

extern "C" const char* spec_last_error(void) { return g_err; }

extern "C" size_t spec_kv_cache_bytes(const spec_model_cfg* c)
{
    if (check_cfg(c, true) != SPEC_OK) return 0;
    CacheGeom g = make_cache_geom(*c);
    return g.layer_stride * (size_t)c->n_layers * (c->dtype == SPEC_DTYPE_BF16 ? 2 : 4);
}

extern "C" size_t spec_kv_page_bytes(const spec_model_cfg* c)
{
    if (check_cfg(c, true) != SPEC_OK || c->dtype != SPEC_DTYPE_BF16) return 0;
    return (size_t)c->n_layers * c->n_kv_heads * 64 * c->head_dim * 2;
}

static int init_common(const spec_model_cfg* cfg, const spec_weights* weights, void* kv_cache, size_t kv_cache_bytes,
                       int32_t* kv_len, bool paged, spec_handle** out);

extern "C" int spec_verify_init(const spec_model_cfg* cfg, const spec_weights* weights, void* kv_cache,
                                size_t kv_cache_bytes, int32_t* kv_len, spec_handle** out)
{
    return init_common(cfg, weights, kv_cache, kv_cache_bytes, kv_len, false, out);
}

extern "C" int spec_verify_init_paged(const spec_model_cfg* cfg, const spec_weights* weights, void* kv_pool,
                                      size_t kv_pool_bytes, int32_t* kv_len, spec_handle** out)
{
    if (!weights) return fail(SPEC_ERR_INVALID_ARG, "a paged handle needs a model");
    return init_common(cfg, weights, kv_pool, kv_pool_bytes, kv_len, true, out);
}

static int init_common(const spec_model_cfg* cfg, const spec_weights* weights, void* kv_cache, size_t kv_cache_bytes,
                       int32_t* kv_len, bool paged, spec_handle** out)
{
    if (!out) return fail(SPEC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    const bool has_model = weights != nullptr;
    int rc = check_cfg(cfg, has_model);
    if (rc) return rc;
    if (has_model) {
        if (!kv_cache || !kv_len) return fail(SPEC_ERR_INVALID_ARG, "a handle with weights needs kv_cache and kv_len");
        if (!weights->tok_embed || !weights->final_norm || !weights->lm_head || !weights->layers)
            return fail(SPEC_ERR_INVALID_ARG, "weights has a NULL member");
        for (int l = 0; l < cfg->n_layers; ++l) {
            const spec_layer_weights& w = weights->layers[l];
            if (!w.attn_norm || !w.w_qkv || !w.w_o || !w.ffn_norm || !w.w_gate_up || !w.w_down)
                return fail(SPEC_ERR_INVALID_ARG, "layer %d has a NULL weight", l);
        }
        if (paged) {
            if (cfg->dtype != SPEC_DTYPE_BF16) return fail(SPEC_ERR_SHAPE, "a paged cache needs the bf16 storage type");
            if (kv_cache_bytes < spec_kv_page_bytes(cfg)) return fail(SPEC_ERR_INVALID_ARG, "the pool holds no whole page");
        } else {
            const size_t need = spec_kv_cache_bytes(cfg);
            if (kv_cache_bytes < need)
                return fail(SPEC_ERR_INVALID_ARG, "kv_cache_bytes %zu is below the required %zu", kv_cache_bytes, need);
        }
    } else if (kv_cache) {
        return fail(SPEC_ERR_INVALID_ARG, "kv_cache given without weights");
    }

    spec_handle* h = new (std::nothrow) spec_handle();
    if (!h) return fail(SPEC_ERR_ALLOC, "out of host memory");
    h->cfg = *cfg;
    h->has_model = has_model;
    h->kv_cache = kv_cache;
    h->kv_len = kv_len;
    hipError_t e = hipGetDevice(&h->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, h->device);
    if (e != hipSuccess) {
        delete h;
        return fail(SPEC_ERR_DEVICE, "no usable HIP device: %s", hipGetErrorString(e));
    }
    h->cu_count = prop.multiProcessorCount;

    const int B = cfg->max_batch, Kmax = cfg->max_lookahead, V = cfg->vocab;
    const int max_rows = B * (Kmax + 1);
    const int max_stat = B * (2 * Kmax + 2);   // a tree has a draft row for its root as well
    const int n_stat_chunks = (V + STAT_CHUNK - 1) / STAT_CHUNK;
    const int n_res_chunks = (V + RES_CHUNK - 1) / RES_CHUNK;
    Arena& a = h->arena;
    rc = SPEC_OK;
    auto A = [&](auto** p, size_t count) {
        if (rc == SPEC_OK) rc = a.alloc(reinterpret_cast<void**>(p), count * sizeof(**p));
    };
    A(&h->flag, 4);
    A(&h->tables.seq_row0, B + 1);
    A(&h->tables.seq_stat0, B + 1);
    A(&h->tables.seq_n, B);
    A(&h->tables.seq_ok, B);
    A(&h->tables.seq_slot, B);
    A(&h->tables.row_seq, max_rows);
    A(&h->tables.row_pos, max_rows);
    A(&h->tables.row_tok, max_rows);
    A(&h->tables.row_rope, max_rows);
    A(&h->tables.row_mask, max_rows);
    if (cfg->dtype == SPEC_DTYPE_BF16 && max_rows > GEMM_MAX_ROWS && weights) {
        // a step may need several decoder passes: tables for one pass's share
        StepTables& g = h->group_tables;
        A(&g.seq_row0, B + 1);
        A(&g.seq_stat0, B + 1);
        A(&g.seq_n, B);
        A(&g.seq_ok, B);
        A(&g.seq_slot, B);
        A(&g.row_seq, GEMM_MAX_ROWS);
        A(&g.row_pos, GEMM_MAX_ROWS);
        A(&g.row_tok, GEMM_MAX_ROWS);
        A(&g.row_rope, GEMM_MAX_ROWS);
        A(&g.row_mask, GEMM_MAX_ROWS);
    }
    A(&h->sampler.part_max, (size_t)max_stat * n_stat_chunks);
    A(&h->sampler.part_sum, (size_t)max_stat * n_stat_chunks);
    A(&h->sampler.chunk_mass, (size_t)B * n_res_chunks);
    A(&h->sampler.accepted, B);
    A(&h->sampler.row_inv_z, 2 * (size_t)B);
    A(&h->sampler.row_max, 2 * (size_t)B);
    A(&h->sampler.part_idx, (size_t)max_stat * n_stat_chunks);
    if (rc == SPEC_OK && hipMemset(h->flag, 0, 16) != hipSuccess) rc = fail(SPEC_ERR_DEVICE, "hipMemset failed");
    if (rc == SPEC_OK && paged) {
        // page table (all -1), stack of free pages (all of them), geometry of the pool
        const int bps = (cfg->max_kv_len + 31) / 32;
        const size_t page_elems = (size_t)cfg->n_layers * cfg->n_kv_heads * 64 * cfg->head_dim;
        const size_t n_pages = kv_cache_bytes / (page_elems * 2);
        h->n_pages = (int)(n_pages > 0x7fffffff ? 0x7fffffff : n_pages);
        PagePool& pp = h->tables.pool;
        pp.blocks_per_slot = bps;
        A(&pp.table, (size_t)B * bps);
        A(&pp.free_stack, (size_t)h->n_pages);
        A(&pp.free_top, 4);
        if (rc == SPEC_OK) {
            std::vector<int32_t> init((size_t)B * bps, -1), stack((size_t)h->n_pages);
            for (int i = 0; i < h->n_pages; ++i) stack[i] = h->n_pages - 1 - i;   // page 0 is handed out first
            const int32_t top = h->n_pages;
            if (hipMemcpy(pp.table, init.data(), init.size() * 4, hipMemcpyHostToDevice) != hipSuccess
                || hipMemcpy(pp.free_stack, stack.data(), stack.size() * 4, hipMemcpyHostToDevice) != hipSuccess
                || hipMemcpy(pp.free_top, &top, 4, hipMemcpyHostToDevice) != hipSuccess)
                rc = fail(SPEC_ERR_DEVICE, "hipMemcpy failed");
        }
        h->geom = make_cache_geom(*cfg);
        h->geom.table = pp.table;
        h->geom.blocks_per_slot = bps;
        h->geom.page_stride = page_elems;
    }
    if (rc == SPEC_OK && has_model) {
        h->layers.assign(weights->layers, weights->layers + cfg->n_layers);
        h->tok_embed = weights->tok_embed;
        h->final_norm = weights->final_norm;
        h->lm_head = weights->lm_head;
        rc = forward_init(h, max_rows);
    }
    if (rc != SPEC_OK) {
        a.release();
        delete h;
        return rc;
    }
    *out = h;
    return SPEC_OK;
}

extern "C" int spec_verify_profile_begin(spec_handle* h)
{
    if (!h) return fail(SPEC_ERR_INVALID_ARG, "NULL handle");
    h->prof.used = 0;
    h->prof.on = true;
    return SPEC_OK;
}

extern "C" int spec_verify_profile_end(spec_handle* h, void* stream, double* ms, int32_t* launches,
                                       double* empty_pair_ms)
{
    if (!h || !ms || !launches) return fail(SPEC_ERR_INVALID_ARG, "NULL argument");
    h->prof.on = false;
    hipStream_t s = (hipStream_t)stream;
    SPECV_HIP(hipStreamSynchronize(s));
    for (int i = 0; i < SPEC_PROF_COUNT; ++i) {
        ms[i] = 0.0;
        launches[i] = 0;
    }
    for (int i = 0; i < h->prof.used; ++i) {
        float t = 0.f;
        SPECV_HIP(hipEventElapsedTime(&t, h->prof.recs[i].start, h->prof.recs[i].stop));
        const int cls = h->prof.recs[i].cls;
        ms[cls] += t;
        launches[cls] += 1;
        if (cls >= SPEC_PROF_GEMM_QKV && cls <= SPEC_PROF_GEMM_LM_HEAD) {   // every projection also counts as a GEMM
            ms[SPEC_PROF_GEMM] += t;
            launches[SPEC_PROF_GEMM] += 1;
        }
    }
    if (empty_pair_ms) {
        // what a start/stop pair measures with nothing in between (median of 33): the part of every
        // bracketed time that is event handling rather than kernel execution
        *empty_pair_ms = 0.0;
        const int n = h->prof.cap < 33 ? h->prof.cap : 33;
        if (n > 0) {
            for (int i = 0; i < n; ++i) {
                SPECV_HIP(hipEventRecord(h->prof.recs[i].start, s));
                SPECV_HIP(hipEventRecord(h->prof.recs[i].stop, s));
            }
            SPECV_HIP(hipStreamSynchronize(s));
            float v[33];
            for (int i = 0; i < n; ++i) SPECV_HIP(hipEventElapsedTime(&v[i], h->prof.recs[i].start, h->prof.recs[i].stop));
            for (int i = 1; i < n; ++i)
                for (int j = i; j > 0 && v[j] < v[j - 1]; --j) {
                    const float tmp = v[j];
                    v[j] = v[j - 1];
                    v[j - 1] = tmp;
                }
            *empty_pair_ms = v[n / 2];
        }
    }
    h->prof.used = 0;
    return SPEC_OK;
}

extern "C" void spec_verify_destroy(spec_handle* h)
{
    if (!h) return;
    for (int i = 0; i < h->prof.cap; ++i) {
        (void)hipEventDestroy(h->prof.recs[i].start);
        (void)hipEventDestroy(h->prof.recs[i].stop);
    }
    free(h->prof.recs);
    h->arena.release();
    delete h;
}

extern "C" int spec_verify_step(spec_handle* h, const spec_step_args* args, const spec_step_out* out, void* stream)
{
    if (!h || !args || !out) return fail(SPEC_ERR_INVALID_ARG, "NULL handle, args or out");
    const spec_model_cfg& c = h->cfg;
    const int B = args->batch, Kmax = c.max_lookahead;
    if (B < 1 || B > c.max_batch) return fail(SPEC_ERR_INVALID_ARG, "batch %d outside 1..%d", B, c.max_batch);
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
    const bool run_model = args->target_logits_in == nullptr;
    if (run_model) {
        if (!h->has_model) return fail(SPEC_ERR_INVALID_ARG, "sampler-only handle needs target_logits_in");
        if (!args->seq_slot || !args->last_token) return fail(SPEC_ERR_INVALID_ARG, "seq_slot or last_token is NULL");
    }
    hipStream_t s = (hipStream_t)stream;
    // draft_tokens may be NULL when every K_b is 0; the kernels then never read it
    int rc;
    h->tables.tree = 0;
    // without a decoder pass nothing needs the row tables before the sampler's second kernel: its first
    // one fills them (the greedy rule's kernels read them from the start)
    const bool prepare_in_sampler = !run_model && !greedy;
    if (!prepare_in_sampler) {
        ProfScope ps(&h->prof, SPEC_PROF_PREPARE, s);
        rc = launch_prepare(h->tables, ks, B, Kmax, c.vocab, c.max_batch, c.max_kv_len, run_model, args->seq_slot,
                            run_model ? args->last_token : nullptr, args->draft_tokens, h->kv_len, h->flag, s);
        if (rc) return rc;
    }
    const float* logits = args->target_logits_in;
    if (run_model) {
        float* dst = out->logits_out ? out->logits_out : h->logits;
        rc = forward_run_grouped(h, ks, B, M, dst, s);
        if (rc) return rc;
        logits = dst;
    } else if (out->logits_out) {
        SPECV_HIP(hipMemcpyAsync(out->logits_out, logits, (size_t)M * c.vocab * sizeof(float),
                                 hipMemcpyDeviceToDevice, s));
    }
    if (greedy)
        return launch_greedy(h->tables, h->sampler, ks, B, Kmax, c.vocab, M, logits, args->draft_tokens,
                             args->auto_rollback, run_model ? h->kv_len : nullptr, out->n_accepted, out->out_tokens,
                             nullptr, &h->prof, s);
    return launch_sampler(h->tables, h->sampler, ks, B, Kmax, c.vocab, n_stat, logits, args->draft_logits,
                          args->draft_tokens, args->uniforms, Kmax + 1, args->temperature, args->auto_rollback,
                          run_model ? h->kv_len : nullptr, out->n_accepted, out->out_tokens, nullptr, &h->prof, s,
                          prepare_in_sampler ? h->flag : nullptr);
}

extern "C" int spec_verify_tree_step(spec_handle* h, const spec_tree_args* args, const spec_tree_out* out, void* stream)
{
    if (!h || !args || !out) return fail(SPEC_ERR_INVALID_ARG, "NULL handle, args or out");
    const spec_model_cfg& c = h->cfg;
    const int B = args->batch, Kmax = c.max_lookahead;
    if (B < 1 || B > c.max_batch) return fail(SPEC_ERR_INVALID_ARG, "batch %d outside 1..%d", B, c.max_batch);
    if (!args->n_nodes) return fail(SPEC_ERR_INVALID_ARG, "n_nodes is NULL");
    if (!(args->temperature >= 0.f)) return fail(SPEC_ERR_INVALID_ARG, "temperature must be >= 0");
    const bool greedy = args->temperature == 0.f;
    if (!greedy && !args->uniforms) return fail(SPEC_ERR_INVALID_ARG, "uniforms is NULL");
    if (!out->n_accepted || !out->out_tokens || !out->path)
        return fail(SPEC_ERR_INVALID_ARG, "n_accepted, out_tokens or path is NULL");
    LookaheadPack ks;
    memset(&ks, 0, sizeof(ks));
    int M = 0, any = 0;
    for (int b = 0; b < B; ++b) {
        const int k = args->n_nodes[b];
        if (k < 0 || k > Kmax) return fail(SPEC_ERR_INVALID_ARG, "n_nodes[%d] = %d outside 0..%d", b, k, Kmax);
        ks.k[b] = (uint8_t)k;
        M += k + 1;
        any |= k;
    }
    if (!greedy && !args->draft_logits) return fail(SPEC_ERR_INVALID_ARG, "draft_logits is NULL");
    if (any && (!args->draft_tokens || !args->parent))
        return fail(SPEC_ERR_INVALID_ARG, "draft_tokens or parent is NULL");
    const bool run_model = args->target_logits_in == nullptr;
    if (run_model) {
        if (!h->has_model) return fail(SPEC_ERR_INVALID_ARG, "sampler-only handle needs target_logits_in");
        if (!args->seq_slot || !args->last_token) return fail(SPEC_ERR_INVALID_ARG, "seq_slot or last_token is NULL");
    }
    hipStream_t s = (hipStream_t)stream;
    int rc;
    h->tables.tree = 1;
    {
        ProfScope ps(&h->prof, SPEC_PROF_PREPARE, s);
        rc = launch_prepare_tree(h->tables, ks, B, Kmax, c.vocab, c.max_batch, c.max_kv_len, run_model, args->seq_slot,
                                 run_model ? args->last_token : nullptr, args->parent, args->draft_tokens, h->kv_len,
                                 h->flag, s);
    }
    if (rc) return rc;
    const float* logits = args->target_logits_in;
    if (run_model) {
        float* dst = out->logits_out ? out->logits_out : h->logits;
        rc = forward_run_grouped(h, ks, B, M, dst, s);
        if (rc) return rc;
        logits = dst;
    } else if (out->logits_out) {
        SPECV_HIP(hipMemcpyAsync(out->logits_out, logits, (size_t)M * c.vocab * sizeof(float),
                                 hipMemcpyDeviceToDevice, s));
    }
    if (greedy)
        rc = launch_tree_greedy(h->tables, h->sampler, ks, B, Kmax, c.vocab, M, logits, args->parent, args->draft_tokens,
                                args->auto_rollback, run_model ? h->kv_len : nullptr, out->n_accepted, out->out_tokens,
                                out->path, &h->prof, s);
    else
        rc = launch_tree_sampler(h->tables, h->sampler, ks, B, Kmax, c.vocab, 2 * M, logits, args->draft_logits,
                                 args->parent, args->draft_tokens, args->uniforms, args->temperature,
                                 args->auto_rollback, run_model ? h->kv_len : nullptr, out->n_accepted,
                                 out->out_tokens, out->path, &h->prof, s);
    if (rc) return rc;
    if (run_model && args->auto_rollback) {
        ProfScope ps(&h->prof, SPEC_PROF_GLUE, s);
        rc = launch_kv_compact(h->geom, h->kv_cache, h->tables, B, Kmax, out->n_accepted, out->path, s);
        if (rc == SPEC_OK) rc = launch_tree_trim(h->tables, B, out->n_accepted, s);
    }
    return rc;
}

extern "C" int spec_kv_rollback(spec_handle* h, const int32_t* seq_slot, const int32_t* new_len, int32_t n,
                                void* stream)
{
    if (!h || !seq_slot || !new_len) return fail(SPEC_ERR_INVALID_ARG, "NULL handle or array");
    if (!h->has_model) return fail(SPEC_ERR_INVALID_ARG, "sampler-only handle has no KV cache");
    if (n < 0 || n > SPEC_MAX_BATCH) return fail(SPEC_ERR_INVALID_ARG, "n outside 0..%d", SPEC_MAX_BATCH);
    if (n == 0) return SPEC_OK;
    RollbackPack p;
    memset(&p, 0, sizeof(p));
    for (int i = 0; i < n; ++i) {
        if (seq_slot[i] < 0 || seq_slot[i] >= h->cfg.max_batch)
            return fail(SPEC_ERR_INVALID_ARG, "seq_slot[%d] = %d outside 0..%d", i, seq_slot[i], h->cfg.max_batch - 1);
        if (new_len[i] < 0 || new_len[i] > h->cfg.max_kv_len)
            return fail(SPEC_ERR_INVALID_ARG, "new_len[%d] = %d outside 0..%d", i, new_len[i], h->cfg.max_kv_len);
        for (int j = 0; j < i; ++j)
            if (seq_slot[j] == seq_slot[i]) return fail(SPEC_ERR_INVALID_ARG, "seq_slot[%d] repeats a slot", i);
        p.slot[i] = seq_slot[i];
        p.len[i] = new_len[i];
    }
    return launch_rollback(p, n, h->cfg.max_batch, h->kv_len, h->flag, h->tables.pool, (hipStream_t)stream);
}

static int kv_copy_common(spec_handle* h, int32_t slot, int32_t pos0, int32_t n_pos, void* plain, bool to_cache,
                          void* stream)
{
    if (!h) return fail(SPEC_ERR_INVALID_ARG, "NULL handle");
    if (!plain && n_pos != 0) return fail(SPEC_ERR_INVALID_ARG, "NULL tensor");   // (an empty tensor has no address)
    if (!h->has_model) return fail(SPEC_ERR_INVALID_ARG, "sampler-only handle has no KV cache");
    if (slot < 0 || slot >= h->cfg.max_batch) return fail(SPEC_ERR_INVALID_ARG, "slot outside 0..%d", h->cfg.max_batch - 1);
    if (pos0 < 0 || n_pos < 0 || pos0 + n_pos > h->cfg.max_kv_len)
        return fail(SPEC_ERR_INVALID_ARG, "positions [%d, %d) outside the slot", pos0, pos0 + n_pos);
    if (n_pos == 0) return SPEC_OK;
    if (to_cache) {
        // pages are always taken from a slot's first block on, so that a slot's table has no holes
        const int rc = launch_pool_cover(h->tables.pool, slot, 0, pos0 + n_pos, h->flag, (hipStream_t)stream);
        if (rc) return rc;
    }
    return launch_kv_copy(h->geom, h->kv_cache, slot, pos0, n_pos, plain, to_cache, (hipStream_t)stream);
}

extern "C" int spec_kv_import(spec_handle* h, int32_t slot, int32_t pos0, int32_t n_pos, const void* src, void* stream)
{
    return kv_copy_common(h, slot, pos0, n_pos, const_cast<void*>(src), true, stream);
}

extern "C" int spec_kv_export(spec_handle* h, int32_t slot, int32_t pos0, int32_t n_pos, void* dst, void* stream)
{
    return kv_copy_common(h, slot, pos0, n_pos, dst, false, stream);
}

extern "C" int spec_kv_pages(spec_handle* h, int32_t* free_pages, int32_t* total_pages, void* stream)
{
    if (!h || !free_pages || !total_pages) return fail(SPEC_ERR_INVALID_ARG, "NULL argument");
    if (!h->tables.pool.table) return fail(SPEC_ERR_INVALID_ARG, "the handle's cache is not paged");
    SPECV_HIP(hipStreamSynchronize((hipStream_t)stream));
    SPECV_HIP(hipMemcpy(free_pages, h->tables.pool.free_top, 4, hipMemcpyDeviceToHost));
    *total_pages = h->n_pages;
    return SPEC_OK;
}

extern "C" int spec_verify_poll(spec_handle* h, void* stream)
{
    if (!h) return fail(SPEC_ERR_INVALID_ARG, "NULL handle");
    int32_t v = 0;
    SPECV_HIP(hipStreamSynchronize((hipStream_t)stream));
    SPECV_HIP(hipMemcpy(&v, h->flag, 4, hipMemcpyDeviceToHost));
    if (v != 0) {
        SPECV_HIP(hipMemset(h->flag, 0, 4));
        return fail(v, "a sequence was skipped on the device (status %d)", v);
    }
    return SPEC_OK;
}

extern "C" int spec_k_plan_step(const spec_model_cfg* cfg, int32_t batch, const int32_t* lookahead, int32_t cu_count,
                                int32_t paged, spec_step_plan* out)
{
    if (!cfg || !lookahead || !out) return fail(SPEC_ERR_INVALID_ARG, "spec_k_plan_step: NULL argument");
    int rc = check_cfg(cfg, true);
    if (rc) return rc;
    if (cfg->dtype != SPEC_DTYPE_BF16) return fail(SPEC_ERR_INVALID_ARG, "spec_k_plan_step: bf16 models only");
    if (batch < 1 || batch > cfg->max_batch) return fail(SPEC_ERR_INVALID_ARG, "batch %d outside 1..%d", batch, cfg->max_batch);
    if (cu_count < 1) return fail(SPEC_ERR_INVALID_ARG, "cu_count must be positive");
    memset(out, 0, sizeof(*out));
    LookaheadPack ks;
    memset(&ks, 0, sizeof(ks));
    int M = 0;
    for (int b = 0; b < batch; ++b) {
        const int k = lookahead[b];
        if (k < 0 || k > cfg->max_lookahead)
            return fail(SPEC_ERR_INVALID_ARG, "lookahead[%d] = %d outside 0..%d", b, k, cfg->max_lookahead);
        ks.k[b] = (uint8_t)k;
        M += k + 1;
    }
    out->rows = M;
    int seqs[SPEC_PLAN_MAX_PASSES], rows[SPEC_PLAN_MAX_PASSES];
    const int n = plan_passes(ks, batch, M, GEMM_MAX_ROWS, seqs, rows, SPEC_PLAN_MAX_PASSES);
    if (n == 0) return fail(SPEC_ERR_SHAPE, "a step of %d rows needs more than %d decoder passes", M, SPEC_PLAN_MAX_PASSES);
    out->n_passes = n;
    for (int i = 0; i < n; ++i) {
        out->pass_seqs[i] = seqs[i];
        out->pass_rows[i] = rows[i];
    }
    const int max_rows = std::min(cfg->max_batch * (cfg->max_lookahead + 1), GEMM_MAX_ROWS);
    int n_out[SPEC_PLAN_PROJECTIONS], n_in[SPEC_PLAN_PROJECTIONS];
    projection_shapes(*cfg, n_out, n_in);
    for (int i = 0; i < SPEC_PLAN_PROJECTIONS; ++i) {
        const GemmPlan p = plan_gemm(rows[0], n_out[i], n_in[i], cu_count, true);
        out->gemm_row_tiles[i] = p.mt;
        out->gemm_col_tiles[i] = p.nt;
        out->gemm_k_ranges[i] = p.n_split;
        out->gemm_k_blocks_per_range[i] = p.kb_per_split;
        out->gemm_row_parts[i] = p.rs;
        out->gemm_col_groups[i] = p.cg;
        const int n_tiles = p.n_pad / 16;
        out->gemm_workgroups[i] = (n_tiles + p.cg * p.nt - 1) / (p.cg * p.nt) * p.n_split;
        out->gemm_partial_floats[i] = gemm_partial_elems(p, rows[0]);
    }
    out->gemm_partial_capacity = gemm_partial_capacity(*cfg, max_rows, cu_count);
    const int widest = std::max(std::max(cfg->d_model, cfg->n_q_heads * cfg->head_dim), cfg->d_ffn);
    out->gate_up_swiglu_inside = gemm_swiglu_fits(rows[0], cfg->d_ffn, cu_count) ? 1 : 0;
    out->xfrag_units = xfrag_uint4s(gemm_row_tiles(rows[0]), 2, widest);
    out->xfrag_capacity = xfrag_uint4s(gemm_row_tiles(max_rows), 2, widest);
    out->xfrag_act_units = out->gate_up_swiglu_inside ? xfrag_uint4s(gemm_row_tiles(rows[0]), 2, cfg->d_ffn) : 0;
    out->xfrag_act_capacity = xfrag_uint4s(gemm_row_tiles(std::min(max_rows, 64)), 2, cfg->d_ffn);
    int kmax = 0;
    for (int b = 0; b < seqs[0]; ++b) kmax = ks.k[b] > kmax ? ks.k[b] : kmax;
    const CacheGeom g = make_cache_geom(*cfg);
    const AttnDescription d = describe_attention(g, paged != 0, cfg->n_q_heads, kmax, seqs[0], cfg->max_kv_len,
                                                 cfg->max_lookahead + 1, cu_count);
    out->attn_kv_share = d.share;
    out->attn_small = d.small;
    out->attn_chunks = d.max_chunks;
    out->attn_chunk_keys = d.chunk_keys;
    out->attn_row_tiles = d.row_tiles;
    out->attn_wavefronts = d.wavefronts;
    out->attn_fused = d.fused;
    out->attn_partial_floats = d.partial_floats;
    out->attn_partial_capacity = attn_partial_floats(cfg->max_kv_len, cfg->max_batch, cfg->n_kv_heads,
                                                     cfg->n_q_heads / cfg->n_kv_heads, cfg->max_lookahead + 1, cfg->head_dim,
                                                     cu_count, paged != 0);
    return SPEC_OK;
}
