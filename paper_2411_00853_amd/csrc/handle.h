// The opaque handle behind spec_verify.h and the decoder-pass entry points it drives.
#pragma once

#include <vector>

#include "common.h"

namespace specv {

struct Arena {
    std::vector<void*> blocks;
    size_t total = 0;
    int alloc(void** out, size_t bytes);
    void release();
};

enum GemmId { G_QKV = 0, G_O, G_GATE_UP, G_DOWN, G_LM_HEAD, G_COUNT };

}  // namespace specv

struct spec_handle {
    spec_model_cfg cfg;
    bool has_model = false;
    int device = 0;
    int cu_count = 256;
    void* kv_cache = nullptr;
    int32_t* kv_len = nullptr;
    int32_t* flag = nullptr;
    specv::Arena arena;
    specv::StepTables tables{};
    specv::StepTables group_tables{};   // one pass's share of `tables` when a step is scored in several passes
    specv::SamplerWorkspace sampler{};
    specv::Profiler prof;

    // decoder pass
    std::vector<spec_layer_weights> layers;
    const void* tok_embed = nullptr;
    const float* final_norm = nullptr;
    const void* lm_head = nullptr;
    specv::CacheGeom geom{};
    int n_pages = 0;           // paged cache: pages in the caller's pool (0: contiguous cache)
    bool split_act = true;     // feed activations to the matrix cores as bf16 head + remainder
    bool fuse_rope = true;     // bf16: rotary + KV append happen inside the attention kernel
    float* x = nullptr;        // [rows][d_model] residual stream
    float* hn = nullptr;       // [rows][d_model] normalised activations (fp32 path only)
    void* xf = nullptr;        // operand fragments of the current GEMM's input (bf16 path)
    void* xf_act = nullptr;    // second fragment buffer: the down projection's operand when the gate/up GEMM writes it
    float* ssq = nullptr;      // [rows][ssq chunks] partial sums of squares of x
    float* q = nullptr;        // [rows][n_q_heads*head_dim] rotated queries
    float* att = nullptr;      // [rows][n_q_heads*head_dim] attention output
    float* act = nullptr;      // [rows][d_ffn]
    float* partial = nullptr;  // K-range partial sums of the current GEMM
    size_t partial_cap = 0;    // its capacity in floats (sized at init from the plans of every row count)
    float* logits = nullptr;   // [rows][vocab] when the caller gives no logits_out
    float* cos_sin = nullptr;  // rotary table
    float* attn_part_o = nullptr;
    float* attn_part_ml = nullptr;
    size_t attn_part_cap = 0;  // capacity of attn_part_o in floats (attn_part_ml holds 2/head_dim of that)
    int max_rows = 0;   // max_batch * (max_lookahead + 1): what the row tables hold
    int row_cap = 0;    // window rows one step may carry (the activation buffers are sized for it)
};

namespace specv {
int forward_init(spec_handle* h, int max_rows);
// one decoder pass over the B sequences (M <= row_cap window rows) that t describes
int forward_run(spec_handle* h, const StepTables& t, const LookaheadPack& ks, int B, int M, float* logits_out, hipStream_t s);
// the same for any M: sequences are taken in groups of at most row_cap rows, one pass each (t = h->tables)
int forward_run_grouped(spec_handle* h, const LookaheadPack& ks, int B, int M, float* logits_out, hipStream_t s);
// host logic behind the two (no device work): see forward.hip
size_t gemm_partial_capacity(const spec_model_cfg& c, int max_rows, int cu_count);
void projection_shapes(const spec_model_cfg& c, int* n_out, int* n_in);   // [SPEC_PLAN_PROJECTIONS]
int plan_passes(const LookaheadPack& ks, int B, int M, int cap, int* pass_seqs, int* pass_rows, int max_passes);
}  // namespace specv
