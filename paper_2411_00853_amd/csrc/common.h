// Shared declarations of the verify-step library (host + device helpers).  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/spec_verify.h"
#include "../../include/spec_kernels.h"

namespace specv {

// ---- error plumbing -------------------------------------------------------------------------
void set_error(const char* fmt, ...);
int fail(int status, const char* fmt, ...);

#define SPECV_HIP(call)                                                                  \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess)                                                            \
            return ::specv::fail(SPEC_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define SPECV_LAUNCH_CHECK(name)                                                         \
    do {                                                                                 \
        hipError_t e_ = hipGetLastError();                                               \
        if (e_ != hipSuccess)                                                            \
            return ::specv::fail(SPEC_ERR_DEVICE, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

// ---- optional per-kernel-class timing with HIP events on the launch stream ----------------------
// Classes follow SPEC_PROF_* in spec_kernels.h.  Off by default: then begin/end do nothing.
struct Profiler {
    bool on = false;
    struct Rec {
        hipEvent_t start, stop;
        int cls;
    };
    Rec* recs = nullptr;
    int cap = 0, used = 0;
    void begin(int cls, hipStream_t s);
    void end(hipStream_t s);
};
struct ProfScope {
    Profiler* p;
    hipStream_t s;
    ProfScope(Profiler* p_, int cls, hipStream_t s_) : p(p_), s(s_)
    {
        if (p && p->on) p->begin(cls, s);
    }
    ~ProfScope()
    {
        if (p && p->on) p->end(s);
    }
};

// The page pool of a paged cache: a stack of free page numbers.  Pages are taken only by the row
// bookkeeping kernels (before a window is appended) and by imports, and returned only where a cache
// length shrinks -- never both in one kernel, so plain atomic counters suffice.
struct PagePool {
    int32_t* table;        // NULL: contiguous cache, everything below is a no-op
    int32_t* free_stack;   // [n_pages]
    int32_t* free_top;     // number of entries in free_stack
    int blocks_per_slot;
};

// ---- per-step row bookkeeping built on the device by the prepare kernel ------------------------
struct LookaheadPack {
    uint8_t k[SPEC_MAX_BATCH];
};

struct StepTables {
    int32_t* seq_row0;   // [B+1] first target row of each sequence (prefix of K_b+1)
    int32_t* seq_stat0;  // [B+1] first statistics row of each sequence (prefix of 2K_b+1)
    int32_t* seq_n;      // [B] cached length n_b read at the start of the step
    int32_t* seq_ok;     // [B] 1 = sequence takes part, 0 = skipped (device-side error)
    int32_t* seq_slot;   // [B] cache slot (copied so later kernels need not re-validate)
    int32_t* row_seq;    // [M]
    int32_t* row_pos;    // [M] cache position n_b + j of the row's key/value (or -1 for rows of skipped sequences)
    int32_t* row_tok;    // [M] token id fed at this row
    int32_t* row_rope;   // [M] position the rotary embedding uses: n_b + depth of the row in its window
    uint32_t* row_mask;  // [M] bit i set: the row attends to window slot i (position n_b + i)
    PagePool pool;       // the cache's page pool (table == NULL: contiguous cache)
    int tree;            // set by the host: 0 = the windows are chains (row_rope = row_pos, row_mask = slots
                         // 0..j, so the kernels need not load them), 1 = token trees
};

// ---- sampler (sampler.hip) ---------------------------------------------------------------------
constexpr int STAT_CHUNK = 16384;   // logits per workgroup in the statistics pass
constexpr int RES_CHUNK = 4096;    // logits per workgroup in the residual pass / final scan

struct SamplerWorkspace {
    float* part_max;      // [stat rows][stat chunks] chunk maxima of raw logits
    double* part_sum;     // [stat rows][stat chunks] sum exp((l - chunk max)/T)
    double* chunk_mass;   // [B][res chunks] mass of the final-draw distribution per chunk
    int32_t* accepted;    // [B] a_b
    double* row_inv_z;    // [B][2] 1/Z of the two rows the final draw reads (p, q)
    float* row_max;       // [B][2] their maxima
    int32_t* part_idx;    // [stat rows][stat chunks] greedy rule: lowest id holding the chunk maximum
};

int launch_prepare(const StepTables& t, const LookaheadPack& ks, int B, int Kmax, int V, int max_batch,
                   int max_kv_len, bool has_cache, const int32_t* seq_slot, const int32_t* last_token,
                   const int32_t* draft_tokens, const int32_t* kv_len, int32_t* flag, hipStream_t s);

// Temperature 0: keep a proposal iff it is the target row's most likely token (lowest id among equal
// maxima); the final token is the most likely token of the first mismatching row, or of row K_b.
struct DrawEmit;
// emit != NULL: every K_b = 0 and M rows = all rows of the step; the token of sequence b comes from row seq_row0[b]
int launch_greedy(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax, int V,
                  int M, const float* target_logits, const int32_t* draft_tokens, int auto_rollback, int32_t* kv_len,
                  int32_t* n_accepted, int32_t* out_tokens, const DrawEmit* emit, Profiler* prof, hipStream_t s);

// Where a plain draw (every K_b = 0: one token from each sequence's row) puts its results when the
// sampler serves a proposing model instead of a verification.  tokens == NULL: verification mode.
struct DrawEmit {
    int32_t* tokens;       // tokens[b * stride + offset] = drawn token
    int stride, offset;
    int32_t* next_token;   // [B] the drawn token again: the next decode step's input
    int32_t* kv_len;       // kv_len[slot] = cached length at the start of the step + kv_add
    int kv_add;
    float* logits_copy;    // the row the token was drawn from, copied to logits_copy + b * copy_stride
    size_t copy_stride;
};

// uniforms: sequence b reads uniforms[b * u_stride + i] (i < K_b: proposal i; i = K_b: the final draw)
// prepare_flag != NULL: no launch_prepare ran for this step (no decoder pass, no cache); the statistics pass
// fills t itself, reporting bad tokens through that flag
int launch_sampler(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax,
                   int V, int n_stat_rows, const float* target_logits, const float* draft_logits,
                   const int32_t* draft_tokens, const float* uniforms, int u_stride, float temperature,
                   int auto_rollback, int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens,
                   const DrawEmit* emit, Profiler* prof, hipStream_t s, int32_t* prepare_flag = nullptr);

// Token-tree variants: parent/tokens [B][Kmax], draft logits [B][Kmax+1][V] (row 0: the root)
int launch_prepare_tree(const StepTables& t, const LookaheadPack& ks, int B, int Kmax, int V, int max_batch,
                        int max_kv_len, bool has_cache, const int32_t* seq_slot, const int32_t* last_token,
                        const int32_t* parent, const int32_t* tokens, const int32_t* kv_len, int32_t* flag,
                        hipStream_t s);
int launch_tree_sampler(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax,
                        int V, int n_stat_rows, const float* target_logits, const float* draft_logits,
                        const int32_t* parent, const int32_t* tokens, const float* uniforms, float temperature,
                        int auto_rollback, int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens,
                        int32_t* path, Profiler* prof, hipStream_t s);

struct RollbackPack {
    int32_t slot[SPEC_MAX_BATCH];
    int32_t len[SPEC_MAX_BATCH];
};
int launch_rollback(const RollbackPack& p, int n, int max_batch, int32_t* kv_len, int32_t* flag, const PagePool& pool,
                    hipStream_t s);
// paged caches, after launch_kv_compact: return the pages beyond n + n_accepted + 1 of every sequence
int launch_tree_trim(const StepTables& t, int B, const int32_t* n_accepted, hipStream_t s);
// sub := the tables of sequences [b0, b0 + Bg) of full, rows and sequence numbers counted from that group's start
int launch_slice_tables(const StepTables& full, const StepTables& sub, int b0, int Bg, hipStream_t s);
// paged caches: make sure positions [pos0, pos1) of a slot have pages (flags SPEC_ERR_KV_OVERFLOW if not)
int launch_pool_cover(const PagePool& pool, int slot, int pos0, int pos1, int32_t* flag, hipStream_t s);

// ---- decoder pass (elementwise.hip, gemm.hip, attention.hip) -----------------------------------
struct RopeTable {
    const float* cos_sin;   // [max_kv_len][head_dim/2][2] cos, sin of pos * theta^(-2i/hd)
};

// bf16 cache tile order: per (layer, slot) a run of 32-position blocks, each holding that block of
// every kv head in turn; a head's block is a key part then a value part of 32*hd elements each (see
// cache_layout.h for the element order).
struct CacheGeom {
    int dtype;
    int n_layers, n_slots, n_kv_heads, head_dim;
    int t_pad;            // max_kv_len rounded up to 32
    size_t layer_stride;  // elements
    size_t slot_stride;
    size_t head_stride;   // bf16: one block of one head (64*hd); fp32: one plane (t_pad*hd)
    size_t blk_stride;    // bf16: from a head's block to its next one (n_kv_heads*64*hd); fp32: unused
    // paged mode (bf16 only): the 32-position blocks of a slot live in pages of a shared pool,
    // [page][layer][kv head][block]; table[slot * blocks_per_slot + blk] names the page (-1: none)
    const int32_t* table; // NULL: contiguous mode
    int blocks_per_slot;
    size_t page_stride;   // elements of one page: n_layers * n_kv_heads * 64 * head_dim
};

CacheGeom make_cache_geom(const spec_model_cfg& c);

// Row-wise sums of squares travel as SSQ_CHUNK-column partial sums ([M][n_ssq]).  RMSNorm is split
// in two: the producer of a GEMM's input multiplies by the gain; the row's 1/rms factors out of the
// dot product and is applied by the consumer of the GEMM's output (NormScale).
constexpr int SSQ_CHUNK = 1024;
inline int ssq_chunks(int d) { return (d + SSQ_CHUNK - 1) / SSQ_CHUNK; }
struct NormScale {
    const float* ssq;   // NULL: no scaling
    int n_ssq;
    int d;              // row length the mean is taken over
    float eps;
};
// Where a producer puts a GEMM operand: fragment buffer (bf16 path) and/or plain fp32 rows.
struct XOut {
    void* frags;        // NULL on the fp32 path
    int mt, planes;
    float* plain;       // NULL on the bf16 path
};
int launch_embed(int dtype, const void* tok_embed, const int32_t* row_tok, int M, int d, float* x, float* ssq,
                 const float* gain, const XOut& xo, hipStream_t s);
// x[m] += sum of the n_split partial ranges ([n_split][M][ld], added in index order); ssq updated;
// x * gain written as the next GEMM's operand
int launch_resid(const float* partial, int n_split, size_t split_stride, int ld, int M, int d, float* x, float* ssq,
                 const float* gain, const XOut& xo, hipStream_t s);
// h = x * inv_rms * gain (only the fp32 path materialises normalised activations)
int launch_rmsnorm_apply(const float* x, const float* ssq, const float* gain, float eps, int M, int d, float* h,
                         hipStream_t s);
int launch_silu_mul(const float* partial, int n_split, size_t split_stride, int ld, int M, int F, bool interleaved,
                    const NormScale& ns, const XOut& xo, hipStream_t s);
int launch_rope_append(const float* partial, int n_split, size_t split_stride, int ld, const StepTables& t, int M,
                       const CacheGeom& g, int n_q_heads, int layer, const float* cos_sin, const NormScale& ns,
                       void* cache, float* q_out, hipStream_t s);
int launch_reduce_splits(const float* partial, int n_split, size_t split_stride, int M, int N, int ld,
                         const float* ssq, int n_ssq, int d, float eps, float* out, hipStream_t s);
int launch_kv_copy(const CacheGeom& g, void* cache, int slot, int pos0, int n_pos, void* plain, bool to_cache,
                   hipStream_t s);
int launch_tree_greedy(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax, int V,
                       int M, const float* target_logits, const int32_t* parent, const int32_t* tokens,
                       int auto_rollback, int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens, int32_t* path,
                       Profiler* prof, hipStream_t s);
// keys/values of the kept path (slot path[k]+1 of the window) moved to positions n+1..n+a, all layers
int launch_kv_compact(const CacheGeom& g, void* cache, const StepTables& t, int B, int Kmax, const int32_t* n_accepted,
                      const int32_t* path, hipStream_t s);

// Y[M][N] (+)= X[M][K] * W[N][K]^T.  bf16: W packed, result left as n_split partial sums in
// `partial` ([n_split][M][N_pad]); the plan says how many.  fp32: direct result (n_split = 1).
struct GemmPlan {
    int n_split;      // K ranges summed later by the consumer
    int n_pad;        // N rounded up to 16
    int mt;           // 16-row tiles
    int nt;           // 16-column tiles per wavefront
    int planes;       // 2: bf16 head + remainder; 1: bf16 head only
    int kb_per_split; // 32-wide K blocks per range
    int rs;           // row parts per workgroup: 1 (every wavefront takes all row tiles), 2 or 4
    int cg;           // column groups (of nt tiles) per workgroup: 4, or 3 for many-row launches that then fill more compute units
};
constexpr int GEMM_MAX_ROWS = SPEC_MAX_STEP_ROWS;   // rows the largest variant of the bf16 GEMM takes
GemmPlan plan_gemm(int M, int N, int K, int cu_count, bool split_x);
int gemm_row_tiles(int M);   // row tiles (mt) of the variant that serves M rows; 0 if none
size_t gemm_partial_elems(const GemmPlan& p, int M);
// x_frags: X as operand fragments (frag.h) with p.mt row tiles and p.planes planes
int launch_gemm_bf16(const GemmPlan& p, const void* x_frags, const void* w_packed, int M, int N, int K,
                     float* partial, hipStream_t s);
int launch_pack_x(const float* x, const float* gain, int M, int K, int mt_count, int planes, void* x_frags,
                  hipStream_t s);
void set_gemm_wg_target(int workgroups);
// Gate/up projection that finishes SwiGLU itself and writes the down projection's operand fragments
// (see gemm.hip); `fits` says whether the shape allows it.
bool gemm_swiglu_fits(int M, int F, int cu_count);
void set_swiglu_min_wgs(int workgroups);
void set_swiglu_column_groups(int groups);
int launch_gemm_swiglu(const void* x_frags, int planes, const void* w_gate_up, int M, int F, int K, const float* ssq,
                       int n_ssq, int d, float eps, void* act_frags, int act_mt, int act_planes, int cu_count, hipStream_t s);
int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* y, hipStream_t s);

// The QKV projection's result as the attention kernel can take it directly (bf16 path): K-range
// partial sums [n_split][M][ld] with columns q heads | k heads | v heads, the row scale of the
// attention norm, and the rotary table.  partial == NULL: queries come rotated from `q`, and the
// window's keys and values are already in the cache.
struct QkvSrc {
    const float* partial;
    int n_split;
    size_t stride;
    int ld;
    NormScale ns;
    const float* cos_sin;
};

struct AttnPlan {
    int chunk_keys;   // most keys a wavefront work item can get (multiple of 32): a sequence at max_kv_len
    int max_chunks;   // chunks per (sequence, kv head) at max_kv_len
    int lag_keys;     // positions by which the chunks before a sequence's last one are longer (multiple of 32)
};
AttnPlan plan_attention(int max_kv_len, int batch, int n_kv_heads, int cu_count, bool paged = false);
void set_attn_items_per_cu(int n);
void set_attn_merge_min_pairs(int n);
void set_attn_max_chunks(int n);
void set_attn_small_positions(int n);
size_t attn_partial_floats(int max_kv_len, int max_batch, int n_kv_heads, int group, int max_window, int hd,
                           int cu_count, bool paged = false);
// part_cap: capacity of part_o in floats (part_ml holds 2/head_dim of that); a plan that needs more
// (the tuning knobs changed after the buffers were sized) is refused with SPEC_ERR_SHAPE.
// Whether the bf16 attention kernel can take the QKV projection's partial sums itself (QkvSrc) for
// this step's shapes; if not, launch_rope_append has to run first.
bool attention_takes_qkv(const CacheGeom& g, int n_q_heads, const LookaheadPack& ks, int B, int max_kv_len, int cu_count);
// What launch_attention would do for a step of B sequences whose longest window has kmax + 1 rows (host logic only)
struct AttnDescription {
    int share, small, max_chunks, chunk_keys, row_tiles, wavefronts, fused;
    size_t partial_floats;   // chunk results the launch writes when they go through memory
};
AttnDescription describe_attention(const CacheGeom& g, bool paged, int n_q_heads, int kmax, int B, int max_kv_len,
                                   int max_window, int cu_count);
int launch_attention(int max_kv_len, int cu_count, const StepTables& t, const LookaheadPack& ks, int B, int M,
                     const CacheGeom& g, int n_q_heads, int layer, const void* cache, const float* q,
                     float* part_o, float* part_ml, size_t part_cap, const XOut& xo, int max_window, Profiler* prof,
                     hipStream_t s, const QkvSrc* qkv = nullptr, void* cache_w = nullptr);

}  // namespace specv
