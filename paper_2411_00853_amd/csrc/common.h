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
    int32_t* row_pos;    // [M] absolute position n_b + j (or -1 for rows of skipped sequences)
    int32_t* row_tok;    // [M] token id fed at this row
};

// ---- sampler (sampler.hip) ---------------------------------------------------------------------
constexpr int STAT_CHUNK = 8192;   // logits per workgroup in the statistics pass
constexpr int RES_CHUNK = 4096;    // logits per workgroup in the residual pass / final scan

struct SamplerWorkspace {
    float* part_max;      // [stat rows][stat chunks] chunk maxima of raw logits
    double* part_sum;     // [stat rows][stat chunks] sum exp((l - chunk max)/T)
    double* chunk_mass;   // [B][res chunks] mass of the final-draw distribution per chunk
    int32_t* accepted;    // [B] a_b
    double* row_inv_z;    // [B][2] 1/Z of the two rows the final draw reads (p, q)
    float* row_max;       // [B][2] their maxima
};

int launch_prepare(const StepTables& t, const LookaheadPack& ks, int B, int Kmax, int V, int max_batch,
                   int max_kv_len, bool has_cache, const int32_t* seq_slot, const int32_t* last_token,
                   const int32_t* draft_tokens, const int32_t* kv_len, int32_t* flag, hipStream_t s);

int launch_sampler(const StepTables& t, const SamplerWorkspace& w, const LookaheadPack& ks, int B, int Kmax,
                   int V, int n_stat_rows, const float* target_logits, const float* draft_logits,
                   const int32_t* draft_tokens, const float* uniforms, float temperature, int auto_rollback,
                   int32_t* kv_len, int32_t* n_accepted, int32_t* out_tokens, Profiler* prof, hipStream_t s);

struct RollbackPack {
    int32_t slot[SPEC_MAX_BATCH];
    int32_t len[SPEC_MAX_BATCH];
};
int launch_rollback(const RollbackPack& p, int n, int max_batch, int32_t* kv_len, int32_t* flag, hipStream_t s);

// ---- decoder pass (elementwise.hip, gemm.hip, attention.hip) -----------------------------------
struct RopeTable {
    const float* cos_sin;   // [max_kv_len][head_dim/2][2] cos, sin of pos * theta^(-2i/hd)
};

// bf16 cache tile order: per (layer, slot, kv head) a run of 32-key blocks; each block holds a key
// part then a value part of 32*hd elements each (see attention.hip for the element order).
struct CacheGeom {
    int dtype;
    int n_layers, n_slots, n_kv_heads, head_dim;
    int t_pad;            // max_kv_len rounded up to 32
    size_t layer_stride;  // elements
    size_t slot_stride;
    size_t head_stride;   // bf16: keys and values of one head (2*t_pad*hd); fp32: one plane (t_pad*hd)
};
CacheGeom make_cache_geom(const spec_model_cfg& c);

int launch_embed_rmsnorm(int dtype, const void* tok_embed, const int32_t* row_tok, const float* gain, float eps,
                         int M, int d, float* x, float* h, hipStream_t s);
// `partial` is [n_split][M][ld]; consumers add the ranges in index order.
int launch_resid_rmsnorm(const float* partial, int n_split, size_t split_stride, int ld, const float* gain, float eps,
                         int M, int d, float* x, float* h, hipStream_t s);
int launch_silu_mul(const float* partial, int n_split, size_t split_stride, int ld, int M, int F, bool interleaved,
                    float* act, hipStream_t s);
int launch_rope_append(const float* partial, int n_split, size_t split_stride, int ld, const StepTables& t, int M,
                       const CacheGeom& g, int n_q_heads, int layer, const float* cos_sin, void* cache,
                       float* q_out, hipStream_t s);
int launch_reduce_splits(const float* partial, int n_split, size_t split_stride, int M, int N, int ld, float* out,
                         hipStream_t s);
int launch_kv_copy(const CacheGeom& g, void* cache, int slot, int pos0, int n_pos, void* plain, bool to_cache,
                   hipStream_t s);

// Y[M][N] (+)= X[M][K] * W[N][K]^T.  bf16: W packed, result left as n_split partial sums in
// `partial` ([n_split][M][N_pad]); the plan says how many.  fp32: direct result (n_split = 1).
struct GemmPlan {
    int n_split;      // K ranges summed later by the consumer
    int n_pad;        // N rounded up to 16
    int mt;           // 16-row tiles
    int nt;           // 16-column tiles per wavefront
    int kb_per_split; // 32-wide K blocks per range
};
GemmPlan plan_gemm(int M, int N, int K, int cu_count);
size_t gemm_partial_elems(const GemmPlan& p, int M);
int launch_gemm_bf16(const GemmPlan& p, const float* x, const void* w_packed, int M, int N, int K,
                     bool split_x, float* partial, hipStream_t s);
int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* y, hipStream_t s);

struct AttnPlan {
    int chunk_keys;   // keys per wavefront work item (multiple of 32)
    int max_chunks;   // chunks per (sequence, kv head) at max_kv_len
};
AttnPlan plan_attention(int max_kv_len, int batch, int n_kv_heads, int cu_count);
size_t attn_partial_floats(int max_kv_len, int max_batch, int n_kv_heads, int group, int max_window, int hd,
                           int cu_count);
int launch_attention(const AttnPlan& p, int max_kv_len, int cu_count, const StepTables& t, const LookaheadPack& ks, int B, int M,
                     const CacheGeom& g, int n_q_heads, int layer, const void* cache, const float* q,
                     float* part_o, float* part_ml, float* out, int max_window, Profiler* prof, hipStream_t s);

}  // namespace specv
