/*
 * spec_kernels.h -- single-kernel entry points of the verify-step library, exported so that each
 * building block of spec_verify_step can be tested against the CPU oracle and profiled on its
 * own.  Same conventions as spec_verify.h: plain device pointers, asynchronous on the given
 * stream, negative spec_status on failure.  Not needed by an application.
 */
#ifndef SPEC_KERNELS_H
#define SPEC_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#include "spec_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* dst[i] = src[i] for n_bytes (multiple of 16; both device, 16-byte aligned).  A plain streaming
 * copy of known size: the yardstick that HBM byte counters and achieved bandwidth are scaled by. */
int spec_k_copy(const void* src, void* dst, size_t n_bytes, void* stream);

/* sum of n_bytes of device memory read as fp32 -> out[0] per workgroup slot (read-only stream). */
int spec_k_read(const void* src, size_t n_bytes, float* out, void* stream);

/* D = A * B for one 16x16x32 bf16 MFMA tile, operands and result in plain row-major device arrays
 * (A bf16[16][32], B bf16[32][16], D fp32[16][16]).  Checks the register layout the GEMM and
 * attention kernels assume for the matrix instruction. */
int spec_k_mfma_tile(const void* a_bf16, const void* b_bf16, float* d, void* stream);

/* Y[M][N] = X[M][K] * W^T for a packed bf16 W (see spec_pack_weight): the decoder's skinny GEMM
 * including the reduction of its K-range partial sums.  X, Y fp32 row-major.  split_x != 0 feeds
 * each activation as a bf16 head plus a bf16 remainder (two matrix instructions per tile) so that
 * activation rounding stays near fp32 level.  workspace: device scratch of at least
 * spec_k_gemm_workspace_bytes(M, N, K). */
size_t spec_k_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K);
int spec_k_gemm_bf16(const float* x, const void* w_packed, float* y, int32_t M, int32_t N, int32_t K,
                     int32_t split_x, void* workspace, void* stream);

/* Tuning knob: number of workgroups a GEMM launch aims for when it cuts K into ranges
 * (0 = default, two thirds of the compute units).  Process-wide; affects launches made after the
 * call.  Set it before spec_verify_init: a handle's partial-sum workspace is sized for the plans in
 * force at init, and a step whose plan needs more (a larger target set later) fails with
 * SPEC_ERR_SHAPE instead of writing past the workspace. */
void spec_k_set_gemm_wg_target(int32_t workgroups);

/* Tuning knob: launches of more than 112 rows whose twelve column tiles per workgroup would run as
 * three column groups of four tiles (six wavefronts) run as four groups of three tiles instead
 * (eight wavefronts, two on every SIMD); 1 = on (default), 0 = off.  Process-wide. */
void spec_k_set_gemm_balance_groups(int32_t on);

/* Tuning knob: the gate/up projection finishes SwiGLU inside the GEMM (one K range, 128-column
 * workgroups, up to 64 rows) when that launch has at least this many workgroups; 0 = default
 * (a third of the compute units).  1 forces it wherever the shape allows. */
void spec_k_set_swiglu_min_wgs(int32_t workgroups);

/* Tuning knob: wavefronts per workgroup of that SwiGLU GEMM (each takes a gate tile and its up
 * tile): 2, 3 or 4; 0 = default (as few as still give no more workgroups than compute units).
 * Process-wide; affects launches made after the call. */
void spec_k_set_swiglu_column_groups(int32_t groups);

/* Tuning knob: wavefront work items (sequence, kv head, position chunk) per compute unit that the
 * attention kernel's position split aims for (0 = default).  Set before spec_verify_init: the
 * workspace for chunk results is sized with it, and a step whose plan needs more than the handle
 * holds fails with SPEC_ERR_SHAPE.  Process-wide. */
void spec_k_set_attn_items_per_cu(int32_t items);

/* Tuning knob: the attention workgroups merge the chunk results of a (sequence, kv head) themselves
 * (one workgroup of up to 8 wavefronts per pair, no merge kernel) when the launch has at least this
 * many pairs; 0 = default (half the compute units).  1 forces it wherever the shape allows. */
void spec_k_set_attn_merge_min_pairs(int32_t pairs);

/* Tuning knob: most position chunks per (sequence, kv head), 1..16 (anything else restores the
 * default 16).  Set before spec_verify_init, like spec_k_set_attn_items_per_cu. */
void spec_k_set_attn_max_chunks(int32_t chunks);

/* Same product for a plain fp32 W[N][K]. */
int spec_k_gemm_f32(const float* x, const float* w, float* y, int32_t M, int32_t N, int32_t K, void* stream);

/* Per-kernel-class timing of spec_verify_step with HIP events recorded on the launch stream.
 * Between profile_begin and profile_end every kernel (or short group of kernels) of a step is
 * bracketed by two events; profile_end synchronises the stream, adds the elapsed times per class
 * into ms[SPEC_PROF_COUNT] and the number of bracketed launches into launches[SPEC_PROF_COUNT]
 * (host arrays), and switches timing off again.  If empty_pair_ms is not NULL it receives what a
 * start/stop event pair measures with no work in between (median of 33 pairs on the same stream):
 * every bracketed time contains about that much event handling on top of the kernel's execution.
 * Event recording costs a little time per launch, so profiled steps are slower than plain ones;
 * kernel durations themselves are unaffected. */
enum {
    SPEC_PROF_GEMM = 0,          /* projection GEMMs (QKV, O, gate/up, down, LM head) */
    SPEC_PROF_ATTENTION = 1,     /* windowed-causal attention, position-chunk pass */
    SPEC_PROF_ATTN_MERGE = 2,    /* merge of the chunk results */
    SPEC_PROF_GLUE = 3,          /* embedding, norms, rotary + KV append, SiLU gating, partial sums */
    SPEC_PROF_SAMPLER_STATS = 4, /* softmax statistics over all target and draft rows */
    SPEC_PROF_SAMPLER_DRAW = 5,  /* accept scan, residual mass, final draw, KV length update */
    SPEC_PROF_PREPARE = 6,       /* row bookkeeping */
    /* the projection GEMMs one by one (each is also counted in SPEC_PROF_GEMM) */
    SPEC_PROF_GEMM_QKV = 7,
    SPEC_PROF_GEMM_O = 8,
    SPEC_PROF_GEMM_GATE_UP = 9,  /* with SwiGLU where the GEMM finishes it itself */
    SPEC_PROF_GEMM_DOWN = 10,
    SPEC_PROF_GEMM_LM_HEAD = 11,
    SPEC_PROF_COUNT = 12
};
struct spec_handle;
int spec_verify_profile_begin(struct spec_handle* h);
int spec_verify_profile_end(struct spec_handle* h, void* stream, double* ms, int32_t* launches,
                            double* empty_pair_ms);

/* Tuning knob: an attention launch of a model with several query heads per kv head, at most an eighth as
 * many (sequence, kv head) pairs as compute units and a cache capacity (max_kv_len, counted in positions of
 * 64-dim heads) of at most this many positions uses the small-launch plan -- a kv
 * head's query heads as work items of their own, at most four position chunks, merged inside the
 * workgroup; negative = default (2816), 0 = never.  Process-wide; set before spec_verify_init. */
void spec_k_set_attn_small_positions(int32_t positions);

/* What a step would launch, without touching a device: the host-side planning of spec_verify_step
 * for a bf16 model of cfg and a batch with the given lookaheads, on a chip with cu_count compute
 * units.  For tests of that logic and for sizing questions ("how many passes, how much workspace").
 * The figures are those of the tuning knobs in force at the call. */
#define SPEC_PLAN_MAX_PASSES 32
#define SPEC_PLAN_PROJECTIONS 5   /* QKV, output, gate/up, down, LM head */
typedef struct {
    int32_t rows;                 /* sum of K_b + 1 */
    int32_t n_passes;             /* decoder passes (1 unless rows > SPEC_MAX_STEP_ROWS) */
    int32_t pass_seqs[SPEC_PLAN_MAX_PASSES], pass_rows[SPEC_PLAN_MAX_PASSES];
    /* the projections of the first pass: variant and launch shape (gate/up: the plan used when SwiGLU is
     * not finished inside the GEMM) */
    int32_t gemm_row_tiles[SPEC_PLAN_PROJECTIONS], gemm_col_tiles[SPEC_PLAN_PROJECTIONS];
    int32_t gemm_k_ranges[SPEC_PLAN_PROJECTIONS], gemm_k_blocks_per_range[SPEC_PLAN_PROJECTIONS];
    int32_t gemm_row_parts[SPEC_PLAN_PROJECTIONS], gemm_col_groups[SPEC_PLAN_PROJECTIONS];
    int32_t gemm_workgroups[SPEC_PLAN_PROJECTIONS];
    uint64_t gemm_partial_floats[SPEC_PLAN_PROJECTIONS];
    uint64_t gemm_partial_capacity;   /* what spec_verify_init would allocate for them */
    int32_t gate_up_swiglu_inside;    /* 1: the gate/up projection finishes SwiGLU itself (one K range) */
    int32_t reserved0;
    /* operand-fragment buffers, in 16-byte units: what the first pass writes and what init allocates;
     * the second pair is the down projection's operand when SwiGLU is finished inside the GEMM */
    uint64_t xfrag_units, xfrag_capacity, xfrag_act_units, xfrag_act_capacity;
    /* the attention launch of the first pass */
    int32_t attn_kv_share;        /* work items per kv head */
    int32_t attn_small;           /* 1: the small-launch plan */
    int32_t attn_chunks, attn_chunk_keys, attn_row_tiles;
    int32_t attn_wavefronts;      /* per workgroup when the chunks merge there; 0: merge kernel */
    int32_t attn_fused;           /* 1: rotary/append inside the attention kernel */
    uint64_t attn_partial_floats, attn_partial_capacity;
} spec_step_plan;
int spec_k_plan_step(const spec_model_cfg* cfg, int32_t batch, const int32_t* lookahead, int32_t cu_count,
                     int32_t paged, spec_step_plan* out);

#ifdef __cplusplus
}
#endif
#endif
