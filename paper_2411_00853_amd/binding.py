"""ctypes binding of libspecverify.so: the same entry points as include/spec_verify.h,
include/spec_decode.h and include/spec_kernels.h, taking torch tensors where the C side takes device pointers.  Argument
marshalling only -- no arithmetic of the method happens here, and there is no fallback: if the
HIP library is missing or fails to load, every call raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

from . import build as _build

SPEC_DTYPE_FP32, SPEC_DTYPE_BF16 = 0, 1
SPEC_MAX_BATCH, SPEC_MAX_LOOKAHEAD = 256, 15
SPEC_OK = 0


class SpecError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"spec status {status}: {msg}")
        self.status = status


class spec_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                         "vocab", "max_batch", "max_kv_len", "max_lookahead", "dtype")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class spec_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down")]


class spec_weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(spec_layer_weights))]


class spec_step_args(C.Structure):
    _fields_ = [("batch", C.c_int32), ("lookahead", C.POINTER(C.c_int32)), ("seq_slot", C.c_void_p),
                ("last_token", C.c_void_p), ("draft_tokens", C.c_void_p), ("draft_logits", C.c_void_p),
                ("uniforms", C.c_void_p), ("temperature", C.c_float), ("target_logits_in", C.c_void_p),
                ("auto_rollback", C.c_int32)]


class spec_step_out(C.Structure):
    _fields_ = [("n_accepted", C.c_void_p), ("out_tokens", C.c_void_p), ("logits_out", C.c_void_p)]


class spec_tree_args(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_nodes", C.POINTER(C.c_int32)), ("seq_slot", C.c_void_p),
                ("last_token", C.c_void_p), ("parent", C.c_void_p), ("draft_tokens", C.c_void_p),
                ("draft_logits", C.c_void_p), ("uniforms", C.c_void_p), ("temperature", C.c_float),
                ("target_logits_in", C.c_void_p), ("auto_rollback", C.c_int32)]


class spec_tree_out(C.Structure):
    _fields_ = [("n_accepted", C.c_void_p), ("out_tokens", C.c_void_p), ("path", C.c_void_p),
                ("logits_out", C.c_void_p)]


class spec_decode_cfg(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("max_new_tokens", C.c_int32)]


class spec_round_args(C.Structure):
    _fields_ = [("lookahead", C.c_int32), ("draft_uniforms", C.c_void_p), ("verify_uniforms", C.c_void_p),
                ("temperature", C.c_float), ("lookahead_per_seq", C.POINTER(C.c_int32))]


class spec_lookahead_cfg(C.Structure):
    _fields_ = [("draft_ms", C.c_double), ("verify_ms", C.c_double), ("verify_ms_per_token", C.c_double),
                ("k_min", C.c_int32), ("k_max", C.c_int32), ("forget", C.c_double), ("prior_accept", C.c_double),
                ("prior_weight", C.c_double)]


class spec_decode_view(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("tokens", "n_tokens", "n_accepted", "draft_tokens", "draft_logits",
                                          "target_logits", "prev_token", "last_token", "counters")]


PLAN_MAX_PASSES, PLAN_PROJECTIONS = 32, 5


class spec_step_plan(C.Structure):
    _fields_ = [("rows", C.c_int32), ("n_passes", C.c_int32),
                ("pass_seqs", C.c_int32 * PLAN_MAX_PASSES), ("pass_rows", C.c_int32 * PLAN_MAX_PASSES)] + \
               [(n, C.c_int32 * PLAN_PROJECTIONS) for n in ("gemm_row_tiles", "gemm_col_tiles", "gemm_k_ranges",
                                                            "gemm_k_blocks_per_range", "gemm_row_parts",
                                                            "gemm_col_groups", "gemm_workgroups")] + \
               [("gemm_partial_floats", C.c_uint64 * PLAN_PROJECTIONS), ("gemm_partial_capacity", C.c_uint64),
                ("gate_up_swiglu_inside", C.c_int32), ("reserved0", C.c_int32), ("xfrag_units", C.c_uint64),
                ("xfrag_capacity", C.c_uint64), ("xfrag_act_units", C.c_uint64), ("xfrag_act_capacity", C.c_uint64)] + \
               [(n, C.c_int32) for n in ("attn_kv_share", "attn_small", "attn_chunks", "attn_chunk_keys",
                                         "attn_row_tiles", "attn_wavefronts", "attn_fused")] + \
               [("attn_partial_floats", C.c_uint64), ("attn_partial_capacity", C.c_uint64)]


_lib = None


def lib():
    """Load the HIP library (building it first only if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build_library()
        L = C.CDLL(_build.LIB)
        L.spec_last_error.restype = C.c_char_p
        L.spec_packed_weight_bytes.restype = C.c_size_t
        L.spec_packed_weight_bytes.argtypes = [C.c_int32, C.c_int32]
        L.spec_kv_cache_bytes.restype = C.c_size_t
        L.spec_kv_cache_bytes.argtypes = [C.POINTER(spec_model_cfg)]
        L.spec_k_gemm_workspace_bytes.restype = C.c_size_t
        L.spec_k_gemm_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.spec_verify_destroy.restype = None
        L.spec_verify_destroy.argtypes = [C.c_void_p]
        L.spec_verify_init.argtypes = [C.POINTER(spec_model_cfg), C.POINTER(spec_weights), C.c_void_p, C.c_size_t,
                                       C.c_void_p, C.POINTER(C.c_void_p)]
        L.spec_verify_init_paged.argtypes = L.spec_verify_init.argtypes
        L.spec_kv_page_bytes.restype = C.c_size_t
        L.spec_kv_page_bytes.argtypes = [C.POINTER(spec_model_cfg)]
        L.spec_kv_pages.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]
        L.spec_verify_step.argtypes = [C.c_void_p, C.POINTER(spec_step_args), C.POINTER(spec_step_out), C.c_void_p]
        L.spec_sample_step_noalloc.argtypes = [C.c_int32, C.c_int32, C.POINTER(spec_step_args), C.POINTER(spec_step_out),
                                               C.c_void_p]
        L.spec_verify_tree_step.argtypes = [C.c_void_p, C.POINTER(spec_tree_args), C.POINTER(spec_tree_out), C.c_void_p]
        L.spec_kv_rollback.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32, C.c_void_p]
        L.spec_kv_import.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.spec_kv_export.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.spec_verify_poll.argtypes = [C.c_void_p, C.c_void_p]
        L.spec_pack_weight.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.spec_k_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.spec_k_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.spec_k_mfma_tile.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.spec_k_gemm_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_void_p, C.c_void_p]
        L.spec_k_gemm_f32.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.spec_k_set_gemm_wg_target.restype = None
        L.spec_k_set_gemm_wg_target.argtypes = [C.c_int32]
        L.spec_k_set_gemm_balance_groups.restype = None
        L.spec_k_set_gemm_balance_groups.argtypes = [C.c_int32]
        L.spec_k_set_swiglu_min_wgs.restype = None
        L.spec_k_set_swiglu_min_wgs.argtypes = [C.c_int32]
        L.spec_k_set_swiglu_column_groups.restype = None
        L.spec_k_set_swiglu_column_groups.argtypes = [C.c_int32]
        L.spec_k_set_attn_items_per_cu.restype = None
        L.spec_k_set_attn_items_per_cu.argtypes = [C.c_int32]
        L.spec_k_set_attn_merge_min_pairs.restype = None
        L.spec_k_set_attn_merge_min_pairs.argtypes = [C.c_int32]
        L.spec_k_set_attn_max_chunks.restype = None
        L.spec_k_set_attn_max_chunks.argtypes = [C.c_int32]
        L.spec_k_set_attn_small_positions.restype = None
        L.spec_k_set_attn_small_positions.argtypes = [C.c_int32]
        L.spec_verify_profile_begin.argtypes = [C.c_void_p]
        L.spec_verify_profile_end.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32),
                                              C.POINTER(C.c_double)]
        L.spec_decode_init.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(spec_decode_cfg), C.POINTER(C.c_void_p)]
        L.spec_decode_destroy.restype = None
        L.spec_decode_destroy.argtypes = [C.c_void_p]
        L.spec_decode_begin.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.spec_decode_round.argtypes = [C.c_void_p, C.POINTER(spec_round_args), C.c_void_p]
        L.spec_decode_get_view.argtypes = [C.c_void_p, C.POINTER(spec_decode_view)]
        L.spec_lookahead_init.argtypes = [C.POINTER(spec_lookahead_cfg), C.c_int32, C.POINTER(C.c_void_p)]
        L.spec_lookahead_destroy.restype = None
        L.spec_lookahead_destroy.argtypes = [C.c_void_p]
        L.spec_lookahead_update.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32]
        L.spec_lookahead_next.argtypes = [C.c_void_p]
        L.spec_lookahead_next.restype = C.c_int32
        L.spec_lookahead_next_per_seq.restype = C.c_int32
        L.spec_lookahead_next_per_seq.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.spec_lookahead_update_per_seq.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.spec_lookahead_accept.argtypes = [C.c_void_p, C.c_int32]
        L.spec_lookahead_accept.restype = C.c_double
        _lib = L
    return _lib


def last_error() -> str:
    return lib().spec_last_error().decode()


def _check(rc: int):
    if rc != SPEC_OK:
        raise SpecError(rc, last_error())


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    """Device pointer of a contiguous CUDA tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def make_cfg(shape, max_batch: int, max_kv_len: int, max_lookahead: int) -> spec_model_cfg:
    """spec_model_cfg from a workload.ModelShape-like object."""
    return spec_model_cfg(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                          shape.d_ffn, shape.vocab, max_batch, max_kv_len, max_lookahead,
                          SPEC_DTYPE_BF16 if shape.dtype == "bf16" else SPEC_DTYPE_FP32, shape.rms_eps, shape.rope_theta)


def sampler_cfg(vocab: int, max_batch: int, max_lookahead: int) -> spec_model_cfg:
    return spec_model_cfg(0, 0, 0, 0, 0, 0, vocab, max_batch, 0, max_lookahead, 0, 0.0, 0.0)


def spec_packed_weight_bytes(n_out: int, n_in: int) -> int:
    return int(lib().spec_packed_weight_bytes(n_out, n_in))


def spec_pack_weight(src: torch.Tensor, interleave_halves: bool = False, stream=None) -> torch.Tensor:
    """Row-major bf16 [n_out][n_in] device matrix -> new device buffer in streaming tile order."""
    n_out, n_in = src.shape
    nbytes = spec_packed_weight_bytes(n_out, n_in)
    if nbytes == 0:
        raise SpecError(-2, "matrix shape cannot be packed (n_in must be a multiple of 32)")
    dst = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=src.device)
    _check(lib().spec_pack_weight(_ptr(src, torch.bfloat16), _ptr(dst), n_out, n_in, int(interleave_halves),
                                  _stream(stream)))
    return dst


def spec_kv_cache_bytes(cfg: spec_model_cfg) -> int:
    return int(lib().spec_kv_cache_bytes(C.byref(cfg)))


class Handle:
    """Owns a spec_handle* and keeps the caller-owned tensors it points into alive."""

    def __init__(self, ptr, cfg, keep):
        self.ptr, self.cfg, self._keep = ptr, cfg, keep

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def close(self):
        if getattr(self, "ptr", None):
            lib().spec_verify_destroy(self.ptr)
            self.ptr = None


def spec_kv_page_bytes(cfg: spec_model_cfg) -> int:
    return int(lib().spec_kv_page_bytes(C.byref(cfg)))


def spec_kv_pages(h: Handle, stream=None):
    """(free pages, total pages) of a paged handle."""
    f, t = C.c_int32(0), C.c_int32(0)
    _check(lib().spec_kv_pages(h.ptr, C.byref(f), C.byref(t), _stream(stream)))
    return int(f.value), int(t.value)


def spec_verify_init_paged(cfg: spec_model_cfg, weights: dict, kv_pool: torch.Tensor, kv_len: torch.Tensor) -> Handle:
    return spec_verify_init(cfg, weights, kv_pool, kv_len, paged=True)


def spec_verify_init(cfg: spec_model_cfg, weights: Optional[dict], kv_cache: Optional[torch.Tensor],
                     kv_len: Optional[torch.Tensor], paged: bool = False) -> Handle:
    """weights: {"tok_embed", "final_norm", "lm_head", "layers": [{"attn_norm", "w_qkv", "w_o", "ffn_norm",
    "w_gate_up", "w_down"}]} of device tensors already in the layout the header prescribes (bf16
    projection matrices packed with spec_pack_weight), or None for a sampler-only handle."""
    out = C.c_void_p()
    keep = [weights, kv_cache, kv_len]
    wp = None
    if weights is not None:
        L = cfg.n_layers
        arr = (spec_layer_weights * L)()
        for l, lw in enumerate(weights["layers"]):
            arr[l] = spec_layer_weights(_ptr(lw["attn_norm"], torch.float32), _ptr(lw["w_qkv"]), _ptr(lw["w_o"]),
                                        _ptr(lw["ffn_norm"], torch.float32), _ptr(lw["w_gate_up"]), _ptr(lw["w_down"]))
        w = spec_weights(_ptr(weights["tok_embed"]), _ptr(weights["final_norm"], torch.float32),
                         _ptr(weights["lm_head"]), C.cast(arr, C.POINTER(spec_layer_weights)))
        keep.append(arr)
        wp = C.byref(w)
    nbytes = kv_cache.numel() * kv_cache.element_size() if kv_cache is not None else 0
    init = lib().spec_verify_init_paged if paged else lib().spec_verify_init
    _check(init(C.byref(cfg), wp, _ptr(kv_cache), nbytes, _ptr(kv_len, torch.int32), C.byref(out)))
    return Handle(out.value, cfg, keep)


def spec_verify_destroy(h: Handle):
    h.close()


def spec_verify_step(h: Handle, lookahead: Sequence[int], uniforms: torch.Tensor, temperature: float,
                     n_accepted: torch.Tensor, out_tokens: torch.Tensor, seq_slot: Optional[torch.Tensor] = None,
                     last_token: Optional[torch.Tensor] = None, draft_tokens: Optional[torch.Tensor] = None,
                     draft_logits: Optional[torch.Tensor] = None, target_logits_in: Optional[torch.Tensor] = None,
                     logits_out: Optional[torch.Tensor] = None, auto_rollback: bool = True, stream=None):
    B = len(lookahead)
    ks = (C.c_int32 * B)(*[int(k) for k in lookahead])
    args = spec_step_args(B, ks, _ptr(seq_slot, torch.int32), _ptr(last_token, torch.int32),
                          _ptr(draft_tokens, torch.int32), _ptr(draft_logits, torch.float32),
                          _ptr(uniforms, torch.float32), float(temperature), _ptr(target_logits_in, torch.float32),
                          int(auto_rollback))
    out = spec_step_out(_ptr(n_accepted, torch.int32), _ptr(out_tokens, torch.int32), _ptr(logits_out, torch.float32))
    _check(lib().spec_verify_step(h.ptr, C.byref(args), C.byref(out), _stream(stream)))


def spec_sample_step_noalloc(vocab: int, max_lookahead: int, lookahead: Sequence[int], uniforms: Optional[torch.Tensor],
                             temperature: float, n_accepted: torch.Tensor, out_tokens: torch.Tensor,
                             target_logits_in: torch.Tensor, draft_tokens: Optional[torch.Tensor] = None,
                             draft_logits: Optional[torch.Tensor] = None, logits_out: Optional[torch.Tensor] = None,
                             stream=None):
    B = len(lookahead)
    ks = (C.c_int32 * max(B, 1))(*[int(k) for k in lookahead])
    args = spec_step_args(B, ks, None, None, _ptr(draft_tokens, torch.int32), _ptr(draft_logits, torch.float32),
                          _ptr(uniforms, torch.float32), float(temperature), _ptr(target_logits_in, torch.float32), 0)
    out = spec_step_out(_ptr(n_accepted, torch.int32), _ptr(out_tokens, torch.int32), _ptr(logits_out, torch.float32))
    _check(lib().spec_sample_step_noalloc(int(vocab), int(max_lookahead), C.byref(args), C.byref(out), _stream(stream)))


def spec_verify_tree_step(h: Handle, n_nodes: Sequence[int], parent: Optional[torch.Tensor],
                          draft_tokens: Optional[torch.Tensor], draft_logits: torch.Tensor, uniforms: torch.Tensor,
                          temperature: float, n_accepted: torch.Tensor, out_tokens: torch.Tensor, path: torch.Tensor,
                          seq_slot: Optional[torch.Tensor] = None, last_token: Optional[torch.Tensor] = None,
                          target_logits_in: Optional[torch.Tensor] = None, logits_out: Optional[torch.Tensor] = None,
                          auto_rollback: bool = True, stream=None):
    B = len(n_nodes)
    ns = (C.c_int32 * B)(*[int(k) for k in n_nodes])
    args = spec_tree_args(B, ns, _ptr(seq_slot, torch.int32), _ptr(last_token, torch.int32),
                          _ptr(parent, torch.int32), _ptr(draft_tokens, torch.int32),
                          _ptr(draft_logits, torch.float32), _ptr(uniforms, torch.float32), float(temperature),
                          _ptr(target_logits_in, torch.float32), int(auto_rollback))
    out = spec_tree_out(_ptr(n_accepted, torch.int32), _ptr(out_tokens, torch.int32), _ptr(path, torch.int32),
                        _ptr(logits_out, torch.float32))
    _check(lib().spec_verify_tree_step(h.ptr, C.byref(args), C.byref(out), _stream(stream)))


def spec_kv_rollback(h: Handle, seq_slot: Sequence[int], new_len: Sequence[int], stream=None):
    n = len(seq_slot)
    a = (C.c_int32 * max(n, 1))(*[int(v) for v in seq_slot])
    b = (C.c_int32 * max(n, 1))(*[int(v) for v in new_len])
    _check(lib().spec_kv_rollback(h.ptr, a, b, n, _stream(stream)))


def spec_kv_import(h: Handle, slot: int, pos0: int, src: torch.Tensor, stream=None):
    """src: device tensor [n_layers][2][n_kv_heads][n_pos][head_dim] in the cache's storage dtype."""
    _check(lib().spec_kv_import(h.ptr, slot, pos0, src.shape[3], _ptr(src), _stream(stream)))


def spec_kv_export(h: Handle, slot: int, pos0: int, dst: torch.Tensor, stream=None):
    _check(lib().spec_kv_export(h.ptr, slot, pos0, dst.shape[3], _ptr(dst), _stream(stream)))


def spec_verify_poll(h: Handle, stream=None):
    _check(lib().spec_verify_poll(h.ptr, _stream(stream)))


# ---- the decoding round (include/spec_decode.h) --------------------------------------------------

class Decoder:
    """Owns a spec_decoder* and keeps the two handles alive."""

    def __init__(self, ptr, target: Handle, draft: Optional[Handle], max_batch: int, max_new_tokens: int):
        self.ptr, self.target, self.draft = ptr, target, draft
        self.max_batch, self.max_new_tokens = max_batch, max_new_tokens

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def close(self):
        if getattr(self, "ptr", None):
            lib().spec_decode_destroy(self.ptr)
            self.ptr = None


def spec_decode_init(target: Handle, draft: Optional[Handle], max_batch: int, max_new_tokens: int) -> Decoder:
    out = C.c_void_p()
    cfg = spec_decode_cfg(max_batch, max_new_tokens)
    _check(lib().spec_decode_init(target.ptr, draft.ptr if draft is not None else None, C.byref(cfg), C.byref(out)))
    return Decoder(out.value, target, draft, max_batch, max_new_tokens)


def spec_decode_destroy(d: Decoder):
    d.close()


def spec_decode_begin(d: Decoder, seq_slot: torch.Tensor, prev_token: Optional[torch.Tensor],
                      last_token: torch.Tensor, stream=None):
    _check(lib().spec_decode_begin(d.ptr, seq_slot.numel(), _ptr(seq_slot, torch.int32), _ptr(prev_token, torch.int32),
                                   _ptr(last_token, torch.int32), _stream(stream)))


def spec_decode_round(d: Decoder, lookahead: int, draft_uniforms: Optional[torch.Tensor],
                      verify_uniforms: torch.Tensor, temperature: float, stream=None, lookahead_per_seq=None):
    per = None
    if lookahead_per_seq is not None:
        per = (C.c_int32 * len(lookahead_per_seq))(*[int(k) for k in lookahead_per_seq])
    args = spec_round_args(int(lookahead), _ptr(draft_uniforms, torch.float32), _ptr(verify_uniforms, torch.float32),
                           float(temperature), per)
    _check(lib().spec_decode_round(d.ptr, C.byref(args), _stream(stream)))


def spec_decode_get_view(d: Decoder) -> spec_decode_view:
    v = spec_decode_view()
    _check(lib().spec_decode_get_view(d.ptr, C.byref(v)))
    return v


class Lookahead:
    """Owns a spec_lookahead* (host-side controller; no GPU needed)."""

    def __init__(self, batch: int, draft_ms: float, verify_ms: float, verify_ms_per_token: float, k_min: int,
                 k_max: int, forget: float = 0.9, prior_accept: float = 0.5, prior_weight: float = 4.0):
        self.batch = batch
        cfg = spec_lookahead_cfg(draft_ms, verify_ms, verify_ms_per_token, k_min, k_max, forget, prior_accept,
                                 prior_weight)
        out = C.c_void_p()
        _check(lib().spec_lookahead_init(C.byref(cfg), batch, C.byref(out)))
        self.ptr = out.value

    def update(self, n_accepted: Sequence[int], K: int):
        arr = (C.c_int32 * self.batch)(*[int(v) for v in n_accepted])
        _check(lib().spec_lookahead_update(self.ptr, arr, int(K)))

    def next(self) -> int:
        k = int(lib().spec_lookahead_next(self.ptr))
        if k < 0:
            raise SpecError(k, last_error())
        return k

    def next_per_seq(self):
        """(K of the round, [K_b per sequence])"""
        out = (C.c_int32 * self.batch)()
        k = int(lib().spec_lookahead_next_per_seq(self.ptr, out))
        if k < 0:
            raise SpecError(k, last_error())
        return k, list(out)

    def update_per_seq(self, n_accepted: Sequence[int], K_per_seq: Sequence[int]):
        arr = (C.c_int32 * self.batch)(*[int(v) for v in n_accepted])
        ks = (C.c_int32 * self.batch)(*[int(v) for v in K_per_seq])
        _check(lib().spec_lookahead_update_per_seq(self.ptr, arr, ks))

    def accept(self, b: int) -> float:
        return float(lib().spec_lookahead_accept(self.ptr, int(b)))

    def close(self):
        if getattr(self, "ptr", None):
            lib().spec_lookahead_destroy(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def device_array(ptr: Optional[int], shape, dtype, device="cuda") -> torch.Tensor:
    """A copy of library-owned device memory as a tensor (spec_k_copy on the current stream; the
    library's allocations are 256-byte granular, so rounding the size up to 16 bytes stays inside)."""
    n = 1
    for v in shape:
        n *= int(v)
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    raw = torch.empty((nbytes + 15) // 16 * 16, dtype=torch.uint8, device=device)
    if nbytes:
        _check(lib().spec_k_copy(C.c_void_p(ptr), _ptr(raw), raw.numel(), _stream(None)))
    return raw[:nbytes].view(dtype).reshape(shape)


# ---- single-kernel entry points (include/spec_kernels.h) -----------------------------------------

def spec_k_copy(src: torch.Tensor, dst: torch.Tensor, stream=None):
    _check(lib().spec_k_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream(stream)))


def spec_k_read(src: torch.Tensor, out: torch.Tensor, stream=None):
    _check(lib().spec_k_read(_ptr(src), src.numel() * src.element_size(), _ptr(out, torch.float32), _stream(stream)))


def spec_k_mfma_tile(a: torch.Tensor, b: torch.Tensor, d: torch.Tensor, stream=None):
    _check(lib().spec_k_mfma_tile(_ptr(a, torch.bfloat16), _ptr(b, torch.bfloat16), _ptr(d, torch.float32),
                                  _stream(stream)))


def spec_k_gemm_bf16(x: torch.Tensor, w_packed: torch.Tensor, n_out: int, split_x: bool = True,
                     workspace: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None, stream=None):
    M, K = x.shape
    if y is None:
        y = torch.empty((M, n_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        nb = int(lib().spec_k_gemm_workspace_bytes(M, n_out, K))
        workspace = torch.empty(max(nb // 4, 4), dtype=torch.float32, device=x.device)
    _check(lib().spec_k_gemm_bf16(_ptr(x, torch.float32), _ptr(w_packed), _ptr(y), M, n_out, K, int(split_x),
                                  _ptr(workspace), _stream(stream)))
    return y


def spec_k_set_gemm_wg_target(workgroups: int):
    lib().spec_k_set_gemm_wg_target(int(workgroups))


def spec_k_set_gemm_balance_groups(on: bool):
    lib().spec_k_set_gemm_balance_groups(int(on))


def spec_k_set_swiglu_min_wgs(workgroups: int):
    lib().spec_k_set_swiglu_min_wgs(int(workgroups))


def spec_k_set_swiglu_column_groups(groups: int):
    lib().spec_k_set_swiglu_column_groups(int(groups))


def spec_k_set_attn_items_per_cu(items: int):
    lib().spec_k_set_attn_items_per_cu(int(items))


def spec_k_set_attn_merge_min_pairs(pairs: int):
    lib().spec_k_set_attn_merge_min_pairs(int(pairs))


def spec_k_set_attn_max_chunks(chunks: int):
    lib().spec_k_set_attn_max_chunks(int(chunks))


def spec_k_set_attn_small_positions(n: int):
    lib().spec_k_set_attn_small_positions(int(n))


def spec_k_gemm_f32(x: torch.Tensor, w: torch.Tensor, stream=None):
    M, K = x.shape
    N = w.shape[0]
    y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    _check(lib().spec_k_gemm_f32(_ptr(x, torch.float32), _ptr(w, torch.float32), _ptr(y), M, N, K, _stream(stream)))
    return y


PROF_CLASSES = ("gemm", "attention", "attn_merge", "glue", "sampler_stats", "sampler_draw", "prepare",
                "gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head")


def spec_verify_profile_begin(h: Handle):
    _check(lib().spec_verify_profile_begin(h.ptr))


def spec_verify_profile_end(h: Handle, stream=None):
    """Returns ({class name: (total ms, bracketed launches)}, empty event-pair ms) since
    spec_verify_profile_begin."""
    n = len(PROF_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int32 * n)()
    empty = C.c_double(0.0)
    _check(lib().spec_verify_profile_end(h.ptr, _stream(stream), ms, cnt, C.byref(empty)))
    return {PROF_CLASSES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}, float(empty.value)


def spec_k_plan_step(cfg, lookahead, cu_count=256, paged=False) -> spec_step_plan:
    """Host-side planning of one step (no device work): passes, projection launch shapes, attention plan."""
    out = spec_step_plan()
    look = (C.c_int32 * len(lookahead))(*[int(k) for k in lookahead])
    _check(lib().spec_k_plan_step(C.byref(cfg), len(lookahead), look, int(cu_count), 1 if paged else 0, C.byref(out)))
    return out
