"""ctypes front end of the CPU oracle (oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It knows nothing about the GPU library and takes plain CPU tensors.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SRC = [os.path.join(_HERE, "oracle.c"), os.path.join(_HERE, "oracle.h")]


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (generic x86-64 code, OpenMP, no fp contraction)."""
    if not force and os.path.exists(_LIB_PATH) and all(
            os.path.getmtime(_LIB_PATH) >= os.path.getmtime(s) for s in _SRC):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra",
           "-o", _LIB_PATH, _SRC[0], "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def build_sanitized(out_dir: str) -> str:
    """Compile oracle.c together with its driver (sanitize_main.c) under AddressSanitizer and
    UndefinedBehaviorSanitizer into an executable in out_dir; returns its path.  Run it directly: it
    exercises every exported routine on small seeded inputs and exits non-zero on a failed check,
    the sanitizers abort on anything they find."""
    exe = os.path.join(out_dir, "oracle_sanitized")
    here = os.path.dirname(os.path.abspath(__file__))
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-o", exe, os.path.join(here, "sanitize_main.c"), _SRC[0], "-lm"]
    subprocess.run(cmd, check=True)
    return exe


class _Model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_ffn", "vocab", "dtype", "max_kv_len")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _Weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("w_qkv", C.POINTER(C.c_void_p)),
                ("w_o", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


class _Cache(C.Structure):
    _fields_ = [("base", C.c_void_p), ("layer_stride", C.c_int64)]


class SampleDiag(C.Structure):
    _fields_ = [("accept_ratio", C.c_double * 16), ("final_S", C.c_double), ("final_target", C.c_double),
                ("final_cdf_lo", C.c_double), ("final_cdf_hi", C.c_double), ("final_row", C.c_int32),
                ("final_is_residual", C.c_int32)]


class TreeDiag(C.Structure):
    _fields_ = [("accept_ratio", C.c_double * 16), ("final_S", C.c_double), ("final_target", C.c_double),
                ("final_cdf_lo", C.c_double), ("final_cdf_hi", C.c_double), ("final_node", C.c_int32),
                ("final_level", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.oracle_round_bf16.restype = C.c_float
        _lib.oracle_round_bf16.argtypes = [C.c_float]
        _lib.oracle_inverse_cdf.restype = C.c_int32
        _lib.oracle_threads.restype = C.c_int
    return _lib


def threads() -> int:
    return int(lib().oracle_threads())


def _cpu(t: torch.Tensor) -> torch.Tensor:
    assert t.device.type == "cpu" and t.is_contiguous(), "oracle takes contiguous CPU tensors"
    return t


def _fptr(t: torch.Tensor):
    return C.c_void_p(_cpu(t).data_ptr())


class Model:
    """Target-model description + weights held for the oracle."""

    def __init__(self, shape, weights: Dict[str, object], max_kv_len: int):
        self.shape = shape
        self.max_kv_len = int(max_kv_len)
        self.dtype = shape.torch_dtype
        self._keep = weights
        self.m = _Model(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                        shape.d_ffn, shape.vocab, 1 if shape.dtype == "bf16" else 0, self.max_kv_len,
                        shape.rms_eps, shape.rope_theta)
        L = shape.n_layers
        arr = {}
        for key in ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down"):
            a = (C.c_void_p * L)()
            for l in range(L):
                t = weights["layers"][l][key]
                want = torch.float32 if key.endswith("norm") else self.dtype
                assert t.dtype == want, (key, t.dtype)
                a[l] = _cpu(t).data_ptr()
            arr[key] = a
        self._arr = arr
        assert weights["tok_embed"].dtype == self.dtype and weights["lm_head"].dtype == self.dtype
        self.w = _Weights(_cpu(weights["tok_embed"]).data_ptr(), _cpu(weights["final_norm"]).data_ptr(),
                          _cpu(weights["lm_head"]).data_ptr(),
                          *[C.cast(arr[k], C.POINTER(C.c_void_p)) for k in
                            ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down")])

    def new_cache(self, fill: float = 0.0) -> torch.Tensor:
        """One sequence's cache [L][2][Hkv][T][hd] in the storage dtype."""
        s = self.shape
        return torch.full((s.n_layers, 2, s.n_kv_heads, self.max_kv_len, s.head_dim), fill, dtype=self.dtype)

    def _cache(self, cache: torch.Tensor) -> _Cache:
        s = self.shape
        assert cache.dtype == self.dtype and cache.device.type == "cpu"
        assert tuple(cache.shape[1:]) == (2, s.n_kv_heads, self.max_kv_len, s.head_dim), cache.shape
        assert cache[0].is_contiguous()
        return _Cache(cache.data_ptr(), cache.stride(0))

    def decode_one(self, cache: torch.Tensor, pos: int, token: int) -> torch.Tensor:
        out = torch.empty(self.shape.vocab, dtype=torch.float32)
        c = self._cache(cache)
        rc = lib().oracle_decode_one(C.byref(self.m), C.byref(self.w), C.byref(c), C.c_int32(pos),
                                     C.c_int32(token), _fptr(out))
        if rc:
            raise ValueError("oracle_decode_one rejected its arguments")
        return out

    def verify_sequential(self, cache: torch.Tensor, n: int, window: Sequence[int]) -> torch.Tensor:
        win = (C.c_int32 * len(window))(*[int(t) for t in window])
        out = torch.empty((len(window), self.shape.vocab), dtype=torch.float32)
        c = self._cache(cache)
        rc = lib().oracle_verify_sequential(C.byref(self.m), C.byref(self.w), C.byref(c), C.c_int32(n), win,
                                            C.c_int32(len(window)), _fptr(out))
        if rc:
            raise ValueError("oracle_verify_sequential rejected its arguments")
        return out

    def verify_rows(self, caches: List[torch.Tensor], n: Sequence[int],
                    windows: Sequence[Sequence[int]]) -> torch.Tensor:
        S = len(caches)
        cs = (_Cache * S)(*[self._cache(c) for c in caches])
        nn = (C.c_int32 * S)(*[int(v) for v in n])
        nw = (C.c_int32 * S)(*[len(wd) for wd in windows])
        flat = [int(t) for wd in windows for t in wd]
        win = (C.c_int32 * len(flat))(*flat)
        out = torch.empty((len(flat), self.shape.vocab), dtype=torch.float32)
        rc = lib().oracle_verify_rows(C.byref(self.m), C.byref(self.w), C.c_int32(S), cs, nn, nw, win, _fptr(out))
        if rc:
            raise ValueError("oracle_verify_rows rejected its arguments")
        return out

    def attend(self, cache: torch.Tensor, layer: int, kv_head: int, n_pos: int, q: torch.Tensor) -> torch.Tensor:
        out = torch.empty(self.shape.head_dim, dtype=torch.float32)
        c = self._cache(cache)
        lib().oracle_attend(C.byref(self.m), C.byref(c), C.c_int32(layer), C.c_int32(kv_head),
                            C.c_int32(n_pos), _fptr(q.float().contiguous()), _fptr(out))
        return out


def sample(target_logits: torch.Tensor, draft_logits: torch.Tensor, draft_tokens: Sequence[int],
           uniforms: Sequence[float], temperature: float):
    """One sequence.  target_logits [K+1,V] fp32, draft_logits [K,V] fp32 (K may be 0).
    Returns (n_accepted, out_tokens list of K+1 ints, SampleDiag)."""
    K = len(draft_tokens)
    V = target_logits.shape[-1]
    assert target_logits.shape == (K + 1, V) and target_logits.dtype == torch.float32
    if K:
        assert draft_logits.shape[0] >= K and draft_logits.shape[1] == V and draft_logits.dtype == torch.float32
    dl = _cpu(draft_logits) if K else torch.zeros((1, V), dtype=torch.float32)
    toks = (C.c_int32 * max(K, 1))(*[int(t) for t in draft_tokens])
    us = (C.c_float * (K + 1))(*[float(u) for u in uniforms[:K + 1]])
    na = C.c_int32(0)
    out = (C.c_int32 * (K + 1))()
    diag = SampleDiag()
    rc = lib().oracle_sample(C.c_int32(V), C.c_int32(K), _fptr(target_logits), _fptr(dl), toks, us,
                             C.c_float(temperature), C.byref(na), out, C.byref(diag))
    if rc:
        raise ValueError("oracle_sample rejected its arguments")
    return int(na.value), list(out), diag


def greedy(target_logits: torch.Tensor, draft_tokens: Sequence[int]):
    """Temperature-0 verification of one sequence: (n_accepted, out_tokens [K+1], smallest deciding gap)."""
    K = len(draft_tokens)
    V = target_logits.shape[-1]
    assert target_logits.shape == (K + 1, V) and target_logits.dtype == torch.float32
    toks = (C.c_int32 * max(K, 1))(*[int(t) for t in draft_tokens])
    na = C.c_int32(0)
    out = (C.c_int32 * (K + 1))()
    gap = C.c_float(0.0)
    rc = lib().oracle_greedy(C.c_int32(V), C.c_int32(K), _fptr(target_logits), toks, C.byref(na), out, C.byref(gap))
    if rc:
        raise ValueError("oracle_greedy rejected its arguments")
    return int(na.value), list(out), float(gap.value)


def tree_sample(parent: Sequence[int], tokens: Sequence[int], target_logits: torch.Tensor,
                draft_logits: torch.Tensor, uniforms: Sequence[float], temperature: float):
    """One sequence's token tree.  target_logits, draft_logits [N+1,V] fp32 (row 0: the root, row i+1:
    node i), uniforms [N+1].  Returns (n_accepted, path, out_tokens [N+1], TreeDiag)."""
    N = len(tokens)
    V = target_logits.shape[-1]
    assert len(parent) == N and target_logits.shape == (N + 1, V) and draft_logits.shape[0] >= N + 1
    assert target_logits.dtype == torch.float32 and draft_logits.dtype == torch.float32
    par = (C.c_int32 * max(N, 1))(*[int(v) for v in parent])
    tok = (C.c_int32 * max(N, 1))(*[int(v) for v in tokens])
    us = (C.c_float * (N + 1))(*[float(u) for u in uniforms[:N + 1]])
    na = C.c_int32(0)
    path = (C.c_int32 * max(N, 1))()
    out = (C.c_int32 * (N + 1))()
    diag = TreeDiag()
    rc = lib().oracle_tree_sample(C.c_int32(V), C.c_int32(N), par, tok, _fptr(target_logits), _fptr(draft_logits),
                                  us, C.c_float(temperature), C.byref(na), path, out, C.byref(diag))
    if rc:
        raise ValueError("oracle_tree_sample rejected its arguments")
    return int(na.value), list(path)[:int(na.value)], list(out), diag


def tree_greedy(parent: Sequence[int], tokens: Sequence[int], target_logits: torch.Tensor):
    """Temperature-0 verification of one sequence's tree: (n_accepted, path, out_tokens [N+1], smallest gap)."""
    N = len(tokens)
    V = target_logits.shape[-1]
    assert len(parent) == N and target_logits.shape == (N + 1, V) and target_logits.dtype == torch.float32
    par = (C.c_int32 * max(N, 1))(*[int(v) for v in parent])
    tok = (C.c_int32 * max(N, 1))(*[int(v) for v in tokens])
    na = C.c_int32(0)
    path = (C.c_int32 * max(N, 1))()
    out = (C.c_int32 * (N + 1))()
    gap = C.c_float(0.0)
    rc = lib().oracle_tree_greedy(C.c_int32(V), C.c_int32(N), par, tok, _fptr(target_logits), C.byref(na), path, out,
                                  C.byref(gap))
    if rc:
        raise ValueError("oracle_tree_greedy rejected its arguments")
    return int(na.value), list(path)[:int(na.value)], list(out), float(gap.value)


def tree_paths(parent: Sequence[int]):
    """For every node its path from the root (list of node indices ending in the node itself)."""
    paths = []
    for i, p in enumerate(parent):
        paths.append((paths[p] if p >= 0 else []) + [i])
    return paths


def tree_logits(model: "Model", cache: torch.Tensor, n: int, last_token: int, parent: Sequence[int],
                tokens: Sequence[int]) -> torch.Tensor:
    """Rows [N+1,V]: row 0 = the model's distribution after the last token, row i+1 after the path
    to node i -- each by ordinary decoding along that path (the definition; shared prefixes are
    simply decoded again).  Cache entries from position n on are scratch."""
    V = model.shape.vocab
    rows = torch.empty((len(tokens) + 1, V), dtype=torch.float32)
    rows[0] = model.decode_one(cache, n, int(last_token))
    for i, path in enumerate(tree_paths(parent)):
        lg = model.verify_sequential(cache, n, [int(last_token)] + [int(tokens[j]) for j in path])
        rows[i + 1] = lg[-1]
    return rows


def softmax(logits: torch.Tensor, temperature: float) -> torch.Tensor:
    V = logits.numel()
    p = torch.empty(V, dtype=torch.float64)
    lib().oracle_softmax(C.c_int32(V), _fptr(logits.float().contiguous()), C.c_float(temperature), _fptr(p))
    return p


def residual(p: torch.Tensor, q: torch.Tensor):
    V = p.numel()
    r = torch.empty(V, dtype=torch.float64)
    S = C.c_double(0.0)
    lib().oracle_residual(C.c_int32(V), _fptr(p), _fptr(q), _fptr(r), C.byref(S))
    return r, float(S.value)


def inverse_cdf(r: torch.Tensor, target: float):
    lo, hi = C.c_double(0.0), C.c_double(0.0)
    y = lib().oracle_inverse_cdf(C.c_int32(r.numel()), _fptr(r), C.c_double(target), C.byref(lo), C.byref(hi))
    return int(y), float(lo.value), float(hi.value)


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    out = torch.empty_like(x)
    lib().oracle_rmsnorm(C.c_int32(x.numel()), _fptr(x), _fptr(gain), C.c_float(eps), _fptr(out))
    return out


def rope(vec: torch.Tensor, theta: float, pos: int) -> torch.Tensor:
    out = vec.clone().contiguous()
    lib().oracle_rope(C.c_int32(out.numel()), C.c_float(theta), C.c_int32(pos), _fptr(out))
    return out


def linear(W: torch.Tensor, x: torch.Tensor) -> torch.Tensor:
    n_out, n_in = W.shape
    y = torch.empty(n_out, dtype=torch.float32)
    lib().oracle_linear(C.c_int32(1 if W.dtype == torch.bfloat16 else 0), _fptr(W), C.c_int32(n_out),
                        C.c_int32(n_in), _fptr(x), _fptr(y))
    return y


def round_bf16(x: float) -> float:
    return float(lib().oracle_round_bf16(C.c_float(x)))
