"""Seeded synthetic inputs for the speculative-sampling verify step.

This module only *makes inputs*: model shapes, random weights, KV-cache contents,
draft tokens, draft logits and uniforms.  It contains none of the method's
arithmetic (no transformer layer, no softmax, no acceptance test) and is the one
module shared by the CPU oracle's tests and the HIP path's tests and benchmark.

Every value is a pure function of (seed, stream id, flat index): a counter-based
generator built on the splitmix64 finaliser, evaluated with int64 tensor ops so
that any slice of any tensor can be regenerated on its own and on any device.
Normals come from Box-Muller in fp32; transcendental rounding may differ by an
ulp between devices, so one run generates on one device and copies the bytes to
whoever else needs them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import torch

# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------

_M64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed value torch wants."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 lanes (torch's >> is arithmetic)."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """Key of one tensor's stream: two rounds of the finaliser over (seed, stream)."""
    return _mix_py(_mix_py(seed * 0x9E3779B97F4A7C15 + 0x632BE59BD9B4E019) ^ (stream * 0xD1342543DE82EF95))


def hash64(key: int, idx: torch.Tensor) -> torch.Tensor:
    """splitmix64 output for counters ``idx`` (int64 tensor) under ``key``; wraps mod 2^64."""
    z = idx * _GOLDEN + _s64(key)
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


_CHUNK = 1 << 24  # elements generated per pass (bounds temporaries to ~1 GB)


class Rng:
    """Named, counter-based random tensors on one device."""

    def __init__(self, seed: int, device: str | torch.device = "cpu"):
        self.seed = int(seed)
        self.device = torch.device(device)

    def _bits(self, stream: int, start: int, n: int) -> torch.Tensor:
        idx = torch.arange(start, start + n, dtype=torch.int64, device=self.device)
        return hash64(stream_key(self.seed, stream), idx)

    def _fill(self, out_flat: torch.Tensor, stream: int, fn, offset: int = 0):
        n = out_flat.numel()
        for s in range(0, n, _CHUNK):
            m = min(_CHUNK, n - s)
            out_flat[s:s + m] = fn(self._bits(stream, offset + s, m)).to(out_flat.dtype)

    def uniform(self, stream: int, shape, offset: int = 0) -> torch.Tensor:
        """fp32 uniforms in [0,1): top 24 bits of the hash times 2^-24."""
        out = torch.empty(shape, dtype=torch.float32, device=self.device)
        self._fill(out.view(-1), stream, lambda z: _lsr(z, 40).to(torch.float32) * (2.0 ** -24), offset)
        return out

    def normal(self, stream: int, shape, std: float = 1.0, dtype=torch.float32,
               offset: int = 0) -> torch.Tensor:
        """N(0, std^2) by Box-Muller on two 24-bit fields of one hash, rounded (RNE) to dtype."""
        out = torch.empty(shape, dtype=dtype, device=self.device)

        def bm(z):
            u1 = (_lsr(z, 40).to(torch.float32) + 0.5) * (2.0 ** -24)
            u2 = ((_lsr(z, 16) & 0xFFFFFF).to(torch.float32) + 0.5) * (2.0 ** -24)
            return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2) * std

        self._fill(out.view(-1), stream, bm, offset)
        return out

    def gumbel(self, stream: int, shape, offset: int = 0) -> torch.Tensor:
        """Standard Gumbel noise, -log(-log(u)), fp32."""
        out = torch.empty(shape, dtype=torch.float32, device=self.device)

        def g(z):
            u = (_lsr(z, 40).to(torch.float32) + 0.5) * (2.0 ** -24)
            return -torch.log(-torch.log(u))

        self._fill(out.view(-1), stream, g, offset)
        return out

    def randint(self, stream: int, shape, high: int, offset: int = 0) -> torch.Tensor:
        """int32 in [0, high): 32 hash bits scaled down (bias < 2^-32 * high, irrelevant here)."""
        out = torch.empty(shape, dtype=torch.int32, device=self.device)
        self._fill(out.view(-1), stream, lambda z: (_lsr(z, 32) * high) >> 32, offset)
        return out

    def binomial(self, stream: int, shape, n: int, p: float) -> torch.Tensor:
        """Binomial(n, p) as a sum of n Bernoulli draws from n separate counters."""
        numel = int(torch.Size(shape).numel()) if not isinstance(shape, int) else shape
        u = self.uniform(stream, (numel, n))
        return (u < p).sum(dim=1).to(torch.int32).reshape(shape)


# ----------------------------------------------------------------------------
# model shapes and workloads (the five configurations of the benchmark definition)
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"            # storage of weights and KV cache: "bf16" or "fp32"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def d_q(self):
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self):
        return self.n_kv_heads * self.head_dim

    def weight_elems(self) -> int:
        per_layer = (self.d_model * (self.d_q + 2 * self.d_kv) + self.d_q * self.d_model
                     + 3 * self.d_model * self.d_ffn + 2 * self.d_model)
        return self.n_layers * per_layer + 2 * self.vocab * self.d_model + self.d_model


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    batch: int
    kv_lens: tuple            # cached tokens n_b per sequence
    lookahead: tuple          # K_b per sequence
    max_lookahead: int
    max_kv_len: int
    temperature: float
    seed: int
    kv_kind: str              # "prefill" (made by running the model) or "synthetic" N(0,1)

    @property
    def rows(self) -> int:
        return sum(k + 1 for k in self.lookahead)


SEED_BASE = 20241100
# stream ids (added to per-tensor offsets below)
S_WEIGHTS, S_KV, S_TOKENS, S_DRAFT_NOISE, S_DRAFT_PICK, S_UNIFORMS, S_K, S_N, S_STRESS = (
    1 << 20, 2 << 20, 3 << 20, 4 << 20, 5 << 20, 6 << 20, 7 << 20, 8 << 20, 9 << 20)

TINY = ModelShape(2, 256, 4, 4, 64, 1024, 1024, dtype="fp32")
ONE_B = ModelShape(16, 2048, 32, 8, 64, 8192, 32000)
SEVEN_B = ModelShape(32, 4096, 32, 32, 128, 11008, 32000)
# The draft models the configurations name ("draft 2 layers d_model 1024", "draft 4 layers d_model
# 2048"); what they leave open is filled in like the target: same head_dim, same heads-to-width and
# FFN-to-width ratios, same vocabulary.
ONE_B_DRAFT = ModelShape(2, 1024, 16, 4, 64, 4096, 32000)
SEVEN_B_DRAFT = ModelShape(4, 2048, 16, 16, 128, 5504, 32000)


def workload_tiny() -> Workload:
    return Workload("tiny", TINY, 1, (128,), (4,), 4, 128 + 5, 1.0, SEED_BASE + 0, "prefill")


def workload_1b() -> Workload:
    return Workload("1b", ONE_B, 1, (1024,), (5,), 5, 1024 + 6, 1.0, SEED_BASE + 1000, "synthetic")


def workload_7b() -> Workload:
    return Workload("7b", SEVEN_B, 8, (2048,) * 8, (5,) * 8, 5, 2048 + 6, 1.0,
                    SEED_BASE + 2000, "synthetic")


def workload_dyn(batch: int = 32) -> Workload:
    """Dynamic lookahead: n_b uniform in [512, 4096]; K_b = 1 + Binomial(9, 1/3) (support 1..10, mean 4)."""
    seed = SEED_BASE + 3000
    rng = Rng(seed, "cpu")
    n = (512 + rng.randint(S_N, (batch,), 4096 - 512 + 1)).tolist()
    k = (1 + rng.binomial(S_K, (batch,), 9, 1.0 / 3.0)).tolist()
    return Workload("dyn", SEVEN_B, batch, tuple(n), tuple(k), 10, 4096 + 11, 1.0, seed, "synthetic")


def workload_rows352() -> Workload:
    """The largest window the projection kernels take: 32 sequences x (10 proposals + 1) = 352 rows on
    the 7B-shape weights, with short caches (64 positions) so that the step is almost only the
    projections.  Not one of the benchmark's configurations: the point at which the GEMM family's
    matrix-core utilisation is reported (its intensity, 352 flop/B, is just past the ridge)."""
    return Workload("rows352", SEVEN_B, 32, (64,) * 32, (10,) * 32, 10, 64 + 11, 1.0, SEED_BASE + 5000, "synthetic")


# A drafted token tree of 10 nodes (3 candidates for the first token, 2 for the second below the
# first two of them, then single continuations): depth 4, 5 leaves.
TREE10_PARENT = (-1, -1, -1, 0, 0, 1, 3, 3, 4, 6)


def workload_tree() -> Workload:
    """7B-shape target, 8 sequences of 2048 cached tokens, each verifying the 10-node tree above
    (11 window rows per sequence; `lookahead` holds the node count)."""
    n_nodes = len(TREE10_PARENT)
    return Workload("tree", SEVEN_B, 8, (2048,) * 8, (n_nodes,) * 8, n_nodes, 2048 + n_nodes + 1, 1.0,
                    SEED_BASE + 4000, "synthetic")


def make_tree_drafts(w: Workload, parent, device="cpu", logit_std: float = 1.28):
    """Draft logits rows [B][N+1][V] (row 0: the root's, row i+1: node i's), independent of the target,
    N(0, logit_std^2); node tokens drawn from softmax(row of their parent / T)."""
    rng = Rng(w.seed, device)
    B, N, V = w.batch, w.max_lookahead, w.shape.vocab
    logits = rng.normal(S_DRAFT_NOISE, (B, N + 1, V), logit_std)
    idx = torch.tensor([p + 1 for p in parent], device=device)
    tokens = pick_tokens(rng, logits[:, idx, :], w.temperature, S_DRAFT_PICK)
    par = torch.tensor(parent, dtype=torch.int32, device=device).repeat(B, 1).contiguous()
    return par, tokens, logits


def scaled(w: Workload, **shape_overrides) -> Workload:
    """Same workload on a reduced model shape (used for CPU-sized test cases)."""
    return replace(w, shape=replace(w.shape, **shape_overrides))


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------

def make_weights(shape: ModelShape, seed: int, device="cpu", std: float = 0.02) -> Dict[str, object]:
    """All matrices N(0, std^2) in the storage dtype, laid out [out_features, in_features]
    (each output feature's weights contiguous); norm gains are 1.  q|k|v and gate|up are
    concatenated along the output dimension."""
    rng = Rng(seed, device)
    dt = shape.torch_dtype
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    w: Dict[str, object] = {
        "tok_embed": rng.normal(S_WEIGHTS + 0, (V, d), std, dt),
        "final_norm": torch.ones(d, dtype=torch.float32, device=device),
        "lm_head": rng.normal(S_WEIGHTS + 1, (V, d), std, dt),
        "layers": [],
    }
    for l in range(shape.n_layers):
        b = S_WEIGHTS + 16 * (l + 1)
        w["layers"].append({
            "attn_norm": torch.ones(d, dtype=torch.float32, device=device),
            "w_qkv": rng.normal(b + 0, (shape.d_q + 2 * shape.d_kv, d), std, dt),
            "w_o": rng.normal(b + 1, (d, shape.d_q), std, dt),
            "ffn_norm": torch.ones(d, dtype=torch.float32, device=device),
            "w_gate_up": rng.normal(b + 2, (2 * F, d), std, dt),
            "w_down": rng.normal(b + 3, (d, F), std, dt),
        })
    return w


def kv_cache_shape(shape: ModelShape, n_slots: int, max_kv_len: int):
    """[layer][slot][k|v][kv_head][position][head_dim]"""
    return (shape.n_layers, n_slots, 2, shape.n_kv_heads, max_kv_len, shape.head_dim)


def fill_synthetic_kv(cache: torch.Tensor, w: Workload, slot: int, n: int, seq_index: int):
    """Write N(0,1) keys and values (storage dtype) into positions [0, n) of one slot, every layer.
    The stream depends on (sequence, layer) only, so one sequence can be regenerated alone."""
    rng = Rng(w.seed, cache.device)
    L, _, _, H, T, hd = cache.shape
    for l in range(L):
        blk = rng.normal(S_KV + seq_index * 4096 + l, (2, H, n, hd), 1.0, cache.dtype)
        cache[l, slot, :, :, :n, :] = blk


def make_context(w: Workload, device="cpu"):
    """Last emitted token t0 per sequence and (for prefill-built caches) the prompt tokens."""
    rng = Rng(w.seed, device)
    t0 = rng.randint(S_TOKENS + 0, (w.batch,), w.shape.vocab)
    prompts = [rng.randint(S_TOKENS + 1 + b, (w.kv_lens[b],), w.shape.vocab) for b in range(w.batch)]
    return t0, prompts


def make_uniforms(w: Workload, device="cpu") -> torch.Tensor:
    return Rng(w.seed, device).uniform(S_UNIFORMS, (w.batch, w.max_lookahead + 1))


def make_free_drafts(w: Workload, device="cpu", logit_std: float = 1.28):
    """Draft logits that do not depend on the target: N(0, logit_std^2) per entry, and draft
    tokens drawn from softmax(draft_logits / T) with the Gumbel-max trick."""
    rng = Rng(w.seed, device)
    B, K, V = w.batch, w.max_lookahead, w.shape.vocab
    logits = rng.normal(S_DRAFT_NOISE, (B, K, V), logit_std)
    tokens = pick_tokens(rng, logits, w.temperature, S_DRAFT_PICK)
    return tokens, logits


def pick_tokens(rng: Rng, logits: torch.Tensor, temperature: float, stream: int) -> torch.Tensor:
    """One token per row distributed as softmax(logits/T): argmax of logits/T + Gumbel noise."""
    g = rng.gumbel(stream, logits.shape)
    return torch.argmax(logits / temperature + g, dim=-1).to(torch.int32)


def perturbed_drafts(w: Workload, target_logits_rows: List[torch.Tensor], sigma: float, device="cpu"):
    """Draft logits = given per-sequence target logits rows [K_b+1, V] (first K_b used) plus
    N(0, sigma^2); sigma = 0 gives q == p.  Draft *tokens* are NOT drawn here because the
    target rows already depend on them; callers pass the tokens the rows were scored with."""
    rng = Rng(w.seed, device)
    B, K, V = w.batch, w.max_lookahead, w.shape.vocab
    out = torch.zeros((B, K, V), dtype=torch.float32, device=device)
    for b in range(B):
        kb = w.lookahead[b]
        noise = rng.normal(S_DRAFT_NOISE + 64 + b, (kb, V), sigma) if sigma > 0 else 0.0
        out[b, :kb] = target_logits_rows[b][:kb].to(device) + noise
    return out


@dataclass
class StressInputs:
    target_logits: torch.Tensor   # fp32 [B*(K+1), V], rows ordered (sequence, window offset)
    draft_logits: torch.Tensor    # fp32 [B, K, V]
    draft_tokens: torch.Tensor    # int32 [B, K]
    uniforms: torch.Tensor        # fp32 [B, K+1]
    lookahead: tuple
    temperature: float
    vocab: int


def make_stress(batch: int = 64, K: int = 8, vocab: int = 128256, temperature: float = 0.7,
                seed: int = SEED_BASE + 4000, device="cpu", variant: int = 0) -> StressInputs:
    """Sampling-kernel stress inputs: per row a seeded permutation ranks the tokens, the target
    logit is -1.1*ln(rank) + N(0, 0.5^2) and the draft logit is the target's plus N(0, 0.3^2).
    ``variant`` selects an independent copy (benchmarks rotate several)."""
    rng = Rng(seed + 17 * variant, device)
    R = batch * (K + 1)
    tl = torch.empty((R, vocab), dtype=torch.float32, device=device)
    for r in range(R):
        key = rng.uniform(S_STRESS + 0, (vocab,), offset=r * vocab)
        rank = torch.empty(vocab, dtype=torch.float32, device=device)
        rank[torch.argsort(key)] = torch.arange(1, vocab + 1, dtype=torch.float32, device=device)
        tl[r] = -1.1 * torch.log(rank) + rng.normal(S_STRESS + 1, (vocab,), 0.5, offset=r * vocab)
    dl = torch.empty((batch, K, vocab), dtype=torch.float32, device=device)
    tl3 = tl.view(batch, K + 1, vocab)
    for b in range(batch):
        dl[b] = tl3[b, :K] + rng.normal(S_STRESS + 2, (K, vocab), 0.3, offset=b * K * vocab)
    toks = pick_tokens(rng, dl, temperature, S_STRESS + 3)
    u = rng.uniform(S_STRESS + 4, (batch, K + 1))
    return StressInputs(tl, dl, toks, u, (K,) * batch, temperature, vocab)
