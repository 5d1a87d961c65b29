"""The speculative decoding loop, spelled out on top of the oracle's primitives.  TEST INFRASTRUCTURE ONLY.

Section "Speculative Sampling Results" of the paper describes one round: a small draft model
decodes several tokens in the ordinary autoregressive way; the target model then scores all of
them in one pass; the two models' probabilities of each proposed token are compared and a prefix
of the proposals is kept; the first rejected position is resampled from a combination of the two
distributions, and if nothing was rejected one more token is drawn from the target.  Repeating the
round generates text from the target's distribution in fewer target passes.

Everything below is plain Python around `oracle.Model.decode_one`, `oracle.Model.verify_sequential`
and `oracle.sample`: one token at a time, one sequence at a time, caches passed explicitly.  Random
numbers are inputs (one uniform per draft draw, K+1 per verification).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import torch

from . import Model, SampleDiag, greedy, sample


def draw(logits: torch.Tensor, temperature: float, u: float):
    """One token from softmax(logits / T) by inverse CDF in ascending token id (the K = 0 case of
    `oracle.sample`: a single draw from the row's distribution); at temperature 0 the most likely
    token (the K = 0 case of `oracle.greedy`).  Returns (token, diagnostics)."""
    if temperature == 0:
        _, out, gap = greedy(logits.reshape(1, -1), [])
        return int(out[0]), gap
    _, out, diag = sample(logits.reshape(1, -1), torch.zeros((0, logits.numel())), [], [u], temperature)
    return int(out[0]), diag


@dataclass
class SequenceState:
    """One sequence being generated: its tokens and, per model, a cache plus the number of leading
    positions of it that hold keys/values of `tokens` (entries beyond are stale)."""
    tokens: List[int]
    target_cache: torch.Tensor
    target_len: int
    draft_cache: torch.Tensor = None
    draft_len: int = 0


@dataclass
class RoundTrace:
    length_before: int                     # len(tokens) when the round started
    draft_tokens: List[int]
    draft_logits: torch.Tensor             # [K, V]
    draft_diags: List[SampleDiag]
    target_logits: torch.Tensor            # [K+1, V]
    n_accepted: int
    emitted: List[int]                     # n_accepted kept proposals + the final token
    diag: SampleDiag = None


def feed(model: Model, cache: torch.Tensor, have: int, tokens: Sequence[int], upto: int) -> int:
    """Decode tokens[have:upto] into the cache one by one (logits discarded); returns upto."""
    for pos in range(have, upto):
        model.decode_one(cache, pos, int(tokens[pos]))
    return max(have, upto)


def speculative_round(target: Model, draft: Model, st: SequenceState, K: int, temperature: float,
                      draft_uniforms: Sequence[float], verify_uniforms: Sequence[float]) -> RoundTrace:
    L = len(st.tokens)
    assert st.target_len == L - 1, "the target cache holds every token but the last"
    # the draft first reads whatever part of the sequence it has not seen (all but the last token)...
    st.draft_len = feed(draft, st.draft_cache, st.draft_len, st.tokens, L - 1)
    # ...then decodes K tokens autoregressively, starting from the last token of the sequence
    cur = st.tokens[-1]
    proposals, q_logits, q_diags = [], [], []
    for i in range(K):
        lg = draft.decode_one(st.draft_cache, L - 1 + i, cur)
        x, dg = draw(lg, temperature, float(draft_uniforms[i]))
        proposals.append(x)
        q_logits.append(lg)
        q_diags.append(dg)
        cur = x
    st.draft_len = L - 1 + K
    # the target scores the last token and the K proposals; row i is its distribution after
    # proposals[:i], i.e. the one proposal i is tested against, row K the extra token's
    p_logits = target.verify_sequential(st.target_cache, L - 1, [st.tokens[-1]] + proposals)
    ql = torch.stack(q_logits) if K else torch.zeros((0, p_logits.shape[1]))
    if temperature == 0:
        a, out, diag = greedy(p_logits, proposals)      # diag: the smallest deciding logit gap
    else:
        a, out, diag = sample(p_logits, ql, proposals, list(verify_uniforms[:K + 1]), temperature)
    emitted = [int(t) for t in out[:a + 1]]
    st.tokens.extend(emitted)
    # caches: the target appended the whole window, of which last token + a proposals remain valid;
    # the draft processed last token + proposals[:K-1]
    st.target_len = L + a
    st.draft_len = min(st.draft_len, L + a)
    return RoundTrace(L, proposals, ql, q_diags, p_logits, a, emitted, diag)


def speculative_decode(target: Model, draft: Model, st: SequenceState, rounds: int, K: int, temperature: float,
                       draft_uniforms, verify_uniforms) -> List[RoundTrace]:
    """`rounds` rounds on one sequence.  draft_uniforms[r][i], verify_uniforms[r][i]."""
    return [speculative_round(target, draft, st, K, temperature, draft_uniforms[r], verify_uniforms[r])
            for r in range(rounds)]


def autoregressive_decode(model: Model, st: SequenceState, n_new: int, temperature: float,
                          uniforms: Sequence[float]) -> List[int]:
    """Plain sampling from the target: the loop speculative decoding is meant to speed up."""
    new = []
    for i in range(n_new):
        L = len(st.tokens)
        assert st.target_len == L - 1
        lg = model.decode_one(st.target_cache, L - 1, st.tokens[-1])
        y, _ = draw(lg, temperature, float(uniforms[i]))
        st.tokens.append(y)
        st.target_len = L
        new.append(y)
    return new


# ---- choosing the lookahead ------------------------------------------------------------------------
# The paper motivates sampling schemes that adapt to the data; it does not give one.  The rule below
# is this project's reading (stated in full in include/spec_decode.h): per-sequence acceptance
# estimates with exponential forgetting, and the K with the best predicted tokens per millisecond.

class LookaheadRule:
    def __init__(self, batch, draft_ms, verify_ms, verify_ms_per_token, k_min, k_max, forget=0.9,
                 prior_accept=0.5, prior_weight=4.0):
        self.c = (draft_ms, verify_ms, verify_ms_per_token)
        self.k_min, self.k_max = k_min, k_max
        self.forget, self.prior_accept, self.prior_weight = forget, prior_accept, prior_weight
        self.tested = [0.0] * batch
        self.kept = [0.0] * batch

    def accept(self, b):
        return (self.kept[b] + self.prior_accept * self.prior_weight) / (self.tested[b] + self.prior_weight)

    def update(self, n_accepted, K):
        for b, a in enumerate(n_accepted):
            if a < 0:
                continue
            self.tested[b] = self.forget * self.tested[b] + float(min(a + 1, K))
            self.kept[b] = self.forget * self.kept[b] + float(a)

    def expected_tokens(self, K):
        total = 0.0
        for b in range(len(self.tested)):
            al = self.accept(b)
            total += (1.0 - al ** (K + 1)) / (1.0 - al) if al < 1.0 else float(K + 1)
        return total

    def next(self):
        d, v, vt = self.c
        best, best_k = -1.0, self.k_min
        for K in range(self.k_min, self.k_max + 1):
            rate = self.expected_tokens(K) / (K * d + v + K * vt)
            if rate > best:
                best, best_k = rate, K
        return best_k

    def next_per_seq(self):
        """The batch's K and every sequence's own window (at least 1): proposal k is put to the target
        while alpha_b^k >= rate * verify_ms_per_token / batch (rate = predicted tokens per ms at that K)."""
        d, v, vt = self.c
        K = self.next()
        rate = self.expected_tokens(K) / (K * d + v + K * vt)
        worth = rate * vt / len(self.tested)
        out = []
        for b in range(len(self.tested)):
            al, reach, kb = self.accept(b), 1.0, 1          # one proposal is always tested
            for k in range(1, K + 1):
                reach *= al
                if reach >= worth:
                    kb = k
                else:
                    break
            out.append(kb)
        return K, out

    def update_per_seq(self, n_accepted, K_per_seq):
        for b, (a, K) in enumerate(zip(n_accepted, K_per_seq)):
            if a < 0:
                continue
            self.tested[b] = self.forget * self.tested[b] + float(min(a + 1, K))
            self.kept[b] = self.forget * self.kept[b] + float(a)
