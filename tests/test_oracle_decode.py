"""Pins of the oracle's speculative decoding loop (oracle/decode.py) against facts that do not
depend on it: the output law of speculative sampling (the emitted text is distributed as the
target's own sampling, whatever the draft), its degenerate cases, and a from-scratch recomputation
of every logit it used."""
import math

import pytest
import torch

import oracle
from oracle import decode as od
from paper_2411_00853_amd import workload as wl

SMALL = wl.ModelShape(2, 64, 2, 2, 32, 128, 96, dtype="fp32")
SMALL_DRAFT = wl.ModelShape(1, 32, 2, 1, 16, 64, 96, dtype="fp32")
T_MAX = 64


def model(shape, seed, std=0.2):
    return oracle.Model(shape, wl.make_weights(shape, seed, std=std), T_MAX)


def uniforms(seed, shape):
    return wl.Rng(seed).uniform(wl.S_UNIFORMS, shape).tolist()


def fresh_state(target, draft, tokens):
    st = od.SequenceState(list(tokens), target.new_cache(), 0, draft.new_cache() if draft else None, 0)
    st.target_len = od.feed(target, st.target_cache, 0, st.tokens, len(st.tokens) - 1)
    return st


CONTEXT = [5, 17, 3, 88, 41, 2, 60]


def test_draft_equal_to_target_accepts_everything():
    """q == p: u*q(x) < p(x) holds for every u in [0,1), so each round keeps all K proposals, and the
    text is what plain sampling from the target gives when fed the same uniforms in the order used."""
    tgt = model(SMALL, 11)
    same = model(SMALL, 11)
    R, K, T = 4, 3, 0.9
    du, vu = uniforms(1, (R, K)), uniforms(2, (R, K + 1))
    st = fresh_state(tgt, same, CONTEXT)
    trace = od.speculative_decode(tgt, same, st, R, K, T, du, vu)
    assert [t.n_accepted for t in trace] == [K] * R
    flat = []
    for r in range(R):
        flat += du[r] + [vu[r][K]]
    ref = fresh_state(tgt, None, CONTEXT)
    assert od.autoregressive_decode(tgt, ref, R * (K + 1), T, flat) == st.tokens[len(CONTEXT):]


def test_bookkeeping_matches_recomputation_from_scratch():
    """Every logit row a round used equals the one obtained by decoding the whole prefix into an
    empty cache (no reuse, no rollback): stale cache entries or a wrong position would show."""
    tgt, drf = model(SMALL, 21), model(SMALL_DRAFT, 22)
    R, K, T = 6, 4, 1.0
    du, vu = uniforms(3, (R, K)), uniforms(4, (R, K + 1))
    st = fresh_state(tgt, drf, CONTEXT)
    trace = od.speculative_decode(tgt, drf, st, R, K, T, du, vu)
    assert {t.n_accepted for t in trace} - {K} and any(t.n_accepted > 0 for t in trace), "want rejections and accepts"
    seq = list(CONTEXT)
    for t in trace:
        assert t.length_before == len(seq)
        assert len(t.emitted) == t.n_accepted + 1 and t.emitted[:-1] == t.draft_tokens[:t.n_accepted]
        window = [seq[-1]] + t.draft_tokens
        for mdl, rows, n_rows in ((tgt, t.target_logits, K + 1), (drf, t.draft_logits, K)):
            cache = mdl.new_cache(float("nan"))
            od.feed(mdl, cache, 0, seq, len(seq) - 1)
            for i in range(n_rows):
                lg = mdl.decode_one(cache, len(seq) - 1 + i, window[i])
                assert torch.equal(lg, rows[i])
        seq += t.emitted
    assert seq == st.tokens and st.target_len == len(seq) - 1 and st.draft_len <= len(seq) - 1


def test_low_temperature_reproduces_greedy_target_text():
    """T -> 0: both models put all mass on their argmax; speculative sampling must then emit the
    target's greedy continuation whatever the draft proposes."""
    tgt, drf = model(SMALL, 31), model(SMALL_DRAFT, 32)
    R, K, T = 5, 3, 1e-3
    st = fresh_state(tgt, drf, CONTEXT)
    od.speculative_decode(tgt, drf, st, R, K, T, uniforms(5, (R, K)), uniforms(6, (R, K + 1)))
    new = st.tokens[len(CONTEXT):]
    cache = tgt.new_cache()
    seq = list(CONTEXT)
    od.feed(tgt, cache, 0, seq, len(seq) - 1)
    gaps = []
    for _ in new:
        lg = tgt.decode_one(cache, len(seq) - 1, seq[-1])
        top = torch.topk(lg, 2).values
        gaps.append(float(top[0] - top[1]))
        seq.append(int(torch.argmax(lg)))
    assert min(gaps) > 20 * T, "seed gives a near-tie; the limit argument needs a clear argmax"
    assert seq[len(CONTEXT):] == new


def chi_square(counts, probs, n):
    stat, dof, rest_c, rest_p = 0.0, 0, 0.0, 0.0
    for c, p in zip(counts, probs):
        if n * p >= 8:
            stat += (c - n * p) ** 2 / (n * p)
            dof += 1
        else:
            rest_c += c
            rest_p += p
    if n * rest_p >= 8:
        stat += (rest_c - n * rest_p) ** 2 / (n * rest_p)
        dof += 1
    return stat, dof - 1


def test_first_two_emitted_tokens_follow_the_target_law():
    """The theorem behind the method: the text has the target's distribution.  Monte Carlo over the
    uniforms: the first emitted token ~ p(.|context), and given it, the second ~ p(.|context, first)."""
    tgt, drf = model(SMALL, 41, std=0.12), model(SMALL_DRAFT, 42, std=0.12)
    K, T, N = 2, 1.0, 6000
    V = SMALL.vocab
    base = fresh_state(tgt, drf, CONTEXT)
    p1 = oracle.softmax(tgt.decode_one(base.target_cache.clone(), len(CONTEXT) - 1, CONTEXT[-1]), T).tolist()
    q1 = oracle.softmax(drf.decode_one(od_fed_draft(drf, CONTEXT), len(CONTEXT) - 1, CONTEXT[-1]), T).tolist()
    du = wl.Rng(7).uniform(wl.S_UNIFORMS + 1, (N, K)).tolist()
    vu = wl.Rng(8).uniform(wl.S_UNIFORMS + 2, (N, K + 1)).tolist()
    du2 = wl.Rng(7).uniform(wl.S_UNIFORMS + 3, (N, K)).tolist()      # a second round, when needed, draws afresh
    vu2 = wl.Rng(8).uniform(wl.S_UNIFORMS + 4, (N, K + 1)).tolist()
    first = [0] * V
    pairs = {}
    n_acc = 0
    for i in range(N):
        st = od.SequenceState(list(CONTEXT), base.target_cache.clone(), base.target_len, drf.new_cache(), 0)
        tr = od.speculative_round(tgt, drf, st, K, T, du[i], vu[i])
        # the second token comes from this round only if the first proposal was kept
        if len(st.tokens) < len(CONTEXT) + 2:
            tr2 = od.speculative_round(tgt, drf, st, K, T, du2[i], vu2[i])
            assert tr2.length_before == len(CONTEXT) + 1
        a, b = st.tokens[len(CONTEXT)], st.tokens[len(CONTEXT) + 1]
        first[a] += 1
        pairs.setdefault(a, [0] * V)[b] += 1
        n_acc += tr.n_accepted
    assert 0.2 < n_acc / (N * K) < 0.8, "both outcomes must be common for the test to bite"
    stat, dof = chi_square(first, p1, N)
    assert stat < dof + 5 * math.sqrt(2 * dof), (stat, dof)
    stat_q, dof_q = chi_square(first, q1, N)
    assert stat_q > dof_q + 20 * math.sqrt(2 * dof_q), "the statistic cannot tell p from q: test too weak"
    # conditional law of the second token for the most frequent first token
    a = max(range(V), key=lambda t: first[t])
    cache = tgt.new_cache()
    seq = CONTEXT + [a]
    od.feed(tgt, cache, 0, seq, len(seq) - 1)
    p2 = oracle.softmax(tgt.decode_one(cache, len(seq) - 1, a), T).tolist()
    stat2, dof2 = chi_square(pairs[a], p2, first[a])
    assert first[a] > 300 and stat2 < dof2 + 5 * math.sqrt(2 * dof2), (first[a], stat2, dof2)


def od_fed_draft(drf, tokens):
    cache = drf.new_cache()
    od.feed(drf, cache, 0, tokens, len(tokens) - 1)
    return cache


def test_draw_is_inverse_cdf_of_softmax():
    """draw() against the definition written out with torch in fp64."""
    lg = wl.Rng(9).normal(wl.S_TOKENS, (50,), 1.5, torch.float32)
    p = torch.softmax(lg.double() / 0.7, 0)
    cdf = torch.cumsum(p, 0)
    for u in (0.0, 0.013, 0.37, 0.5, 0.99, 0.999999):
        want = int(torch.searchsorted(cdf, torch.tensor(u * float(cdf[-1]), dtype=torch.float64), right=True))
        got, _ = od.draw(lg, 0.7, u)
        assert got == min(want, 49)


def test_autoregressive_decode_feeds_positions_in_order():
    tgt = model(SMALL, 51)
    st = fresh_state(tgt, None, CONTEXT)
    us = uniforms(10, (5,))
    new = od.autoregressive_decode(tgt, st, 5, 0.8, us)
    seq = list(CONTEXT)
    for i, y in enumerate(new):
        cache = tgt.new_cache()
        od.feed(tgt, cache, 0, seq, len(seq) - 1)
        lg = tgt.decode_one(cache, len(seq) - 1, seq[-1])
        assert od.draw(lg, 0.8, us[i])[0] == y
        seq.append(y)


def test_temperature_zero_rounds_emit_the_targets_greedy_text_exactly():
    """Greedy speculative decoding: whatever the draft proposes, the text is the target's greedy
    continuation, token for token; a draft equal to the target has every proposal kept."""
    tgt, drf = model(SMALL, 61), model(SMALL_DRAFT, 62)
    R, K = 6, 4
    zeros_d, zeros_v = [[0.0] * K] * R, [[0.0] * (K + 1)] * R
    st = fresh_state(tgt, drf, CONTEXT)
    trace = od.speculative_decode(tgt, drf, st, R, K, 0.0, zeros_d, zeros_v)
    new = st.tokens[len(CONTEXT):]
    cache = tgt.new_cache()
    seq = list(CONTEXT)
    od.feed(tgt, cache, 0, seq, len(seq) - 1)
    for _ in range(max(len(new), 3 * (K + 1))):
        seq.append(int(torch.argmax(tgt.decode_one(cache, len(seq) - 1, seq[-1]))))
    assert seq[len(CONTEXT):len(CONTEXT) + len(new)] == new and len(new) == sum(t.n_accepted + 1 for t in trace)
    same = model(SMALL, 61)
    st2 = fresh_state(tgt, same, CONTEXT)
    trace2 = od.speculative_decode(tgt, same, st2, 3, K, 0.0, zeros_d, zeros_v)
    assert [t.n_accepted for t in trace2] == [K] * 3 and st2.tokens == seq[:len(CONTEXT) + 3 * (K + 1)]
