"""Pins of the CPU oracle's rejection sampler (no GPU).

The paper states the procedure in prose (section "Speculative Sampling Results"): compare
target and draft probabilities, keep a prefix of the drafts, resample the first rejected
token from a combination of the two distributions, and sample one extra token from the target
when every draft is kept -- all "without compromising the sample quality".  The tests below
check the oracle against what that fixes: exactness of the output distribution by brute-force
enumeration on tiny vocabularies, closed forms for the acceptance probability and residual
mass, library routines on the special cases, and the structural invariants.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from paper_2411_00853_amd import workload as wl


def logits_of(probs):
    """fp32 logits whose softmax is the given probability vector (zeros become -inf)."""
    p = np.asarray([float(x) for x in probs], dtype=np.float64)
    with np.errstate(divide="ignore"):
        return torch.tensor(np.log(p), dtype=torch.float32)


def mid(i, n):
    return (i + 0.5) / n


# ------------------------------------------------------------------ library special cases

@pytest.mark.parametrize("T", [1.0, 0.7, 2.5])
def test_softmax_with_temperature_matches_library(T):
    g = torch.Generator().manual_seed(0)
    l = torch.randn(1000, generator=g) * 4 + 30.0
    p = oracle.softmax(l, T).numpy()
    want = scipy.special.softmax(l.double().numpy() / np.float64(np.float32(T)))
    assert np.abs(p - want).max() < 1e-15 and abs(p.sum() - 1) < 1e-12


def test_inverse_cdf_matches_searchsorted():
    g = np.random.default_rng(1)
    r = g.random(500)
    r[g.random(500) < 0.3] = 0.0
    c = np.cumsum(r)
    rt = torch.tensor(r)
    for t in np.concatenate([g.random(200) * c[-1], [0.0, c[3], c[-1] * (1 - 1e-16)]]):
        y, lo, hi = oracle.inverse_cdf(rt, float(t))
        want = int(np.searchsorted(c, t, side="right"))     # first index with cumsum > t
        assert y == want and r[y] > 0 and lo <= t < hi
    # target at or beyond the total (rounding): last id with positive mass
    r[-3:] = 0.0
    y, _, _ = oracle.inverse_cdf(torch.tensor(r), float(np.cumsum(r)[-1]) + 1.0)
    assert y == int(np.nonzero(r)[0][-1])


def test_zero_lookahead_is_textbook_inverse_cdf_sampling():
    g = torch.Generator().manual_seed(2)
    l = torch.randn(1, 300, generator=g) * 2
    for T in (1.0, 0.5):
        c = np.cumsum(scipy.special.softmax(l[0].double().numpy() / T))
        for u in (0.0, 0.123, 0.5, 0.9999):
            a, out, d = oracle.sample(l, torch.zeros(0, 300), [], [u], T)
            assert a == 0 and out == [int(np.searchsorted(c, u * c[-1], side="right"))]
            assert d.final_row == 0 and not d.final_is_residual


def test_identical_distributions_accept_everything():
    g = torch.Generator().manual_seed(3)
    K, V = 6, 500
    tl = torch.randn(K + 1, V, generator=g) * 3
    toks = torch.randint(0, V, (K,), generator=g).tolist()
    for us in ([0.0] * (K + 1), [math.nextafter(1.0, 0.0)] * K + [0.42], torch.rand(K + 1, generator=g).tolist()):
        us = [float(np.float32(u)) if u < 0.99999997 else float(np.nextafter(np.float32(1), np.float32(0))) for u in us]
        a, out, d = oracle.sample(tl, tl[:K].clone(), toks, us, 0.9)
        assert a == K and out[:K] == toks and d.final_row == K and not d.final_is_residual
        c = np.cumsum(scipy.special.softmax(tl[K].double().numpy() / np.float64(np.float32(0.9))))
        assert out[K] == int(np.searchsorted(c, us[K] * c[-1], side="right"))


# ------------------------------------------------------------------ distribution exactness, brute force

CASES_K1 = [
    # (p numerators, q numerators) over 64; q numerators divide 64*k, residual mass s/64 with s | N
    ([32, 16, 8, 8], [16, 16, 16, 16]),      # s = 16
    ([8, 8, 16, 32], [32, 16, 8, 8]),        # s = 32
    ([0, 32, 32], [16, 16, 32]),             # a zero-probability target token; s = 16
    ([16, 16, 16, 16, 0, 0], [8, 8, 8, 8, 16, 16]),  # s = 32
    ([64, 0, 0], [16, 16, 32]),              # one-hot target; s = 48
]


@pytest.mark.parametrize("pn,qn", CASES_K1)
def test_first_emitted_token_is_distributed_as_target_K1(pn, qn):
    """Enumerate the draft token (weight q(x)) and sweep both uniforms over the midpoints of an
    N x N grid.  Every accept threshold p/q and every CDF edge is a multiple of 1/N, so the
    counts are exact: P(first emitted token = v) must equal p(v) as a rational number."""
    N = 192
    V = len(pn)
    p = [Fraction(a, 64) for a in pn]
    q = [Fraction(a, 64) for a in qn]
    s = sum(max(Fraction(0), a - b) for a, b in zip(p, q))
    assert (s * N).denominator == 1 and all((Fraction(N) * a / b).denominator == 1 for a, b in zip(p, q) if b)
    tl = torch.stack([logits_of(p), logits_of([Fraction(1, V)] * V)])   # row 1 (bonus) irrelevant to token 1
    dl = logits_of(q)[None]
    prob = [Fraction(0)] * V
    accepted_mass = Fraction(0)
    for x in range(V):
        if q[x] == 0:
            continue
        for ia in range(N):
            a0, out0, _ = oracle.sample(tl, dl, [x], [mid(ia, N), 0.5], 1.0)
            if a0 == 1:                      # accepted: first token is x for every final uniform
                assert out0[0] == x
                prob[x] += q[x] * Fraction(1, N)
                accepted_mass += q[x] * Fraction(1, N)
                continue
            for jf in range(N):
                a, out, d = oracle.sample(tl, dl, [x], [mid(ia, N), mid(jf, N)], 1.0)
                assert a == 0 and out[1] == -1 and d.final_is_residual
                assert p[out[0]] > q[out[0]]          # resampled tokens come from where p exceeds q
                prob[out[0]] += q[x] * Fraction(1, N * N)
    assert prob == p
    # acceptance probability = sum_v min(p, q) = 1 - TV(p, q); residual mass = 1 - that
    assert accepted_mass == sum(min(a, b) for a, b in zip(p, q)) == 1 - s


def test_two_step_joint_distribution_is_exact_K2():
    """K = 2 over a 3-token vocabulary with context-dependent rows.  Checks, exactly:
    P(first = v) = p0(v);  P(x1 kept and second emitted = v) = min(p0,q0)(x1) * p1(v | x1);
    P(both kept and bonus = v) = min(p0,q0)(x1) * min(p1,q1)(x2 | x1) * p2(v | x1, x2)."""
    N = 24
    V = 3
    F8 = lambda *a: [Fraction(x, 8) for x in a]
    p0, q0 = F8(4, 2, 2), F8(2, 4, 2)
    p1 = {0: F8(2, 2, 4), 1: F8(4, 4, 0), 2: F8(1, 1, 6)}
    q1 = {0: F8(4, 2, 2), 1: F8(2, 2, 4), 2: F8(2, 2, 4)}
    p2 = {(a, b): F8(*[(1 + a + b) % 3 + 1, 5 - (a + b) % 3 - ((1 + a + b) % 3), 2 + (a + b) % 3])
          for a in range(V) for b in range(V)}
    for v in p2.values():
        assert sum(v) == 1 and min(v) >= 0
    first = [Fraction(0)] * V
    second = {c: [Fraction(0)] * V for c in range(V)}
    bonus = {k: [Fraction(0)] * V for k in p2}
    w3 = Fraction(1, N ** 3)
    for x1 in range(V):
        for x2 in range(V):
            wx = q0[x1] * q1[x1][x2]
            if wx == 0:
                continue
            tl = torch.stack([logits_of(p0), logits_of(p1[x1]), logits_of(p2[(x1, x2)])])
            dl = torch.stack([logits_of(q0), logits_of(q1[x1])])
            for i in range(N):
                for j in range(N):
                    for k in range(N):
                        a, out, _ = oracle.sample(tl, dl, [x1, x2], [mid(i, N), mid(j, N), mid(k, N)], 1.0)
                        assert out[a + 1:] == [-1] * (2 - a) and out[:a] == [x1, x2][:a]
                        first[out[0]] += wx * w3
                        if a >= 1:
                            second[x1][out[1]] += wx * w3
                        if a == 2:
                            bonus[(x1, x2)][out[2]] += wx * w3
    assert first == p0
    for c in range(V):
        keep = min(p0[c], q0[c])
        assert second[c] == [keep * t for t in p1[c]]
        for b in range(V):
            keep2 = keep * min(p1[c][b], q1[c][b])
            assert bonus[(c, b)] == [keep2 * t for t in p2[(c, b)]]


# ------------------------------------------------------------------ closed forms and invariants

def _random_case(g, K, V, T, noise=0.5):
    tl = torch.randn(K + 1, V, generator=g) * 2
    dl = tl[:K] + torch.randn(K, V, generator=g) * noise
    toks = torch.randint(0, V, (K,), generator=g).tolist()
    us = torch.rand(K + 1, generator=g).tolist()
    return tl, dl.contiguous(), toks, us


def test_accept_ratio_and_residual_mass_closed_forms():
    g = torch.Generator().manual_seed(5)
    for _ in range(20):
        K, V, T = 4, 200, 0.8
        tl, dl, toks, us = _random_case(g, K, V, T)
        a, out, d = oracle.sample(tl, dl, toks, us, T)
        Tn = np.float64(np.float32(T))
        for i in range(min(a + 1, K)):
            p = scipy.special.softmax(tl[i].double().numpy() / Tn)
            q = scipy.special.softmax(dl[i].double().numpy() / Tn)
            assert d.accept_ratio[i] == pytest.approx(min(1.0, p[toks[i]] / q[toks[i]]), rel=1e-12)
            assert (np.float64(np.float32(us[i])) < d.accept_ratio[i]) == (i < a)
        if a < K:
            assert d.final_is_residual and d.final_row == a
            assert d.final_S == pytest.approx(1.0 - np.minimum(p, q).sum(), rel=1e-9)   # 1 - sum min(p,q) = TV
            assert d.final_S == pytest.approx(0.5 * np.abs(p - q).sum(), rel=1e-9)
            assert p[out[a]] > q[out[a]]
        else:
            assert d.final_S == pytest.approx(1.0, rel=1e-12)
        assert d.final_cdf_lo <= d.final_target < d.final_cdf_hi
        assert out[:a] == toks[:a] and all(t == -1 for t in out[a + 1:]) and 0 <= out[a] < V


def test_acceptance_rate_over_many_uniforms_matches_one_minus_tv():
    g = torch.Generator().manual_seed(6)
    V, T = 50, 1.0
    tl = torch.randn(2, V, generator=g)
    dl = (tl[:1] + torch.randn(1, V, generator=g)).contiguous()
    p = scipy.special.softmax(tl[0].double().numpy())
    q = scipy.special.softmax(dl[0].double().numpy())
    N = 400
    acc = 0.0
    for x in range(V):
        kept = sum(oracle.sample(tl, dl, [x], [mid(i, N), 0.5], T)[0] for i in range(N))
        acc += q[x] * kept / N
    assert acc == pytest.approx(np.minimum(p, q).sum(), abs=1.0 / N)


def test_one_hot_limits():
    V = 5
    hot = lambda i: logits_of([1.0 if j == i else 0.0 for j in range(V)])
    flat = logits_of([0.2] * V)
    # target certain of the drafted token: kept whatever the uniform
    a, out, _ = oracle.sample(torch.stack([hot(2), flat]), flat[None], [2], [0.999999, 0.3], 1.0)
    assert a == 1 and out[0] == 2
    # draft certain of a token the target gives zero mass: rejected even at u = 0, resampled from p
    p = logits_of([0.5, 0.5, 0.0, 0.0, 0.0])
    a, out, d = oracle.sample(torch.stack([p, flat]), hot(2)[None], [2], [0.0, 0.75], 1.0)
    assert a == 0 and out[0] == 1 and d.final_S == pytest.approx(1.0)
    # drafted token has zero draft mass but positive target mass: kept (ratio is infinite)
    a, out, _ = oracle.sample(torch.stack([flat, flat]), hot(1)[None], [3], [0.999, 0.1], 1.0)
    assert a == 1


def test_monotone_in_the_uniforms_and_prefix_property():
    g = torch.Generator().manual_seed(7)
    K, V, T = 5, 64, 1.3
    tl, dl, toks, us = _random_case(g, K, V, T, noise=1.0)
    grid = [mid(i, 40) for i in range(40)]
    for pos in range(K):
        prev = K + 1
        for u in grid:
            uu = list(us)
            uu[pos] = u
            a, out, _ = oracle.sample(tl, dl, toks, uu, T)
            assert a <= prev
            prev = a
            assert out[:a] == toks[:a] and sum(t >= 0 for t in out) == a + 1
    prev = -1
    a0 = oracle.sample(tl, dl, toks, us, T)[0]
    for u in grid:
        uu = list(us)
        uu[K] = u
        a, out, _ = oracle.sample(tl, dl, toks, uu, T)
        assert a == a0 and out[a] >= prev      # final uniform never changes the kept prefix
        prev = out[a]


def test_uniform_index_convention_ragged():
    # sequence with lookahead K uses uniforms[0..K-1] for the tests and uniforms[K] for the final draw
    g = torch.Generator().manual_seed(8)
    tl, dl, toks, _ = _random_case(g, 3, 40, 1.0)
    base = [0.0, 0.0, 0.0, 0.37, 0.99, 0.99]     # u = 0 keeps every draft with p(x) > 0
    a, out, _ = oracle.sample(tl, dl, toks, base, 1.0)
    c = np.cumsum(scipy.special.softmax(tl[3].double().numpy()))
    assert a == 3 and out[3] == int(np.searchsorted(c, np.float64(np.float32(0.37)) * c[-1], side="right"))


def test_bad_arguments_are_rejected():
    l = torch.zeros(2, 4)
    with pytest.raises(ValueError):
        oracle.sample(l, l[:1].clone(), [4], [0.1, 0.1], 1.0)     # token id out of range
    with pytest.raises(ValueError):
        oracle.sample(l, l[:1].clone(), [0], [0.1, 0.1], 0.0)     # temperature must be positive


def test_greedy_rule_is_the_zero_temperature_limit_and_plain_argmax():
    """oracle_greedy against (a) torch.argmax row by row and (b) oracle_sample at a temperature so low
    that all mass sits on the argmax (whatever the draft distribution and the uniforms are)."""
    rng = wl.Rng(77)
    V, K = 200, 5
    hits = set()
    for case in range(60):
        tl = rng.normal(500 + case, (K + 1, V), 2.0)
        best = torch.argmax(tl, dim=1).tolist()
        toks = list(best[:K])
        cut = case % (K + 2)                      # first mismatching position (K+1: none)
        if cut < K:
            toks[cut] = (toks[cut] + 1 + case) % V
            if toks[cut] == best[cut]:
                toks[cut] = (toks[cut] + 1) % V
        a, out, gap = oracle.greedy(tl, toks)
        want_a = min(cut, K)
        assert a == want_a and out[:a] == best[:a] and out[a] == best[a] and out[a + 1:] == [-1] * (K - a)
        hits.add(a)
        # the limit of the stochastic rule: a draft that proposes its own most likely token (q(x) -> 1),
        # so that u q(x) < p(x) holds iff p(x) -> 1, i.e. iff x is the target's most likely token too
        dl = rng.normal(900 + case, (K, V), 2.0)
        for i in range(K):
            dl[i, toks[i]] = dl[i].max() + 1.0
        us = [max(u, 1e-3) for u in rng.uniform(1300 + case, (K + 1,)).tolist()]
        assert gap > 1e-3
        T = min(gap, 1.0) / 60.0                  # every runner-up has relative mass <= e^-60
        a2, out2, _ = oracle.sample(tl, dl, toks, us, T)
        assert (a2, out2) == (a, out)
    assert hits == set(range(K + 1))
    ties = torch.zeros((1, 7))
    ties[0, 3] = ties[0, 5] = 2.0
    assert oracle.greedy(ties, [])[1] == [3]      # lowest id among equal maxima
