"""Pins of the oracle's tree verification (oracle_tree_sample, oracle.tree_logits): the chain case
must be the linear sampler, the emitted tokens must follow the target's law whatever the draft
(Monte Carlo on a toy Markov pair of models), and special cases with closed forms."""
import math

import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl


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


def test_chain_tree_is_the_linear_sampler():
    rng = wl.Rng(3)
    V, K = 40, 5
    seen = set()
    for case in range(200):
        tl = rng.normal(1000 + case, (K + 1, V), 1.0)
        dl = tl + rng.normal(2000 + case, (K + 1, V), 0.7)
        toks = wl.pick_tokens(rng, dl[None, :K], 1.0, 3000 + case)[0].tolist()
        us = rng.uniform(4000 + case, (K + 1,)).tolist()
        a, out, d = oracle.sample(tl, dl[:K].contiguous(), toks, us, 0.9)
        ta, path, tout, td = oracle.tree_sample(list(range(-1, K - 1)), toks, tl, dl, us, 0.9)
        assert (ta, tout) == (a, out) and path == list(range(a))
        assert td.final_target == d.final_target and td.final_cdf_hi == d.final_cdf_hi
        seen.add(a)
    assert len(seen) >= 4


def test_no_nodes_is_one_draw_from_the_root_row():
    rng = wl.Rng(4)
    tl = rng.normal(1, (1, 30), 1.5)
    for u in (0.0, 0.3, 0.77, 0.9999):
        a, path, out, _ = oracle.tree_sample([], [], tl, torch.zeros((1, 30)), [u], 0.8)
        _, want, _ = oracle.sample(tl, torch.zeros((0, 30)), [], [u], 0.8)
        assert a == 0 and path == [] and out == want


def test_second_rejection_uses_the_renormalised_residual():
    """Root with three children, all rejected: the final token comes from r3 with
    r1 = norm(max(0,p-q)), r2 = norm(max(0,r1-q)), r3 = norm(max(0,r2-q)) -- every rejection is one
    update, also that of a repeated child token, which has r(x) = 0 after its first rejection and
    can never be kept (not even with u ~ 0)."""
    rng = wl.Rng(5)
    V, T = 24, 1.0
    tl = rng.normal(1, (4, V), 1.0)
    dl = rng.normal(2, (4, V), 1.0)
    p = torch.softmax(tl[0].double() / T, 0)
    q = torch.softmax(dl[0].double() / T, 0)
    order = torch.argsort(q / p, descending=True).tolist()     # tokens the draft over-weights most
    x0, x1 = order[0], order[1]
    assert q[x0] > p[x0] and q[x1] > p[x1]
    toks = [x0, x0, x1]                                         # the second child repeats the first
    r = p.clone()
    for _ in range(3):
        r = torch.clamp(r - q, min=0)
        r = r / r.sum()
    cdf = torch.cumsum(r, 0)
    for u in (0.05, 0.4, 0.93):
        a, path, out, d = oracle.tree_sample([-1, -1, -1], toks, tl, dl, [0.999999, 1e-9, 0.999999, u], T)
        assert a == 0 and d.final_level == 3 and d.final_node == -1
        want = int(torch.searchsorted(cdf, torch.tensor(u, dtype=torch.float64), right=True))
        assert out[0] == want and out[1:] == [-1, -1, -1]


def test_emitted_tokens_follow_the_target_law():
    """Toy pair of Markov models over 12 tokens: p(.|t), q(.|t) from fixed logit tables.  Trees: 3
    children of the root and 2 children of each of them, all drawn independently from q at their
    parent.  First emitted token ~ p(.|root); given a first token t1 that was a kept child, the
    second ~ p(.|t1)."""
    V, T, N = 12, 1.0, 30000
    g = torch.Generator().manual_seed(11)
    lp = torch.randn((V, V), generator=g) * 1.2
    lq = lp * 0.5 + torch.randn((V, V), generator=g) * 0.9
    root_tok = 7
    P = torch.softmax(lp.double() / T, 1)
    Q = torch.softmax(lq.double() / T, 1)
    first = [0] * V
    second = {}
    kept = 0
    parent = [-1, -1, -1, 0, 0, 1, 1, 2, 2]
    u_all = torch.rand((N, len(parent) + 1), generator=g)
    for i in range(N):
        kids = torch.multinomial(Q[root_tok], 3, replacement=True, generator=g).tolist()
        toks = list(kids)
        for k in kids:
            toks += torch.multinomial(Q[k], 2, replacement=True, generator=g).tolist()
        ctx = [root_tok] + toks                                   # row j belongs to the node with token ctx[j]
        tl = lp[ctx].float().contiguous()
        dl = lq[ctx].float().contiguous()
        a, path, out, _ = oracle.tree_sample(parent, toks, tl, dl, u_all[i].tolist(), T)
        first[out[0]] += 1
        kept += a
        if a >= 1:
            second.setdefault(out[0], [0] * V)[out[1]] += 1
    assert 0.3 < kept / N < 1.7
    stat, dof = chi_square(first, P[root_tok].tolist(), N)
    assert stat < dof + 5 * math.sqrt(2 * dof), (stat, dof)
    stat_q, dof_q = chi_square(first, Q[root_tok].tolist(), N)
    assert stat_q > dof_q + 20 * math.sqrt(2 * dof_q), "cannot tell p from q: test too weak"
    t1 = max(second, key=lambda t: sum(second[t]))
    n2 = sum(second[t1])
    stat2, dof2 = chi_square(second[t1], P[t1].tolist(), n2)
    assert n2 > 1500 and stat2 < dof2 + 5 * math.sqrt(2 * dof2), (n2, stat2, dof2)
    stat2q, dof2q = chi_square(second[t1], Q[t1].tolist(), n2)
    assert stat2q > dof2q + 10 * math.sqrt(2 * dof2q)


def test_tree_logits_rows_depend_on_their_own_path_only():
    shape = wl.ModelShape(2, 64, 2, 2, 32, 128, 96, dtype="fp32")
    m = oracle.Model(shape, wl.make_weights(shape, 9, std=0.2), 48)
    ctx = [3, 9, 27, 81, 5]
    cache = m.new_cache()
    for i, t in enumerate(ctx[:-1]):
        m.decode_one(cache, i, t)
    parent = [-1, -1, 0, 0, 1, 3]
    toks = [11, 12, 13, 14, 15, 16]
    rows = oracle.tree_logits(m, cache, len(ctx) - 1, ctx[-1], parent, toks)
    # node 5 sits on the path 0 -> 3 -> 5: the same row comes out of a chain holding only that path
    chain = m.verify_sequential(cache, len(ctx) - 1, [ctx[-1], toks[0], toks[3], toks[5]])
    assert torch.equal(rows[0], chain[0]) and torch.equal(rows[1], chain[1])
    assert torch.equal(rows[4], chain[2]) and torch.equal(rows[6], chain[3])
    # siblings see the same prefix: rows of nodes 2 and 3 differ only through their own token
    assert not torch.equal(rows[3], rows[4])


def test_greedy_tree_walk_follows_the_argmax_path_and_is_the_cold_limit():
    """oracle_tree_greedy: (a) a chain is oracle_greedy; (b) on a tree the kept path is the unique
    root-down path whose tokens are the row-wise argmaxes, found with plain torch; (c) it is what
    oracle_tree_sample gives at a temperature so low that all mass sits on the argmax, for a draft
    that proposes its own most likely token."""
    rng = wl.Rng(31)
    V, N = 50, 9
    parent = [-1, -1, -1, 0, 0, 1, 3, 3, 4]
    depths = set()
    for case in range(80):
        tl = rng.normal(100 + case, (N + 1, V), 2.0)
        best = torch.argmax(tl, dim=1).tolist()
        toks = rng.randint(300 + case, (N,), V).tolist()
        # plant the argmax along a path of random depth
        want_path, cur = [], -1
        for d in range(case % 5):
            kids = [c for c in range(N) if parent[c] == cur]
            if not kids:
                break
            c = kids[(case + d) % len(kids)]
            toks[c] = best[cur + 1]
            want_path.append(c)
            cur = c
        for c in range(N):                      # no accidental matches elsewhere
            if c not in want_path and toks[c] == best[parent[c] + 1]:
                toks[c] = (toks[c] + 1) % V
                if toks[c] == best[parent[c] + 1]:
                    toks[c] = (toks[c] + 1) % V
        a, path, out, gap = oracle.tree_greedy(parent, toks, tl)
        assert path == want_path and a == len(want_path)
        assert out[:a] == [toks[c] for c in path] and out[a] == best[cur + 1] and out[a + 1:] == [-1] * (N - a)
        depths.add(a)
        # (c) on the kept path taken as a chain, with a draft whose most likely token is the proposal
        T = min(gap, 1.0) / 60.0
        ctoks = [toks[c] for c in want_path]
        rows = [0] + [c + 1 for c in want_path]
        ctl = tl[rows].contiguous()
        cdl = torch.zeros((len(rows), V))
        for i, c in enumerate(want_path):
            cdl[i] = rng.normal(700 + case, (V,), 1.0)
            cdl[i, toks[c]] = cdl[i].max() + 1.0
        us = [max(u, 1e-3) for u in rng.uniform(900 + case, (len(rows),)).tolist()]
        a2, path2, out2, _ = oracle.tree_sample(list(range(-1, len(want_path) - 1)), ctoks, ctl, cdl, us, T)
        assert a2 == a and out2[:a + 1] == out[:a + 1]
    assert depths == {0, 1, 2, 3, 4} or depths == {0, 1, 2, 3}
    tl = rng.normal(1, (4, V), 2.0)
    chain_toks = torch.argmax(tl[:3], dim=1).tolist()
    chain_toks[2] = (chain_toks[2] + 1) % V
    assert oracle.tree_greedy([-1, 0, 1], chain_toks, tl)[::2] == oracle.greedy(tl, chain_toks)[:2]
