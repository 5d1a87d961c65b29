"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

1B-shape, 7B-shape (contiguous and paged cache), dynamic lookahead (32 ragged sequences, 157 rows)
and the 7B-shape token tree: every window row of every sequence against the oracle (<= 3e-2), tokens
on identical logits under the margin rules; the oracle takes the sequences a few at a time, their
caches regenerated from the seed.  Sampler stress: every sequence against the oracle.
Weights are made on the GPU by the seeded generator and copied to the host for the oracle; KV
contents are synthetic N(0,1) (stated in the workload recipe)."""
import sys
import time

import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


class BigWeights:
    """Generator-made weights of one shape on both sides (made on the GPU, copied to the host)."""

    def __init__(self, shape, seed):
        from paper_2411_00853_amd import binding as sv
        t = time.time()
        self.shape = shape
        raw = wl.make_weights(shape, seed, "cuda")
        self.cpu = {"tok_embed": raw["tok_embed"].cpu(), "final_norm": raw["final_norm"].cpu(),
                    "lm_head": raw["lm_head"].cpu(), "layers": [{k: v.cpu() for k, v in lw.items()} for lw in raw["layers"]]}
        pk = sv.spec_pack_weight
        self.dev = {"tok_embed": raw["tok_embed"], "final_norm": raw["final_norm"], "lm_head": pk(raw["lm_head"]),
                    "layers": [{"attn_norm": lw["attn_norm"], "ffn_norm": lw["ffn_norm"], "w_qkv": pk(lw["w_qkv"]),
                                "w_o": pk(lw["w_o"]), "w_gate_up": pk(lw["w_gate_up"], True),
                                "w_down": pk(lw["w_down"])} for lw in raw["layers"]]}
        torch.cuda.synchronize()
        say(f"  [weights] generated, packed and copied to the host in {time.time() - t:.1f}s")


class BigRig:
    def __init__(self, weights, n_slots, max_kv_len, Kmax, paged_lens=None):
        """paged_lens: the sequences' cached lengths -- the cache then lives in a page pool of exactly
        the pages one step of those sequences can touch (the handle `bench.py --paged` builds)."""
        from paper_2411_00853_amd import binding as sv
        shape = weights.shape
        self.sv, self.shape, self.Kmax, self.max_kv_len = sv, shape, Kmax, max_kv_len
        self.om = oracle.Model(shape, weights.cpu, max_kv_len)
        self.cfg = sv.make_cfg(shape, n_slots, max_kv_len, Kmax)
        self.kv_len = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        if paged_lens is None:
            self.kv = torch.empty(sv.spec_kv_cache_bytes(self.cfg), dtype=torch.uint8, device="cuda")
            self.h = sv.spec_verify_init(self.cfg, weights.dev, self.kv, self.kv_len)
        else:
            self.n_pages = sum((n + Kmax + 1 + 31) // 32 for n in paged_lens)
            self.kv = torch.empty(self.n_pages * sv.spec_kv_page_bytes(self.cfg), dtype=torch.uint8, device="cuda")
            self.h = sv.spec_verify_init_paged(self.cfg, weights.dev, self.kv, self.kv_len)

    def synthetic(self, w, n, seq_index):
        """The sequence's synthetic N(0,1) keys and values [layer][k|v][head][n][dim], on the GPU."""
        s = self.shape
        rng = wl.Rng(w.seed, "cuda")
        plain = torch.empty((s.n_layers, 2, s.n_kv_heads, n, s.head_dim), dtype=s.torch_dtype, device="cuda")
        for l in range(s.n_layers):
            plain[l] = rng.normal(wl.S_KV + seq_index * 4096 + l, (2, s.n_kv_heads, n, s.head_dim), 1.0, s.torch_dtype)
        return plain

    def fill_slot(self, w, slot, n, seq_index):
        self.sv.spec_kv_import(self.h, slot, 0, self.synthetic(w, n, seq_index))
        self.kv_len[slot] = n

    def oracle_cache(self, w, n, seq_index):
        """The same contents as an oracle-side cache (regenerated from the seed: a cache is 1-2 GB on
        the host at these sizes, so the oracle takes the sequences a few at a time)."""
        s = self.shape
        c = torch.zeros((s.n_layers, 2, s.n_kv_heads, self.max_kv_len, s.head_dim), dtype=s.torch_dtype)
        c[:, :, :, :n] = self.synthetic(w, n, seq_index).cpu()
        return c

    def close(self):
        self.h.close()


def _run_and_check(rig, w, label, group=8):
    """One step of workload w; EVERY sequence is verified against the oracle, `group` at a time:
    all window rows' logits (<= 3e-2) and the decisions on identical logits."""
    from helpers import SamplerCheck
    sv, shape = rig.sv, w.shape
    B, Kmax, V = w.batch, w.max_lookahead, shape.vocab
    look = list(w.lookahead)
    for b in range(B):
        rig.fill_slot(w, b, w.kv_lens[b], b)
    t0, _ = wl.make_context(w, "cuda")
    toks, dl = wl.make_free_drafts(w, "cuda")
    us = wl.make_uniforms(w, "cuda")
    M = w.rows
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    ot = torch.zeros((B, Kmax + 1), dtype=torch.int32, device="cuda")
    lo = torch.zeros((M, V), dtype=torch.float32, device="cuda")
    slots = torch.arange(B, dtype=torch.int32, device="cuda")
    sv.spec_verify_step(rig.h, look, us, w.temperature, na, ot, seq_slot=slots, last_token=t0, draft_tokens=toks,
                        draft_logits=dl, logits_out=lo, auto_rollback=True)
    torch.cuda.synchronize()
    sv.spec_verify_poll(rig.h)
    na_c, ot_c, lo_c = na.cpu(), ot.cpu(), lo.cpu()
    t0_c, toks_c, dl_c, us_c = t0.cpu(), toks.cpu(), dl.cpu(), us.cpu()
    # bookkeeping of every sequence
    kl = rig.kv_len.cpu().tolist()
    row0 = [0]
    for k in look:
        row0.append(row0[-1] + k + 1)
    for b in range(B):
        a = int(na_c[b])
        assert 0 <= a <= look[b] and kl[b] == w.kv_lens[b] + a + 1
        assert ot_c[b, :a].tolist() == toks_c[b, :a].tolist() and 0 <= int(ot_c[b, a]) < V
        assert (ot_c[b, a + 1:] == -1).all()
    assert torch.isfinite(lo_c).all()
    # the oracle, a group of sequences at a time
    worst, rows_checked, t_or = 0.0, 0, 0.0
    chk = SamplerCheck()
    for g0 in range(0, B, group):
        seqs = list(range(g0, min(g0 + group, B)))
        caches = [rig.oracle_cache(w, w.kv_lens[b], b) for b in seqs]
        t = time.time()
        want = rig.om.verify_rows(caches, [w.kv_lens[b] for b in seqs],
                                  [[int(t0_c[b])] + toks_c[b, :look[b]].tolist() for b in seqs])
        t_or += time.time() - t
        del caches
        r = 0
        for b in seqs:
            got = lo_c[row0[b]:row0[b + 1]]
            err = (got - want[r:r + look[b] + 1]).abs().max().item()
            assert err <= 3e-2, f"[{label}] sequence {b} (n={w.kv_lens[b]}, K={look[b]}): logits max-abs error {err}"
            worst = max(worst, err)
            r += look[b] + 1
        rows_checked += r
        # token parity on identical logits: replay the sampler on the oracle's logits for this group
        Bs = len(seqs)
        na2 = torch.zeros(Bs, dtype=torch.int32, device="cuda")
        ot2 = torch.zeros((Bs, Kmax + 1), dtype=torch.int32, device="cuda")
        idx = torch.tensor(seqs, device="cuda")
        sv.spec_verify_step(rig.h, [look[b] for b in seqs], us[idx].contiguous(), w.temperature, na2, ot2,
                            draft_tokens=toks[idx].contiguous(), draft_logits=dl[idx].contiguous(),
                            target_logits_in=want.cuda())
        torch.cuda.synchronize()
        r = 0
        for i, b in enumerate(seqs):
            chk.compare(want[r:r + look[b] + 1], dl_c[b], toks_c[b, :look[b]].tolist(), us_c[b, :look[b] + 1].tolist(),
                        w.temperature, int(na2[i]), ot2[i].cpu().tolist(), Kmax)
            r += look[b] + 1
        say(f"  [{label}] sequences {seqs[0]}..{seqs[-1]} checked, worst logits error so far {worst:.3e}")
    assert rows_checked == M
    say(f"  [{label}] oracle: all {rows_checked} rows of {B} sequences in {t_or:.1f}s; logits max-abs error {worst:.3e}")
    say(f"  [{label}] sampler: exact accept {chk.exact_accept}, margin {chk.margin_accept}; "
        f"exact token {chk.exact_token}, margin {chk.margin_token}; accepted {na_c.tolist()}")
    assert chk.exact_accept + chk.margin_accept == B
    return worst, chk


def test_1b_shape_full():
    w = wl.workload_1b()
    rig = BigRig(BigWeights(w.shape, w.seed), w.batch, w.max_kv_len, w.max_lookahead)
    try:
        _run_and_check(rig, w, "1b")
    finally:
        rig.close()


@pytest.mark.parametrize("hd,paged", [(64, False), (128, False), (64, True), (128, True)])
def test_long_contexts_on_a_small_model(hd, paged):
    """Caches of 32768 positions (on a page pool 16 chunks of 2048 positions, a wavefront holding the
    page numbers of 64 blocks) on a small model: sequences of 30000, 17001 and 40
    cached positions in one step, every row against the oracle, contiguous and paged."""
    shape = wl.ModelShape(2, 256, 8, 2, hd, 512, 1000)
    w = wl.Workload(f"long-{hd}", shape, 3, (30000, 17001, 40), (5, 3, 5), 5, 32768, 1.0, wl.SEED_BASE + 7000 + hd,
                    "synthetic")
    weights = BigWeights(shape, w.seed)
    rig = BigRig(weights, w.batch, w.max_kv_len, w.max_lookahead, paged_lens=w.kv_lens if paged else None)
    try:
        worst, chk = _run_and_check(rig, w, w.name + ("-paged" if paged else ""))
        assert worst < 5e-3
    finally:
        rig.close()


@pytest.mark.parametrize("paged", [False, True])
def test_a_hundred_thousand_positions(paged):
    """A slot of 131072 positions: 16 chunks of 8192 on a contiguous cache; on a page pool, where a
    wavefront keeps the page numbers of at most 64 blocks, 64 chunks of 2048 through the merge kernel."""
    shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    w = wl.Workload("long-100k", shape, 2, (100000, 513), (5, 2), 5, 131072, 1.0, wl.SEED_BASE + 7500, "synthetic")
    rig = BigRig(BigWeights(shape, w.seed), w.batch, w.max_kv_len, w.max_lookahead,
                 paged_lens=w.kv_lens if paged else None)
    try:
        worst, chk = _run_and_check(rig, w, w.name)
        assert worst < 5e-3
    finally:
        rig.close()


@pytest.fixture(scope="module")
def weights7b():
    return BigWeights(wl.SEVEN_B, wl.workload_7b().seed)


def test_7b_shape_full_all_rows(weights7b):
    # exactly the handle bench.py builds: 8 slots, 2054 positions, lookahead 5
    w = wl.workload_7b()
    rig = BigRig(weights7b, w.batch, w.max_kv_len, w.max_lookahead)
    try:
        _run_and_check(rig, w, "7b")
    finally:
        rig.close()


def test_7b_shape_paged_all_rows(weights7b):
    """The handle `bench.py --paged` builds (a pool of exactly the pages the step can touch): all 48
    rows against the oracle, decisions on identical logits, and the pages of rejected proposals back
    in the pool afterwards."""
    w = wl.workload_7b()
    rig = BigRig(weights7b, w.batch, w.max_kv_len, w.max_lookahead, paged_lens=w.kv_lens)
    try:
        _run_and_check(rig, w, "7b-paged")
        kl = rig.kv_len.cpu().tolist()
        assert rig.sv.spec_kv_pages(rig.h)[0] == rig.n_pages - sum((n + 31) // 32 for n in kl)
    finally:
        rig.close()


def test_dynamic_lookahead_all_sequences(weights7b):
    # same target weights as the 7B-shape case; 32 ragged sequences, every one of them through the oracle
    w = wl.workload_dyn()
    say(f"  [dyn] rows {w.rows}, n={list(w.kv_lens)} K={list(w.lookahead)}")
    rig = BigRig(weights7b, w.batch, w.max_kv_len, w.max_lookahead)
    try:
        _run_and_check(rig, w, "dyn")
    finally:
        rig.close()


def test_7b_shape_token_tree(weights7b):
    """The 10-node tree per sequence at 7B-shape (88 window rows): for every sequence the logits of all
    nodes against the oracle decoding along every root-to-leaf path, decisions on identical logits,
    the bookkeeping and the compacted cache length."""
    from helpers import TreeCheck
    w = wl.workload_tree()
    rig = BigRig(weights7b, w.batch, w.max_kv_len, w.max_lookahead)
    try:
        sv, shape = rig.sv, w.shape
        B, N, V = w.batch, w.max_lookahead, shape.vocab
        for b in range(B):
            rig.fill_slot(w, b, w.kv_lens[b], b)
        t0, _ = wl.make_context(w, "cuda")
        par, toks, dl = wl.make_tree_drafts(w, wl.TREE10_PARENT, "cuda")
        us = wl.make_uniforms(w, "cuda")
        M = B * (N + 1)
        na = torch.zeros(B, dtype=torch.int32, device="cuda")
        ot = torch.zeros((B, N + 1), dtype=torch.int32, device="cuda")
        pt = torch.zeros((B, N), dtype=torch.int32, device="cuda")
        lo = torch.zeros((M, V), dtype=torch.float32, device="cuda")
        sv.spec_verify_tree_step(rig.h, [N] * B, par, toks, dl, us, w.temperature, na, ot, pt,
                                 seq_slot=torch.arange(B, dtype=torch.int32, device="cuda"), last_token=t0,
                                 logits_out=lo, auto_rollback=True)
        torch.cuda.synchronize()
        sv.spec_verify_poll(rig.h)
        na_c, ot_c, pt_c, lo_c = na.cpu(), ot.cpu(), pt.cpu(), lo.cpu()
        toks_c, dl_c, us_c, t0_c = toks.cpu(), dl.cpu(), us.cpu(), t0.cpu()
        parent = list(wl.TREE10_PARENT)
        kl = rig.kv_len.cpu().tolist()
        for b in range(B):
            a = int(na_c[b])
            assert 0 <= a <= 4 and kl[b] == w.kv_lens[b] + a + 1          # the tree is 4 deep
            path = pt_c[b, :a].tolist()
            assert all(parent[path[k]] == (path[k - 1] if k else -1) for k in range(a))
            assert ot_c[b, :a].tolist() == [int(toks_c[b, i]) for i in path] and 0 <= int(ot_c[b, a]) < V
        assert torch.isfinite(lo_c).all()
        paths = oracle.tree_paths(parent)
        leaves = [i for i in range(N) if i not in parent]
        worst = 0.0
        chk = TreeCheck()
        t_or = 0.0
        for b in range(B):
            # every root-to-leaf path is one ordinary window on a cache of its own (they share the prefix)
            base = rig.oracle_cache(w, w.kv_lens[b], b)
            caches = [base] + [base.clone() for _ in leaves[1:]]
            t = time.time()
            rows = rig.om.verify_rows(caches, [w.kv_lens[b]] * len(leaves),
                                      [[int(t0_c[b])] + [int(toks_c[b, i]) for i in paths[leaf]] for leaf in leaves])
            t_or += time.time() - t
            del caches, base
            want = torch.zeros((N + 1, V))
            r = 0
            for leaf in leaves:
                want[0] = rows[r]
                for d, node in enumerate(paths[leaf]):
                    want[node + 1] = rows[r + d + 1]
                r += len(paths[leaf]) + 1
            got = lo_c[b * (N + 1):(b + 1) * (N + 1)]
            err = (got - want).abs().max().item()
            assert err <= 3e-2, f"tree logits of sequence {b}: max-abs error {err}"
            worst = max(worst, err)
            # decisions: replay the walk on the oracle's logits through the sampler-only entry
            na2 = torch.zeros(1, dtype=torch.int32, device="cuda")
            ot2 = torch.zeros((1, N + 1), dtype=torch.int32, device="cuda")
            pt2 = torch.zeros((1, N), dtype=torch.int32, device="cuda")
            sv.spec_verify_tree_step(rig.h, [N], par[b:b + 1].contiguous(), toks[b:b + 1].contiguous(),
                                     dl[b:b + 1].contiguous(), us[b:b + 1].contiguous(), w.temperature, na2, ot2, pt2,
                                     target_logits_in=want.cuda())
            torch.cuda.synchronize()
            chk.compare(parent, toks_c[b].tolist(), want, dl_c[b], us_c[b].tolist(), w.temperature, int(na2[0]),
                        pt2[0].cpu().tolist(), ot2[0].cpu().tolist(), N)
            say(f"  [tree] sequence {b} checked, worst logits error so far {worst:.3e}")
        say(f"  [tree] oracle {t_or:.1f}s; logits max-abs error {worst:.3e}; kept {na_c.tolist()}; "
            f"exact walks {chk.exact_walk}, margin walks {chk.margin_walk}; exact tokens {chk.exact_token}, "
            f"margin tokens {chk.margin_token}")
        assert chk.exact_walk + chk.margin_walk == B
    finally:
        rig.close()


def test_sampler_stress_full():
    from helpers import check_sampler_against_oracle, run_sampler_gpu
    t = time.time()
    s = wl.make_stress(device="cuda")      # 64 x (8+1) x 128256 target rows, 64 x 8 draft rows
    tl, dl, toks, us = s.target_logits.cpu(), s.draft_logits.cpu(), s.draft_tokens.cpu(), s.uniforms.cpu()
    say(f"  [stress] inputs in {time.time() - t:.1f}s")
    na, ot = run_sampler_gpu(tl, dl, toks, us, s.lookahead, s.temperature, 8)
    t = time.time()
    chk = check_sampler_against_oracle(tl, dl, toks, us, s.lookahead, s.temperature, 8, na, ot)
    say(f"  [stress] oracle {time.time() - t:.1f}s; exact accept {chk.exact_accept}, margin {chk.margin_accept}; "
        f"exact token {chk.exact_token}, margin {chk.margin_token}; mean accepted {na.float().mean().item():.2f}")
    assert chk.exact_accept >= 60 and chk.exact_token >= 50
