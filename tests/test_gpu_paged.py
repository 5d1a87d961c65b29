"""Paged KV cache (spec_verify_init_paged) against the oracle: logits of every window row within the
bf16 bound, decisions on identical logits under the margin rules, cache contents against the
oracle's cache -- and, on top, results bit-identical to the contiguous cache, pages taken on append
and handed back when a cache length shrinks, a pool smaller than the worst case, and the
out-of-pages error."""
import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu

SHAPE = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)     # bf16, grouped-query attention
DRAFT = wl.ModelShape(1, 128, 2, 1, 64, 256, 1000)
LOGIT_TOL = 3e-2                                        # bf16 models (the stated bound); measured < 5e-3


def _linear(rig_like, sv, slots, t0, look, toks, dl, us, T, Kmax, V, target_logits_in=None):
    B, M = len(slots), sum(k + 1 for k in look)
    na = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -9, dtype=torch.int32, device="cuda")
    lo = torch.zeros((M, V), dtype=torch.float32, device="cuda")
    sv.spec_verify_step(rig_like.h, look, us.cuda(), T, na, ot, seq_slot=torch.tensor(slots, dtype=torch.int32, device="cuda"),
                        last_token=torch.tensor(t0, dtype=torch.int32, device="cuda"), draft_tokens=toks.cuda(),
                        draft_logits=dl.cuda(), logits_out=lo, auto_rollback=True, target_logits_in=target_logits_in)
    torch.cuda.synchronize()
    return lo.cpu(), na.cpu(), ot.cpu()


def _against_oracle(paged, slots, t0, look, toks, dl, us, T, Kmax, V, got):
    """got = the paged handle's (logits, n_accepted, out_tokens): logits against the oracle's K+1
    single-token decodes, decisions on identical logits (the sampler replayed on the oracle's rows
    through the paged handle)."""
    from helpers import check_sampler_against_oracle
    want = paged.oracle_logits(slots, t0, look, toks)
    err = (got[0] - want).abs().max().item()
    assert err <= LOGIT_TOL, f"paged logits max-abs error {err}"
    _, na2, ot2 = _linear(paged, paged.sv, slots, t0, look, toks, dl, us, T, Kmax, V, target_logits_in=want.cuda())
    chk = check_sampler_against_oracle(want, dl, toks, us, look, T, Kmax, na2, ot2)
    return want, err, chk


def _export(rig, slot, pos0, n_pos):
    s = rig.shape
    x = torch.empty((s.n_layers, 2, s.n_kv_heads, n_pos, s.head_dim), dtype=torch.bfloat16, device="cuda")
    rig.sv.spec_kv_export(rig.h, slot, pos0, x)
    torch.cuda.synchronize()
    return x.cpu()


def test_paged_cache_gives_the_same_results_and_returns_pages():
    from test_gpu_forward import Rig, PagedRig
    from test_gpu_tree import _tree_step
    Kmax, T, V = 7, 1.0, SHAPE.vocab
    base = Rig(SHAPE, 3, 160, Kmax, seed=5, std=0.05)
    rng = wl.Rng(9, "cpu")
    lens = {0: 40, 1: 0, 2: 95}
    for s, n in lens.items():
        base.prefill(s, rng.randint(20 + s, (n,), V).tolist())
    paged = PagedRig(base, 3, 160, Kmax, n_pages=9)            # worst case would be 3 * 5 = 15 pages
    assert paged.free() == 9
    for s in lens:
        paged.load(base, s)
    assert paged.free() == 9 - (2 + 0 + 3)
    slots, t0, look = [2, 0, 1], [5, 6, 7], [7, 2, 4]
    toks = rng.randint(60, (3, Kmax), V)
    dl = rng.normal(61, (3, Kmax, V), 1.0)
    us = rng.uniform(62, (3, Kmax + 1))
    want = _linear(base, base.sv, slots, t0, look, toks, dl, us, T, Kmax, V)
    got = _linear(paged, paged.sv, slots, t0, look, toks, dl, us, T, Kmax, V)
    paged.sv.spec_verify_poll(paged.h)
    _, err, chk = _against_oracle(paged, slots, t0, look, toks, dl, us, T, Kmax, V, got)
    assert err < 5e-3 and chk.exact_accept + chk.margin_accept == 3
    assert torch.equal(want[0], got[0]) and torch.equal(want[1], got[1]) and torch.equal(want[2], got[2])
    kl = paged.kv_len.cpu().tolist()
    assert kl == base.kv_len.cpu().tolist()
    # slot 2 grew from 95 to 96 + a <= 103: positions 96.. need a fourth page only if something stayed there
    assert paged.free() == 9 - sum((kl[s] + 31) // 32 for s in range(3))
    # the appended window sits in the pages where the oracle's cache has it
    for b, s in enumerate(slots):
        a = int(got[1][b])
        ref = base.caches[s][:, :, :, lens[s]:lens[s] + a + 1]
        assert (_export(paged, s, lens[s], a + 1).float() - ref.float()).abs().max().item() < 2e-2
    # a tree step (with compaction) from here, on both
    n_nodes = [7, 4, 6]
    parent = torch.full((3, Kmax), -1, dtype=torch.int32)
    parent[0] = torch.tensor([-1, -1, 0, 0, 1, 2, 5])
    parent[1, :4] = torch.tensor([-1, 0, 1, 2])
    parent[2, :6] = torch.tensor([-1, -1, -1, 1, 3, 3])
    ttoks = rng.randint(70, (3, Kmax), V)
    tdl = rng.normal(71, (3, Kmax + 1, V), 1.0)
    tus = rng.uniform(72, (3, Kmax + 1))
    nxt = [int(want[2][b, int(want[1][b])]) for b in range(3)]
    a1 = _tree_step(base, slots, nxt, n_nodes, parent, ttoks, tdl, tus, T)
    a2 = _tree_step(paged, slots, nxt, n_nodes, parent, ttoks, tdl, tus, T)
    for x, y in zip(a1, a2):
        assert torch.equal(x, y)
    # ... and its logits against the oracle decoding along every path from the state after the first step
    r0 = 0
    for b, s in enumerate(slots):
        c = base.caches[s].clone()
        rows = oracle.tree_logits(base.om, c, kl[s], nxt[b], parent[b, :n_nodes[b]].tolist(), ttoks[b, :n_nodes[b]].tolist())
        err = (a2[0][r0:r0 + n_nodes[b] + 1] - rows).abs().max().item()
        assert err <= LOGIT_TOL, f"paged tree logits of sequence {b}: max-abs error {err}"
        r0 += n_nodes[b] + 1
    kl = paged.kv_len.cpu().tolist()
    assert kl == base.kv_len.cpu().tolist()
    assert paged.free() == 9 - sum((kl[s] + 31) // 32 for s in range(3))
    # the caches hold the same keys and values
    for s in range(3):
        if kl[s]:
            shape = (SHAPE.n_layers, 2, SHAPE.n_kv_heads, kl[s], SHAPE.head_dim)
            x = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
            y = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
            base.sv.spec_kv_export(base.h, s, 0, x)
            paged.sv.spec_kv_export(paged.h, s, 0, y)
            torch.cuda.synchronize()
            assert torch.equal(x, y)
    # dropping a sequence gives its pages back
    paged.sv.spec_kv_rollback(paged.h, [2, 0], [0, 33])
    assert paged.free() == 9 - (2 + (kl[1] + 31) // 32)
    paged.sv.spec_kv_rollback(paged.h, [0, 1], [0, 0])
    assert paged.free() == 9


def _planted_tree(rig, slot, t0, T, rng, stream):
    """A 7-node tree whose walk is known in advance: the root's children 0..2 are tokens the draft
    favours far more than the target (rejected at uniforms near 1), child 3 the token the target
    favours most over the draft (kept at uniform 0); node 3's children 4, 5 are rejected likewise and
    child 6 kept.  The kept path [3, 6] sits in window slots 4 and 7.  Rows come from the oracle."""
    V, om, n = rig.shape.vocab, rig.om, rig.n[slot]
    parent = [-1, -1, -1, -1, 3, 3, 3]
    dl = rng.normal(stream, (8, V), 1.5)
    c = rig.caches[slot].clone()
    p0 = oracle.softmax(om.verify_sequential(c, n, [t0])[0], T)
    q0 = oracle.softmax(dl[0], T)
    toks = torch.topk(q0 - p0, 3).indices.tolist() + [int(torch.argmax(p0 - q0))]
    p3 = oracle.softmax(om.verify_sequential(c, n, [t0, toks[3]])[1], T)
    q3 = oracle.softmax(dl[4], T)
    toks += torch.topk(q3 - p3, 2).indices.tolist() + [int(torch.argmax(p3 - q3))]
    us = [0.999, 0.999, 0.999, 0.0, 0.999, 0.999, 0.0, 0.37]
    return parent, toks, dl, us


def test_tree_step_whose_kept_nodes_sit_beyond_a_block_boundary():
    """A sequence of 28 positions keeps nodes 3 and 6 of its tree: their keys and values were written
    at positions 32 and 35 (second block) and move to 29 and 30, and the new length 31 needs the first
    block only.  The page of the second block must go back to the pool after that move, not before
    it: results equal to the contiguous cache's and to the oracle's, cache contents included."""
    from test_gpu_forward import Rig, PagedRig, _check_step
    from test_gpu_tree import _tree_step
    from helpers import TreeCheck
    Kmax, T, V = 7, 1.0, SHAPE.vocab
    base = Rig(SHAPE, 2, 96, Kmax, seed=7, std=0.05)
    rng = wl.Rng(19, "cpu")
    lens = {0: 28, 1: 61}                       # slot 1: kept nodes move from positions 65, 68 to 62, 63
    for s, n in lens.items():
        base.prefill(s, rng.randint(20 + s, (n,), V).tolist())
    paged = PagedRig(base, 2, 96, Kmax, n_pages=6)
    for s in lens:
        paged.load(base, s)
    # the second sequence's pool neighbour: whatever page is handed back too early is the one a
    # later append of the other sequence would take, so both run in one step
    slots, t0 = [0, 1], [11, 12]
    par, toks, dl, us = [], [], [], []
    for b, s in enumerate(slots):
        p, t, d, u = _planted_tree(base, s, t0[b], T, rng, 40 + b)
        par.append(p); toks.append(t); dl.append(d); us.append(u)
    parent = torch.tensor(par, dtype=torch.int32)
    ttoks = torch.tensor(toks, dtype=torch.int32)
    tdl = torch.stack(dl)
    tus = torch.tensor(us, dtype=torch.float32)
    a1 = _tree_step(base, slots, t0, [7, 7], parent, ttoks, tdl, tus, T)
    a2 = _tree_step(paged, slots, t0, [7, 7], parent, ttoks, tdl, tus, T)
    for x, y in zip(a1, a2):
        assert torch.equal(x, y)
    logits, na, ot, pt = a2
    chk = TreeCheck()
    for b, s in enumerate(slots):
        c = base.caches[s].clone()
        want = oracle.tree_logits(base.om, c, lens[s], t0[b], par[b], toks[b])
        rows = logits[8 * b:8 * b + 8]
        assert (rows - want).abs().max().item() <= LOGIT_TOL
        # the planted walk, as the oracle takes it on the GPU's own rows
        a, path, out, _ = oracle.tree_sample(par[b], toks[b], rows.contiguous(), tdl[b], us[b], T)
        assert (a, path) == (2, [3, 6]), "the planted walk should keep nodes 3 and 6"
        chk.compare(par[b], toks[b], rows.contiguous(), tdl[b], us[b], T, int(na[b]), pt[b].tolist(), ot[b].tolist(), Kmax)
    assert chk.exact_walk == 2
    kl = paged.kv_len.cpu().tolist()
    assert kl == [31, 64] and kl == base.kv_len.cpu().tolist()
    assert paged.free() == 6 - (1 + 2)
    # cache contents: paged == contiguous bit for bit, and both hold what ordinary decoding of
    # root + kept path leaves behind
    for b, s in enumerate(slots):
        x, y = _export(base, s, 0, kl[s]), _export(paged, s, 0, kl[s])
        assert torch.equal(x, y)
        ref = base.caches[s]
        base.om.verify_sequential(ref, lens[s], [t0[b], toks[b][3], toks[b][6]])
        diff = (y[:, :, :, lens[s]:].float() - ref[:, :, :, lens[s]:kl[s]].float()).abs().max().item()
        assert diff <= 0.07, f"compacted cache of slot {s} differs from the oracle's by {diff}"
        base.n[s] = kl[s]
    # the next step reads those positions: logits against the oracle continuing from its own cache
    nxt = [int(ot[b, 2]) for b in range(2)]
    err, *_ = _check_step(paged, slots, nxt, [3, 2], T, 321)
    assert err < 5e-3


def test_greedy_tree_step_whose_kept_nodes_sit_beyond_a_block_boundary():
    """The same situation at temperature 0 (the greedy walk has its own kernel): nodes 3 and 6 carry the
    most likely tokens of their parents' rows, every other node a different token."""
    from test_gpu_forward import Rig, PagedRig
    from test_gpu_tree import _tree_step
    Kmax, V = 7, SHAPE.vocab
    base = Rig(SHAPE, 2, 96, Kmax, seed=7, std=0.3)           # large weights: clear logit gaps
    rng = wl.Rng(23, "cpu")
    lens = {0: 28, 1: 61}
    for s, n in lens.items():
        base.prefill(s, rng.randint(20 + s, (n,), V).tolist())
    paged = PagedRig(base, 2, 96, Kmax, n_pages=6)
    for s in lens:
        paged.load(base, s)
    slots, t0 = [0, 1], [11, 12]
    parent = [-1, -1, -1, -1, 3, 3, 3]
    toks = []
    for b, s in enumerate(slots):
        c = base.caches[s].clone()
        top0 = int(torch.argmax(base.om.verify_sequential(c, lens[s], [t0[b]])[0]))
        top3 = int(torch.argmax(base.om.verify_sequential(c, lens[s], [t0[b], top0])[1]))
        toks.append([(top0 + 1) % V, (top0 + 2) % V, (top0 + 3) % V, top0, (top3 + 1) % V, (top3 + 2) % V, top3])
    par_t = torch.tensor([parent, parent], dtype=torch.int32)
    tok_t = torch.tensor(toks, dtype=torch.int32)
    dl = torch.zeros((2, Kmax + 1, V))
    us = torch.zeros((2, Kmax + 1))
    a1 = _tree_step(base, slots, t0, [7, 7], par_t, tok_t, dl, us, 0.0)
    a2 = _tree_step(paged, slots, t0, [7, 7], par_t, tok_t, dl, us, 0.0)
    for x, y in zip(a1, a2):
        assert torch.equal(x, y)
    logits, na, ot, pt = a2
    for b, s in enumerate(slots):
        rows = logits[8 * b:8 * b + 8].contiguous()
        a, path, out, gap = oracle.tree_greedy(parent, toks[b], rows)
        assert (a, path) == (2, [3, 6]) and gap > 1e-2, "the planted walk should keep nodes 3 and 6 by a clear gap"
        assert int(na[b]) == 2 and pt[b, :2].tolist() == [3, 6] and ot[b, :3].tolist() == out[:3]
    kl = paged.kv_len.cpu().tolist()
    assert kl == [31, 64] and kl == base.kv_len.cpu().tolist()
    assert paged.free() == 6 - (1 + 2)
    for b, s in enumerate(slots):
        x, y = _export(base, s, 0, kl[s]), _export(paged, s, 0, kl[s])
        assert torch.equal(x, y)
        ref = base.caches[s]
        base.om.verify_sequential(ref, lens[s], [t0[b], toks[b][3], toks[b][6]])
        diff = (y[:, :, :, lens[s]:].float() - ref[:, :, :, lens[s]:kl[s]].float()).abs().max().item()
        assert diff <= 0.5, f"compacted cache of slot {s} differs from the oracle's by {diff}"   # bf16 ulp at |v| ~ 30


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 5, 7, 9, 11, 12, 13])
def test_random_small_models_on_a_page_pool(seed):
    """The seeded random cases of test_gpu_forward (bf16 ones) on a page pool: logits against the
    oracle, decisions on identical logits, and the same tokens and lengths as the contiguous cache."""
    from test_gpu_forward import Rig, PagedRig, _random_case
    shape, n_slots, cap, kmax, lens, look, order, T = _random_case(1000 + seed)
    if shape.dtype != "bf16":
        pytest.skip("a page pool holds bf16 caches only")
    base = Rig(shape, n_slots, cap, kmax, seed=20 + seed, std=0.05)
    rng = wl.Rng(300 + seed, "cpu")
    for s, n in enumerate(lens):
        base.prefill(s, rng.randint(70 + s, (n,), shape.vocab).tolist())
    n_pages = sum((n + kmax + 1 + 31) // 32 for n in lens)          # exactly what the step can touch
    paged = PagedRig(base, n_slots, cap, kmax, n_pages=n_pages)
    for s in range(n_slots):
        paged.load(base, s)
    V = shape.vocab
    t0 = rng.randint(90, (n_slots,), V).tolist()
    lk = [look[s] for s in order]
    toks = rng.randint(91, (n_slots, max(kmax, 1)), V)[:, :kmax].contiguous()
    dl = rng.normal(92, (n_slots, max(kmax, 1), V), 1.0)[:, :kmax].contiguous()
    us = rng.uniform(93, (n_slots, kmax + 1))
    want = _linear(base, base.sv, order, t0, lk, toks, dl, us, T, kmax, V)
    got = _linear(paged, paged.sv, order, t0, lk, toks, dl, us, T, kmax, V)
    paged.sv.spec_verify_poll(paged.h)
    _, err, chk = _against_oracle(paged, order, t0, lk, toks, dl, us, T, kmax, V, got)
    assert err <= 5e-3, (err, shape, lens, look)
    assert torch.equal(want[1], got[1]) and torch.equal(want[2], got[2])
    assert (want[0] - got[0]).abs().max().item() <= 1e-5      # same arithmetic unless the chunk plans differ
    kl = paged.kv_len.cpu().tolist()
    assert kl == base.kv_len.cpu().tolist()
    assert paged.free() == n_pages - sum((n + 31) // 32 for n in kl)


def test_long_slots_of_a_small_model_on_a_page_pool():
    """A handle whose slots can grow to 16384 positions while the model and the batch are small (a
    launch with a few MiB of keys and values): a paged wavefront keeps the page numbers of at most 64
    blocks, so such a launch still cuts its sequences into chunks of at most 2048 positions.  Logits
    against the oracle, results equal to the contiguous cache's."""
    from test_gpu_forward import Rig, PagedRig
    shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    cap, kmax = 16384, 5
    base = Rig(shape, 2, cap, kmax, seed=41, std=0.05)
    rng = wl.Rng(42, "cpu")
    lens = [40, 2100]
    for s, n in enumerate(lens):
        base.prefill(s, rng.randint(70 + s, (n,), shape.vocab).tolist())
    paged = PagedRig(base, 2, cap, kmax, n_pages=80)
    for s in range(2):
        paged.load(base, s)
    V = shape.vocab
    t0 = rng.randint(90, (2,), V).tolist()
    lk = [kmax, 3]
    toks = rng.randint(91, (2, kmax), V)
    dl = rng.normal(92, (2, kmax, V), 1.0)
    us = rng.uniform(93, (2, kmax + 1))
    want = _linear(base, base.sv, [0, 1], t0, lk, toks, dl, us, 1.0, kmax, V)
    got = _linear(paged, paged.sv, [0, 1], t0, lk, toks, dl, us, 1.0, kmax, V)
    paged.sv.spec_verify_poll(paged.h)
    _, err, chk = _against_oracle(paged, [0, 1], t0, lk, toks, dl, us, 1.0, kmax, V, got)
    assert err <= 5e-3
    assert torch.equal(want[1], got[1]) and torch.equal(want[2], got[2])
    assert (want[0] - got[0]).abs().max().item() <= 1e-4      # the two caches cut the positions differently
    assert paged.kv_len.cpu().tolist() == base.kv_len.cpu().tolist()


def test_pool_exhaustion_skips_the_sequence_and_is_reported():
    from test_gpu_forward import Rig, PagedRig
    Kmax, T, V = 4, 1.0, SHAPE.vocab
    base = Rig(SHAPE, 2, 96, Kmax, seed=6, std=0.05)
    rng = wl.Rng(3, "cpu")
    base.prefill(0, rng.randint(1, (30,), V).tolist())       # the window will cross into a second block
    base.prefill(1, rng.randint(2, (10,), V).tolist())
    paged = PagedRig(base, 2, 96, Kmax, n_pages=2)
    paged.load(base, 0)
    paged.load(base, 1)
    assert paged.free() == 0
    toks = rng.randint(60, (2, Kmax), V)
    dl = rng.normal(61, (2, Kmax, V), 1.0)
    us = rng.uniform(62, (2, Kmax + 1))
    lo, na, ot = _linear(paged, paged.sv, [0, 1], [5, 6], [4, 4], toks, dl, us, T, Kmax, V)
    with pytest.raises(paged.sv.SpecError) as e:
        paged.sv.spec_verify_poll(paged.h)
    assert e.value.status == -3                                # SPEC_ERR_KV_OVERFLOW
    assert int(na[0]) == -1 and int(na[1]) >= 0
    # the healthy neighbour's rows are the oracle's
    want = paged.oracle_logits([1], [6], [4], toks[1:])
    assert (lo[5:] - want).abs().max().item() <= 5e-3
    same = _linear(base, base.sv, [1], [6], [4], toks[1:], dl[1:], us[1:], T, Kmax, V)
    assert torch.equal(same[0], lo[5:]) and int(same[1][0]) == int(na[1])


def test_decode_rounds_on_paged_caches_follow_the_oracle():
    """Five decoding rounds with both models' caches on page pools: the oracle follows the GPU round
    by round (every draft and target row, every proposal and decision, all bookkeeping), and the pools
    hold exactly the pages of the valid positions afterwards."""
    from test_gpu_decode import run_following, CONTEXTS
    pair, chk, tally, kept = run_following(SHAPE, DRAFT, CONTEXTS, K=3, Kt=3, rounds=5, T=1.0, seed=8, paged=(7, 7))
    assert tally["draft_err"] < 5e-3 and tally["target_err"] < 5e-3
    assert chk.exact_accept + chk.margin_accept == 5 * len(CONTEXTS)
    lt, ld = pair.tg.kv_len.cpu().tolist(), pair.dr.kv_len.cpu().tolist()
    assert pair.tg.free() == 7 - sum((x + 31) // 32 for x in lt) and pair.dr.free() == 7 - sum((x + 31) // 32 for x in ld)


def test_decode_rounds_on_paged_caches_match_contiguous_ones():
    from test_gpu_forward import PagedRig
    from test_gpu_decode import Pair, CONTEXTS
    from paper_2411_00853_amd import binding as sv
    K, R, T = 3, 5, 1.0
    pair = Pair(SHAPE, DRAFT, CONTEXTS, 96, K, 64, seed=8)
    B = len(CONTEXTS)
    ptg = PagedRig(pair.tg, B, 96, K, n_pages=7)
    pdr = PagedRig(pair.dr, B, 96, 1, n_pages=7)
    for b in range(B):
        ptg.load(pair.tg, b)
        pdr.load(pair.dr, b)
    dec = sv.spec_decode_init(ptg.h, pdr.h, B, 64)
    sv.spec_decode_begin(dec, torch.arange(B, dtype=torch.int32, device="cuda"),
                         torch.tensor([c[-2] for c in CONTEXTS], dtype=torch.int32, device="cuda"),
                         torch.tensor([c[-1] for c in CONTEXTS], dtype=torch.int32, device="cuda"))
    rng = wl.Rng(8, "cpu")
    for r in range(R):
        du, vu = rng.uniform(100 + r, (B, K)).cuda(), rng.uniform(200 + r, (B, K + 1)).cuda()
        g = pair.round(K, du.cpu(), vu.cpu(), T)
        sv.spec_decode_round(dec, K, du, vu, T)
    torch.cuda.synchronize()
    sv.spec_verify_poll(ptg.h)
    sv.spec_verify_poll(pdr.h)
    v = sv.spec_decode_get_view(dec)
    toks = sv.device_array(v.tokens, (B, 64), torch.int32).cpu()
    n = sv.device_array(v.n_tokens, (B,), torch.int32).cpu()
    assert torch.equal(n, g["n_tokens"])
    for b in range(B):
        assert toks[b, :int(n[b])].tolist() == g["tokens"][b, :int(n[b])].tolist()
    lt, ld = ptg.kv_len.cpu().tolist(), pdr.kv_len.cpu().tolist()
    assert lt == pair.tg.kv_len.cpu().tolist() and ld == pair.dr.kv_len.cpu().tolist()
    assert ptg.free() == 7 - sum((x + 31) // 32 for x in lt) and pdr.free() == 7 - sum((x + 31) // 32 for x in ld)
