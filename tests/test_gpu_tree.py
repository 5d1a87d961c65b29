"""GPU parity of token-tree verification (spec_verify_tree_step) against the oracle
(oracle_tree_sample, oracle.tree_logits): the sampler alone on given logits, the chain case against
spec_verify_step, and the whole step on small models including the cache compaction."""
import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu

LOGIT_TOL = {"fp32": 1e-4, "bf16": 3e-2}


def random_tree(rng, stream, N, branch=0.5):
    """parent[i] in {-1, 0..i-1}: with probability `branch` a uniformly chosen earlier node (or the
    root), otherwise the previous node (chains dominate, as in drafted trees)."""
    u = rng.uniform(stream, (max(N, 1), 2)).tolist()
    parent = []
    for i in range(N):
        if i == 0 or u[i][0] < branch:
            parent.append(int(u[i][1] * (i + 1)) - 1)
        else:
            parent.append(i - 1)
    return parent


def make_tree_inputs(seed, B, Kmax, V, T, sigma=0.5):
    rng = wl.Rng(seed, "cpu")
    n_nodes = [int(v) for v in rng.randint(1, (B,), Kmax + 1).tolist()]
    n_nodes[0] = Kmax
    if B > 1:
        n_nodes[1] = 0
    parent = torch.full((B, Kmax), -1, dtype=torch.int32)
    for b in range(B):
        parent[b, :n_nodes[b]] = torch.tensor(random_tree(rng, 10 + b, n_nodes[b]), dtype=torch.int32)[:n_nodes[b]] \
            if n_nodes[b] else parent[b, :0]
    M = sum(n + 1 for n in n_nodes)
    tl = rng.normal(100, (M, V), 1.0)
    dl = torch.zeros((B, Kmax + 1, V))
    r0 = 0
    for b, n in enumerate(n_nodes):
        dl[b, :n + 1] = tl[r0:r0 + n + 1] + rng.normal(200 + b, (n + 1, V), sigma)
        r0 += n + 1
    # children are draws from the draft distribution at their parent
    toks = torch.zeros((B, Kmax), dtype=torch.int32)
    for b, n in enumerate(n_nodes):
        if n:
            rows = torch.stack([dl[b, parent[b, i] + 1] for i in range(n)])
            toks[b, :n] = wl.pick_tokens(rng, rows[None], T, 300 + b)[0]
    us = rng.uniform(400, (B, Kmax + 1))
    return n_nodes, parent, toks, tl, dl, us


def run_tree_sampler(n_nodes, parent, toks, tl, dl, us, T, Kmax):
    from paper_2411_00853_amd import binding as sv
    B, V = len(n_nodes), tl.shape[1]
    h = sv.spec_verify_init(sv.sampler_cfg(V, B, Kmax), None, None, None)
    na = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -7, dtype=torch.int32, device="cuda")
    pt = torch.full((B, Kmax), -7, dtype=torch.int32, device="cuda")
    sv.spec_verify_tree_step(h, n_nodes, parent.cuda(), toks.cuda(), dl.cuda().contiguous(), us.cuda(), T, na, ot, pt,
                             target_logits_in=tl.cuda().contiguous())
    torch.cuda.synchronize()
    sv.spec_verify_poll(h)
    h.close()
    return na.cpu(), ot.cpu(), pt.cpu()


def check_trees(n_nodes, parent, toks, tl, dl, us, T, Kmax, na, ot, pt):
    from helpers import TreeCheck
    chk = TreeCheck()
    r0 = 0
    for b, n in enumerate(n_nodes):
        chk.compare(parent[b, :n].tolist(), toks[b, :n].tolist(), tl[r0:r0 + n + 1], dl[b, :n + 1], us[b].tolist()[:n]
                    + [float(us[b, n])], T, int(na[b]), pt[b].tolist(), ot[b].tolist(), Kmax)
        r0 += n + 1
    return chk


@pytest.mark.parametrize("V,Kmax,T", [(1000, 8, 1.0), (301, 5, 0.7), (32000, 15, 1.3)])
def test_tree_sampler_against_oracle(V, Kmax, T):
    B = 12
    inp = make_tree_inputs(50 + Kmax, B, Kmax, V, T)
    na, ot, pt = run_tree_sampler(*inp, T, Kmax)
    chk = check_trees(*inp, T, Kmax, na, ot, pt)
    assert chk.exact_walk >= B - 2 and chk.exact_token >= B - 3
    assert len(set(na.tolist())) >= 3, "walks of different lengths should occur"


@pytest.mark.parametrize("V,k", [(50257, 20), (1000, 2)])
def test_tree_sampler_on_top_k_filtered_rows(V, k):
    """Rows after top-k filtering (all but the k largest logits of a row are -inf, on both sides): whole
    statistics chunks without a finite value, siblings that repeat a token, children the target excludes."""
    Kmax, T, B = 8, 1.0, 9
    n_nodes, parent, toks, tl, dl, us = make_tree_inputs(77 + V, B, Kmax, V, T, 0.3)

    def top_k(x):
        kth = x.topk(k, dim=-1).values[..., -1:]
        return x.masked_fill(x < kth, float("-inf"))
    tl, dl = top_k(tl), top_k(dl)
    rng = wl.Rng(78 + V, "cpu")
    for b, n in enumerate(n_nodes):                  # children drawn from the filtered draft row of their parent
        if n:
            rows = torch.stack([dl[b, parent[b, i] + 1] for i in range(n)])
            toks[b, :n] = wl.pick_tokens(rng, rows[None], T, 300 + b)[0]
    na, ot, pt = run_tree_sampler(n_nodes, parent, toks, tl, dl, us, T, Kmax)
    chk = check_trees(n_nodes, parent, toks, tl, dl, us, T, Kmax, na, ot, pt)
    assert chk.exact_walk >= B - 1
    r0 = 0
    for b, n in enumerate(n_nodes):                  # the final token has positive probability at the last kept node
        a = int(na[b])
        last = int(pt[b, a - 1]) + 1 if a else 0
        assert torch.isfinite(tl[r0 + last, int(ot[b, a])])
        r0 += n + 1


def test_chain_tree_equals_the_linear_step():
    from helpers import run_sampler_gpu
    B, K, V, T = 10, 6, 2000, 0.9
    rng = wl.Rng(77, "cpu")
    look = [K, 0, 3, K, 1, 5, 2, K, 4, K]
    M = sum(k + 1 for k in look)
    tl = rng.normal(1, (M, V), 1.0)
    dl = torch.zeros((B, K + 1, V))
    r0 = 0
    for b, k in enumerate(look):
        dl[b, :k + 1] = tl[r0:r0 + k + 1] + rng.normal(10 + b, (k + 1, V), 0.4)
        r0 += k + 1
    toks = wl.pick_tokens(rng, dl[:, :K].contiguous(), T, 30)
    us = rng.uniform(40, (B, K + 1))
    na1, ot1 = run_sampler_gpu(tl, dl[:, :K].contiguous(), toks, us, look, T, K)
    parent = torch.arange(-1, K - 1, dtype=torch.int32).repeat(B, 1)
    na2, ot2, pt2 = run_tree_sampler(look, parent, toks, tl, dl, us, T, K)
    assert torch.equal(na1, na2) and torch.equal(ot1, ot2)
    for b in range(B):
        a = int(na2[b])
        assert pt2[b, :a].tolist() == list(range(a)) and (pt2[b, a:] == -1).all()
    assert len(set(na1.tolist())) >= 3


def _tree_step(rig, slots, t0, n_nodes, parent, toks, dl, us, T, auto_rollback=True):
    B, V, Kmax = len(slots), rig.shape.vocab, rig.Kmax
    M = sum(n + 1 for n in n_nodes)
    na = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -9, dtype=torch.int32, device="cuda")
    pt = torch.full((B, Kmax), -9, dtype=torch.int32, device="cuda")
    lo = torch.zeros((M, V), dtype=torch.float32, device="cuda")
    rig.sv.spec_verify_tree_step(rig.h, n_nodes, parent.cuda(), toks.cuda(), dl.cuda().contiguous(), us.cuda(), T,
                                 na, ot, pt, seq_slot=torch.tensor(slots, dtype=torch.int32, device="cuda"),
                                 last_token=torch.tensor(t0, dtype=torch.int32, device="cuda"), logits_out=lo,
                                 auto_rollback=auto_rollback)
    torch.cuda.synchronize()
    rig.sv.spec_verify_poll(rig.h)
    return lo.cpu(), na.cpu(), ot.cpu(), pt.cpu()


@pytest.mark.parametrize("shape", [
    wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype="fp32"),
    wl.ModelShape(2, 256, 8, 2, 64, 512, 1000),               # bf16, grouped-query attention
    wl.ModelShape(2, 512, 4, 4, 128, 736, 1000),              # bf16, head_dim 128
])
def test_tree_step_on_small_models(shape):
    from test_gpu_forward import Rig
    from helpers import TreeCheck
    Kmax, T = 7, 1.0
    rig = Rig(shape, 3, 120, Kmax, seed=5, std=0.05)
    rng = wl.Rng(9, "cpu")
    lens = {0: 40, 1: 0, 2: 77}
    for s, n in lens.items():
        rig.prefill(s, rng.randint(20 + s, (n,), shape.vocab).tolist())
    slots, t0 = [2, 0, 1], [5, 6, 7]
    n_nodes = [7, 4, 6]
    parent = torch.full((3, Kmax), -1, dtype=torch.int32)
    parent[0] = torch.tensor([-1, -1, 0, 0, 1, 2, 5])
    parent[1, :4] = torch.tensor([-1, 0, 1, 2])            # a chain
    parent[2, :6] = torch.tensor([-1, -1, -1, 1, 3, 3])
    V = shape.vocab
    toks = rng.randint(60, (3, Kmax), V)
    # oracle logits along every path, from copies of the caches (tree_logits scribbles past n)
    want_rows, r0s = [], []
    for b, s in enumerate(slots):
        c = rig.caches[s].clone()
        want_rows.append(oracle.tree_logits(rig.om, c, rig.n[s], t0[b], parent[b, :n_nodes[b]].tolist(),
                                            toks[b, :n_nodes[b]].tolist()))
    want = torch.cat(want_rows)
    dl = torch.zeros((3, Kmax + 1, V))
    r0 = 0
    for b, n in enumerate(n_nodes):
        dl[b, :n + 1] = want[r0:r0 + n + 1] + rng.normal(70 + b, (n + 1, V), 0.3)
        r0 += n + 1
    us = rng.uniform(80, (3, Kmax + 1))
    n_before = [rig.n[s] for s in slots]
    logits, na, ot, pt = _tree_step(rig, slots, t0, n_nodes, parent, toks, dl, us, T)
    err = (logits - want).abs().max().item()
    assert err <= LOGIT_TOL[shape.dtype], f"tree logits max-abs error {err}"
    if shape.dtype == "bf16":
        assert err < 5e-3
    # decisions on the GPU's own rows
    chk = TreeCheck()
    r0 = 0
    for b, n in enumerate(n_nodes):
        chk.compare(parent[b, :n].tolist(), toks[b, :n].tolist(), logits[r0:r0 + n + 1].contiguous(), dl[b, :n + 1],
                    us[b, :n + 1].tolist(), T, int(na[b]), pt[b].tolist(), ot[b].tolist(), Kmax)
        r0 += n + 1
    assert chk.exact_walk == 3
    # the cache now holds root + kept path at n .. n+a, as ordinary decoding of those tokens would
    kl = rig.kv_len.cpu().tolist()
    for b, s in enumerate(slots):
        a = int(na[b])
        assert kl[s] == n_before[b] + a + 1
        kept = [int(toks[b, i]) for i in pt[b, :a].tolist()]
        ref = rig.caches[s]
        rig.om.verify_sequential(ref, n_before[b], [t0[b]] + kept)       # appends root + path in place
        got = torch.empty((shape.n_layers, 2, shape.n_kv_heads, a + 1, shape.head_dim), dtype=shape.torch_dtype,
                          device="cuda")
        rig.sv.spec_kv_export(rig.h, s, n_before[b], got)
        torch.cuda.synchronize()
        diff = (got.cpu().float() - ref[:, :, :, n_before[b]:n_before[b] + a + 1].float()).abs().max().item()
        assert diff <= (1e-5 if shape.dtype == "fp32" else 0.07), f"compacted cache differs by {diff}"
        rig.n[s] = n_before[b] + a + 1
    assert int(na.max()) >= 1, "at least one node should have been kept for the compaction to be exercised"
    # and the next (linear) step from that state agrees with the oracle continuing from its own
    from test_gpu_forward import _check_step
    nxt = [int(ot[b, int(na[b])]) for b in range(3)]
    err2, chk2, *_ = _check_step(rig, slots, nxt, [2, 3, 1], T, 123)
    assert err2 <= LOGIT_TOL[shape.dtype]


def test_bad_parent_is_flagged_and_skipped():
    from paper_2411_00853_amd import binding as sv
    B, Kmax, V = 2, 4, 64
    n_nodes, parent, toks, tl, dl, us = make_tree_inputs(5, B, Kmax, V, 1.0)
    n_nodes = [3, 2]
    M = 7
    tl = tl[:1].repeat(M, 1).contiguous()
    parent[0, :3] = torch.tensor([-1, 2, 0])      # node 1 names a later node as its parent
    parent[1, :2] = torch.tensor([-1, 0])
    h = sv.spec_verify_init(sv.sampler_cfg(V, B, Kmax), None, None, None)
    na = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -7, dtype=torch.int32, device="cuda")
    pt = torch.full((B, Kmax), -7, dtype=torch.int32, device="cuda")
    sv.spec_verify_tree_step(h, n_nodes, parent.cuda(), toks.cuda(), dl.cuda().contiguous(), us.cuda(), 1.0, na, ot, pt,
                             target_logits_in=tl.cuda())
    torch.cuda.synchronize()
    with pytest.raises(sv.SpecError):
        sv.spec_verify_poll(h)
    assert int(na[0]) == -1 and int(na[1]) >= 0
    h.close()


def test_greedy_tree_walk_at_temperature_zero():
    from paper_2411_00853_amd import binding as sv
    B, Kmax, V = 10, 9, 32003
    n_nodes, parent, toks, tl, dl, us = make_tree_inputs(91, B, Kmax, V, 1.0)
    # plant argmax tokens on some children so that walks of several depths occur
    r0 = 0
    for b, n in enumerate(n_nodes):
        best = torch.argmax(tl[r0:r0 + n + 1], dim=1)
        for i in range(n):
            if (b + i) % 2 == 0:
                toks[b, i] = int(best[int(parent[b, i]) + 1])
        r0 += n + 1
    h = sv.spec_verify_init(sv.sampler_cfg(V, B, Kmax), None, None, None)
    na = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -7, dtype=torch.int32, device="cuda")
    pt = torch.full((B, Kmax), -7, dtype=torch.int32, device="cuda")
    sv.spec_verify_tree_step(h, n_nodes, parent.cuda(), toks.cuda(), None, None, 0.0, na, ot, pt,
                             target_logits_in=tl.cuda().contiguous())
    torch.cuda.synchronize()
    sv.spec_verify_poll(h)
    h.close()
    r0, seen = 0, set()
    for b, n in enumerate(n_nodes):
        a, path, out, _ = oracle.tree_greedy(parent[b, :n].tolist(), toks[b, :n].tolist(), tl[r0:r0 + n + 1].contiguous())
        assert int(na[b]) == a and pt[b, :a].tolist() == path and (pt[b, a:] == -1).all()
        assert ot[b, :n + 1].tolist() == out and (ot[b, n + 1:] == -1).all()
        seen.add(a)
        r0 += n + 1
    assert len(seen) >= 3


@pytest.mark.parametrize("n_q", [8, 16])
def test_tree_step_with_more_rows_than_one_decoder_pass(n_q):
    """36 token trees of up to 10 nodes (390-odd window rows, more than one launch of the projections
    takes): the step scores them in two passes; logits of every node against the oracle's path-by-path
    decoding, every walk against the oracle's rule, and the compacted caches of all sequences.  With 16
    query heads on 2 kv heads a tree also has 88 query rows per kv head, more than a wavefront of the
    attention kernel holds: the heads of a kv head are then dealt to two work items."""
    from test_gpu_forward import Rig
    from helpers import TreeCheck
    shape = wl.ModelShape(2, 256, n_q, 2, 64, 512, 1000)
    B, Kmax, T = 36, 10, 1.0
    rig = Rig(shape, B, 64, Kmax, seed=31, std=0.05)
    rng = wl.Rng(32, "cpu")
    lens = rng.randint(1, (B,), 36).tolist()
    for s, n in enumerate(lens):
        rig.prefill(s, rng.randint(40 + s, (n,), shape.vocab).tolist())
    slots = list(range(B))
    t0 = rng.randint(2, (B,), shape.vocab).tolist()
    n_nodes = [Kmax] * B
    n_nodes[3], n_nodes[20] = 0, 4
    V = shape.vocab
    parent = torch.full((B, Kmax), -1, dtype=torch.int32)
    for b in range(B):
        if n_nodes[b]:
            parent[b, :n_nodes[b]] = torch.tensor(random_tree(rng, 100 + b, n_nodes[b]), dtype=torch.int32)
    toks = rng.randint(60, (B, Kmax), V)
    want = torch.cat([oracle.tree_logits(rig.om, rig.caches[s].clone(), rig.n[s], t0[b],
                                         parent[b, :n_nodes[b]].tolist(), toks[b, :n_nodes[b]].tolist())
                      for b, s in enumerate(slots)])
    M = sum(n + 1 for n in n_nodes)
    assert M > 352 and want.shape[0] == M
    dl = torch.zeros((B, Kmax + 1, V))
    r0 = 0
    for b, n in enumerate(n_nodes):
        dl[b, :n + 1] = want[r0:r0 + n + 1] + rng.normal(700 + b, (n + 1, V), 0.3)
        r0 += n + 1
    us = rng.uniform(80, (B, Kmax + 1))
    logits, na, ot, pt = _tree_step(rig, slots, t0, n_nodes, parent, toks, dl, us, T)
    err = (logits - want).abs().max().item()
    assert err < 5e-3, f"tree logits max-abs error {err}"
    chk = TreeCheck()
    r0 = 0
    for b, n in enumerate(n_nodes):
        chk.compare(parent[b, :n].tolist(), toks[b, :n].tolist(), logits[r0:r0 + n + 1].contiguous(), dl[b, :n + 1],
                    us[b, :n + 1].tolist(), T, int(na[b]), pt[b].tolist(), ot[b].tolist(), Kmax)
        r0 += n + 1
    assert chk.exact_walk >= B - 2
    kl = rig.kv_len.cpu().tolist()
    for b, s in enumerate(slots):
        a = int(na[b])
        assert kl[s] == lens[s] + a + 1
        kept = [int(toks[b, i]) for i in pt[b, :a].tolist()]
        ref = rig.caches[s]
        rig.om.verify_sequential(ref, lens[s], [t0[b]] + kept)
        got = torch.empty((shape.n_layers, 2, shape.n_kv_heads, a + 1, shape.head_dim), dtype=shape.torch_dtype,
                          device="cuda")
        rig.sv.spec_kv_export(rig.h, s, lens[s], got)
        torch.cuda.synchronize()
        diff = (got.cpu().float() - ref[:, :, :, lens[s]:lens[s] + a + 1].float()).abs().max().item()
        assert diff <= 0.07, f"compacted cache of sequence {b} differs by {diff}"
    assert int(na.max()) >= 1
