"""Paged KV cache (spec_verify_init_paged): identical results to the contiguous cache, pages taken
on append and handed back when a cache length shrinks, a pool smaller than the worst case, and the
out-of-pages error."""
import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu

SHAPE = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)     # bf16, grouped-query attention
DRAFT = wl.ModelShape(1, 128, 2, 1, 64, 256, 1000)


class PagedRig:
    """Like test_gpu_forward.Rig (same weights), but on a page pool of n_pages pages."""

    def __init__(self, base, n_slots, max_kv_len, max_lookahead, n_pages):
        from paper_2411_00853_amd import binding as sv
        self.sv, self.shape, self.Kmax = sv, base.shape, max_lookahead
        self.cfg = sv.make_cfg(base.shape, n_slots, max_kv_len, max_lookahead)
        self.kv = torch.zeros(n_pages * sv.spec_kv_page_bytes(self.cfg), dtype=torch.uint8, device="cuda")
        self.kv_len = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        self.h = sv.spec_verify_init_paged(self.cfg, base.w_dev, self.kv, self.kv_len)

    def load(self, base, slot):
        n = base.n[slot]
        if n:
            self.sv.spec_kv_import(self.h, slot, 0, base.caches[slot][:, :, :, :n, :].contiguous().cuda())
        self.kv_len[slot] = n

    def free(self):
        return self.sv.spec_kv_pages(self.h)[0]


def _linear(rig_like, sv, slots, t0, look, toks, dl, us, T, Kmax, V):
    B, M = len(slots), sum(k + 1 for k in look)
    na = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -9, dtype=torch.int32, device="cuda")
    lo = torch.zeros((M, V), dtype=torch.float32, device="cuda")
    sv.spec_verify_step(rig_like.h, look, us.cuda(), T, na, ot, seq_slot=torch.tensor(slots, dtype=torch.int32, device="cuda"),
                        last_token=torch.tensor(t0, dtype=torch.int32, device="cuda"), draft_tokens=toks.cuda(),
                        draft_logits=dl.cuda(), logits_out=lo, auto_rollback=True)
    torch.cuda.synchronize()
    return lo.cpu(), na.cpu(), ot.cpu()


def test_paged_cache_gives_the_same_results_and_returns_pages():
    from test_gpu_forward import Rig
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
    assert torch.equal(want[0], got[0]) and torch.equal(want[1], got[1]) and torch.equal(want[2], got[2])
    kl = paged.kv_len.cpu().tolist()
    assert kl == base.kv_len.cpu().tolist()
    # slot 2 grew from 95 to 96 + a <= 103: positions 96.. need a fourth page only if something stayed there
    assert paged.free() == 9 - sum((kl[s] + 31) // 32 for s in range(3))
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


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 5, 7, 9, 11, 12, 13])
def test_random_small_models_on_a_page_pool(seed):
    """The seeded random cases of test_gpu_forward (bf16 ones) give the same logits, tokens and
    lengths on a page pool as on the contiguous cache."""
    from test_gpu_forward import Rig, _random_case
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
    assert torch.equal(want[1], got[1]) and torch.equal(want[2], got[2])
    assert (want[0] - got[0]).abs().max().item() <= 1e-5      # same arithmetic unless the chunk plans differ
    kl = paged.kv_len.cpu().tolist()
    assert kl == base.kv_len.cpu().tolist()
    assert paged.free() == n_pages - sum((n + 31) // 32 for n in kl)


def test_pool_exhaustion_skips_the_sequence_and_is_reported():
    from test_gpu_forward import Rig
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
    want = _linear(base, base.sv, [1], [6], [4], toks[1:], dl[1:], us[1:], T, Kmax, V)
    assert torch.equal(want[0], lo[5:]) and int(want[1][0]) == int(na[1])


def test_decode_rounds_on_paged_caches_match_contiguous_ones():
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
