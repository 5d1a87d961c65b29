"""GPU parity of the whole verify step (decoder pass + sampler + KV bookkeeping) against the oracle.

Verify logits must equal what K+1 ordinary single-token decodes give (the oracle's definition):
max-abs error <= 1e-4 for fp32 models and <= 3e-2 for bf16 models.  Tokens are compared under the
margin rules of helpers.SamplerCheck; for bf16 models the sampler comparison uses identical logits
(the oracle's), because a 3e-2 logit difference moves p/q by far more than the 1e-3 accept margin."""
import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu

LOGIT_TOL = {"fp32": 1e-4, "bf16": 3e-2}


class Rig:
    """One model on both sides: oracle (CPU) and library handle (GPU) with identical weights/cache."""

    def __init__(self, shape, n_slots, max_kv_len, max_lookahead, seed=1, std=0.02, w_cpu=None):
        from helpers import device_weights
        from paper_2411_00853_amd import binding as sv
        self.sv, self.shape = sv, shape
        self.w_cpu = w_cpu if w_cpu is not None else wl.make_weights(shape, seed, "cpu", std=std)
        self.om = oracle.Model(shape, self.w_cpu, max_kv_len)
        self.cfg = sv.make_cfg(shape, n_slots, max_kv_len, max_lookahead)
        self.w_dev = device_weights(shape, self.w_cpu)
        self.kv = torch.zeros(sv.spec_kv_cache_bytes(self.cfg), dtype=torch.uint8, device="cuda")
        self.kv_len = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        self.h = sv.spec_verify_init(self.cfg, self.w_dev, self.kv, self.kv_len)
        self.caches = [self.om.new_cache() for _ in range(n_slots)]
        self.n = [0] * n_slots
        self.Kmax = max_lookahead

    def prefill(self, slot, tokens):
        """Build the slot's cache with the oracle (ordinary decoding) and upload it."""
        for i, t in enumerate(tokens):
            self.om.decode_one(self.caches[slot], i, int(t))
        self.set_cache(slot, len(tokens))

    def set_cache(self, slot, n):
        self.n[slot] = n
        if n:
            self.sv.spec_kv_import(self.h, slot, 0, self.caches[slot][:, :, :, :n, :].contiguous().cuda())
        self.kv_len[slot] = n

    def step(self, slots, t0, lookahead, draft_tokens, draft_logits, uniforms, T, auto_rollback=True,
             target_logits_in=None):
        B, V = len(slots), self.shape.vocab
        M = sum(k + 1 for k in lookahead)
        na = torch.full((B,), -9, dtype=torch.int32, device="cuda")
        ot = torch.full((B, self.Kmax + 1), -9, dtype=torch.int32, device="cuda")
        lo = torch.zeros((M, V), dtype=torch.float32, device="cuda")
        self.sv.spec_verify_step(
            self.h, lookahead, uniforms.cuda(), T, na, ot,
            seq_slot=torch.tensor(slots, dtype=torch.int32, device="cuda"),
            last_token=torch.tensor(t0, dtype=torch.int32, device="cuda"),
            draft_tokens=draft_tokens.cuda() if self.Kmax else None,
            draft_logits=draft_logits.cuda() if self.Kmax else None,
            target_logits_in=target_logits_in, logits_out=lo, auto_rollback=auto_rollback)
        torch.cuda.synchronize()
        self.sv.spec_verify_poll(self.h)
        return lo.cpu(), na.cpu(), ot.cpu()

    def oracle_logits(self, slots, t0, lookahead, draft_tokens):
        windows = [[t0[i]] + draft_tokens[i, :k].tolist() for i, k in enumerate(lookahead)]
        caches = [self.caches[s] for s in slots]          # the oracle appends the window to these
        return self.om.verify_rows(caches, [self.n[s] for s in slots], windows)


class PagedRig:
    """The same model and sequences as a Rig (it shares the Rig's oracle, weights and oracle-side
    caches), but the library handle keeps its cache in a page pool of n_pages pages."""

    def __init__(self, base, n_slots, max_kv_len, max_lookahead, n_pages):
        sv = base.sv
        self.sv, self.shape, self.Kmax = sv, base.shape, max_lookahead
        self.om, self.caches, self.n, self.w_cpu, self.w_dev = base.om, base.caches, base.n, base.w_cpu, base.w_dev
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

    step = Rig.step
    oracle_logits = Rig.oracle_logits


def _drafts(rng, B, Kmax, V, T):
    dl = rng.normal(50, (B, max(Kmax, 1), V), 1.0)[:, :Kmax].contiguous()
    toks = wl.pick_tokens(rng, dl, T, 51) if Kmax else torch.zeros((B, 0), dtype=torch.int32)
    return toks, dl


def _check_step(rig, slots, t0, lookahead, T, seed, perturb=0.3):
    """Run one step on both sides with drafts q = p_oracle + noise; returns the tallies."""
    from helpers import check_sampler_against_oracle
    rng = wl.Rng(seed, "cpu")
    B, V, Kmax = len(slots), rig.shape.vocab, rig.Kmax
    toks, dl = _drafts(rng, B, Kmax, V, T)
    us = rng.uniform(52, (B, Kmax + 1))
    n_before = [rig.n[s] for s in slots]
    want = rig.oracle_logits(slots, t0, lookahead, toks)
    # drafts close to the target so that both keep and reject outcomes occur
    r0 = 0
    for b, k in enumerate(lookahead):
        dl[b, :k] = want[r0:r0 + k] + rng.normal(60 + b, (k, V), perturb)
        r0 += k + 1
    logits, na, ot = rig.step(slots, t0, lookahead, toks, dl, us, T)
    err = (logits - want).abs().max().item()
    assert err <= LOGIT_TOL[rig.shape.dtype], f"logits max-abs error {err}"
    # KV bookkeeping: kv_len = n + accepted + 1, fp32 and bf16 models alike
    kl = rig.kv_len.cpu().tolist()
    for b, s in enumerate(slots):
        assert 0 <= int(na[b]) <= lookahead[b] and kl[s] == n_before[b] + int(na[b]) + 1, (b, s, kl, n_before, na)
    if rig.shape.dtype == "fp32":
        chk = check_sampler_against_oracle(want, dl, toks, us, lookahead, T, Kmax, na, ot)
    else:
        # identical logits for the token comparison: replay the sampler on the oracle's logits (a
        # sampler-only step neither reads nor writes the cache lengths)
        _, na2, ot2 = rig.step(slots, t0, lookahead, toks, dl, us, T, target_logits_in=want.cuda())
        chk = check_sampler_against_oracle(want, dl, toks, us, lookahead, T, Kmax, na2, ot2)
        assert rig.kv_len.cpu().tolist() == kl
    return err, chk, na, ot, logits, want


def test_tiny_config_end_to_end():
    w = wl.workload_tiny()
    rig = Rig(w.shape, 1, w.max_kv_len, w.max_lookahead, seed=w.seed)
    t0, prompts = wl.make_context(w)
    rig.prefill(0, prompts[0].tolist())
    err, chk, na, ot, logits, want = _check_step(rig, [0], t0.tolist(), list(w.lookahead), w.temperature, w.seed)
    assert chk.exact_accept == 1
    # the window's keys and values landed in the cache where the oracle put them
    got = torch.empty((w.shape.n_layers, 2, w.shape.n_kv_heads, 5, w.shape.head_dim), device="cuda")
    rig.sv.spec_kv_export(rig.h, 0, 128, got)
    torch.cuda.synchronize()
    assert (got.cpu() - rig.caches[0][:, :, :, 128:133, :]).abs().max().item() < 1e-5


@pytest.mark.parametrize("shape", [
    wl.ModelShape(3, 256, 8, 2, 64, 512, 1000),      # grouped-query attention, head_dim 64
    wl.ModelShape(2, 512, 4, 4, 128, 736, 2048),     # multi-head, head_dim 128, FFN not a multiple of 64
])
def test_small_bf16_models_ragged_batch(shape):
    rig = Rig(shape, 4, 200, 5, seed=3, std=0.05)
    rng = wl.Rng(8, "cpu")
    lens = {0: 70, 1: 33, 2: 0, 3: 150}
    for s, n in lens.items():
        rig.prefill(s, rng.randint(20 + s, (n,), shape.vocab).tolist())
    slots = [3, 0, 2, 1]
    err, chk, na, ot, logits, want = _check_step(rig, slots, [5, 6, 7, 8], [5, 0, 3, 2], 0.9, 12)
    assert chk.exact_accept >= 3
    assert err < 5e-3     # head + remainder operands keep the error far below the bf16 bound


@pytest.mark.parametrize("shape,kmax,look", [
    # 8 query heads per kv head: (K+1)*8 query rows per kv head
    (wl.ModelShape(2, 512, 8, 1, 128, 512, 1000), 5, [5, 0, 3, 2]),   # 48 rows, 128-dim heads: separate rotary kernel
    (wl.ModelShape(2, 512, 8, 1, 128, 512, 1000), 7, [7, 1, 4, 0]),   # 64 rows, 128-dim heads
    (wl.ModelShape(2, 512, 8, 1, 64, 512, 1000), 7, [7, 1, 4, 0]),    # 64 rows, 64-dim heads: merged kernel
])
def test_wide_query_groups(shape, kmax, look):
    rig = Rig(shape, 4, 200, kmax, seed=4, std=0.05)
    rng = wl.Rng(9, "cpu")
    lens = {0: 61, 1: 35, 2: 0, 3: 140}
    for s, n in lens.items():
        rig.prefill(s, rng.randint(30 + s, (n,), shape.vocab).tolist())
    slots = [3, 0, 2, 1]
    err, chk, na, ot, logits, want = _check_step(rig, slots, [5, 6, 7, 8], look, 0.9, 13)
    assert err < 5e-3
    # the window's keys and values are where the oracle put them (whichever kernel wrote them)
    for s, k in zip(slots, look):
        n = lens[s]
        got = torch.empty((shape.n_layers, 2, shape.n_kv_heads, k + 1, shape.head_dim), dtype=torch.bfloat16, device="cuda")
        rig.sv.spec_kv_export(rig.h, s, n, got)
        torch.cuda.synchronize()
        ref = rig.caches[s][:, :, :, n:n + k + 1, :]
        assert (got.cpu().float() - ref.float()).abs().max().item() < 2e-2


def test_sequences_far_below_the_cache_capacity():
    """The launch is sized for max_kv_len; every sequence cuts its own length into the chunks."""
    shape = wl.ModelShape(2, 256, 4, 2, 64, 256, 512)
    rig = Rig(shape, 3, 4000, 4, seed=6, std=0.05)
    rng = wl.Rng(10, "cpu")
    lens = {0: 700, 1: 130, 2: 3}
    for s, n in lens.items():
        rig.prefill(s, rng.randint(40 + s, (n,), shape.vocab).tolist())
    err, chk, na, ot, logits, want = _check_step(rig, [0, 1, 2], [5, 6, 7], [4, 2, 3], 0.9, 14)
    assert err < 5e-3


@pytest.mark.parametrize("hd,merge_in_workgroup", [(64, False), (64, True), (128, False), (128, True)])
def test_peaked_attention_scores(hd, merge_in_workgroup):
    """Query and key projections scaled up so that the scores spread over tens of units: in some
    blocks a row's running reference exponent jumps, in others a new maximum stays within the
    margin and the reference lags behind it; both must agree with the plain softmax."""
    from paper_2411_00853_amd import binding as sv
    shape = wl.ModelShape(2, 256, 256 // hd, 128 // hd, hd, 256, 512)
    w = wl.make_weights(shape, 21, "cpu", std=0.05)
    for lay in w["layers"]:
        rows = shape.d_q + shape.d_kv                      # the query and key rows of q|k|v
        lay["w_qkv"][:rows] = (lay["w_qkv"][:rows].float() * 4.0).to(lay["w_qkv"].dtype)
    sv.spec_k_set_attn_merge_min_pairs(1 if merge_in_workgroup else 0)
    try:
        rig = Rig(shape, 2, 700, 4, w_cpu=w)
        rng = wl.Rng(33, "cpu")
        for s, n in {0: 610, 1: 150}.items():
            rig.prefill(s, rng.randint(70 + s, (n,), shape.vocab).tolist())
        # the scores really are spread out: the oracle's attention is far from uniform
        err, chk, na, ot, logits, want = _check_step(rig, [0, 1], [9, 11], [4, 3], 1.0, 15)
        assert err < 1e-2
    finally:
        sv.spec_k_set_attn_merge_min_pairs(0)


def _random_case(seed):
    """A seeded small model and batch: shapes, lengths and lookaheads drawn from the ranges the
    library accepts (bf16: 64- or 128-dim heads, widths multiples of 32)."""
    import random
    r = random.Random(seed)
    hd = r.choice([64, 128])
    n_kv = r.choice([1, 2, 4])
    group = r.choice([1, 2, 3, 4, 8])
    n_q = n_kv * group
    d = r.choice([128, 224, 384])
    ffn = r.choice([160, 352, 736])
    vocab = r.choice([257, 1000, 4099])
    dtype = r.choice(["bf16", "bf16", "fp32"])
    kmax = r.choice([1, 3, 6, 9, 15])
    shape = wl.ModelShape(r.choice([1, 2]), d, n_q, n_kv, hd, ffn, vocab, dtype=dtype)
    n_slots = r.choice([1, 2, 3, 5])
    cap = r.choice([96, 300, 1500])
    lens = [r.choice([0, 1, 31, 32, 33, r.randrange(2, cap - kmax - 1), cap - kmax - 1]) for _ in range(n_slots)]
    look = [r.randrange(0, kmax + 1) for _ in range(n_slots)]
    look[r.randrange(n_slots)] = kmax
    order = list(range(n_slots))
    r.shuffle(order)
    return shape, n_slots, cap, kmax, lens, look, order, r.choice([0.6, 1.0, 1.7])


@pytest.mark.parametrize("seed", range(72))
def test_random_small_models(seed):
    shape, n_slots, cap, kmax, lens, look, order, T = _random_case(1000 + seed)
    rig = Rig(shape, n_slots, cap, kmax, seed=20 + seed, std=0.05)
    rng = wl.Rng(300 + seed, "cpu")
    for s, n in enumerate(lens):
        rig.prefill(s, rng.randint(70 + s, (n,), shape.vocab).tolist())
    t0 = rng.randint(90, (n_slots,), shape.vocab).tolist()
    err, chk, na, ot, logits, want = _check_step(rig, order, t0, [look[s] for s in order], T, 40 + seed)
    assert err <= (1e-4 if shape.dtype == "fp32" else 5e-3), (err, shape, lens, look)


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 5, 7, 9, 11, 12, 13, 14, 15])
def test_random_small_models_with_swiglu_inside_the_gemm(seed):
    """The same seeded cases with the gate/up projection forced to finish SwiGLU itself (by default
    only launches with enough workgroups do, i.e. large models), with 2, 3 or 4 wavefronts per
    workgroup in turn (left alone, a small model always gets 2)."""
    from paper_2411_00853_amd import binding as sv
    shape, n_slots, cap, kmax, lens, look, order, T = _random_case(1000 + seed)
    if shape.dtype != "bf16":
        pytest.skip("bf16 path only")
    sv.spec_k_set_swiglu_min_wgs(1)
    sv.spec_k_set_swiglu_column_groups(2 + seed % 3)
    try:
        rig = Rig(shape, n_slots, cap, kmax, seed=20 + seed, std=0.05)
        rng = wl.Rng(300 + seed, "cpu")
        for s, n in enumerate(lens):
            rig.prefill(s, rng.randint(70 + s, (n,), shape.vocab).tolist())
        t0 = rng.randint(90, (n_slots,), shape.vocab).tolist()
        err, chk, na, ot, logits, want = _check_step(rig, order, t0, [look[s] for s in order], T, 40 + seed)
        assert err <= 5e-3, (err, shape, lens, look)
    finally:
        sv.spec_k_set_swiglu_min_wgs(0)
        sv.spec_k_set_swiglu_column_groups(0)


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 5, 7, 9, 11, 12, 13, 14, 15, 16, 18, 20, 22])
@pytest.mark.parametrize("max_chunks", [1, 2, 3, 8])
def test_random_small_models_with_chunks_merged_in_the_workgroup(seed, max_chunks):
    """The same seeded cases with the attention workgroups forced to merge their chunks themselves
    (by default only launches with enough (sequence, kv head) pairs do), at 1, 2, 4 (for 3 chunks) and
    8 wavefronts per workgroup; shapes whose chunk results do not fit fall back to the merge kernel."""
    from paper_2411_00853_amd import binding as sv
    shape, n_slots, cap, kmax, lens, look, order, T = _random_case(1000 + seed)
    if shape.dtype != "bf16":
        pytest.skip("bf16 path only")
    sv.spec_k_set_attn_merge_min_pairs(1)
    sv.spec_k_set_attn_max_chunks(max_chunks)
    try:
        rig = Rig(shape, n_slots, cap, kmax, seed=20 + seed, std=0.05)
        rng = wl.Rng(300 + seed, "cpu")
        for s, n in enumerate(lens):
            rig.prefill(s, rng.randint(70 + s, (n,), shape.vocab).tolist())
        t0 = rng.randint(90, (n_slots,), shape.vocab).tolist()
        err, chk, na, ot, logits, want = _check_step(rig, order, t0, [look[s] for s in order], T, 40 + seed)
        assert err <= 5e-3, (err, shape, lens, look)
    finally:
        sv.spec_k_set_attn_merge_min_pairs(0)
        sv.spec_k_set_attn_max_chunks(0)


def test_step_rollback_step_reproduces_bits_and_ignores_stale_slots():
    shape = wl.ModelShape(2, 256, 4, 2, 64, 256, 512)
    rig = Rig(shape, 2, 96, 4, seed=5, std=0.05)
    rng = wl.Rng(9, "cpu")
    rig.prefill(0, rng.randint(1, (40,), shape.vocab).tolist())
    rig.prefill(1, rng.randint(2, (17,), shape.vocab).tolist())
    toks, dl = _drafts(rng, 2, 4, shape.vocab, 1.0)
    us = rng.uniform(3, (2, 5))
    a = rig.step([0, 1], [1, 2], [4, 3], toks, dl, us, 1.0, auto_rollback=False)
    assert rig.kv_len.cpu().tolist() == [45, 21]            # whole window appended
    rig.sv.spec_kv_rollback(rig.h, [0, 1], [40, 17])
    b = rig.step([0, 1], [1, 2], [4, 3], toks, dl, us, 1.0, auto_rollback=True)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
    assert rig.kv_len.cpu().tolist() == [40 + int(b[1][0]) + 1, 17 + int(b[1][1]) + 1]
    # poison everything beyond the valid length: the next step must not see it
    n0 = int(rig.kv_len[0])
    junk = torch.full((shape.n_layers, 2, shape.n_kv_heads, 96 - n0, shape.head_dim), float("nan"),
                      dtype=torch.bfloat16, device="cuda")
    rig.sv.spec_kv_import(rig.h, 0, n0, junk)
    c = rig.step([0], [3], [2], toks[:1], dl[:1], us[:1], 1.0)
    assert torch.isfinite(c[0]).all()
    # copying no positions is not an error (an empty tensor has no address)
    empty = torch.empty((shape.n_layers, 2, shape.n_kv_heads, 0, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    rig.sv.spec_kv_import(rig.h, 1, 5, empty)
    rig.sv.spec_kv_export(rig.h, 1, 0, empty)
    # rolling back above the current length is refused on the device and reported
    rig.sv.spec_kv_rollback(rig.h, [1], [90])
    with pytest.raises(rig.sv.SpecError) as e:
        rig.sv.spec_verify_poll(rig.h)
    assert e.value.status == -7


def test_two_handles_on_two_streams_at_once():
    """Handles share no device state: two models queued step by step on two streams, nothing waited
    for in between, give the bits each gives alone (and the first step of each matches the oracle)."""
    shapes = (wl.ModelShape(2, 256, 4, 2, 64, 256, 512), wl.ModelShape(3, 384, 8, 2, 128, 352, 1000))
    rigs, plans = [], []
    for i, shape in enumerate(shapes):
        rig = Rig(shape, 3, 160, 4, seed=31 + i, std=0.05)
        rng = wl.Rng(77 + i, "cpu")
        lens = [(60, 33, 5), (90, 1, 47)][i]
        for s_, n in enumerate(lens):
            rig.prefill(s_, rng.randint(1 + s_, (n,), shape.vocab).tolist())
        look = [(4, 2, 3), (1, 4, 4)][i]
        t0 = rng.randint(9, (3,), shape.vocab).tolist()
        _check_step(rig, [0, 1, 2], t0, list(look), 1.0, 500 + i)       # parity of this handle, alone
        rig.sv.spec_kv_rollback(rig.h, [0, 1, 2], list(lens))
        steps = []
        for j in range(6):                                               # inputs of six consecutive steps
            toks, dl = _drafts(wl.Rng(900 + 10 * i + j, "cpu"), 3, 4, shape.vocab, 1.0)
            steps.append((rng.randint(20 + j, (3,), shape.vocab).int().cuda(), toks.cuda(), dl.cuda(),
                          rng.uniform(40 + j, (3, 5)).cuda()))
        rigs.append(rig)
        plans.append((lens, look, steps))

    def queue(i, j, stream, outs):
        rig, (lens, look, steps) = rigs[i], plans[i]
        t0, toks, dl, us = steps[j]
        na = torch.full((3,), -9, dtype=torch.int32, device="cuda")
        ot = torch.full((3, 5), -9, dtype=torch.int32, device="cuda")
        lo = torch.zeros((sum(k + 1 for k in look), rig.shape.vocab), dtype=torch.float32, device="cuda")
        rig.sv.spec_verify_step(rig.h, list(look), us, 1.0, na, ot,
                                seq_slot=torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda"), last_token=t0,
                                draft_tokens=toks, draft_logits=dl, logits_out=lo, stream=stream)
        outs.append((lo, na, ot))

    def run(streams):
        outs = ([], [])
        torch.cuda.synchronize()
        for j in range(6):
            for i in (0, 1):
                with torch.cuda.stream(streams[i]):      # the small input tensors are made on that stream too
                    queue(i, j, streams[i], outs[i])
        torch.cuda.synchronize()
        for i in (0, 1):
            rigs[i].sv.spec_verify_poll(rigs[i].h)
            kl = rigs[i].kv_len.cpu().tolist()
            rigs[i].sv.spec_kv_rollback(rigs[i].h, [0, 1, 2], list(plans[i][0]))
            outs[i].append(kl)
        torch.cuda.synchronize()
        return outs

    one = torch.cuda.current_stream()
    alone = run((one, one))
    both = run((torch.cuda.Stream(), torch.cuda.Stream()))
    for i in (0, 1):
        assert alone[i][-1] == both[i][-1]
        for j in range(6):
            for x, y in zip(alone[i][j], both[i][j]):
                assert torch.equal(x, y), (i, j)
        assert any(int(v) >= 0 for v in both[i][0][1].tolist())


@pytest.mark.parametrize("merge_in_workgroup", [False, True])
def test_kv_overflow_skips_the_sequence(merge_in_workgroup):
    from paper_2411_00853_amd import binding as sv
    sv.spec_k_set_attn_merge_min_pairs(1 if merge_in_workgroup else 0)   # both ways of writing a skipped row
    try:
        _kv_overflow_case()
    finally:
        sv.spec_k_set_attn_merge_min_pairs(0)


def _kv_overflow_case():
    shape = wl.ModelShape(1, 128, 2, 2, 64, 128, 300)
    rig = Rig(shape, 2, 40, 4, seed=6)
    rng = wl.Rng(4, "cpu")
    rig.prefill(0, rng.randint(1, (38,), shape.vocab).tolist())     # 38 + 4 + 1 > 40
    rig.prefill(1, rng.randint(2, (10,), shape.vocab).tolist())
    toks, dl = _drafts(rng, 2, 4, shape.vocab, 1.0)
    us = rng.uniform(3, (2, 5))
    B = 2
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    ot = torch.zeros((B, 5), dtype=torch.int32, device="cuda")
    rig.sv.spec_verify_step(rig.h, [4, 4], us.cuda(), 1.0, na, ot,
                            seq_slot=torch.tensor([0, 1], dtype=torch.int32, device="cuda"),
                            last_token=torch.tensor([1, 2], dtype=torch.int32, device="cuda"),
                            draft_tokens=toks.cuda(), draft_logits=dl.cuda())
    with pytest.raises(rig.sv.SpecError) as e:
        rig.sv.spec_verify_poll(rig.h)
    assert e.value.status == -3
    assert na.cpu().tolist()[0] == -1 and na.cpu().tolist()[1] >= 0
    assert rig.kv_len.cpu().tolist()[0] == 38                        # untouched
    # the healthy neighbour is unaffected: a second step on it alone matches the oracle
    rig.kv_len[1] = 10
    err, chk, na2, ot2, logits, want = _check_step(rig, [1], [2], [4], 1.0, 77)
    assert err < 5e-3


def test_tuning_knobs_raised_after_init_are_refused_not_overrun():
    """The handle's partial-sum and chunk-result buffers are sized for the plans in force at init; a
    knob raised afterwards makes the step fail on the host with SPEC_ERR_SHAPE (nothing is launched
    past the buffers), and the step works again once the knob is back.  The shape is chosen so that the
    defaults leave room to grow: an LM head wide enough for two K ranges by default (four when asked
    for more workgroups), and 32 sequences x 8 kv heads, which get two position chunks each by default
    (sixteen when asked for more work items)."""
    from paper_2411_00853_amd import binding as sv
    shape = wl.ModelShape(1, 512, 8, 8, 64, 512, 24000)
    B = 32
    rig = Rig(shape, B, 2048, 1, seed=3, std=0.05)
    rng = wl.Rng(2, "cpu")
    toks, dl = _drafts(rng, B, 1, shape.vocab, 1.0)
    us = rng.uniform(3, (B, 2))
    slots, t0, look = list(range(B)), rng.randint(4, (B,), shape.vocab).tolist(), [1] * B
    for setter, value in ((sv.spec_k_set_gemm_wg_target, 4096), (sv.spec_k_set_attn_items_per_cu, 64)):
        setter(value)
        try:
            with pytest.raises(sv.SpecError) as e:
                rig.step(slots, t0, look, toks, dl, us, 1.0)
            assert e.value.status == -2 and "before spec_verify_init" in str(e.value)
        finally:
            setter(0)
        torch.cuda.synchronize()
        rig.kv_len.zero_()                                  # the refused step's bookkeeping kernel had run
    err, *_ = _check_step(rig, slots, t0, look, 1.0, 5)
    assert err < 5e-3


@pytest.mark.parametrize("B,Kmax", [(32, 10), (20, 9), (13, 15)])
def test_largest_windows_on_a_small_model(B, Kmax):
    """Up to 352 window rows in one step (32 sequences x 11 rows: the most the projections take), and
    the row counts between 192 and 352 whose GEMM variants the benchmark's configurations do not reach:
    every row against the oracle."""
    shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    rig = Rig(shape, B, 80, Kmax, seed=13, std=0.05)
    rng = wl.Rng(14, "cpu")
    lens = rng.randint(1, (B,), 60).tolist()
    for s, n in enumerate(lens):
        rig.prefill(s, rng.randint(100 + s, (n,), shape.vocab).tolist())
    look = [Kmax] * B
    look[1] = Kmax - 1 if B == 20 else Kmax          # 20 x 10 - 1 = 199 rows: a ragged tail inside a row tile
    t0 = rng.randint(3, (B,), shape.vocab).tolist()
    err, chk, na, ot, logits, want = _check_step(rig, list(range(B)), t0, look, 1.0, 99)
    assert logits.shape[0] == sum(k + 1 for k in look)
    assert err < 5e-3
    assert chk.exact_accept + chk.margin_accept == B


def test_steps_with_more_rows_than_one_decoder_pass():
    """40 sequences x 11 window rows = 440 rows, more than one launch of the projections takes (352): the
    step scores its sequences in two passes, and nothing else changes -- every row against the oracle,
    the sampler rules, the cache lengths; the same on a page pool, bit for bit; a ragged 408-row step
    from the state the first left; and a slot named by a sequence of each pass is refused for the
    later one only, as in a single pass."""
    shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    B, Kmax = 40, 10
    rig = Rig(shape, B, 80, Kmax, seed=17, std=0.05)
    rng = wl.Rng(18, "cpu")
    lens = rng.randint(1, (B,), 40).tolist()
    for s, n in enumerate(lens):
        rig.prefill(s, rng.randint(200 + s, (n,), shape.vocab).tolist())
    paged = PagedRig(rig, B, 80, Kmax, n_pages=B * 3)
    for s in range(B):
        paged.load(rig, s)
    slots = list(range(B))
    t0 = rng.randint(3, (B,), shape.vocab).tolist()
    look = [Kmax] * B
    # the paged handle first, on the same inputs _check_step will build (it advances the oracle's caches)
    r2 = wl.Rng(77, "cpu")
    toks, dl = _drafts(r2, B, Kmax, shape.vocab, 1.0)
    us = r2.uniform(52, (B, Kmax + 1))
    err, chk, na, ot, logits, want = _check_step(rig, slots, t0, look, 1.0, 77)
    assert logits.shape[0] == 440 and err < 5e-3
    assert chk.exact_accept + chk.margin_accept == B
    r0 = 0
    for b, k in enumerate(look):
        dl[b, :k] = want[r0:r0 + k] + r2.normal(60 + b, (k, shape.vocab), 0.3)
        r0 += k + 1
    lp, nap, otp = paged.step(slots, t0, look, toks, dl, us, 1.0)
    assert torch.equal(lp, logits) and torch.equal(nap, na) and torch.equal(otp, ot)
    assert torch.equal(paged.kv_len, rig.kv_len)
    # next step: ragged windows, 360 rows, sequences in another order
    for b in range(B):
        rig.n[b] = lens[b] + int(na[b]) + 1
    order = list(reversed(slots))
    look2 = [Kmax if i % 5 else 6 for i in range(B)]
    assert sum(k + 1 for k in look2) == 408
    nxt = [int(ot[s, int(na[s])]) for s in order]
    err2, chk2, na2, ot2, logits2, _ = _check_step(rig, order, nxt, look2, 1.0, 78)
    assert logits2.shape[0] == 408 and err2 < 5e-3
    assert chk2.exact_accept + chk2.margin_accept == B
    # one slot named twice, by a sequence of the first pass and one of the second
    before = rig.kv_len.clone()
    dup = list(slots)
    dup[B - 1] = dup[0]
    toks3, dl3 = _drafts(rng, B, Kmax, shape.vocab, 1.0)
    us3 = rng.uniform(9, (B, Kmax + 1))
    from paper_2411_00853_amd import binding as sv
    lo = torch.zeros((440, shape.vocab), device="cuda")
    na3 = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot3 = torch.full((B, Kmax + 1), -9, dtype=torch.int32, device="cuda")
    sv.spec_verify_step(rig.h, look, us3.cuda(), 1.0, na3, ot3,
                        seq_slot=torch.tensor(dup, dtype=torch.int32, device="cuda"),
                        last_token=torch.tensor(t0, dtype=torch.int32, device="cuda"), draft_tokens=toks3.cuda(),
                        draft_logits=dl3.cuda(), logits_out=lo)
    torch.cuda.synchronize()
    with pytest.raises(sv.SpecError):
        sv.spec_verify_poll(rig.h)
    na3 = na3.cpu()
    assert int(na3[B - 1]) == -1 and (na3[:B - 1] >= 0).all()
    after = rig.kv_len.cpu()
    assert int(after[B - 1]) == int(before[B - 1])                     # the slot the refused sequence did not get
    assert int(after[0]) == int(before[0]) + int(na3[0]) + 1


@pytest.mark.parametrize("n_kv,group,hd,Kmax", [(2, 8, 64, 15), (1, 8, 128, 15), (2, 6, 64, 11), (1, 16, 64, 15),
                                                 (2, 8, 128, 9)])
def test_more_than_64_query_rows_per_kv_head(n_kv, group, hd, Kmax):
    """(query heads per kv head) x (window length) beyond the 64 rows a wavefront holds: the heads of a
    kv head are dealt to two or four work items that stream the same cache head.  Every row against
    the oracle, on a contiguous cache and on a page pool (bit-identical), short and long windows in
    one step, then a second step from the state the first left."""
    shape = wl.ModelShape(2, 256, n_kv * group, n_kv, hd, 512, 1000)
    B = 5
    rig = Rig(shape, B, 400, Kmax, seed=21, std=0.05)
    rng = wl.Rng(22, "cpu")
    lens = [0, 31, 150, 333, 64]
    for s, n in enumerate(lens):
        rig.prefill(s, rng.randint(300 + s, (n,), shape.vocab).tolist())
    paged = PagedRig(rig, B, 400, Kmax, n_pages=40)
    for s in range(B):
        paged.load(rig, s)
    slots = [3, 0, 4, 1, 2]
    t0 = rng.randint(3, (B,), shape.vocab).tolist()
    look = [Kmax, 2, Kmax, 0, Kmax - 1]
    r2 = wl.Rng(91, "cpu")
    toks, dl = _drafts(r2, B, Kmax, shape.vocab, 1.0)
    us = r2.uniform(52, (B, Kmax + 1))
    err, chk, na, ot, logits, want = _check_step(rig, slots, t0, look, 1.0, 91)
    assert err < 5e-3
    assert chk.exact_accept + chk.margin_accept == B
    r0 = 0
    for b, k in enumerate(look):
        dl[b, :k] = want[r0:r0 + k] + r2.normal(60 + b, (k, shape.vocab), 0.3)
        r0 += k + 1
    lp, nap, otp = paged.step(slots, t0, look, toks, dl, us, 1.0)
    assert torch.equal(lp, logits) and torch.equal(nap, na) and torch.equal(otp, ot)
    for b, s in enumerate(slots):
        rig.n[s] += int(na[b]) + 1
    nxt = [int(ot[b, int(na[b])]) for b in range(B)]
    err2, chk2, *_ = _check_step(rig, slots, nxt, [Kmax] * B, 1.0, 92)
    assert err2 < 5e-3
