"""The verify step and the no-alloc sampling step under HIP graph capture: both only queue kernels
(no allocation, no synchronisation, no memset node), so a serving loop can capture them once and
replay.  Each graph is replayed several times, with eager work and synchronisations between the
replays, on changing inputs, and every replay is compared with the eager call."""
import pytest
import torch

from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu


def test_noalloc_sampling_step_replayed_from_a_graph():
    from paper_2411_00853_amd import binding as sv
    B, Kmax, V, T = 6, 4, 4099, 0.9
    look = [4, 0, 3, 4, 1, 2]
    M = sum(k + 1 for k in look)
    rng = wl.Rng(71, "cuda")
    tl = torch.zeros((M, V), device="cuda")
    dl = torch.zeros((B, Kmax, V), device="cuda")
    toks = torch.zeros((B, Kmax), dtype=torch.int32, device="cuda")
    us = torch.zeros((B, Kmax + 1), device="cuda")
    na = torch.zeros(B, dtype=torch.int32, device="cuda")
    ot = torch.zeros((B, Kmax + 1), dtype=torch.int32, device="cuda")

    def new_inputs(i):
        tl.copy_(rng.normal(10 + i, (M, V), 1.0))
        dl.copy_(rng.normal(20 + i, (B, Kmax, V), 0.4))
        r0 = 0
        for b, k in enumerate(look):
            dl[b, :k] += tl[r0:r0 + k]
            r0 += k + 1
        toks.copy_(wl.pick_tokens(rng, dl, T, 30 + i))
        us.copy_(rng.uniform(40 + i, (B, Kmax + 1)))

    new_inputs(0)
    sv.spec_sample_step_noalloc(V, Kmax, look, us, T, na, ot, tl, draft_tokens=toks, draft_logits=dl)   # first call: address look-up
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            sv.spec_sample_step_noalloc(V, Kmax, look, us, T, na, ot, tl, draft_tokens=toks, draft_logits=dl,
                                        stream=torch.cuda.current_stream())
    h = sv.spec_verify_init(sv.sampler_cfg(V, B, Kmax), None, None, None)
    na_e = torch.zeros_like(na)
    ot_e = torch.zeros_like(ot)
    seen = set()
    for i in range(1, 5):
        new_inputs(i)
        torch.cuda.synchronize()
        na.fill_(-5)
        ot.fill_(-5)
        g.replay()
        torch.cuda.synchronize()
        sv.spec_verify_step(h, look, us, T, na_e, ot_e, draft_tokens=toks, draft_logits=dl, target_logits_in=tl)
        torch.cuda.synchronize()
        assert torch.equal(na, na_e) and torch.equal(ot, ot_e), f"replay {i} differs from the eager step"
        seen.add(tuple(na.tolist()))
    assert len(seen) >= 3, "the replays should have seen different inputs"
    h.close()


def test_verify_step_replayed_from_a_graph():
    from test_gpu_forward import Rig, _drafts
    from paper_2411_00853_amd import binding as sv
    shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    rig = Rig(shape, 2, 96, 4, seed=3, std=0.05)
    rng = wl.Rng(8, "cpu")
    lens = [40, 9]
    for s, n in enumerate(lens):
        rig.prefill(s, rng.randint(20 + s, (n,), shape.vocab).tolist())
    look, V, Kmax = [4, 2], shape.vocab, 4
    M = sum(k + 1 for k in look)
    toks_c, dl_c = _drafts(rng, 2, Kmax, V, 1.0)
    toks, dl = toks_c.cuda(), dl_c.cuda()
    us = rng.uniform(3, (2, Kmax + 1)).cuda()
    slots = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    t0 = torch.tensor([5, 6], dtype=torch.int32, device="cuda")
    na = torch.zeros(2, dtype=torch.int32, device="cuda")
    ot = torch.zeros((2, Kmax + 1), dtype=torch.int32, device="cuda")
    lo = torch.zeros((M, V), device="cuda")

    def step(stream=None):
        sv.spec_kv_rollback(rig.h, [0, 1], lens, stream=stream)
        sv.spec_verify_step(rig.h, look, us, 1.0, na, ot, seq_slot=slots, last_token=t0, draft_tokens=toks,
                            draft_logits=dl, logits_out=lo, auto_rollback=True, stream=stream)

    sv.spec_verify_step(rig.h, look, us, 1.0, na, ot, seq_slot=slots, last_token=t0, draft_tokens=toks, draft_logits=dl,
                        logits_out=lo, auto_rollback=True)
    torch.cuda.synchronize()
    want = (lo.clone(), na.clone(), ot.clone(), rig.kv_len.clone())
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(torch.cuda.current_stream())
    for i in range(4):
        lo.zero_()
        na.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(lo, want[0]) and torch.equal(na, want[1]) and torch.equal(ot, want[2]), f"replay {i}"
        assert torch.equal(rig.kv_len, want[3])
        # eager work between the replays: a step with other uniforms, then back
        us2 = rng.uniform(50 + i, (2, Kmax + 1)).cuda()
        sv.spec_kv_rollback(rig.h, [0, 1], lens)
        sv.spec_verify_step(rig.h, look, us2, 1.0, na, ot, seq_slot=slots, last_token=t0, draft_tokens=toks,
                            draft_logits=dl, auto_rollback=True)
        torch.cuda.synchronize()
    rig.sv.spec_verify_poll(rig.h)
