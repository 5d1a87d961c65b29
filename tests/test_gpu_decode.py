"""GPU parity of the whole speculative decoding round (draft loop + verification + bookkeeping,
include/spec_decode.h) against the oracle's loop (oracle/decode.py).

The GPU runs free; after every round the oracle is made to follow it token by token:
  * logits: the oracle's draft model decodes the GPU's proposals one by one, the oracle's target
    scores the GPU's window -- every row must agree with the GPU's (1e-4 fp32, 3e-2 bf16);
  * decisions on identical logits: every proposal must be the oracle's inverse-CDF draw from the
    GPU's own draft row, and n_accepted / emitted tokens the oracle's verification of the GPU's own
    rows (margin rules of helpers.SamplerCheck);
  * bookkeeping: output lists, the two trailing tokens, both cache lengths.
A second test lets the oracle run free as well (fp32) and compares the generated text itself."""
import pytest
import torch

import oracle
from oracle import decode as od
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu

LOGIT_TOL = {"fp32": 1e-4, "bf16": 3e-2}


class Pair:
    """Target + draft on both sides, a batch of sequences with oracle-built caches."""

    def __init__(self, t_shape, d_shape, contexts, max_kv_len, Kt, max_new, seed=5, std=0.05, paged=None):
        """paged = (target pages, draft pages): both handles keep their caches in page pools."""
        from test_gpu_forward import Rig, PagedRig
        from paper_2411_00853_amd import binding as sv
        self.sv = sv
        B = len(contexts)
        self.B, self.Kt = B, Kt
        self.tg = Rig(t_shape, B, max_kv_len, Kt, seed=seed, std=std)
        self.dr = Rig(d_shape, B, max_kv_len, 1, seed=seed + 1, std=std)
        self.states = []
        for b, ctx in enumerate(contexts):
            st = od.SequenceState(list(ctx), self.tg.caches[b], 0, self.dr.caches[b], 0)
            st.target_len = od.feed(self.tg.om, st.target_cache, 0, st.tokens, len(ctx) - 1)
            st.draft_len = od.feed(self.dr.om, st.draft_cache, 0, st.tokens, len(ctx) - 2)
            self.tg.set_cache(b, len(ctx) - 1)
            self.dr.set_cache(b, len(ctx) - 2)
            self.states.append(st)
        if paged:
            ptg = PagedRig(self.tg, B, max_kv_len, Kt, n_pages=paged[0])
            pdr = PagedRig(self.dr, B, max_kv_len, 1, n_pages=paged[1])
            for b in range(B):
                ptg.load(self.tg, b)
                pdr.load(self.dr, b)
            self.tg, self.dr = ptg, pdr
        self.dec = sv.spec_decode_init(self.tg.h, self.dr.h, B, max_new)
        self.max_new = max_new
        dev = "cuda"
        sv.spec_decode_begin(self.dec, torch.arange(B, dtype=torch.int32, device=dev),
                             torch.tensor([c[-2] for c in contexts], dtype=torch.int32, device=dev),
                             torch.tensor([c[-1] for c in contexts], dtype=torch.int32, device=dev))

    def view(self, K, rows=None):
        sv, v, B, Kt, V = self.sv, self.sv.spec_decode_get_view(self.dec), self.B, self.Kt, self.tg.shape.vocab
        get = lambda p, shape, dt: sv.device_array(p, shape, dt).cpu()
        out = {
            "tokens": get(v.tokens, (B, self.max_new), torch.int32),
            "n_tokens": get(v.n_tokens, (B,), torch.int32),
            "n_accepted": get(v.n_accepted, (B,), torch.int32),
            "draft_tokens": get(v.draft_tokens, (B, Kt), torch.int32),
            "draft_logits": get(v.draft_logits, (B, Kt, V), torch.float32),
            "target_logits": get(v.target_logits, (rows if rows is not None else B * (K + 1), V), torch.float32),
            "prev": get(v.prev_token, (B,), torch.int32),
            "last": get(v.last_token, (B,), torch.int32),
            "counters": get(v.counters, (3,), torch.int64),
        }
        torch.cuda.synchronize()
        return out

    def round(self, K, du, vu, T, per_seq=None):
        self.sv.spec_decode_round(self.dec, K, du.cuda(), vu.cuda(), T, lookahead_per_seq=per_seq)
        torch.cuda.synchronize()
        self.sv.spec_verify_poll(self.tg.h)
        self.sv.spec_verify_poll(self.dr.h)
        return self.view(K, None if per_seq is None else sum(k + 1 for k in per_seq))


def follow_round(pair, g, K, du, vu, T, chk, tally, per_seq=None):
    """Make the oracle take the round the GPU took (g = the GPU's view after it) and compare.
    per_seq: the proposals of each sequence that were put to the target (all K by default)."""
    from helpers import CDF_MARGIN
    tol = LOGIT_TOL[pair.tg.shape.dtype]
    row0 = 0
    for b, st in enumerate(pair.states):
        Kb = K if per_seq is None else per_seq[b]
        L = len(st.tokens)
        a = int(g["n_accepted"][b])
        props = g["draft_tokens"][b, :K].tolist()
        # ---- draft side: oracle decodes the GPU's proposals -----------------------------------
        st.draft_len = od.feed(pair.dr.om, st.draft_cache, st.draft_len, st.tokens, L - 1)
        cur = st.tokens[-1]
        for i in range(K):
            want = pair.dr.om.decode_one(st.draft_cache, L - 1 + i, cur)
            got = g["draft_logits"][b, i]
            err = (want - got).abs().max().item()
            tally["draft_err"] = max(tally["draft_err"], err)
            assert err <= tol, f"draft logits row {i} of sequence {b}: max-abs error {err}"
            # the proposal is the inverse-CDF draw from the GPU's own row
            y, dg = od.draw(got.contiguous(), T, float(du[b, i]))
            if min(dg.final_target - dg.final_cdf_lo, dg.final_cdf_hi - dg.final_target) > CDF_MARGIN:
                assert props[i] == y, f"proposal {i} of sequence {b}: {props[i]} != oracle {y}"
                tally["draws_exact"] += 1
            else:
                tally["draws_margin"] += 1
            cur = props[i]
        st.draft_len = L - 1 + K
        # ---- target side ---------------------------------------------------------------------
        props = props[:Kb]                      # the rest of the draft's proposals were dropped
        want = pair.tg.om.verify_sequential(st.target_cache, L - 1, [st.tokens[-1]] + props)
        got = g["target_logits"][row0:row0 + Kb + 1]
        row0 += Kb + 1
        err = (want - got).abs().max().item()
        tally["target_err"] = max(tally["target_err"], err)
        assert err <= tol, f"target logits of sequence {b}: max-abs error {err}"
        # verification on the GPU's own rows: the emitted tokens of this round are the tail of its list
        n_out = int(g["n_tokens"][b])
        emitted = g["tokens"][b, n_out - (a + 1):n_out].tolist()
        out_gpu = emitted + [-1] * (pair.Kt - a)
        chk.compare(got.contiguous(), g["draft_logits"][b].contiguous(), props, vu[b, :Kb + 1].tolist(), T, a, out_gpu,
                    pair.Kt)
        # ---- bookkeeping ---------------------------------------------------------------------
        assert emitted[:a] == props[:a]
        st.tokens.extend(emitted)
        st.target_len = L + a
        st.draft_len = min(st.draft_len, L + a)
        assert n_out == len(st.tokens) - tally["ctx_len"][b]
        assert int(g["last"][b]) == st.tokens[-1] and int(g["prev"][b]) == st.tokens[-2]
    kt = pair.tg.kv_len.cpu().tolist()
    kd = pair.dr.kv_len.cpu().tolist()
    for b, st in enumerate(pair.states):
        assert kt[b] == len(st.tokens) - 1 and kd[b] == len(st.tokens) - 2


def run_following(t_shape, d_shape, contexts, K, Kt, rounds, T, seed, paged=None, per_seq=None):
    from helpers import SamplerCheck
    pair = Pair(t_shape, d_shape, contexts, 96, Kt, 64, seed=seed, paged=paged)
    chk = SamplerCheck()
    tally = {"draft_err": 0.0, "target_err": 0.0, "draws_exact": 0, "draws_margin": 0,
             "ctx_len": [len(c) for c in contexts]}
    rng = wl.Rng(seed, "cpu")
    B = len(contexts)
    kept = 0
    Ks = K if isinstance(K, (list, tuple)) else [K] * rounds
    for r in range(rounds):
        K = Ks[r]
        du = rng.uniform(wl.S_UNIFORMS + 10 + 2 * r, (B, Kt))
        vu = rng.uniform(wl.S_UNIFORMS + 11 + 2 * r, (B, Kt + 1))
        ps = per_seq[r] if per_seq is not None else None
        g = pair.round(K, du, vu, T, per_seq=ps)
        follow_round(pair, g, K, du, vu, T, chk, tally, per_seq=ps)
        kept += int(g["n_accepted"].sum())
        c = g["counters"].tolist()
        assert c[0] == B * (r + 1) and c[1] == kept and c[2] == kept + B * (r + 1)
    # the generated text is in the output lists
    g = pair.view(0)
    for b, st in enumerate(pair.states):
        n = int(g["n_tokens"][b])
        assert g["tokens"][b, :n].tolist() == st.tokens[len(contexts[b]):]
    return pair, chk, tally, kept


CONTEXTS = [[5, 17, 3, 88, 41, 2, 60], [9, 1], [7] * 33 + [4, 250, 6]]


def test_rounds_fp32_oracle_follows_gpu():
    t_shape = wl.ModelShape(2, 256, 4, 4, 64, 512, 301, dtype="fp32")     # vocabulary not a multiple of 4
    d_shape = wl.ModelShape(1, 128, 2, 2, 64, 256, 301, dtype="fp32")
    pair, chk, tally, kept = run_following(t_shape, d_shape, CONTEXTS, K=4, Kt=4, rounds=5, T=1.0, seed=31)
    assert chk.exact_accept >= 13 and chk.exact_token >= 12
    assert tally["draws_exact"] >= 55
    assert 0 < kept < 5 * 3 * 4, "both outcomes should occur"


def test_rounds_bf16_lookahead_below_maximum():
    t_shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    d_shape = wl.ModelShape(1, 128, 2, 1, 64, 256, 1000)
    pair, chk, tally, kept = run_following(t_shape, d_shape, CONTEXTS, K=3, Kt=5, rounds=4, T=0.8, seed=32)
    assert chk.exact_accept >= 10
    assert tally["draft_err"] < 5e-3 and tally["target_err"] < 5e-3


def test_rounds_with_a_lookahead_that_changes_every_round():
    """What the lookahead controller does to the loop: K differs from round to round."""
    t_shape = wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype="fp32")
    d_shape = wl.ModelShape(1, 128, 2, 2, 64, 256, 300, dtype="fp32")
    pair, chk, tally, kept = run_following(t_shape, d_shape, CONTEXTS, K=[3, 1, 5, 2, 1, 4], Kt=5, rounds=6, T=1.0,
                                           seed=33)
    assert chk.exact_accept >= 16


@pytest.mark.parametrize("B,K", [(40, 10), (180, 1)])
def test_rounds_with_more_rows_than_one_decoder_pass(B, K):
    """Rounds whose verification window (40 x 11 = 440 rows), or whose first draft step and window
    (180 x 2 = 360 rows each), exceed what one launch of the projections takes: the models score their
    sequences in two passes and the oracle follows every row, draw, decision and length as usual."""
    import random
    r = random.Random(B)
    contexts = [[r.randrange(1000) for _ in range(r.choice([2, 3, 5, 8]))] for _ in range(B)]
    t_shape = wl.ModelShape(2, 256, 8, 2, 64, 512, 1000)
    d_shape = wl.ModelShape(1, 128, 2, 1, 64, 256, 1000)
    pair, chk, tally, kept = run_following(t_shape, d_shape, contexts, K=K, Kt=K, rounds=2, T=0.9, seed=40 + K)
    assert chk.exact_accept + chk.margin_accept == 2 * B
    assert tally["draft_err"] < 5e-3 and tally["target_err"] < 5e-3
    assert 0 < kept < 2 * B * K


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_rounds_with_a_lookahead_of_its_own_for_every_sequence(dtype):
    """The draft proposes K tokens for the whole batch, each sequence puts only its own K_b of them to the
    target (0 = none: the sequence just draws its next token from the target): ragged verification
    windows inside the round, the oracle following every row, draw and decision, lengths included."""
    V = 300 if dtype == "fp32" else 1000
    t_shape = wl.ModelShape(2, 256, 8, 2, 64, 512, V, dtype=dtype)
    d_shape = wl.ModelShape(1, 128, 2, 1, 64, 256, V, dtype=dtype)
    contexts = CONTEXTS + [[3, 1, 4, 1, 5, 9, 2, 6], [8, 8]]
    per = [[5, 0, 3, 1, 2], [0, 5, 5, 2, 4], [4, 4, 0, 0, 1], [1, 2, 3, 4, 4]]
    Ks = [5, 5, 4, 4]
    pair, chk, tally, kept = run_following(t_shape, d_shape, contexts, K=Ks, Kt=5, rounds=4, T=0.9, seed=61, per_seq=per)
    assert chk.exact_accept + chk.margin_accept == 4 * 5
    assert kept <= sum(sum(p) for p in per)
    from paper_2411_00853_amd import binding as sv
    du = torch.zeros((5, 5)); vu = torch.zeros((5, 6))
    with pytest.raises(sv.SpecError):
        pair.round(3, du, vu, 0.9, per_seq=[4, 0, 0, 0, 0])          # beyond the round's lookahead


def test_free_running_text_equals_the_oracles_fp32():
    """Both sides run on their own from the same start; the generated text must be the same for as
    long as no decision of the oracle's run was closer to its threshold than the margins that the
    1e-4 logit tolerance can move."""
    t_shape = wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype="fp32")
    d_shape = wl.ModelShape(1, 128, 2, 2, 64, 256, 300, dtype="fp32")
    K, R, T, seed = 3, 6, 1.0, 41
    pair = Pair(t_shape, d_shape, CONTEXTS, 96, K, 64, seed=seed)
    B = len(CONTEXTS)
    rng = wl.Rng(seed, "cpu")
    du = [rng.uniform(wl.S_UNIFORMS + 100 + r, (B, K)) for r in range(R)]
    vu = [rng.uniform(wl.S_UNIFORMS + 200 + r, (B, K + 1)) for r in range(R)]
    for r in range(R):
        g = pair.round(K, du[r], vu[r], T)
    compared = 0
    for b, st in enumerate(pair.states):
        trace = od.speculative_decode(pair.tg.om, pair.dr.om, st, R, K, T, [u[b].tolist() for u in du],
                                      [u[b].tolist() for u in vu])
        safe = 0   # tokens generated before the first decision that is too close to call
        for r, t in enumerate(trace):
            gaps = [min(d.final_target - d.final_cdf_lo, d.final_cdf_hi - d.final_target) for d in t.draft_diags]
            gaps.append(min(t.diag.final_target - t.diag.final_cdf_lo, t.diag.final_cdf_hi - t.diag.final_target))
            margins = [abs(float(vu[r][b, i]) - t.diag.accept_ratio[i])
                       for i in range(min(t.n_accepted + 1, K))]
            if min(gaps) < 5e-5 or (margins and min(margins) < 1e-3):   # what a 1e-4 logit error can move
                break
            safe += len(t.emitted)
        n = int(g["n_tokens"][b])
        got = g["tokens"][b, :n].tolist()
        want = st.tokens[len(CONTEXTS[b]):]
        assert got[:safe] == want[:safe], f"sequence {b}: text differs inside the safe prefix ({safe} tokens)"
        compared += safe
    assert compared >= 20, "too few tokens compared for the test to mean anything"


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_greedy_rounds_at_temperature_zero(dtype):
    """T = 0: proposals are the draft's most likely tokens, the verification is the greedy rule, and
    the text is the target's greedy continuation.  Compared with the oracle's run for as long as
    every deciding logit gap of the oracle's run is far above the logit tolerance."""
    t_shape = wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype=dtype)
    d_shape = wl.ModelShape(1, 128, 2, 2, 64, 256, 300, dtype=dtype)
    K, R = 3, 6
    pair = Pair(t_shape, d_shape, CONTEXTS, 96, K, 64, seed=51, std=0.3)   # large weights: clear logit gaps
    B = len(CONTEXTS)
    accepted = []
    for r in range(R):
        pair.sv.spec_decode_round(pair.dec, K, None, None, 0.0)
        torch.cuda.synchronize()
        accepted.append(pair.view(K)["n_accepted"].tolist())
    pair.sv.spec_verify_poll(pair.tg.h)
    pair.sv.spec_verify_poll(pair.dr.h)
    g = pair.view(K)
    tol = 5 * LOGIT_TOL[dtype] if dtype == "fp32" else LOGIT_TOL[dtype]   # a gap that the logit error cannot close
    compared = 0
    for b, st in enumerate(pair.states):
        trace = od.speculative_decode(pair.tg.om, pair.dr.om, st, R, K, 0.0, [[0.0] * K] * R, [[0.0] * (K + 1)] * R)
        safe_rounds = 0
        for t in trace:
            draft_gaps = [float(torch.topk(row, 2).values[0] - torch.topk(row, 2).values[1]) for row in t.draft_logits]
            if min(draft_gaps + [t.diag]) < tol:
                break
            safe_rounds += 1
        safe = sum(len(t.emitted) for t in trace[:safe_rounds])
        n = int(g["n_tokens"][b])
        assert g["tokens"][b, :n].tolist()[:safe] == st.tokens[len(CONTEXTS[b]):][:safe]
        assert [accepted[r][b] for r in range(safe_rounds)] == [t.n_accepted for t in trace[:safe_rounds]]
        compared += safe
    assert compared >= (12 if dtype == "fp32" else 4), compared


def test_plain_sampling_rounds_without_a_draft():
    """lookahead 0, no draft model: one token per round drawn from the target -- the baseline loop."""
    from test_gpu_forward import Rig
    from paper_2411_00853_amd import binding as sv
    shape = wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype="fp32")
    rig = Rig(shape, 2, 64, 0, seed=7, std=0.05)
    ctxs = [[3, 4, 5, 6], [10, 11]]
    sts = []
    for b, c in enumerate(ctxs):
        st = od.SequenceState(list(c), rig.caches[b], 0)
        st.target_len = od.feed(rig.om, st.target_cache, 0, st.tokens, len(c) - 1)
        rig.set_cache(b, len(c) - 1)
        sts.append(st)
    dec = sv.spec_decode_init(rig.h, None, 2, 16)
    sv.spec_decode_begin(dec, torch.arange(2, dtype=torch.int32, device="cuda"), None,
                         torch.tensor([c[-1] for c in ctxs], dtype=torch.int32, device="cuda"))
    R, T = 6, 0.9
    us = wl.Rng(3, "cpu").uniform(wl.S_UNIFORMS + 5, (R, 2, 1))
    for r in range(R):
        sv.spec_decode_round(dec, 0, None, us[r].contiguous().cuda(), T)
    torch.cuda.synchronize()
    sv.spec_verify_poll(rig.h)
    v = sv.spec_decode_get_view(dec)
    toks = sv.device_array(v.tokens, (2, 16), torch.int32).cpu()
    n = sv.device_array(v.n_tokens, (2,), torch.int32).cpu().tolist()
    assert n == [R, R]
    for b, st in enumerate(sts):
        want = od.autoregressive_decode(rig.om, st, R, T, us[:, b, 0].tolist())
        assert toks[b, :R].tolist() == want   # fp32, and these seeds keep clear of the CDF edges
    with pytest.raises(sv.SpecError):
        sv.spec_decode_round(dec, 2, None, us[0].contiguous().cuda(), T)


def test_argument_errors():
    from test_gpu_forward import Rig
    from paper_2411_00853_amd import binding as sv
    a = Rig(wl.ModelShape(1, 128, 2, 2, 64, 256, 300, dtype="fp32"), 2, 64, 2, seed=1)
    b = Rig(wl.ModelShape(1, 128, 2, 2, 64, 256, 301, dtype="fp32"), 2, 64, 1, seed=2)
    with pytest.raises(sv.SpecError):
        sv.spec_decode_init(a.h, b.h, 2, 8)          # vocabularies differ
    with pytest.raises(sv.SpecError):
        sv.spec_decode_init(a.h, None, 3, 8)         # more sequences than the handle holds
    dec = sv.spec_decode_init(a.h, None, 2, 8)
    with pytest.raises(sv.SpecError):
        sv.spec_decode_round(dec, 0, None, torch.zeros(2, 3, device="cuda"), 1.0)   # no active batch


@pytest.mark.parametrize("T,cost,per_seq", [(1.0, (0.4, 5.0, 0.05), False), (2.5, (0.4, 5.0, 0.05), False),
                                             (2.5, (1.0, 4.0, 0.05), False), (2.5, (0.4, 5.0, 1.0), True),
                                             (1.5, (0.4, 5.0, 1.5), True)])
def test_lookahead_controller_in_the_loop_fp32(T, cost, per_seq):
    """The lookahead follows the data inside the loop: every round's K is what the library's
    controller (spec_lookahead_next) chooses from the kept counts the GPU reported so far.  The oracle
    runs its own loop from the same start, its K chosen by its own rule (oracle.decode.LookaheadRule)
    from its own results.  The sequence of K, the kept counts, the generated text and the acceptance
    estimates must be the same, for as long as no decision of the oracle's run was closer to its
    threshold than the margins a 1e-4 logit difference can move.
    per_seq: every sequence also gets a window of its own (spec_lookahead_next_per_seq, with a cost model
    in which verification rows are dear, so that the windows do differ)."""
    from paper_2411_00853_amd import binding as sv
    t_shape = wl.ModelShape(2, 256, 4, 4, 64, 512, 300, dtype="fp32")
    d_shape = wl.ModelShape(1, 128, 2, 2, 64, 256, 300, dtype="fp32")
    Kt, R, seed = 5, 10, 61
    pair = Pair(t_shape, d_shape, CONTEXTS, 128, Kt, 96, seed=seed)
    B = len(CONTEXTS)
    kw = dict(draft_ms=cost[0], verify_ms=cost[1], verify_ms_per_token=cost[2], k_min=1, k_max=Kt)
    ctl = sv.Lookahead(B, **kw)
    rule = od.LookaheadRule(B, **kw)
    rng = wl.Rng(seed, "cpu")
    du = [rng.uniform(wl.S_UNIFORMS + 100 + r, (B, Kt)) for r in range(R)]
    vu = [rng.uniform(wl.S_UNIFORMS + 200 + r, (B, Kt + 1)) for r in range(R)]
    # ---- the GPU's loop, controller in it ----
    ks_gpu, kept_gpu, est_gpu = [], [], []
    win_gpu = []
    for r in range(R):
        if per_seq:
            k, win = ctl.next_per_seq()
            g = pair.round(k, du[r], vu[r], T, per_seq=win)
            a = g["n_accepted"].tolist()
            ctl.update_per_seq(a, win)
        else:
            k, win = ctl.next(), None
            g = pair.round(k, du[r], vu[r], T)
            a = g["n_accepted"].tolist()
            ctl.update(a, k)
        win_gpu.append(win)
        ks_gpu.append(k)
        kept_gpu.append(a)
        est_gpu.append([ctl.accept(b) for b in range(B)])
    text_gpu = [g["tokens"][b, :int(g["n_tokens"][b])].tolist() for b in range(B)]
    # ---- the oracle's loop, its own rule in it ----
    # A round in which every decision of the oracle's run is clear of its threshold must agree in
    # full.  A round with a decision too close to call may go either way: if the GPU took the same
    # decisions the comparison goes on, otherwise the two runs have parted for good and it ends.
    rounds_same, rounds_clear, pos = 0, 0, [0] * B
    for r in range(R):
        if per_seq:
            k, win = rule.next_per_seq()
        else:
            k, win = rule.next(), [0] * B
            win = [k] * B
        traces = [od.speculative_round(pair.tg.om, pair.dr.om, st, win[b], T, du[r][b].tolist(), vu[r][b].tolist())
                  for b, st in enumerate(pair.states)]
        if per_seq:
            rule.update_per_seq([t.n_accepted for t in traces], win)
        else:
            rule.update([t.n_accepted for t in traces], k)
        close = False
        for b, t in enumerate(traces):
            gaps = [min(d.final_target - d.final_cdf_lo, d.final_cdf_hi - d.final_target) for d in t.draft_diags]
            gaps.append(min(t.diag.final_target - t.diag.final_cdf_lo, t.diag.final_cdf_hi - t.diag.final_target))
            margins = [abs(float(vu[r][b, i]) - t.diag.accept_ratio[i]) for i in range(min(t.n_accepted + 1, win[b]))]
            close |= min(gaps) < 5e-5 or (bool(margins) and min(margins) < 1e-3)
        same = ks_gpu[r] == k and (not per_seq or win_gpu[r] == win) and kept_gpu[r] == [t.n_accepted for t in traces] and all(
            text_gpu[b][pos[b]:pos[b] + len(t.emitted)] == t.emitted for b, t in enumerate(traces))
        if not same:
            assert close, (f"round {r}: K {ks_gpu[r]} vs {k}, kept {kept_gpu[r]} vs {[t.n_accepted for t in traces]} "
                           "although every decision of the oracle's run was clear of its threshold")
            break
        for b, t in enumerate(traces):
            assert abs(est_gpu[r][b] - rule.accept(b)) < 1e-12
            pos[b] += len(t.emitted)
        rounds_same += 1
        rounds_clear += not close
    assert rounds_same >= 5 and rounds_clear >= 2 and sum(pos) >= 20, (rounds_same, rounds_clear, pos)
    if T > 1.0 and not per_seq:
        assert len(set(ks_gpu[:rounds_same])) >= 2, f"the lookahead should have moved with the data: {ks_gpu}"
    if per_seq:
        assert any(len(set(w)) >= 2 for w in win_gpu[:rounds_same]), f"the windows should have differed: {win_gpu}"
    ctl.close()
