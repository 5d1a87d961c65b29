"""Shared pieces of the GPU parity tests: moving generator-made inputs onto the device in the
library's layouts, and the margin-aware comparison of sampler outputs with the oracle."""
from __future__ import annotations

from typing import List, Sequence

import torch

import oracle
from paper_2411_00853_amd import binding as sv
from paper_2411_00853_amd import workload as wl

ACCEPT_MARGIN = 1e-3    # |u - min(1, p/q)| above which the accept decision must agree
CDF_MARGIN = 1e-6       # distance (in probability mass) of u*S from the chosen token's CDF edges
                        # above which the final token must agree


def device_weights(shape: wl.ModelShape, w_cpu: dict, device="cuda") -> dict:
    """Upload oracle-layout weights ([out][in] row-major) and repack bf16 matrices for the GPU."""
    bf16 = shape.dtype == "bf16"

    def mat(t, interleave=False):
        d = t.to(device)
        return sv.spec_pack_weight(d, interleave) if bf16 else d.contiguous()

    out = {"tok_embed": w_cpu["tok_embed"].to(device).contiguous(),
           "final_norm": w_cpu["final_norm"].to(device).contiguous(),
           "lm_head": mat(w_cpu["lm_head"]), "layers": []}
    for lw in w_cpu["layers"]:
        out["layers"].append({
            "attn_norm": lw["attn_norm"].to(device).contiguous(), "ffn_norm": lw["ffn_norm"].to(device).contiguous(),
            "w_qkv": mat(lw["w_qkv"]), "w_o": mat(lw["w_o"]),
            "w_gate_up": mat(lw["w_gate_up"], interleave=True), "w_down": mat(lw["w_down"])})
    torch.cuda.synchronize()
    return out


class SamplerCheck:
    """Tallies how many decisions were compared exactly and how many fell inside a margin."""

    def __init__(self):
        self.exact_accept = self.margin_accept = self.exact_token = self.margin_token = 0

    def compare(self, tl: torch.Tensor, dl: torch.Tensor, toks: Sequence[int], us: Sequence[float], T: float,
                a_gpu: int, out_gpu: Sequence[int], Kmax: int):
        """One sequence: tl [K+1,V], dl [>=K,V] CPU fp32; GPU results a_gpu, out_gpu (length Kmax+1)."""
        K = len(toks)
        a, out, d = oracle.sample(tl.contiguous(), dl.contiguous(), toks, us, T)
        assert 0 <= a_gpu <= K, (a_gpu, K)
        # positions whose accept test was evaluated by the oracle: 0..min(a, K-1)
        margins = [abs(float(us[i]) - d.accept_ratio[i]) for i in range(min(a + 1, K))]
        if a_gpu != a:
            # admissible only if the two runs part ways at a position whose test is inside the margin
            i = min(a, a_gpu)
            assert i < len(margins) and margins[i] <= ACCEPT_MARGIN, \
                f"n_accepted {a_gpu} != oracle {a}, margins {margins}"
            self.margin_accept += 1
            return
        self.exact_accept += 1
        assert list(out_gpu[:a]) == list(toks[:a])
        assert all(t == -1 for t in out_gpu[a + 1:Kmax + 1])
        y, yg = out[a], int(out_gpu[a])
        lo_gap = d.final_target - d.final_cdf_lo
        hi_gap = d.final_cdf_hi - d.final_target
        if lo_gap > CDF_MARGIN and hi_gap > CDF_MARGIN:
            assert yg == y, f"final token {yg} != oracle {y} (gaps {lo_gap:.3e}, {hi_gap:.3e})"
            self.exact_token += 1
            return
        # inside the band: the GPU's token must still be a valid draw for a CDF moved by the margin
        p = oracle.softmax(tl[a], T)
        if d.final_is_residual:
            r, _ = oracle.residual(p, oracle.softmax(dl[a], T))
        else:
            r = p
        assert 0 <= yg < r.numel() and r[yg] > 0
        c = torch.cumsum(r, 0)
        lo = float(c[yg - 1]) if yg > 0 else 0.0
        assert lo - 2 * CDF_MARGIN <= d.final_target <= float(c[yg]) + 2 * CDF_MARGIN
        self.margin_token += 1


def run_sampler_gpu(tl_rows: torch.Tensor, dl: torch.Tensor, toks: torch.Tensor, us: torch.Tensor,
                    lookahead: Sequence[int], T: float, Kmax: int):
    """Sampler-only step on the GPU.  tl_rows [M,V], dl [B,Kmax,V], toks [B,Kmax], us [B,Kmax+1] (CPU)."""
    B, V = len(lookahead), tl_rows.shape[1]
    h = sv.spec_verify_init(sv.sampler_cfg(V, B, Kmax), None, None, None)
    na = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ot = torch.full((B, Kmax + 1), -7, dtype=torch.int32, device="cuda")
    sv.spec_verify_step(h, lookahead, us.cuda().contiguous(), T, na, ot,
                        draft_tokens=toks.cuda().contiguous() if Kmax else None,
                        draft_logits=dl.cuda().contiguous() if Kmax else None,
                        target_logits_in=tl_rows.cuda().contiguous())
    torch.cuda.synchronize()
    sv.spec_verify_poll(h)
    h.close()
    return na.cpu(), ot.cpu()


def check_sampler_against_oracle(tl_rows, dl, toks, us, lookahead, T, Kmax, na, ot) -> SamplerCheck:
    chk = SamplerCheck()
    r0 = 0
    for b, K in enumerate(lookahead):
        chk.compare(tl_rows[r0:r0 + K + 1], dl[b] if Kmax else torch.zeros(0, tl_rows.shape[1]),
                    toks[b, :K].tolist() if Kmax else [], us[b, :K + 1].tolist(), T, int(na[b]), ot[b].tolist(), Kmax)
        r0 += K + 1
    return chk


class TreeCheck:
    """Margin-aware comparison of one sequence's tree verification with the oracle's."""

    def __init__(self):
        self.exact_walk = self.margin_walk = self.exact_token = self.margin_token = 0

    def compare(self, parent, toks, tl, dl, us, T, a_gpu, path_gpu, out_gpu, Kmax):
        N = len(toks)
        a, path, out, d = oracle.tree_sample(parent, toks, tl.contiguous(), dl.contiguous(), us, T)
        tested = [i for i in range(min(N, 16)) if d.accept_ratio[i] >= 0.0]
        margins = {i: abs(float(us[i]) - d.accept_ratio[i]) for i in tested}
        gp = [int(v) for v in path_gpu[:max(a_gpu, 0)]]
        if a_gpu != a or gp != path:
            # The two walks may only part ways at a node whose own test is inside the margin.  Both
            # try the children of the current node in index order, so after the common prefix the
            # first child on which they decide differently is the lower of the two nodes they keep
            # next (a walk that keeps none tested every child); the oracle tested that node.
            k = 0
            while k < min(len(gp), len(path)) and gp[k] == path[k]:
                k += 1
            nxt = [w[k] for w in (gp, path) if k < len(w)]
            assert nxt, f"walks {gp} and {path} differ in length only by a common prefix"
            node = min(nxt)
            assert node in margins and margins[node] <= ACCEPT_MARGIN, \
                f"walk {gp} != oracle {path}: they part at node {node}, margins {margins}"
            self.margin_walk += 1
            return
        self.exact_walk += 1
        assert list(out_gpu[:a]) == [toks[i] for i in path]
        assert all(t == -1 for t in out_gpu[a + 1:Kmax + 1]) and all(int(v) == -1 for v in path_gpu[a:Kmax])
        lo_gap = d.final_target - d.final_cdf_lo
        hi_gap = d.final_cdf_hi - d.final_target
        # the mass scale of r at level k >= 1 is S_k, so compare gaps relative to it
        scale = d.final_S if d.final_S > 0 else 1.0
        yg = int(out_gpu[a])
        if lo_gap > CDF_MARGIN * scale and hi_gap > CDF_MARGIN * scale:
            assert yg == out[a], f"final token {yg} != oracle {out[a]} (gaps {lo_gap:.3e}, {hi_gap:.3e})"
            self.exact_token += 1
            return
        # inside the band: the GPU's token must still be a valid draw for a CDF moved by the margin.
        # r at the final node after `final_level` rejections: r <- max(0, r/S - q), starting from p
        row = d.final_node + 1
        q = oracle.softmax(dl[row], T)
        r, S = oracle.softmax(tl[row], T), 1.0
        for _ in range(d.final_level):
            r, S = oracle.residual(r / S, q)
        assert 0 <= yg < r.numel() and r[yg] > 0
        c = torch.cumsum(r, 0)
        lo = float(c[yg - 1]) if yg > 0 else 0.0
        assert lo - 2 * CDF_MARGIN * scale <= d.final_target <= float(c[yg]) + 2 * CDF_MARGIN * scale
        self.margin_token += 1
