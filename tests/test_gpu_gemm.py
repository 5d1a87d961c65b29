"""GPU parity of the projection GEMMs against the oracle's matrix-vector product."""
import pytest
import torch

import oracle
from paper_2411_00853_amd import workload as wl

pytestmark = pytest.mark.gpu


def _case(M, N, K, seed):
    rng = wl.Rng(seed, "cpu")
    x = rng.normal(1, (M, K), 1.0)
    w = rng.normal(2, (N, K), 0.02, torch.bfloat16)
    return x, w


def _oracle_rows(w, x, rows):
    return torch.stack([oracle.linear(w, x[r].contiguous()) for r in rows])


@pytest.mark.parametrize("M,N,K", [
    (1, 64, 32), (6, 3072, 2048), (5, 100, 64), (16, 48, 96), (17, 1000, 320),
    (48, 4096, 4096), (48, 1024, 11008), (33, 2064, 512), (64, 256, 4096),
    (80, 304, 512), (100, 512, 1024), (128, 384, 256), (140, 96, 640), (176, 272, 512), (192, 400, 512),
    (220, 208, 384), (250, 128, 2048), (280, 144, 320), (300, 64, 256), (352, 640, 1024), (157, 352, 1024),
    # many columns: the variants with four column tiles per wavefront
    (8, 6000, 64), (20, 5504, 128), (40, 5456, 96), (64, 5632, 256), (75, 5440, 96), (90, 5440, 64), (185, 5440, 64),
])
@pytest.mark.parametrize("split", [True, False])
def test_bf16_gemm_matches_oracle(M, N, K, split):
    from paper_2411_00853_amd import binding as sv
    x, w = _case(M, N, K, 100 + M + N)
    wp = sv.spec_pack_weight(w.cuda())
    y = sv.spec_k_gemm_bf16(x.cuda(), wp, N, split_x=split)
    torch.cuda.synchronize()
    rows = sorted(set([0, M // 2, M - 1] + list(range(0, M, max(1, M // 5)))))
    want = _oracle_rows(w, x, rows)
    got = y.cpu()[rows]
    scale = want.double().pow(2).mean().sqrt().item()
    err = (got.double() - want.double()).abs().max().item()
    # activations as bf16 head + remainder: only fp32 accumulation order and 2^-17 truncation remain;
    # a single bf16 rounding of the activations costs ~2^-9 per term
    assert err < (3e-5 if split else 1.5e-2) * scale, (err, scale)
    # rows the oracle did not visit agree with a library product at the same tolerance
    full = x.double() @ w.double().T
    assert (y.cpu().double() - full).abs().max().item() < (3e-5 if split else 1.5e-2) * scale


def test_gate_up_interleaved_packing_round_trip():
    # tiles alternate between the two halves of the matrix: column 32t+c is gate unit 16t+c and
    # column 32t+16+c is up unit 16t+c
    from paper_2411_00853_amd import binding as sv
    M, F, K = 7, 96, 64
    x, w = _case(M, 2 * F, K, 9)
    wp = sv.spec_pack_weight(w.cuda(), interleave_halves=True)
    y = sv.spec_k_gemm_bf16(x.cuda(), wp, 2 * F).cpu()
    full = (x.double() @ w.double().T)
    idx = torch.arange(F)
    col_gate = (idx // 16) * 32 + idx % 16
    assert (y[:, col_gate].double() - full[:, :F]).abs().max() < 1e-5
    assert (y[:, col_gate + 16].double() - full[:, F:]).abs().max() < 1e-5


@pytest.mark.parametrize("M,N,K", [(5, 768, 256), (5, 1024, 256), (3, 50, 70), (40, 33, 129)])
def test_fp32_gemm_matches_oracle(M, N, K):
    from paper_2411_00853_amd import binding as sv
    rng = wl.Rng(7, "cpu")
    x = rng.normal(1, (M, K), 1.0)
    w = rng.normal(2, (N, K), 0.05)
    y = sv.spec_k_gemm_f32(x.cuda(), w.cuda()).cpu()
    want = _oracle_rows(w, x, range(M))
    assert (y.double() - want.double()).abs().max().item() < 2e-6 * (1 + want.abs().max().item()) * K ** 0.5


def test_gemm_is_reproducible_bit_for_bit():
    from paper_2411_00853_amd import binding as sv
    x, w = _case(48, 2048, 4096, 5)
    wp = sv.spec_pack_weight(w.cuda())
    xd = x.cuda()
    a = sv.spec_k_gemm_bf16(xd, wp, 2048).clone()
    b = sv.spec_k_gemm_bf16(xd, wp, 2048).clone()
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("M,N,K", [(120, 352, 1024), (157, 352, 1024), (185, 5440, 64), (192, 400, 512)])
@pytest.mark.parametrize("balanced", [True, False])
def test_many_row_gemm_both_workgroup_shapes(M, N, K, balanced):
    """Launches of more than 112 rows that fill too few compute units take twelve column tiles per
    workgroup either as four column groups of three tiles (eight wavefronts, the default) or as three
    groups of four (six wavefronts): both against a library product, and bit-identical to each other
    (the same products are added in the same order)."""
    from paper_2411_00853_amd import binding as sv
    x, w = _case(M, N, K, 300 + M)
    wp = sv.spec_pack_weight(w.cuda())
    sv.spec_k_set_gemm_balance_groups(balanced)
    try:
        y = sv.spec_k_gemm_bf16(x.cuda(), wp, N).cpu()
    finally:
        sv.spec_k_set_gemm_balance_groups(True)
    full = x.double() @ w.double().T
    scale = full.pow(2).mean().sqrt().item()
    assert (y.double() - full).abs().max().item() < 3e-5 * scale
    y2 = sv.spec_k_gemm_bf16(x.cuda(), wp, N).cpu()
    assert torch.equal(y, y2)
