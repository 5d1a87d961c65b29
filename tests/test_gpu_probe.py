"""GPU: the register layout assumed for the bf16 matrix instruction, and the yardstick copy kernel."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_mfma_tile_layout():
    from paper_2411_00853_amd import binding as sv
    g = torch.Generator().manual_seed(0)
    a = torch.randn(16, 32, generator=g).to(torch.bfloat16)
    b = torch.randn(32, 16, generator=g).to(torch.bfloat16)
    d = torch.zeros(16, 16, dtype=torch.float32, device="cuda")
    sv.spec_k_mfma_tile(a.cuda(), b.cuda(), d)
    torch.cuda.synchronize()
    want = a.double() @ b.double()
    assert (d.cpu().double() - want).abs().max() < 1e-4


def test_copy_and_read_kernels():
    from paper_2411_00853_amd import binding as sv
    src = torch.arange(1 << 20, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    sv.spec_k_copy(src, dst)
    out = torch.zeros(256 * 16 * 256, dtype=torch.float32, device="cuda")
    ones = torch.ones(3 * 1024 * 1024 + 64, dtype=torch.float32, device="cuda")
    sv.spec_k_read(ones, out)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert out.sum().item() == ones.numel()
