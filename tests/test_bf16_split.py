"""The arithmetic fact the bf16 gate kernel rests on, checked on the CPU: an fp32 number is the exact sum of
three bf16 numbers (hi = bf16(w), mid = bf16(w - hi), lo = bf16(w - hi - mid), round to nearest even), and a
bf16 x bf16 product is exact in fp32.  Then sum_i x_i*hi_i + x_i*mid_i + x_i*lo_i is a sum of exactly
representable terms of x.Wg: only the order of the fp32 additions separates the kernel from any other fp32
evaluation of the gate logits (paper Sec. 5.4 leaves that order open)."""
import numpy as np
import torch


def _split(w: torch.Tensor):
    hi = w.bfloat16()
    r1 = w - hi.float()
    mid = r1.bfloat16()
    r2 = r1 - mid.float()
    lo = r2.bfloat16()
    return hi, mid, lo


def test_three_bf16_pieces_reconstruct_fp32_exactly():
    g = torch.Generator().manual_seed(0)
    # gate-weight-like values, wide dynamic range, exact powers of two, values with all 24 bits set
    parts = [0.02 * torch.randn(200000, generator=g),
             torch.randn(200000, generator=g) * torch.exp2(torch.randint(-60, 60, (200000,), generator=g).float()),
             torch.exp2(torch.arange(-100, 100).float()),
             torch.tensor([16777215.0, -16777215.0, 1.0 + 2.0 ** -23, 1.0 - 2.0 ** -24, 0.0, -0.0, 3.3e38])]   # beyond the largest finite bf16 (3.39e38) hi would round to infinity
    w = torch.cat(parts).float()
    hi, mid, lo = _split(w)
    rec = hi.double() + mid.double() + lo.double()
    assert torch.equal(rec, w.double())
    # the residuals were exact in fp32 (nothing was lost on the way)
    assert torch.equal((w.double() - hi.double()).float().double(), w.double() - hi.double())


def test_bf16_products_are_exact_in_fp32():
    g = torch.Generator().manual_seed(1)
    a = torch.randn(100000, generator=g).bfloat16()
    b = (0.02 * torch.randn(100000, generator=g)).bfloat16()
    exact = a.double() * b.double()
    assert torch.equal((a.float() * b.float()).double(), exact)


def test_split_logits_match_fp64_reference():
    g = torch.Generator().manual_seed(2)
    x = torch.randn(64, 512, generator=g).bfloat16()
    w = 0.02 * torch.randn(512, 48, generator=g)
    hi, mid, lo = _split(w)
    ref = x.double() @ w.double()
    got = x.double() @ hi.double() + x.double() @ mid.double() + x.double() @ lo.double()
    assert np.max(np.abs((got - ref).numpy())) < 1e-12
