"""hook_steer against the CPU oracle (needs an MI355X)."""
import pytest
import torch

import oracle
from paper_2603_06588_amd import workloads as W
from helpers import bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ulp_diff(a: torch.Tensor, b: torch.Tensor) -> int:
    """Largest distance in units of the last place between same-dtype tensors (finite values)."""
    ia, ib = bits(a).to(torch.int64), bits(b).to(torch.int64)
    if a.dtype == torch.bfloat16:
        ia, ib = ia & 0xFFFF, ib & 0xFFFF
        sign = 0x8000
    else:
        ia, ib = ia & 0xFFFFFFFF, ib & 0xFFFFFFFF
        sign = 0x80000000
    # map sign-magnitude to a monotone integer line
    ma = torch.where(ia >= sign, sign - ia, ia)
    mb = torch.where(ib >= sign, sign - ib, ib)
    return int((ma - mb).abs().max())


def _run(s):
    from paper_2603_06588_amd import binding
    d = s.to(DEV)
    binding.hook_steer(d.hidden, d.vec, d.alpha, d.token_mask)
    torch.cuda.synchronize()
    return d.hidden.cpu()


@pytest.mark.parametrize("dtype,T,D", [(torch.bfloat16, 300, 4096), (torch.bfloat16, 17, 520), (torch.float32, 65, 512),
                                       (torch.float32, 9, 36)])
def test_steer_matches_oracle_within_one_ulp(dtype, T, D):
    s = W.steer_batch(200 + T, T, D, dtype, alpha=3.25, mask_frac=0.6)
    want = oracle.steer_batch(s)
    got = _run(s)
    keep = s.token_mask == 0
    assert torch.equal(bits(got)[keep], bits(s.hidden)[keep])      # unmasked rows bit-identical
    assert _ulp_diff(got, want) <= 1


def test_steer_alpha_zero_and_empty_mask_are_bit_identical():
    s = W.steer_batch(210, 40, 256, torch.bfloat16, alpha=0.0)
    s.hidden[3, 5] = float("nan")
    s.hidden[4, 6] = -0.0
    assert torch.equal(bits(_run(s)), bits(s.hidden))
    s.alpha = 5.0
    s.token_mask.zero_()
    assert torch.equal(bits(_run(s)), bits(s.hidden))


def test_steer_cancels_row_exactly():
    s = W.steer_batch(211, 12, 128, torch.float32, alpha=1.0)
    s.token_mask.zero_()
    s.token_mask[7] = 1
    s.vec = -s.hidden[7].clone()
    got = _run(s)
    assert (got[7] == 0).all()


def test_c1_and_c5_steer():
    _, s1 = W.c1_tiny_prefill()
    assert _ulp_diff(_run(s1), oracle.steer_batch(s1)) <= 1
    _, s5 = W.c5_mixed()
    got, want = _run(s5), oracle.steer_batch(s5)
    assert _ulp_diff(got, want) <= 1
    # the 192 padding rows and the 64 decode rows are untouched
    keep = s5.token_mask == 0
    assert int(keep.sum()) == 64 + 192
    assert torch.equal(bits(got)[keep], bits(s5.hidden)[keep])


# ---- steering fused into the residual add ----

@pytest.mark.parametrize("dtype,T,D", [(torch.bfloat16, 300, 4096), (torch.bfloat16, 17, 520), (torch.float32, 65, 512),
                                       (torch.float32, 9, 36)])
def test_residual_steer_matches_oracle(dtype, T, D):
    from paper_2603_06588_amd import binding
    s = W.steer_batch(300 + T, T, D, dtype, alpha=3.25, mask_frac=0.6)
    gen = torch.Generator().manual_seed(77 + T)
    delta = (torch.randn((T, D), generator=gen) * 2).to(dtype)
    delta[1] = (-s.hidden[1].double()).to(dtype)        # exact cancellation of h + d on one row
    want = oracle.residual_steer(s.hidden, delta, s.vec, s.alpha, s.token_mask)
    d = s.to(DEV)
    binding.hook_residual_add_steer(d.hidden, delta.to(DEV), d.vec, d.alpha, d.token_mask)
    torch.cuda.synchronize()
    got = d.hidden.cpu()
    assert _ulp_diff(got, want) <= 1
    # the kernel adds the same three fp64 terms in the same order, so in practice every bit agrees
    assert int((bits(got) != bits(want)).sum()) == 0
    # plain residual add: null mask, and alpha = 0
    want0 = oracle.residual_steer(s.hidden, delta, s.vec, 0.0, None)
    for alpha, mask in ((3.0, None), (0.0, s.token_mask.to(DEV))):
        h = s.hidden.to(DEV).clone()
        binding.hook_residual_add_steer(h, delta.to(DEV), d.vec, alpha, mask)
        torch.cuda.synchronize()
        assert torch.equal(bits(h.cpu()), bits(want0))


def test_residual_steer_rounding_corner_cases_are_bit_exact():
    """Inputs built to sit where an fp32 evaluation cannot be trusted to round like the fp64 sum:
    results on or next to the midpoint of two bf16 neighbours, cancelling terms, huge exponent gaps,
    subnormal / overflowing results, infinities and NaNs.  Every bit must equal the oracle's."""
    from paper_2603_06588_amd import binding
    gen = torch.Generator().manual_seed(4242)
    T, D = 96, 1024
    h = torch.randn((T, D), generator=gen).to(torch.bfloat16)
    d = torch.randn((T, D), generator=gen).to(torch.bfloat16)
    vec = torch.randn((D,), generator=gen).to(torch.bfloat16)
    # rows 0-15: h = 1 + k 2^-7 (bf16 neighbours), d = 0, alpha * v = 2^-8 +- tiny: exact midpoints and near misses
    k = torch.arange(D) % 64
    for r in range(16):
        h[r] = (1.0 + k.double() * 2.0 ** -7).to(torch.bfloat16)
        d[r] = 0.0
    # rows 16-31: h + d cancels to something far smaller than either, then alpha * v decides
    for r in range(16, 32):
        d[r] = (-h[r].double() * (1.0 + 2.0 ** -(r - 14))).to(torch.bfloat16)
    # rows 32-47: exponent gaps beyond 24 bits between the terms
    for r in range(32, 48):
        d[r] = (h[r].double() * 2.0 ** -(20 + r - 32)).to(torch.bfloat16)
    # rows 48-63: tiny and huge magnitudes (subnormal / overflowing sums)
    h[48:56] = (h[48:56].double() * 2.0 ** -125).to(torch.bfloat16)
    d[48:56] = (d[48:56].double() * 2.0 ** -126).to(torch.bfloat16)
    h[56:64] = (h[56:64].double().sign() * 3.0e38).to(torch.bfloat16)
    d[56:64] = (d[56:64].double().abs() * 1.0e37 * h[56:64].double().sign()).to(torch.bfloat16)
    # rows 64-71: infinities and NaNs in every operand position
    h[64, ::3] = float("inf"); d[65, ::5] = float("-inf"); h[66, ::7] = float("nan"); d[67, ::2] = float("nan")
    h[68, ::4] = float("inf"); d[68, ::4] = float("-inf")
    mask = torch.ones(T, dtype=torch.uint8)
    mask[80:] = 0
    for alpha, v_scale in ((2.0 ** -8, None), (3.25, 1.0), (1.0e-30, 1.0), (-7.0e5, 1.0)):
        v = vec.clone()
        if v_scale is None:     # v = 1 (+- one bf16 step on some columns): alpha * v = 2^-8 exactly or a hair off
            v = torch.ones(D).to(torch.bfloat16)
            v[1::3] = (1.0 + 2.0 ** -7)
            v[2::3] = (1.0 - 2.0 ** -8)
        want = oracle.residual_steer(h, d, v, alpha, mask)
        hh = h.to(DEV).clone()
        binding.hook_residual_add_steer(hh, d.to(DEV), v.to(DEV), alpha, mask.to(DEV))
        torch.cuda.synchronize()
        got = hh.cpu()
        nan_w, nan_g = torch.isnan(want.float()), torch.isnan(got.float())
        assert torch.equal(nan_w, nan_g), alpha
        same = (bits(got) == bits(want)) | nan_w
        assert bool(same.all()), (alpha, int((~same).sum()))


def test_residual_steer_c5_shape_sampled():
    from paper_2603_06588_amd import binding
    _, s = W.c5_mixed()
    gen = torch.Generator().manual_seed(5)
    delta = torch.randn(s.hidden.shape, generator=gen).to(s.hidden.dtype)
    rows = torch.cat([torch.arange(0, 70), torch.arange(8250, 8448), torch.randint(70, 8250, (64,), generator=gen)])
    want = oracle.residual_steer(s.hidden[rows], delta[rows], s.vec, s.alpha, s.token_mask[rows])
    d = s.to(DEV)
    binding.hook_residual_add_steer(d.hidden, delta.to(DEV), d.vec, d.alpha, d.token_mask)
    torch.cuda.synchronize()
    assert _ulp_diff(d.hidden.cpu()[rows], want) <= 1
