"""hook_reduce_mass against its fp64 reference (needs an MI355X)."""
import numpy as np
import pytest
import torch

from oracle.reduce import RATIO_MEAN, RATIO_OF_SUMS, SPAN_MEAN, reduce_mass
from paper_2603_06588_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-6   # fp32 sums of at most a few thousand terms in [0, 1] with weights of order one


def _check(mass, mode, sel=None, cu=None, w=None, a=0, b=1):
    from paper_2603_06588_amd import binding
    want = reduce_mass(mass.numpy(), mode, a, b, None if sel is None else sel.tolist(),
                       None if cu is None else cu.tolist(), None if w is None else w.tolist())
    dv = lambda t: None if t is None else t.to(DEV)
    got = binding.hook_reduce_mass(mass.to(DEV), mode, a, b, dv(sel), dv(cu), dv(w))
    torch.cuda.synchronize()
    scale = 1.0 if w is None else float(w.abs().sum())
    assert np.abs(got.cpu().double().numpy() - want).max() <= TOL * max(scale, 1.0)
    # accumulate: a second call adds the same amount; repeated runs are bit-identical
    again = binding.hook_reduce_mass(mass.to(DEV), mode, a, b, dv(sel), dv(cu), dv(w))
    assert torch.equal(got, again)
    acc = binding.hook_reduce_mass(mass.to(DEV), mode, a, b, dv(sel), dv(cu), dv(w), scores=got.clone(),
                                   accumulate=True)
    torch.cuda.synchronize()
    assert np.abs(acc.cpu().double().numpy() - 2 * want).max() <= 2 * TOL * max(scale, 1.0)


@pytest.mark.parametrize("mode", [SPAN_MEAN, RATIO_MEAN, RATIO_OF_SUMS])
def test_reduce_random(mode):
    g = torch.Generator().manual_seed(17)
    mass = torch.rand((37, 12, 8, 5), generator=g) * 0.2
    mass[3] = 0.0
    sel = torch.tensor([[i % 7 - 1, i % 7 - 1 + (i % 10)] for i in range(37)], dtype=torch.int32)
    n = torch.tensor([(i * 5) % 23 for i in range(37)], dtype=torch.int32)
    cu = torch.zeros(38, dtype=torch.int32)
    cu[1:] = torch.cumsum(n, 0)
    w = torch.randn(12, generator=g)
    _check(mass, mode)
    _check(mass, mode, sel, cu, w, a=4, b=2)
    _check(mass, mode, sel, None, None, a=1, b=1)


def test_reduce_on_probe_output():
    """End to end on device: probe a small batch, reduce its mass, compare with the oracle chain."""
    import oracle
    from paper_2603_06588_amd import binding
    b = W.random_batch(41, [300, 150, 64, 700], [300, 1, 64, 20], 8, 2, 128, torch.bfloat16, num_probe_heads=4,
                       max_sel_q=5, max_spans=3)
    _, mass_ref = oracle.attn_probe_batch(b)
    want = reduce_mass(mass_ref.numpy(), RATIO_MEAN, 0, 2, b.query_sel.tolist(), b.cu_q_lens.tolist())
    bd = b.to(DEV)
    _, mass = binding.hook_attn_probe_batch(bd)
    got = binding.hook_reduce_mass(mass, RATIO_MEAN, 0, 2, bd.query_sel, bd.cu_q_lens)
    torch.cuda.synchronize()
    assert np.abs(got.cpu().double().numpy() - want).max() <= 2e-3


def test_reduce_large_many_rows():
    g = torch.Generator().manual_seed(5)
    mass = torch.rand((3, 16, 512, 8), generator=g) / 512
    for mode in (SPAN_MEAN, RATIO_MEAN, RATIO_OF_SUMS):
        _check(mass, mode, a=7, b=0)
