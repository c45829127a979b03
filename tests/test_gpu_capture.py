"""hook_capture_qk against its reference: pure data movement, so bit for bit (needs an MI355X)."""
import pytest
import torch

from oracle.capture import capture_qk
from paper_2603_06588_amd import workloads as W
from helpers import bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(b_cpu, kvh):
    from paper_2603_06588_amd import binding
    want_q, want_k, cu_k = capture_qk(b_cpu.q, b_cpu.k_cache, b_cpu.block_table, b_cpu.seq_lens, b_cpu.cu_q_lens,
                                      b_cpu.probe_heads, b_cpu.max_sel_q, b_cpu.query_sel, kvh)
    b = b_cpu.to(DEV)
    q_out, k_out = binding.hook_capture_qk(b.q, b.k_cache, b.block_table, b.seq_lens, b.cu_q_lens, b.probe_heads,
                                           b.max_sel_q, b.query_sel, kvh.to(DEV), cu_k.to(DEV), int(cu_k[-1]))
    torch.cuda.synchronize()
    assert torch.equal(bits(q_out), bits(want_q))
    assert torch.equal(bits(k_out), bits(want_k))


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64)])
def test_capture_matches_reference(dtype, d):
    b = W.random_batch(300, [333, 17, 64, 1000], [333, 1, 10, 1], 8, 2, d, dtype, num_probe_heads=5, max_sel_q=6,
                       poison=False)
    _run(b, torch.tensor([1, 0], dtype=torch.int32))
    _run(b, torch.tensor([1], dtype=torch.int32))


def test_capture_with_empty_sequence_and_no_selection():
    b = W.random_batch(301, [40, 0, 25], [40, 0, 25], 4, 4, 128, torch.bfloat16, num_probe_heads=2, max_sel_q=3,
                       poison=False)
    b.query_sel[0, 0], b.query_sel[0, 1] = 5, 5   # empty selection
    _run(b, torch.tensor([0, 3], dtype=torch.int32))


def test_capture_c2_shape():
    b = W.c2_prefill_8b(shrink=2)
    kvh = torch.unique(b.probe_heads // 4).to(torch.int32)
    _run(b, kvh)


def test_capture_with_invalid_device_contents_completes():
    from paper_2603_06588_amd import binding
    b = W.random_batch(302, [40, 70, 25], [40, 1, 25], 4, 4, 128, torch.bfloat16, num_probe_heads=2, max_sel_q=3,
                       poison=False).to(DEV)
    kvh = torch.tensor([0, 99, -3], dtype=torch.int32, device=DEV)            # out-of-range heads: clamped
    cu_k = torch.tensor([0, 40, 110, 135], dtype=torch.int32, device=DEV)
    b.block_table = torch.full_like(b.block_table, -7)                         # out-of-range ids: clamped
    b.query_sel = b.query_sel.clone()
    b.query_sel[0, 0], b.query_sel[0, 1] = -2**31, 2**31 - 1
    ph = torch.tensor([1, 77], dtype=torch.int32, device=DEV)                  # head 77 does not exist
    q_out, k_out = binding.hook_capture_qk(b.q, b.k_cache, b.block_table, b.seq_lens, b.cu_q_lens, ph, 3,
                                           b.query_sel, kvh, cu_k, 135)
    torch.cuda.synchronize()
    assert torch.isfinite(k_out.float()).all() and (q_out[:, 1] == 0).all()
    # a prefix-sum array that does not match the lengths: positions beyond a sequence's length read as zero
    cu_bad = torch.tensor([0, 60, 110, 135], dtype=torch.int32, device=DEV)
    _, k2 = binding.hook_capture_qk(b.q, b.k_cache, b.block_table, b.seq_lens, b.cu_q_lens, None, 1, None, kvh[:1],
                                    cu_bad, 135)
    torch.cuda.synchronize()
    assert (k2[40:60] == 0).all()
