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


# ---- writing the new tokens' K/V into the paged cache ----

@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_kv_write_matches_reference(dtype, d):
    from oracle.capture import kv_write
    from paper_2603_06588_amd import binding
    b = W.random_batch(310, [333, 17, 64, 1000, 9], [100, 1, 64, 1, 0], 8, 2, d, dtype, num_probe_heads=1, max_sel_q=1,
                       poison=False)
    gen = torch.Generator().manual_seed(311)
    k_new = torch.randn((b.total_q, 2, d), generator=gen).to(dtype)
    v_new = torch.randn((b.total_q, 2, d), generator=gen).to(dtype)
    want_k, want_v = kv_write(k_new, v_new, b.block_table, b.seq_lens, b.cu_q_lens, b.k_cache, b.v_cache)
    bd = b.to(DEV)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), bd.block_table, bd.seq_lens, bd.cu_q_lens, bd.k_cache,
                          bd.v_cache)
    torch.cuda.synchronize()
    assert torch.equal(bits(bd.k_cache.cpu()), bits(want_k)) and torch.equal(bits(bd.v_cache.cpu()), bits(want_v))


def test_kv_write_then_attention_and_invalid_contents():
    """The written cache feeds the attention call; nonsense ids and lengths drop writes, never fault."""
    import oracle
    from oracle.capture import kv_write
    from paper_2603_06588_amd import binding
    from helpers import compare_with_oracle
    b = W.random_batch(312, [300, 150, 700], [300, 1, 20], 8, 2, 128, torch.bfloat16, std=1.0, num_probe_heads=2,
                       max_sel_q=2, max_spans=2)
    gen = torch.Generator().manual_seed(313)
    k_new = torch.randn((b.total_q, 2, 128), generator=gen).to(torch.bfloat16)
    v_new = torch.randn((b.total_q, 2, 128), generator=gen).to(torch.bfloat16)
    bd = b.to(DEV)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), bd.block_table, bd.seq_lens, bd.cu_q_lens, bd.k_cache,
                          bd.v_cache)
    out, mass = binding.hook_attn_probe_batch(bd)
    torch.cuda.synchronize()
    b.k_cache, b.v_cache = kv_write(k_new, v_new, b.block_table, b.seq_lens, b.cu_q_lens, b.k_cache, b.v_cache)
    compare_with_oracle(b, out, mass, label="after kv_write")
    before_k = bd.k_cache.clone()
    bad_table = torch.full_like(bd.block_table, 0x7FFFFFF0)
    bad_lens = torch.tensor([2**31 - 1, -5, 3], dtype=torch.int32, device=DEV)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), bad_table, bd.seq_lens, bd.cu_q_lens, bd.k_cache, bd.v_cache)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), bd.block_table, bad_lens, bd.cu_q_lens, bd.k_cache, bd.v_cache)
    torch.cuda.synchronize()
    assert torch.equal(bits(bd.k_cache), bits(before_k))
