"""Block ids whose byte offsets lie beyond 4 GiB: a small batch is relocated into a large device-side block
pool so that every cache address the kernels form needs more than 32 bits (needs an MI355X, about 11 GB of
device memory).  Values are those of the small CPU batch, which is what the oracle sees."""
import pytest
import torch

from paper_2603_06588_amd import binding, workloads as W
from helpers import bits, compare_with_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BIG_BLOCKS = 172_000            # x 32 KB per block (8 kv heads, d 128, bf16) = 5.6 GB per cache


def _relocate(b_cpu, big_blocks=BIG_BLOCKS, seed=0):
    """The batch on the device with its live blocks moved to ids above the 4 GiB mark of a big pool."""
    b = b_cpu.to(DEV)
    Hkv, B, d = b.k_cache.shape[1:]
    block_bytes = Hkv * B * d * b.k_cache.element_size()
    first_high = (1 << 32) // block_bytes + 1
    assert big_blocks > first_high + b.k_cache.shape[0]
    gen = torch.Generator().manual_seed(seed)
    new_ids = (first_high + torch.randperm(big_blocks - first_high, generator=gen)[: b.k_cache.shape[0]]).to(torch.int64)
    kbig = torch.full((big_blocks, Hkv, B, d), float("nan"), dtype=b.k_cache.dtype, device=DEV)
    vbig = torch.full_like(kbig, float("nan"))
    kbig[new_ids.to(DEV)] = b.k_cache
    vbig[new_ids.to(DEV)] = b.v_cache
    table = b.block_table.clone()
    live = (table >= 0) & (table < b.k_cache.shape[0])
    table[live] = new_ids.to(DEV)[table[live].long()].to(torch.int32)
    table[~live] = big_blocks + 12345           # dead entries stay out of range
    kw = dict(b.__dict__)
    kw.update(k_cache=kbig, v_cache=vbig, block_table=table, num_blocks=big_blocks)
    return type(b)(**kw), new_ids


def test_attention_with_block_offsets_beyond_4_gib():
    """Query chunks (direct-to-LDS loads), single rows (register streaming, planned and self-planned)."""
    b_cpu = W.random_batch(1301, [700, 90, 1300, 260, 2100, 33], [700, 1, 300, 1, 1, 33], 32, 8, 128, torch.bfloat16,
                           num_probe_heads=6, max_sel_q=4, max_spans=3)
    big, _ = _relocate(b_cpu)
    out = torch.full_like(big.q, float("nan"))
    call = binding.call_from_batch(big, out=out)
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() == 0
    print(compare_with_oracle(b_cpu, call.out, call.mass, label="large_pool_mixed"), flush=True)
    # the decode-only part once more through the self-planned path
    d_cpu = W.random_batch(1302, [2100, 90, 1300, 260], [1, 1, 1, 1], 32, 8, 128, torch.bfloat16, num_probe_heads=6,
                           max_sel_q=1, max_spans=3)
    d_cpu.query_sel[:, 0], d_cpu.query_sel[:, 1] = 0, 1
    dbig, _ = _relocate(d_cpu, seed=1)
    out = torch.full_like(dbig.q, float("nan"))
    call = binding.call_from_batch(dbig, out=out, batch_kind=binding.BATCH_DECODE_ONLY)
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() == 0
    print(compare_with_oracle(d_cpu, call.out, call.mass, label="large_pool_decode"), flush=True)


def test_cache_write_and_capture_with_block_offsets_beyond_4_gib():
    from oracle.capture import capture_qk, kv_write
    b_cpu = W.random_batch(1303, [333, 17, 64, 1000], [100, 1, 64, 1], 32, 8, 128, torch.bfloat16, num_probe_heads=3,
                           max_sel_q=2, poison=False)
    big, new_ids = _relocate(b_cpu, seed=2)
    gen = torch.Generator().manual_seed(1304)
    k_new = torch.randn((b_cpu.total_q, 8, 128), generator=gen).to(torch.bfloat16)
    v_new = torch.randn((b_cpu.total_q, 8, 128), generator=gen).to(torch.bfloat16)
    want_k, want_v = kv_write(k_new, v_new, b_cpu.block_table, b_cpu.seq_lens, b_cpu.cu_q_lens, b_cpu.k_cache,
                              b_cpu.v_cache)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), big.block_table, big.seq_lens, big.cu_q_lens, big.k_cache,
                          big.v_cache)
    torch.cuda.synchronize()
    assert torch.equal(bits(big.k_cache[new_ids.to(DEV)]), bits(want_k))
    assert torch.equal(bits(big.v_cache[new_ids.to(DEV)]), bits(want_v))
    # capture reads the rows just written, through the relocated table
    after = b_cpu.to("cpu")
    kvh = torch.arange(8, dtype=torch.int32)
    cu_k = torch.zeros(b_cpu.num_seqs + 1, dtype=torch.int32)
    cu_k[1:] = torch.cumsum(b_cpu.seq_lens, 0)
    total_k = int(cu_k[-1])
    ref_q, ref_k, ref_cu = capture_qk(after.q, want_k, after.block_table, after.seq_lens, after.cu_q_lens,
                                      after.probe_heads, after.max_sel_q, after.query_sel, kvh)
    assert ref_cu.tolist() == cu_k.tolist()
    got_q, got_k = binding.hook_capture_qk(big.q, big.k_cache, big.block_table, big.seq_lens, big.cu_q_lens,
                                           big.probe_heads, big.max_sel_q, big.query_sel, kvh.to(DEV), cu_k.to(DEV),
                                           total_k)
    torch.cuda.synchronize()
    assert torch.equal(bits(got_q), bits(ref_q)) and torch.equal(bits(got_k), bits(ref_k))
