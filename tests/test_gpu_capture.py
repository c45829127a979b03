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


# ---- quantising write into an 8-bit (E4M3) cache ----

def test_kv_write_quantises_into_fp8_cache_like_the_reference():
    """Bytes written by the library equal the oracle's search-the-table quantiser, on random rows and on
    rows built from midpoints of the format, saturating, tiny, signed-zero and NaN values."""
    from oracle.capture import kv_write
    from paper_2603_06588_amd import binding
    b = W.random_batch(320, [333, 17, 64, 1000, 9], [100, 1, 64, 1, 0], 8, 2, 128, torch.bfloat16, num_probe_heads=1,
                       max_sel_q=1, poison=False)
    b8 = W.fp8_cache_variant(b, 321, k_std=1.0, v_std=0.3)
    gen = torch.Generator().manual_seed(322)
    k_new = (torch.randn((b.total_q, 2, 128), generator=gen) * 1.5).to(torch.bfloat16)
    v_new = (torch.randn((b.total_q, 2, 128), generator=gen) * 0.4).to(torch.bfloat16)
    ks, vs = b8.k_scale.tolist(), b8.v_scale.tolist()
    # row 5: every number of the format and the midpoints between neighbours, times the head's scale
    vals = torch.arange(0x7F, dtype=torch.uint8).view(torch.float8_e4m3fn).double()
    mids = (vals[:-1] + vals[1:]) / 2
    special = torch.cat([mids[:120], torch.tensor([500.0, 1e6, -1e6, 2.0 ** -10, 2.0 ** -11, -2.0 ** -11, -0.0, 0.0])])
    for g in range(2):
        k_new[5, g] = (special * ks[g]).to(torch.bfloat16)
        v_new[5, g] = (-special * vs[g]).to(torch.bfloat16)
    k_new[6, 0, :4] = torch.tensor([float("nan"), float("inf"), float("-inf"), 0.0]).to(torch.bfloat16)
    want_k, want_v = kv_write(k_new, v_new, b8.block_table, b8.seq_lens, b8.cu_q_lens, b8.k_cache, b8.v_cache,
                              b8.k_scale, b8.v_scale)
    bd = b8.to(DEV)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), bd.block_table, bd.seq_lens, bd.cu_q_lens, bd.k_cache,
                          bd.v_cache, k_scale=bd.k_scale, v_scale=bd.v_scale)
    torch.cuda.synchronize()
    got_k, got_v = bd.k_cache.cpu(), bd.v_cache.cpu()
    for got, want in ((got_k, want_k), (got_v, want_v)):
        nan_w, nan_g = (want & 0x7F) == 0x7F, (got & 0x7F) == 0x7F
        assert torch.equal(nan_w, nan_g)
        diff = (got != want) & ~nan_w
        assert int(diff.sum()) == 0, (got[diff][:8], want[diff][:8])


def test_kv_write_quantises_every_bf16_pattern_like_the_reference():
    """All 65536 bf16 bit patterns (NaNs, infinities, subnormals, both zeros included) as keys, and in
    another order as values, under scales that are not powers of two."""
    from oracle.capture import kv_write
    from paper_2603_06588_amd import binding
    b = W.random_batch(330, [512], [512], 2, 1, 128, torch.bfloat16, num_probe_heads=1, max_sel_q=1, poison=False)
    b8 = W.fp8_cache_variant(b, 331, k_std=1.3, v_std=0.021)
    pats = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    k_new = pats.view(torch.bfloat16).reshape(512, 1, 128).clone()
    v_new = pats.roll(12345).view(torch.bfloat16).reshape(512, 1, 128).clone()
    want_k, want_v = kv_write(k_new, v_new, b8.block_table, b8.seq_lens, b8.cu_q_lens, b8.k_cache, b8.v_cache,
                              b8.k_scale, b8.v_scale)
    bd = b8.to(DEV)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), bd.block_table, bd.seq_lens, bd.cu_q_lens, bd.k_cache,
                          bd.v_cache, k_scale=bd.k_scale, v_scale=bd.v_scale)
    torch.cuda.synchronize()
    for got, want in ((bd.k_cache.cpu(), want_k), (bd.v_cache.cpu(), want_v)):
        nan_w, nan_g = (want & 0x7F) == 0x7F, (got & 0x7F) == 0x7F
        assert torch.equal(nan_w, nan_g)
        diff = (got != want) & ~nan_w
        assert int(diff.sum()) == 0, (got[diff][:8], want[diff][:8])


@pytest.mark.parametrize("variant", ["bf16_mixed", "bf16_plan_reuse", "f32", "fp8_decode"])
def test_attention_call_writes_the_new_rows_itself(variant):
    """k_new / v_new given to hook_attn_probe: the cache ends up as hook_kv_write leaves it and the results
    are those of a call on the written cache, bit for bit; before the call the new tokens' slots hold NaN."""
    from paper_2603_06588_amd import binding
    f32 = variant == "f32"
    dtype, d = (torch.float32, 64) if f32 else (torch.bfloat16, 128)
    if variant == "fp8_decode":
        lens, qlens = [500, 33, 257, 1025], [1, 1, 1, 1]
    elif f32:
        lens, qlens = [90, 40, 33], [30, 1, 33]
    else:
        lens, qlens = [300, 150, 700, 64], [300, 1, 20, 64]
    b = W.random_batch(330, lens, qlens, 8, 2, d, dtype, std=1.0, num_probe_heads=2, max_sel_q=2, max_spans=2)
    if variant == "fp8_decode":
        b.query_sel[:, 0], b.query_sel[:, 1] = 0, 1
        b = W.fp8_cache_variant(b, 331)
    gen = torch.Generator().manual_seed(332)
    k_new = torch.randn((b.total_q, 2, d), generator=gen).to(dtype)
    v_new = torch.randn((b.total_q, 2, d), generator=gen).to(dtype)
    # the slots of the new tokens start out as NaN (NaN bytes in the 8-bit cache)
    cu, L, table = b.cu_q_lens.tolist(), b.seq_lens.tolist(), b.block_table.tolist()
    for i in range(b.num_seqs):
        for t in range(cu[i + 1] - cu[i]):
            pos = L[i] - (cu[i + 1] - cu[i]) + t
            if b.k_cache.dtype == torch.uint8:
                b.k_cache[table[i][pos // 16], :, pos % 16] = 0x7F
                b.v_cache[table[i][pos // 16], :, pos % 16] = 0x7F
            else:
                b.k_cache[table[i][pos // 16], :, pos % 16] = float("nan")
                b.v_cache[table[i][pos // 16], :, pos % 16] = float("nan")
    kind = binding.BATCH_DECODE_ONLY if variant == "fp8_decode" else binding.BATCH_MIXED
    # reference: separate write, then the call
    ref = b.to(DEV)
    binding.hook_kv_write(k_new.to(DEV), v_new.to(DEV), ref.block_table, ref.seq_lens, ref.cu_q_lens, ref.k_cache,
                          ref.v_cache, k_scale=ref.k_scale, v_scale=ref.v_scale)
    ref_call = binding.call_from_batch(ref, batch_kind=kind)
    ref_call.launch()
    torch.cuda.synchronize()
    assert torch.isfinite(ref_call.out.float()).all()
    # the call that writes by itself
    one = b.to(DEV)
    kn, vn = k_new.to(DEV), v_new.to(DEV)
    if variant == "bf16_plan_reuse":
        call = binding.call_from_batch(one, batch_kind=kind, workspace=ref_call.workspace, plan_mode=binding.PLAN_REUSE,
                                       k_new=kn, v_new=vn, mass=torch.zeros_like(ref_call.mass))
    else:
        call = binding.call_from_batch(one, batch_kind=kind, k_new=kn, v_new=vn)
    call.launch()
    torch.cuda.synchronize()
    assert torch.equal(bits(call.out), bits(ref_call.out))
    assert torch.equal(bits(call.mass), bits(ref_call.mass))
    if one.k_cache.dtype == torch.uint8:
        assert torch.equal(one.k_cache, ref.k_cache) and torch.equal(one.v_cache, ref.v_cache)
    else:
        live = ~torch.isnan(ref.k_cache.float())
        assert torch.equal(bits(one.k_cache)[live.cpu()], bits(ref.k_cache)[live.cpu()])
        assert torch.equal(torch.isnan(one.k_cache.float()), ~live)


@pytest.mark.parametrize("d", [128, 64])
def test_capture_copies_the_bytes_of_an_8_bit_cache(d):
    """Keys of an 8-bit cache are gathered as the bytes they are (the caller holds the scales); queries as ever."""
    from oracle.capture import capture_qk
    from paper_2603_06588_amd import binding
    b = W.random_batch(340 + d, [333, 17, 64, 1000, 9], [100, 1, 64, 1, 0], 8, 2, d, torch.bfloat16, num_probe_heads=3,
                       max_sel_q=4)
    b8 = W.fp8_cache_variant(b, 341)
    kvh = torch.tensor([1, 0], dtype=torch.int32)
    ref_q, ref_k, cu_k = capture_qk(b8.q, b8.k_cache, b8.block_table, b8.seq_lens, b8.cu_q_lens, b8.probe_heads,
                                    b8.max_sel_q, b8.query_sel, kvh)
    assert ref_k.dtype == torch.uint8
    bd = b8.to(DEV)
    got_q, got_k = binding.hook_capture_qk(bd.q, bd.k_cache, bd.block_table, bd.seq_lens, bd.cu_q_lens, bd.probe_heads,
                                           bd.max_sel_q, bd.query_sel, kvh.to(DEV), cu_k.to(DEV), int(cu_k[-1]))
    torch.cuda.synchronize()
    assert got_k.dtype == torch.uint8 and torch.equal(got_k.cpu(), ref_k)
    assert torch.equal(bits(got_q), bits(ref_q))
