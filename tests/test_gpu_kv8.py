"""Attention over an 8-bit E4M3 key/value cache against the CPU oracle, through the C ABI (needs an
MI355X): single rows (the bandwidth-bound case the format is for), query chunks and mixed batches.  The
oracle dequantises every byte and runs the plain definition."""
import ctypes

import pytest
import torch

from paper_2603_06588_amd import binding, workloads as W
from helpers import bits, compare_with_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(b8_cpu, probe=True, **kw):
    b = b8_cpu.to(DEV)
    out = torch.full_like(b.q, float("nan"))
    call = binding.call_from_batch(b, probe=probe, batch_kind=binding.BATCH_DECODE_ONLY, out=out, **kw)
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() == 0
    return call


CASES = [
    # seed, context lengths, Hq, Hkv, d, key std, value std
    (901, [500, 33, 257, 1025], 8, 2, 128, 1.0, 1.0),       # ragged contexts, G = 4
    (902, [2100], 8, 8, 128, 1.0, 1.0),                     # one long row, G = 1, several chunks
    (903, [330, 330, 17], 6, 2, 64, 1.0, 1.0),              # G = 3, d = 64
    (904, [700, 90, 1, 260], 16, 2, 128, 0.09, 1.0),        # G = 8, near-uniform attention
    (905, [64, 48, 16, 15, 1], 4, 2, 64, 1.5, 0.7),         # block-edge lengths, G = 2, d = 64
    (906, [3000, 2500, 40], 32, 8, 128, 0.5, 1.0),          # the 8B head geometry
]


@pytest.mark.parametrize("seed,lens,Hq,Hkv,d,kstd,vstd", CASES)
def test_fp8_cache_small_batches(seed, lens, Hq, Hkv, d, kstd, vstd):
    b = W.random_batch(seed, lens, [1] * len(lens), Hq, Hkv, d, torch.bfloat16, num_probe_heads=min(5, Hq),
                       max_sel_q=2, max_spans=3)
    b.query_sel[:, 0], b.query_sel[:, 1] = 0, 1
    b8 = W.fp8_cache_variant(b, seed + 50, k_std=kstd, v_std=vstd)
    call = _run(b8)
    res = compare_with_oracle(b8, call.out, call.mass, label=f"kv8_{seed}")
    print(res, flush=True)
    assert res["out_ref_max"] > 0.05        # the comparison is not vacuous


def test_fp8_cache_bitwise_invariants():
    """Same bytes under another block permutation, a second run, and probing switched off: same bits."""
    kw = dict(num_q_heads=8, num_kv_heads=2, head_dim=128, dtype=torch.bfloat16, num_probe_heads=4)
    lens, qlens = [900, 450, 64], [1, 1, 1]
    shuf = W.fp8_cache_variant(W.random_batch(940, lens, qlens, shuffle=True, poison=True, **kw), 941)
    ident = W.fp8_cache_variant(W.random_batch(940, lens, qlens, shuffle=False, poison=False, **kw), 941)
    ident.q = shuf.q.clone()
    ident.query_sel, ident.key_spans, ident.probe_heads = shuf.query_sel, shuf.key_spans, shuf.probe_heads
    for i, L in enumerate(lens):
        for jb in range((L + 15) // 16):
            ident.k_cache[int(ident.block_table[i, jb])] = shuf.k_cache[int(shuf.block_table[i, jb])]
            ident.v_cache[int(ident.block_table[i, jb])] = shuf.v_cache[int(shuf.block_table[i, jb])]
    c1, c2, c3 = _run(shuf), _run(ident), _run(shuf)
    assert torch.equal(bits(c1.out), bits(c2.out)) and torch.equal(bits(c1.mass), bits(c2.mass))
    assert torch.equal(bits(c1.out), bits(c3.out)) and torch.equal(bits(c1.mass), bits(c3.mass))
    assert torch.isfinite(c1.out.float()).all()           # the NaN bytes of dead slots were never read
    c4 = _run(shuf, probe=False)
    assert torch.equal(bits(c1.out), bits(c4.out))


def test_fp8_cache_every_byte_pattern_decodes_like_the_oracle():
    """One key per byte pattern: a query that is a unit vector makes each score a single dequantised
    element, and values of one kv head run through all 254 finite patterns, so a wrong decoding of any
    byte shows in out or mass."""
    b = W.random_batch(950, [256], [1], 2, 1, 128, torch.bfloat16, num_probe_heads=2, max_sel_q=1, max_spans=2,
                       poison=False, shuffle=False)
    b8 = W.fp8_cache_variant(b, 951, k_std=0.05, v_std=1.0)
    pats = torch.tensor([p for p in range(256) if (p & 0x7F) != 0x7F] + [0, 0], dtype=torch.uint8)   # 256 finite bytes
    for j in range(256):
        blk = int(b8.block_table[0, j // 16])
        b8.k_cache[blk, 0, j % 16, :] = pats.roll(j)[:128]
        b8.v_cache[blk, 0, j % 16, :] = pats.roll(3 * j + 1)[:128]
    b8.q.zero_()
    b8.q[0, 0, 5] = 1.0
    b8.q[0, 1, 77] = -2.0
    b8.query_sel[0, 0], b8.query_sel[0, 1] = 0, 1
    call = _run(b8)
    compare_with_oracle(b8, call.out, call.mass, label="kv8_all_bytes")


def test_c3_full_size_fp8_cache():
    b = W.c3_decode_8b(device="cpu")
    b8 = W.fp8_cache_variant(b, 960, k_std=128 ** -0.5, v_std=128 ** -0.5)
    call = _run(b8)
    print(compare_with_oracle(b8, call.out, call.mass, label="c3_kv8"), flush=True)
    peaked = W.fp8_cache_variant(W.c3_decode_8b(device="cpu", peaked=True), 961)
    call = _run(peaked)
    print(compare_with_oracle(peaked, call.out, call.mass, label="c3_kv8_peaked"), flush=True)


def test_fp8_cache_argument_checks():
    lib = binding.load_library()
    b = W.random_batch(970, [100, 50], [1, 1], 8, 2, 128, torch.bfloat16, num_probe_heads=2)
    b8 = W.fp8_cache_variant(b, 971).to(DEV)
    call = binding.call_from_batch(b8, batch_kind=binding.BATCH_MIXED)
    assert lib.hook_attn_probe(ctypes.byref(call.args)) == 0       # any composition of the batch is served
    call = binding.call_from_batch(b8, batch_kind=binding.BATCH_DECODE_ONLY)
    call.args.k_scale = 0
    assert lib.hook_attn_probe(ctypes.byref(call.args)) == 1       # scales missing
    call = binding.call_from_batch(b8, batch_kind=binding.BATCH_DECODE_ONLY)
    call.args.kv_dtype = 7
    assert lib.hook_attn_probe(ctypes.byref(call.args)) == 2
    call = binding.call_from_batch(b8, batch_kind=binding.BATCH_DECODE_ONLY)
    call.args.k_scale = 0
    assert lib.hook_span_mass(ctypes.byref(call.args)) == 1          # the span pass needs the key scales too


CHUNK_CASES = [
    # seed, context lengths, query rows, Hq, Hkv, d, key std, value std
    (981, [200], [200], 8, 2, 128, 1.0, 1.0),                       # one prompt, 4 tiles, G = 4
    (982, [77, 130, 65, 64], [77, 130, 65, 64], 8, 2, 128, 1.0, 1.0),   # ragged, tile-edge lengths
    (983, [300, 150], [45, 150], 8, 2, 128, 1.0, 0.7),              # a chunk on prior context
    (984, [700, 90, 1, 260], [1, 90, 1, 3], 8, 2, 128, 1.0, 1.0),   # single rows, chunks and a tiny chunk together
    (985, [190, 64], [190, 64], 8, 1, 128, 0.5, 1.0),               # G = 8
    (986, [150, 40], [150, 40], 6, 2, 128, 1.0, 1.0),               # G = 3 (one head per wave)
    (987, [210, 90, 300], [210, 1, 1], 8, 2, 64, 1.0, 1.0),         # d = 64, both kinds
    (988, [129, 512], [129, 1], 16, 2, 128, 0.09, 1.0),             # near-uniform attention
    (989, [40, 0, 25], [40, 0, 25], 8, 2, 64, 1.0, 1.0),            # an empty sequence in the middle, d = 64
]


@pytest.mark.parametrize("seed,lens,qlens,Hq,Hkv,d,kstd,vstd", CHUNK_CASES)
def test_fp8_cache_query_chunks_and_mixed_batches(seed, lens, qlens, Hq, Hkv, d, kstd, vstd):
    from helpers import valid_rows
    b = W.random_batch(seed, lens, qlens, Hq, Hkv, d, torch.bfloat16, num_probe_heads=min(5, Hq), max_sel_q=3,
                       max_spans=3)
    b8 = W.fp8_cache_variant(b, seed + 50, k_std=kstd, v_std=vstd)
    bd = b8.to(DEV)
    out = torch.full_like(bd.q, float("nan"))
    mass = torch.full((b.num_seqs, b.num_probe_heads, b.max_sel_q, b.max_spans), float("nan"), dtype=torch.float32,
                      device=DEV)
    call = binding.call_from_batch(bd, out=out, mass=mass)
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() == 0
    written = torch.isfinite(out.float()).all(dim=2).all(dim=1).cpu()
    assert bool((written == valid_rows(b8)).all())
    res = compare_with_oracle(b8, out, mass, label=f"kv8_chunks_{seed}")
    print(res, flush=True)


def test_fp8_cache_c2_shape_shrunk():
    """The 8B prefill geometry over an 8-bit cache, eight times shorter, every row against the oracle."""
    b = W.c2_prefill_8b(device="cpu", peaked=True, shrink=8)
    b8 = W.fp8_cache_variant(b, 990, k_std=1.0, v_std=1.0)
    bd = b8.to(DEV)
    call = binding.call_from_batch(bd, batch_kind=binding.BATCH_PREFILL_ONLY)
    call.out.fill_(float("nan"))
    call.launch()
    torch.cuda.synchronize()
    assert call.device_status() == 0
    print(compare_with_oracle(b8, call.out, call.mass, label="c2_kv8_shrunk"), flush=True)


def test_fp8_cache_chunk_call_writes_its_new_rows_quantised():
    """k_new / v_new with an 8-bit cache and query chunks: the planning launch quantises the rows into
    the cache, the chunk kernel then reads them back."""
    from oracle.capture import kv_write
    b = W.random_batch(995, [300, 64], [100, 64], 8, 2, 128, torch.bfloat16, num_probe_heads=3, max_sel_q=2,
                       poison=False)
    b8 = W.fp8_cache_variant(b, 996, k_std=1.0, v_std=0.5)
    gen = torch.Generator().manual_seed(997)
    k_new = torch.randn((b.total_q, 2, 128), generator=gen).to(torch.bfloat16)
    v_new = (torch.randn((b.total_q, 2, 128), generator=gen) * 0.5).to(torch.bfloat16)
    want_k, want_v = kv_write(k_new, v_new, b8.block_table, b8.seq_lens, b8.cu_q_lens, b8.k_cache, b8.v_cache,
                              b8.k_scale, b8.v_scale)
    after = b8.to("cpu")
    kw = dict(after.__dict__)
    kw.update(k_cache=want_k, v_cache=want_v)
    after = type(after)(**kw)
    bd = b8.to(DEV)
    call = binding.call_from_batch(bd, k_new=k_new.to(DEV), v_new=v_new.to(DEV))
    call.launch()
    torch.cuda.synchronize()
    assert torch.equal(bd.k_cache.cpu(), want_k) and torch.equal(bd.v_cache.cpu(), want_v)
    print(compare_with_oracle(after, call.out, call.mass, label="kv8_chunks_in_call_write"), flush=True)
