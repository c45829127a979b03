"""Pins of the CPU oracle against things other than itself (no GPU needed).

The paper prints no numerical worked example for this path, so the oracle is
pinned by brute force, closed forms, invariants and library special cases:
each is chosen so that a plausible slip (dropped scale, wrong kv-head mapping,
inclusive span end, off-by-one causal horizon, wrong block/slot index) fails
at least one of them.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2603_06588_amd import workloads as W


# --------------------------------------------------------------------------
# brute force: pure-Python loops that materialise the full probability matrix
# --------------------------------------------------------------------------

def brute_force(b):
    """Independent restatement of the definition with Python floats (fp64)."""
    q = b.q.double().tolist()
    kc = b.k_cache.double().tolist()
    vc = b.v_cache.double().tolist()
    table = b.block_table.tolist()
    lens = b.seq_lens.tolist()
    cu = b.cu_q_lens.tolist()
    heads = b.probe_heads.tolist()
    qsel = b.query_sel.tolist()
    spans = b.key_spans.tolist()
    G = b.num_q_heads // b.num_kv_heads
    B, d = b.block_size, b.head_dim
    out = [[[0.0] * d for _ in range(b.num_q_heads)] for _ in range(b.total_q)]
    mass = np.zeros((b.num_seqs, len(heads), b.max_sel_q, b.max_spans))
    for i in range(b.num_seqs):
        n, L = cu[i + 1] - cu[i], lens[i]
        for t in range(n):
            pos = L - n + t
            for h in range(b.num_q_heads):
                g = h // G
                qv = q[cu[i] + t][h]
                P = []
                for j in range(pos + 1):
                    kv = kc[table[i][j // B]][g][j % B]
                    P.append(b.scale * sum(qv[c] * kv[c] for c in range(d)))
                mx = max(P)
                P = [math.exp(x - mx) for x in P]
                tot = sum(P)
                P = [x / tot for x in P]
                for j in range(pos + 1):
                    vv = vc[table[i][j // B]][g][j % B]
                    for c in range(d):
                        out[cu[i] + t][h][c] += P[j] * vv[c]
                if h in heads and qsel[i][0] <= t < qsel[i][1]:
                    p = heads.index(h)
                    for r in range(b.max_spans):
                        a, e = spans[i][r]
                        mass[i, p, t - qsel[i][0], r] = sum(P[j] for j in range(max(a, 0), min(e, pos + 1)))
    return torch.tensor(out, dtype=torch.float64), torch.from_numpy(mass)


BRUTE_CASES = [
    # seed, seq_lens, q_lens, Hq, Hkv, d, block, dtype
    (11, [7], [7], 2, 2, 4, 1, torch.float32),
    (12, [13, 5], [13, 5], 4, 2, 8, 2, torch.float32),
    (13, [17, 9, 1], [3, 9, 1], 4, 1, 8, 4, torch.bfloat16),
    (14, [32, 20], [1, 20], 8, 2, 8, 16, torch.bfloat16),
    (15, [19, 6, 11], [19, 0, 4], 4, 4, 4, 16, torch.float32),
]


@pytest.mark.parametrize("seed,lens,qlens,Hq,Hkv,d,B,dtype", BRUTE_CASES)
def test_brute_force_tiny(seed, lens, qlens, Hq, Hkv, d, B, dtype):
    b = W.random_batch(seed, lens, qlens, Hq, Hkv, d, dtype, std=1.0, num_probe_heads=3, max_sel_q=3,
                       max_spans=3, block_size=B)
    out, mass = oracle.attn_probe_batch(b)
    ref_out, ref_mass = brute_force(b)
    # rows of empty sequences stay NaN in the oracle output; compare the rest
    valid = ~torch.isnan(out)
    assert valid.sum() == sum(qlens) * Hq * d
    assert torch.allclose(out[valid], ref_out[valid], rtol=0, atol=1e-12)
    assert torch.allclose(mass, ref_mass, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# invariants of a softmax row
# --------------------------------------------------------------------------

def test_row_sums_and_partitions():
    lens, qlens = [70, 33], [70, 5]
    gen = torch.Generator().manual_seed(5)
    # spans: [0, L) ; a partition of [0, L) into three pieces
    cut = [(23, 51), (10, 11)]
    spans = [[(0, L), (0, c0), (c0, c1), (c1, L)] for L, (c0, c1) in zip(lens, cut)]
    b = W.build_paged("partition", lens, qlens, 4, 2, 16, torch.float32, 1.0, gen, [0, 1, 2, 3],
                      [(0, n) for n in qlens], spans, max_sel_q=70, max_spans=4)
    _, mass = oracle.attn_probe_batch(b)
    for i, n in enumerate(qlens):
        m = mass[i, :, :n, :]
        assert (m >= 0).all() and (m <= 1 + 1e-12).all()
        assert torch.allclose(m[..., 0], torch.ones_like(m[..., 0]), atol=1e-12)
        assert torch.allclose(m[..., 1:].sum(-1), torch.ones_like(m[..., 0]), atol=1e-12)
        assert (mass[i, :, n:, :] == 0).all()


# --------------------------------------------------------------------------
# closed forms: uniform attention when Q = 0
# --------------------------------------------------------------------------

def test_uniform_attention_closed_form_c1():
    b, _ = W.c1_tiny_prefill()
    b.q.zero_()
    out, mass = oracle.attn_probe_batch(b)
    # span [16, 64) seen from the last of 256 tokens: 48 / 256
    assert torch.allclose(mass, torch.full_like(mass, 0.1875), atol=1e-13)
    # out = prefix mean of V
    v = b.v_cache.double().permute(1, 0, 2, 3).reshape(8, 256, 64)  # identity table
    prefix_mean = v.cumsum(1) / torch.arange(1, 257, dtype=torch.float64)[None, :, None]
    assert torch.allclose(out, prefix_mean.permute(1, 0, 2), atol=1e-12)


def test_uniform_attention_clipped_spans():
    lens, qlens = [40, 25], [10, 25]
    b = W.random_batch(21, lens, qlens, 4, 2, 8, torch.float32, num_probe_heads=4, max_sel_q=4, max_spans=4)
    b.q.zero_()
    _, mass = oracle.attn_probe_batch(b)
    qs, ks = b.query_sel.tolist(), b.key_spans.tolist()
    for i, (L, n) in enumerate(zip(lens, qlens)):
        for tt in range(qs[i][1] - qs[i][0]):
            pos = L - n + qs[i][0] + tt
            for r in range(4):
                a, e = ks[i][r]
                want = max(0, min(e, pos + 1) - max(a, 0)) / (pos + 1)
                assert torch.allclose(mass[i, :, tt, r], torch.full((4,), want, dtype=torch.float64), atol=1e-13)


# --------------------------------------------------------------------------
# special case: one dominant key
# --------------------------------------------------------------------------

def test_dominant_key_limit():
    L = 48
    gen = torch.Generator().manual_seed(6)
    b = W.build_paged("dominant", [L], [L], 2, 1, 16, torch.float32, 1.0, gen, [0, 1], [(L - 1, L)],
                      [[(8, 24), (24, 40)]], max_sel_q=1, max_spans=2)
    jstar = 19
    table = b.block_table.tolist()
    for h in range(2):
        pass
    qlast = b.q[L - 1]                      # [2, 16]
    # make key j* line up with head 0's last query, strongly
    qhat = qlast[0] / qlast[0].norm()
    b.k_cache[table[0][jstar // 16], 0, jstar % 16] = 400.0 * qhat
    out, mass = oracle.attn_probe_batch(b)
    vstar = b.v_cache[table[0][jstar // 16], 0, jstar % 16].double()
    assert torch.allclose(out[L - 1, 0], vstar, atol=1e-9)
    assert abs(mass[0, 0, 0, 0] - 1.0) < 1e-9 and mass[0, 0, 0, 1] < 1e-9


# --------------------------------------------------------------------------
# reduction to library routines on un-paged, GQA-expanded tensors
# --------------------------------------------------------------------------

def _dense_kv(b, i):
    """[L, Hkv, d] fp64 keys/values of sequence i, gathered with torch indexing."""
    L = int(b.seq_lens[i])
    idx = torch.arange(L)
    blk = b.block_table[i, idx // b.block_size].long()
    slot = idx % b.block_size
    return b.k_cache[blk, :, slot, :].double(), b.v_cache[blk, :, slot, :].double()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_against_torch_softmax_and_sdpa(dtype):
    lens, qlens = [150, 64, 37], [150, 20, 1]
    b = W.random_batch(31, lens, qlens, 8, 2, 32, dtype, num_probe_heads=8, max_sel_q=4, max_spans=2)
    out, mass = oracle.attn_probe_batch(b)
    G = 4
    cu = b.cu_q_lens.tolist()
    for i, (L, n) in enumerate(zip(lens, qlens)):
        k, v = _dense_kv(b, i)
        k = k.repeat_interleave(G, dim=1).permute(1, 0, 2)   # [Hq, L, d]
        v = v.repeat_interleave(G, dim=1).permute(1, 0, 2)
        qq = b.q[cu[i]:cu[i + 1]].double().permute(1, 0, 2)  # [Hq, n, d]
        pos = torch.arange(L - n, L)
        mask = torch.arange(L)[None, :] <= pos[:, None]
        s = (qq @ k.transpose(1, 2)) * b.scale
        s = s.masked_fill(~mask[None], float("-inf"))
        p = torch.softmax(s, dim=-1)
        ref = (p @ v).permute(1, 0, 2)
        assert torch.allclose(out[cu[i]:cu[i + 1]], ref, atol=1e-12)
        ref2 = torch.nn.functional.scaled_dot_product_attention(qq, k, v, attn_mask=mask[None], scale=b.scale)
        assert torch.allclose(out[cu[i]:cu[i + 1]], ref2.permute(1, 0, 2), atol=1e-10)
        # masses from the library softmax
        qb, qe = b.query_sel[i].tolist()
        for tt, t in enumerate(range(qb, qe)):
            for r in range(2):
                a, e = b.key_spans[i, r].tolist()
                a, e = max(a, 0), min(e, L - n + t + 1)
                want = p[:, t, a:e].sum(-1) if e > a else torch.zeros(8, dtype=torch.float64)
                assert torch.allclose(mass[i, :, tt, r], want[b.probe_heads.long()], atol=1e-12)


# --------------------------------------------------------------------------
# GQA mapping, paging, chunked-prefill positions
# --------------------------------------------------------------------------

def test_gqa_equals_replicated_kv_heads():
    lens, qlens = [45, 30], [45, 7]
    b = W.random_batch(41, lens, qlens, 8, 2, 16, torch.float32, num_probe_heads=5, poison=False)
    out, mass = oracle.attn_probe_batch(b)
    b2 = W.random_batch(41, lens, qlens, 8, 2, 16, torch.float32, num_probe_heads=5, poison=False)
    b2.k_cache = b.k_cache.repeat_interleave(4, dim=1)
    b2.v_cache = b.v_cache.repeat_interleave(4, dim=1)
    b2.num_kv_heads = 8
    out2, mass2 = oracle.attn_probe_batch(b2)
    assert torch.equal(out, out2) and torch.equal(mass, mass2)


def test_paging_permutation_invariance_and_poison():
    lens, qlens = [100, 37, 64], [100, 5, 1]
    kw = dict(num_q_heads=4, num_kv_heads=2, head_dim=16, dtype=torch.bfloat16, num_probe_heads=4)
    shuf = W.random_batch(51, lens, qlens, shuffle=True, poison=True, **kw)
    out_s, mass_s = oracle.attn_probe_batch(shuf)
    assert torch.isfinite(out_s).all() and torch.isfinite(mass_s).all()
    # same logical K/V laid out contiguously with an identity table
    ident = W.random_batch(51, lens, qlens, shuffle=False, poison=False, **kw)
    ident.q = shuf.q.clone()
    ident.query_sel, ident.key_spans, ident.probe_heads = shuf.query_sel, shuf.key_spans, shuf.probe_heads
    nb = 0
    for i, L in enumerate(lens):
        for jb in range((L + 15) // 16):
            src = int(shuf.block_table[i, jb])
            dst = int(ident.block_table[i, jb])
            ident.k_cache[dst] = shuf.k_cache[src]
            ident.v_cache[dst] = shuf.v_cache[src]
            nb += 1
    out_i, mass_i = oracle.attn_probe_batch(ident)
    assert torch.equal(out_s, out_i) and torch.equal(mass_s, mass_i)


def test_out_of_range_block_id_is_rejected():
    b = W.random_batch(52, [20], [20], 2, 1, 8, torch.float32)
    b.block_table[0, 1] = b.num_blocks
    with pytest.raises(ValueError):
        oracle.attn_probe_batch(b)


def test_chunked_prefill_positions():
    L = 96
    b = W.random_batch(61, [L], [L], 4, 2, 16, torch.float32, num_probe_heads=4, max_sel_q=4, poison=False)
    b.query_sel[0, 0], b.query_sel[0, 1] = 90, 94
    out, mass = oracle.attn_probe_batch(b)
    # second half as its own call on top of the cached first half: rows 48..95
    h2 = W.random_batch(61, [L], [48], 4, 2, 16, torch.float32, num_probe_heads=4, max_sel_q=4, poison=False)
    h2.k_cache, h2.v_cache, h2.block_table = b.k_cache, b.v_cache, b.block_table
    h2.q = b.q[48:].clone()
    h2.probe_heads, h2.key_spans = b.probe_heads, b.key_spans
    h2.query_sel[0, 0], h2.query_sel[0, 1] = 90 - 48, 94 - 48
    out2, mass2 = oracle.attn_probe_batch(h2)
    assert torch.equal(out[48:], out2) and torch.equal(mass, mass2)
    # first half alone: context is only the first 48 tokens
    h1 = W.random_batch(61, [48], [48], 4, 2, 16, torch.float32, num_probe_heads=4, max_sel_q=4, poison=False)
    h1.k_cache, h1.v_cache, h1.block_table = b.k_cache, b.v_cache, b.block_table[:, :3].contiguous()
    h1.q = b.q[:48].clone()
    out1, _ = oracle.attn_probe_batch(h1)
    assert torch.equal(out[:48], out1)


def test_row_subset_matches_full():
    b = W.random_batch(62, [60, 30], [60, 30], 4, 2, 16, torch.bfloat16, max_sel_q=4)
    out, mass = oracle.attn_probe_batch(b)
    qb, qe = b.query_sel[1].tolist()
    rows = [0, 17, 59, 60, 89] + [60 + t for t in range(qb, qe)]
    out_r, mass_r = oracle.attn_probe_batch(b, rows=rows)
    assert torch.equal(out_r[rows], out[rows])
    others = [r for r in range(90) if r not in rows]
    assert torch.isnan(out_r[others]).all()
    assert torch.equal(mass_r[1], mass[1])


# --------------------------------------------------------------------------
# the merge algebra a split-key evaluation relies on
# --------------------------------------------------------------------------

def test_split_key_merge_algebra_matches_oracle():
    L = 200
    b = W.random_batch(71, [L], [1], 2, 1, 16, torch.float32, num_probe_heads=2, max_sel_q=1, max_spans=1,
                       poison=False, wild_spans=False)
    b.query_sel[0, 0], b.query_sel[0, 1] = 0, 1
    b.key_spans[0, 0, 0], b.key_spans[0, 0, 1] = 30, 130
    out, mass = oracle.attn_probe_batch(b)
    k, v = _dense_kv(b, 0)
    for h in range(2):
        s = (k[:, 0, :] @ b.q[0, h].double()) * b.scale
        parts = []
        for c0 in range(0, L, 64):
            sc = s[c0:c0 + 64]
            m = sc.max()
            e = torch.exp(sc - m)
            in_span = (torch.arange(c0, c0 + len(sc)) >= 30) & (torch.arange(c0, c0 + len(sc)) < 130)
            parts.append((m, e.sum(), e @ v[c0:c0 + 64, 0, :], (e * in_span).sum()))
        mstar = max(p[0] for p in parts)
        w = [torch.exp(p[0] - mstar) for p in parts]
        l = sum(wi * p[1] for wi, p in zip(w, parts))
        o = sum(wi * p[2] for wi, p in zip(w, parts)) / l
        a = sum(wi * p[3] for wi, p in zip(w, parts)) / l
        assert torch.allclose(out[0, h], o, atol=1e-12)
        assert abs(float(mass[0, h, 0, 0]) - float(a)) < 1e-12


# --------------------------------------------------------------------------
# steering
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_steer_identities(dtype):
    s = W.steer_batch(81, 33, 48, dtype, alpha=0.0, mask_frac=0.6)
    s.hidden[3, 5] = float("nan")
    s.hidden[4, 6] = -0.0
    view = torch.int32 if dtype == torch.float32 else torch.int16
    # alpha = 0 with finite vec: values unchanged wherever the input is finite and non-zero
    out = oracle.steer(s.hidden, s.vec, 0.0, s.token_mask)
    fin = torch.isfinite(s.hidden) & (s.hidden != 0)
    assert torch.equal(out.view(view)[fin], s.hidden.view(view)[fin])
    # all-zero mask: bit-identical buffer, NaN payloads and signed zeros included
    out = oracle.steer(s.hidden, s.vec, 3.0, torch.zeros_like(s.token_mask))
    assert torch.equal(out.view(view), s.hidden.view(view))
    # unmasked rows are bit-identical, masked rows change
    out = oracle.steer(s.hidden, s.vec, 2.0, s.token_mask)
    keep = s.token_mask == 0
    assert torch.equal(out.view(view)[keep], s.hidden.view(view)[keep])
    # alpha = 1, vec = -row  =>  that row becomes exactly zero
    row = 7
    mask = torch.zeros_like(s.token_mask)
    mask[row] = 1
    h = s.hidden.clone()
    h[3, 5] = 1.0
    out = oracle.steer(h, -h[row], 1.0, mask)
    assert (out[row] == 0).all()


def _nearest_bf16_exact(x: Fraction) -> int:
    """Round-to-nearest-even over an explicit scan of bf16 neighbours (exact rationals)."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 7)
    lo = int(a / quantum)                      # floor
    cands = [lo, lo + 1]
    dist = [abs(a - c * quantum) for c in cands]
    if dist[0] < dist[1] or (dist[0] == dist[1] and lo % 2 == 0):
        n = lo
    else:
        n = lo + 1
    val = float(n * quantum)
    bits = int(torch.tensor(val, dtype=torch.float32).view(torch.int32)) & 0xFFFFFFFF
    assert bits & 0xFFFF == 0
    return sign | (bits >> 16)


def test_round_bf16_single_rounding():
    # values exactly representable in fp32: torch's fp32->bf16 cast is one RNE step
    gen = torch.Generator().manual_seed(9)
    xs = torch.randn(2000, generator=gen) * torch.tensor(10.0) ** torch.randint(-30, 30, (2000,), generator=gen)
    want = xs.to(torch.bfloat16).view(torch.int16).to(torch.int32) & 0xFFFF
    got = [oracle.round_bf16(float(x)) for x in xs]
    assert got == want.tolist()
    # ties go to even
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # just above a tie: rounding through fp32 first would lose the 2^-30 and round down
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81
    # subnormal, overflow, signed zero
    assert oracle.round_bf16(2.0 ** -133) == 0x0001
    assert oracle.round_bf16(2.0 ** -134) == 0x0000
    assert oracle.round_bf16(-0.0) == 0x8000
    assert oracle.round_bf16(3.4e38) == 0x7F80


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_steer_exact_rational_arithmetic(dtype):
    s = W.steer_batch(82, 6, 16, dtype, alpha=1.7, mask_frac=1.0)
    s.token_mask[:] = 1
    out = oracle.steer(s.hidden, s.vec, s.alpha, s.token_mask)
    alpha = Fraction(float(np.float32(s.alpha)))
    for t in range(6):
        for c in range(16):
            exact = Fraction(float(s.hidden[t, c])) + alpha * Fraction(float(s.vec[c]))
            if dtype == torch.bfloat16:
                want = _nearest_bf16_exact(exact)
                got = int(out[t, c].view(torch.int16)) & 0xFFFF
                assert got == want
            else:
                # nearest fp32 to the exact rational: compare against both neighbours
                got = float(out[t, c])
                near = np.float32(float(exact))
                nb = [near, np.nextafter(near, np.float32(np.inf)), np.nextafter(near, np.float32(-np.inf))]
                best = min(nb, key=lambda z: abs(Fraction(float(z)) - exact))
                assert abs(Fraction(got) - exact) <= abs(Fraction(float(best)) - exact)


# --------------------------------------------------------------------------
# compact q/k capture reference: pinned by torch indexing on an identity table
# --------------------------------------------------------------------------

def test_capture_reference_against_slicing():
    from oracle.capture import capture_qk
    lens, qlens = [37, 64, 5], [37, 3, 1]
    b = W.random_batch(91, lens, qlens, 8, 4, 16, torch.bfloat16, num_probe_heads=3, max_sel_q=4, shuffle=False,
                       poison=False)
    kvh = torch.tensor([3, 0], dtype=torch.int32)
    q_out, k_out, cu_k = capture_qk(b.q, b.k_cache, b.block_table, b.seq_lens, b.cu_q_lens, b.probe_heads,
                                    b.max_sel_q, b.query_sel, kvh)
    assert cu_k.tolist() == [0, 37, 101, 106]
    # identity table: sequence i owns consecutive blocks, so its keys are a reshape of the cache
    first_blk = 0
    for i, L in enumerate(lens):
        nb = (L + 15) // 16
        dense = b.k_cache[first_blk:first_blk + nb].permute(0, 2, 1, 3).reshape(nb * 16, 4, 16)[:L]
        assert torch.equal(k_out[cu_k[i]:cu_k[i + 1]].view(torch.int16), dense[:, kvh.long()].view(torch.int16))
        first_blk += nb
    cu = b.cu_q_lens.tolist()
    for i in range(3):
        qb, qe = b.query_sel[i].tolist()
        rows = list(range(qb, min(qe, qlens[i])))[:4]
        want = b.q[cu[i]:cu[i + 1]][rows][:, b.probe_heads.long()].permute(1, 0, 2)
        assert torch.equal(q_out[i, :, :len(rows)].view(torch.int16), want.view(torch.int16))
        assert (q_out[i, :, len(rows):] == 0).all()


# --------------------------------------------------------------------------
# steering fused into the residual add
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_residual_steer_exact_rational_and_identities(dtype):
    s = W.steer_batch(83, 6, 16, dtype, alpha=-2.3, mask_frac=0.5)
    s.token_mask[:] = torch.tensor([1, 0, 1, 1, 0, 1], dtype=torch.uint8)
    gen = torch.Generator().manual_seed(84)
    delta = (torch.randn((6, 16), generator=gen) * 3).to(dtype)
    delta[2] = (-s.hidden[2].double()).to(dtype)            # cancellation: h + d = 0 exactly on row 2
    out = oracle.residual_steer(s.hidden, delta, s.vec, s.alpha, s.token_mask)
    alpha = Fraction(float(np.float32(s.alpha)))
    for t in range(6):
        for c in range(16):
            exact = Fraction(float(s.hidden[t, c])) + Fraction(float(delta[t, c]))
            if s.token_mask[t]:
                exact += alpha * Fraction(float(s.vec[c]))
            if dtype == torch.bfloat16:
                assert (int(out[t, c].view(torch.int16)) & 0xFFFF) == _nearest_bf16_exact(exact)
            else:
                got = float(out[t, c])
                near = np.float32(float(exact))
                nb = [near, np.nextafter(near, np.float32(np.inf)), np.nextafter(near, np.float32(-np.inf))]
                best = min(nb, key=lambda z: abs(Fraction(float(z)) - exact))
                assert abs(Fraction(got) - exact) <= abs(Fraction(float(best)) - exact)
    # delta = 0 reduces to plain steering; no mask / alpha = 0 reduce to a plain add
    zero = torch.zeros_like(delta)
    assert torch.equal(oracle.residual_steer(s.hidden, zero, s.vec, s.alpha, s.token_mask).view(torch.uint8),
                       oracle.steer(s.hidden, s.vec, s.alpha, s.token_mask).view(torch.uint8))
    plain = oracle.residual_steer(s.hidden, delta, s.vec, 0.0, s.token_mask)
    assert torch.equal(plain, oracle.residual_steer(s.hidden, delta, s.vec, 5.0, None))
    if dtype == torch.float32:
        assert torch.equal(plain, (s.hidden.double() + delta.double()).float())


def test_kv_write_reference_round_trip():
    """Writing the new rows and gathering them back through the block table returns them, and
    nothing else in the cache moves (the attention oracle then sees exactly the written values)."""
    from oracle.capture import capture_qk, kv_write
    lens, qlens = [37, 64, 5, 20], [10, 64, 1, 0]
    b = W.random_batch(92, lens, qlens, 8, 4, 16, torch.bfloat16, num_probe_heads=1, max_sel_q=1, poison=False)
    gen = torch.Generator().manual_seed(93)
    k_new = torch.randn((b.total_q, 4, 16), generator=gen).to(torch.bfloat16)
    v_new = torch.randn((b.total_q, 4, 16), generator=gen).to(torch.bfloat16)
    kc, vc = kv_write(k_new, v_new, b.block_table, b.seq_lens, b.cu_q_lens, b.k_cache, b.v_cache)
    kvh = torch.arange(4, dtype=torch.int32)
    _, k_all, cu_k = capture_qk(b.q, kc, b.block_table, b.seq_lens, b.cu_q_lens, b.probe_heads, 1, b.query_sel, kvh)
    _, k_old, _ = capture_qk(b.q, b.k_cache, b.block_table, b.seq_lens, b.cu_q_lens, b.probe_heads, 1, b.query_sel, kvh)
    cu = b.cu_q_lens.tolist()
    for i, (L, n) in enumerate(zip(lens, qlens)):
        got = k_all[cu_k[i]:cu_k[i + 1]]
        assert torch.equal(got[L - n:].view(torch.int16), k_new[cu[i]:cu[i + 1]].view(torch.int16))
        assert torch.equal(got[:L - n].view(torch.int16), k_old[cu_k[i]:cu_k[i + 1]][:L - n].view(torch.int16))
    changed = (kc.view(torch.int16) != b.k_cache.view(torch.int16)).any(-1).any(1).sum()     # (block, slot) pairs
    assert int(changed) <= sum(qlens) and int((vc.view(torch.int16) != b.v_cache.view(torch.int16)).any(-1).any(1).sum()) <= sum(qlens)


# ---- 8-bit (E4M3) key/value cache: dequantise, then the plain definition ----

def test_fp8_decoding_table_matches_the_format_and_a_library():
    """All 256 byte patterns: against the format's published constants and against torch's own
    float8_e4m3fn decoding (a library routine the oracle does not use)."""
    assert oracle.fp8_e4m3_value(0x38) == 1.0 and oracle.fp8_e4m3_value(0xB8) == -1.0
    assert oracle.fp8_e4m3_value(0x7E) == 448.0           # largest finite value
    assert oracle.fp8_e4m3_value(0x08) == 2.0 ** -6        # smallest normal
    assert oracle.fp8_e4m3_value(0x01) == 2.0 ** -9        # smallest subnormal
    assert oracle.fp8_e4m3_value(0x00) == 0.0 and math.copysign(1.0, oracle.fp8_e4m3_value(0x80)) == -1.0
    assert math.isnan(oracle.fp8_e4m3_value(0x7F)) and math.isnan(oracle.fp8_e4m3_value(0xFF))
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double()
    for byte in range(256):
        want, got = float(lib[byte]), oracle.fp8_e4m3_value(byte)
        assert (math.isnan(want) and math.isnan(got)) or (want == got and math.copysign(1, want) == math.copysign(1, got)), byte


def _dequantised(b8):
    """fp64 K / V of an 8-bit batch through torch's decoder (not the oracle's)."""
    Hkv = b8.num_kv_heads
    k = b8.k_cache.view(torch.float8_e4m3fn).double() * b8.k_scale.double().view(1, Hkv, 1, 1)
    v = b8.v_cache.view(torch.float8_e4m3fn).double() * b8.v_scale.double().view(1, Hkv, 1, 1)
    return k, v


def test_fp8_cache_equals_the_16_bit_path_when_bf16_holds_the_dequantised_values():
    """Power-of-two scales: every dequantised value is a bf16 number, so running the (already pinned)
    16-bit path on the dequantised cache must give the very same fp64 results."""
    b = W.random_batch(801, [70, 33, 120, 16], [1, 33, 1, 5], 8, 2, 16, torch.bfloat16, num_probe_heads=4,
                       max_sel_q=3, max_spans=3)
    b8 = W.fp8_cache_variant(b, 802, pow2_scales=True)
    k, v = _dequantised(b8)
    k16, v16 = k.to(torch.bfloat16), v.to(torch.bfloat16)
    live_k = ~torch.isnan(k)
    assert torch.equal(k16.double()[live_k], k[live_k])          # nothing was rounded
    kw = dict(b.__dict__); kw.update(k_cache=k16, v_cache=v16)
    out16, mass16 = oracle.attn_probe_batch(W.AttnBatch(**kw))
    out8, mass8 = oracle.attn_probe_batch(b8)
    assert torch.equal(out8, out16) and torch.equal(mass8, mass16)
    assert torch.isfinite(out8).all()


def test_fp8_cache_matches_torch_softmax_on_dequantised_tensors():
    """Arbitrary scales: un-paged fp64 softmax(Q K^T) V from torch on the dequantised cache."""
    L, n, Hq, Hkv, d = 90, 90, 4, 2, 32
    b = W.random_batch(803, [L], [n], Hq, Hkv, d, torch.bfloat16, num_probe_heads=2, max_sel_q=2, max_spans=2,
                       shuffle=True)
    b8 = W.fp8_cache_variant(b, 804, k_std=0.7, v_std=1.3)
    k, v = _dequantised(b8)
    table = b8.block_table[0].tolist()
    K = torch.stack([k[table[j // 16], :, j % 16] for j in range(L)])     # [L, Hkv, d]
    V = torch.stack([v[table[j // 16], :, j % 16] for j in range(L)])
    out, mass = oracle.attn_probe_batch(b8)
    G = Hq // Hkv
    causal = torch.tril(torch.ones(L, L, dtype=torch.bool))
    for h in range(Hq):
        s = (b8.q[:, h].double() @ K[:, h // G].T) * b8.scale
        p = torch.softmax(s.masked_fill(~causal, float("-inf")), dim=-1)
        assert (p @ V[:, h // G] - out[:, h]).abs().max().item() < 1e-11
    qs, ks, heads = b8.query_sel.tolist(), b8.key_spans.tolist(), b8.probe_heads.tolist()
    for pi, h in enumerate(heads):
        s = (b8.q[:, h].double() @ K[:, h // G].T) * b8.scale
        p = torch.softmax(s.masked_fill(~causal, float("-inf")), dim=-1)
        for slot in range(2):
            t = qs[0][0] + slot
            if not (0 <= t < qs[0][1]):
                continue
            for r in range(2):
                a, e = max(ks[0][r][0], 0), min(ks[0][r][1], t + 1)
                want = p[t, a:e].sum().item() if e > a else 0.0
                assert abs(mass[0, pi, slot, r].item() - want) < 1e-12


def test_fp8_cache_uniform_attention_closed_form():
    """q = 0: every probability is 1 / (pos + 1) whatever the keys are; out is the prefix mean of the
    dequantised values, and a key scale has no effect at all."""
    b = W.random_batch(805, [50], [1], 4, 2, 16, torch.bfloat16, num_probe_heads=4, max_sel_q=1, max_spans=2,
                       wild_spans=False)
    b.q.zero_()
    b.query_sel[0, 0], b.query_sel[0, 1] = 0, 1
    b8 = W.fp8_cache_variant(b, 806)
    out, mass = oracle.attn_probe_batch(b8)
    _, v = _dequantised(b8)
    table = b8.block_table[0].tolist()
    V = torch.stack([v[table[j // 16], :, j % 16] for j in range(50)])
    for h in range(4):
        assert (out[0, h] - V[:, h // 2].mean(dim=0)).abs().max().item() < 1e-12
    for r, (a, e) in enumerate(b8.key_spans[0].tolist()):
        assert abs(mass[0, 0, 0, r].item() - max(0, min(e, 50) - max(a, 0)) / 50) < 1e-12
    b8.k_scale = b8.k_scale * 3.7
    out2, _ = oracle.attn_probe_batch(b8)
    assert torch.equal(out, out2)


def test_fp8_quantiser_is_round_to_nearest_even_with_saturation():
    """oracle.capture.quantize_e4m3: every finite number of the format maps to its own byte, torch's
    own float8_e4m3fn conversion (a library routine) agrees wherever it is defined (|y| <= 448),
    midpoints go to the even neighbour, values beyond the range saturate, signs of zero survive."""
    from oracle.capture import quantize_e4m3
    finite = torch.tensor([b for b in range(256) if (b & 0x7F) != 0x7F], dtype=torch.uint8)
    assert torch.equal(quantize_e4m3(finite.view(torch.float8_e4m3fn).float(), 1.0), finite)
    gen = torch.Generator().manual_seed(11)
    x = torch.cat([torch.randn(3000, generator=gen) * 4, torch.randn(2000, generator=gen) * 0.01,
                   (torch.rand(500, generator=gen) - 0.5) * 890])
    assert torch.equal(quantize_e4m3(x, 1.0), x.to(torch.float8_e4m3fn).view(torch.uint8))
    # a scale: the bytes of x under scale s are the bytes of fl32(x / s) under scale 1
    s = 0.37
    assert torch.equal(quantize_e4m3(x, s), quantize_e4m3((x.double() / float(torch.tensor(s))).float(), 1.0))
    cases = [(1.0625, 0x38), (1.1875, 0x3A), (2.0 ** -10, 0x00), (3 * 2.0 ** -10, 0x02), (449.0, 0x7E), (1e30, 0x7E),
             (-1e30, 0xFE), (464.0, 0x7E), (-0.0, 0x80), (-2.0 ** -12, 0x80), (0.0, 0x00), (432.0, 0x7E), (400.0, 0x7C)]
    for v, want in cases:
        assert int(quantize_e4m3(torch.tensor([v]), 1.0)[0]) == want, v
    assert int(quantize_e4m3(torch.tensor([float("nan")]), 1.0)[0]) == 0x7F


def test_fp8_kv_write_places_quantised_rows():
    """kv_write into an 8-bit cache: positions as for the 16-bit cache, bytes from the quantiser; rows
    holding numbers the format has (times the head's scale) read back exactly."""
    from oracle.capture import kv_write, quantize_e4m3
    b = W.random_batch(811, [40, 9, 33], [7, 9, 1], 4, 2, 16, torch.bfloat16, num_probe_heads=1)
    b8 = W.fp8_cache_variant(b, 812, pow2_scales=True)
    gen = torch.Generator().manual_seed(813)
    k_new = (torch.randn((b.total_q, 2, 16), generator=gen) * 2).to(torch.bfloat16)
    v_new = (torch.randn((b.total_q, 2, 16), generator=gen) * 2).to(torch.bfloat16)
    # row 3: numbers the format holds, times the scale
    exact = torch.tensor([0x38, 0x41, 0xC5, 0x10, 0x01, 0x7E, 0x80, 0x2A] * 2, dtype=torch.uint8)
    for g in range(2):
        k_new[3, g] = (exact.view(torch.float8_e4m3fn).double() * float(b8.k_scale[g])).to(torch.bfloat16)
    k2, v2 = kv_write(k_new, v_new, b8.block_table, b8.seq_lens, b8.cu_q_lens, b8.k_cache, b8.v_cache, b8.k_scale,
                      b8.v_scale)
    cu, lens, table = b8.cu_q_lens.tolist(), b8.seq_lens.tolist(), b8.block_table.tolist()
    touched = torch.zeros_like(b8.k_cache, dtype=torch.bool)
    for i in range(3):
        n = cu[i + 1] - cu[i]
        for t in range(n):
            pos = lens[i] - n + t
            blk = table[i][pos // 16]
            for g in range(2):
                assert torch.equal(k2[blk, g, pos % 16], quantize_e4m3(k_new[cu[i] + t, g].float(), float(b8.k_scale[g])))
                assert torch.equal(v2[blk, g, pos % 16], quantize_e4m3(v_new[cu[i] + t, g].float(), float(b8.v_scale[g])))
            touched[blk, :, pos % 16] = True
    assert torch.equal(k2[~touched], b8.k_cache[~touched]) and torch.equal(v2[~touched], b8.v_cache[~touched])
    blk, slot = table[0][(lens[0] - 7 + 3) // 16], (lens[0] - 7 + 3) % 16
    assert torch.equal(k2[blk, 0, slot], exact) and torch.equal(k2[blk, 1, slot], exact)
