"""Seeded synthetic inputs for the hooked-attention path.

This module only draws shapes, index structures and random tensors.  It holds
none of the method's arithmetic (no scores, no softmax, no span sums), so both
the CPU oracle's tests and the GPU parity tests may build their inputs here
without sharing any computation.

The five named workloads are serving-shaped stand-ins: the paper's example
config probes a handful of heads per layer of a 32-head GQA model with
last-token queries and an instruction / data range pair per prompt (Section 2,
config example; Section 2.2, ``input_range``).  No dataset is involved; every
value is drawn from a seeded generator.

Draw order inside every generator is fixed: lengths, block permutation, probe
heads, spans, then Q, K, V, then the steering tensors.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import torch

BLOCK_SIZE = 16
PAD_BLOCK_ID = 0x7FFFFFF0  # block-table filler past ceil(L/B); never dereferenced


@dataclass
class AttnBatch:
    """One ragged batch for ``hook_attn_probe`` (one layer)."""

    name: str
    num_seqs: int
    total_q: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    max_blocks_per_seq: int
    num_blocks: int
    dtype: torch.dtype
    scale: float                      # softmax scale actually used (1/sqrt(d) unless stated)
    q: torch.Tensor                   # [total_q, Hq, d]
    k_cache: torch.Tensor             # [num_blocks, Hkv, B, d]
    v_cache: torch.Tensor             # [num_blocks, Hkv, B, d]
    block_table: torch.Tensor         # int32 [num_seqs, max_blocks_per_seq]
    seq_lens: torch.Tensor            # int32 [num_seqs]
    cu_q_lens: torch.Tensor           # int32 [num_seqs + 1]
    probe_heads: torch.Tensor         # int32 [P], strictly increasing
    max_sel_q: int                    # NQ
    query_sel: torch.Tensor           # int32 [num_seqs, 2] chunk-local [begin, end)
    max_spans: int                    # S
    key_spans: torch.Tensor           # int32 [num_seqs, S, 2] absolute [start, end)
    seed: int = 0
    notes: dict = field(default_factory=dict)
    # 8-bit cache variant (k_cache / v_cache are uint8 E4M3 bytes): one fp32 scale per kv head
    k_scale: Optional[torch.Tensor] = None
    v_scale: Optional[torch.Tensor] = None

    @property
    def num_probe_heads(self) -> int:
        return int(self.probe_heads.numel())

    def q_lens(self) -> List[int]:
        c = self.cu_q_lens.tolist()
        return [c[i + 1] - c[i] for i in range(self.num_seqs)]

    def to(self, device) -> "AttnBatch":
        kw = dict(self.__dict__)
        for k, v in kw.items():
            if isinstance(v, torch.Tensor):
                kw[k] = v.to(device)
        return AttnBatch(**kw)

    def without_probe(self) -> "AttnBatch":
        kw = dict(self.__dict__)
        kw["probe_heads"] = self.probe_heads[:0].clone()
        return AttnBatch(**kw)


FP8_NAN_BYTE = 0x7F            # the NaN pattern of the 8-bit E4M3 format
_FP8_BYTE_RMS = 3.9            # root mean square of the numbers the bytes drawn below stand for


def fp8_cache_variant(b: AttnBatch, seed: int, k_std: float = 1.0, v_std: float = 1.0,
                      pow2_scales: bool = False) -> AttnBatch:
    """The same batch with an 8-bit (E4M3) key/value cache of the same shape.

    Bytes are drawn directly (no quantisation arithmetic here): sign and mantissa bits uniform,
    exponent field triangular over 4..10, so the stored numbers span 1/8 .. 15 with a root mean
    square of about 3.9; the per-kv-head scales are chosen so that keys / values have roughly the
    requested standard deviation (exact powers of two when ``pow2_scales``).  Slots that were
    poisoned with NaN in the 16-bit cache hold the format's NaN byte.
    """
    gen = torch.Generator().manual_seed(seed)
    shape = tuple(b.k_cache.shape)
    Hkv = b.num_kv_heads

    def draw():
        sign = torch.randint(0, 2, shape, generator=gen, dtype=torch.int32)
        expo = 4 + torch.randint(0, 4, shape, generator=gen, dtype=torch.int32) + torch.randint(0, 4, shape, generator=gen, dtype=torch.int32)
        mant = torch.randint(0, 8, shape, generator=gen, dtype=torch.int32)
        return ((sign << 7) | (expo << 3) | mant).to(torch.uint8)

    k8, v8 = draw(), draw()
    dev = b.k_cache.device
    poisoned_k = torch.isnan(b.k_cache.float()).cpu()
    poisoned_v = torch.isnan(b.v_cache.float()).cpu()
    k8[poisoned_k] = FP8_NAN_BYTE
    v8[poisoned_v] = FP8_NAN_BYTE

    def scales(std):
        base = std / _FP8_BYTE_RMS
        if pow2_scales:
            base = 2.0 ** round(math.log2(base))
            return torch.tensor([base * (2.0 ** (g % 3)) for g in range(Hkv)], dtype=torch.float32)
        return torch.tensor([base * (1.0 + 0.25 * g / max(Hkv, 1)) for g in range(Hkv)], dtype=torch.float32)

    kw = dict(b.__dict__)
    kw.update(name=b.name + "_kv8", k_cache=k8.to(dev), v_cache=v8.to(dev), k_scale=scales(k_std).to(dev),
              v_scale=scales(v_std).to(dev))
    return AttnBatch(**kw)


@dataclass
class SteerBatch:
    """Inputs of ``hook_steer``: hidden is modified in place by the callee."""

    name: str
    hidden: torch.Tensor      # [T, D]
    vec: torch.Tensor         # [D], dtype of hidden
    alpha: float
    token_mask: torch.Tensor  # uint8 [T]

    def to(self, device) -> "SteerBatch":
        return SteerBatch(self.name, self.hidden.to(device), self.vec.to(device), self.alpha,
                          self.token_mask.to(device))


def _randn(shape, gen: torch.Generator, dtype: torch.dtype, std: float, device) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 (chunked along dim 0), stored as ``dtype``."""
    shape = tuple(int(s) for s in shape)
    out = torch.empty(shape, dtype=dtype, device=device)
    if out.numel() == 0:
        return out
    rows = shape[0]
    per_row = max(1, out.numel() // max(rows, 1))
    step = max(1, (1 << 26) // per_row)
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        chunk = torch.randn((r1 - r0,) + shape[1:], generator=gen, dtype=torch.float32, device=device)
        if std != 1.0:
            chunk.mul_(std)
        out[r0:r1] = chunk.to(dtype)
    return out


def build_paged(
    name: str,
    seq_lens: Sequence[int],
    q_lens: Sequence[int],
    num_q_heads: int,
    num_kv_heads: int,
    head_dim: int,
    dtype: torch.dtype,
    std: float,
    gen: torch.Generator,
    probe_heads: Sequence[int],
    query_sel: Sequence[Tuple[int, int]],
    key_spans: Sequence[Sequence[Tuple[int, int]]],
    max_sel_q: Optional[int] = None,
    max_spans: Optional[int] = None,
    block_size: int = BLOCK_SIZE,
    shuffle: bool = True,
    pool_factor: float = 1.25,
    poison: bool = True,
    scale: Optional[float] = None,
    device="cpu",
    seed: int = 0,
    block_perm: Optional[torch.Tensor] = None,
) -> AttnBatch:
    """Assemble a batch: draws the block permutation (unless given), then Q, K, V.

    The KV cache is filled with i.i.d. draws for every slot and then poisoned:
    blocks no sequence owns and the tail slots of each sequence's last block are
    set to NaN, and block-table entries past ceil(L/B) hold ``PAD_BLOCK_ID``, so a
    stray read shows up as a non-finite output or a fault-free wrong value.
    """
    num_seqs = len(seq_lens)
    assert len(q_lens) == num_seqs
    B = block_size
    nblk = [(int(L) + B - 1) // B for L in seq_lens]
    need = sum(nblk)
    num_blocks = max(1, int(math.ceil(need * pool_factor))) if shuffle else max(1, need)
    max_blocks = max(1, max(nblk) if nblk else 1)
    if block_perm is None:
        if shuffle:
            block_perm = torch.randperm(num_blocks, generator=gen)
        else:
            block_perm = torch.arange(num_blocks)
    table = torch.full((num_seqs, max_blocks), PAD_BLOCK_ID, dtype=torch.int32)
    used = 0
    for i in range(num_seqs):
        table[i, : nblk[i]] = block_perm[used: used + nblk[i]].to(torch.int32)
        used += nblk[i]
    cu = [0]
    for n in q_lens:
        cu.append(cu[-1] + int(n))
    total_q = cu[-1]

    gdev = gen
    if str(device) != "cpu":
        gdev = torch.Generator(device=device)
        gdev.manual_seed(int(torch.randint(0, 2**31 - 1, (1,), generator=gen)))
    q = _randn((total_q, num_q_heads, head_dim), gdev, dtype, std, device)
    k_cache = _randn((num_blocks, num_kv_heads, B, head_dim), gdev, dtype, std, device)
    v_cache = _randn((num_blocks, num_kv_heads, B, head_dim), gdev, dtype, std, device)
    if poison:
        owned = torch.zeros(num_blocks, dtype=torch.bool)
        owned[block_perm[:need].long()] = True
        free_ids = (~owned).nonzero().flatten().to(device)
        if free_ids.numel():
            k_cache[free_ids] = float("nan")
            v_cache[free_ids] = float("nan")
        for i in range(num_seqs):
            L = int(seq_lens[i])
            tail = L % B
            if L > 0 and tail:
                blk = int(table[i, nblk[i] - 1])
                k_cache[blk, :, tail:, :] = float("nan")
                v_cache[blk, :, tail:, :] = float("nan")

    P = len(probe_heads)
    NQ = max_sel_q if max_sel_q is not None else max([e - b for b, e in query_sel] + [1])
    S = max_spans if max_spans is not None else max([len(s) for s in key_spans] + [1])
    qs = torch.zeros((num_seqs, 2), dtype=torch.int32)
    ks = torch.zeros((num_seqs, S, 2), dtype=torch.int32)
    for i in range(num_seqs):
        qs[i, 0], qs[i, 1] = int(query_sel[i][0]), int(query_sel[i][1])
        for r, (a, b) in enumerate(key_spans[i]):
            ks[i, r, 0], ks[i, r, 1] = int(a), int(b)
    return AttnBatch(
        name=name, num_seqs=num_seqs, total_q=total_q, num_q_heads=num_q_heads,
        num_kv_heads=num_kv_heads, head_dim=head_dim, block_size=B,
        max_blocks_per_seq=max_blocks, num_blocks=num_blocks, dtype=dtype,
        scale=float(scale) if scale is not None else 1.0 / math.sqrt(head_dim),
        q=q, k_cache=k_cache, v_cache=v_cache, block_table=table.to(device),
        seq_lens=torch.tensor(list(seq_lens), dtype=torch.int32, device=device),
        cu_q_lens=torch.tensor(cu, dtype=torch.int32, device=device),
        probe_heads=torch.tensor(sorted(int(h) for h in probe_heads), dtype=torch.int32, device=device),
        max_sel_q=int(NQ), query_sel=qs.to(device), max_spans=int(S), key_spans=ks.to(device), seed=seed,
    )


def _randint(lo: int, hi: int, n: int, gen: torch.Generator) -> List[int]:
    """n integers uniform in [lo, hi] (inclusive)."""
    return torch.randint(lo, hi + 1, (n,), generator=gen).tolist()


def _distinct_heads(count: int, num_heads: int, gen: torch.Generator) -> List[int]:
    return sorted(torch.randperm(num_heads, generator=gen)[:count].tolist())


# ---------------------------------------------------------------------------
# The five named workloads.  `peaked=True` gives the parity-only twin with
# unscaled N(0,1) values (logit sigma ~ 1 instead of ~ 0.01).  `shrink`
# divides sequence lengths / counts for quick CPU-side checks; shrink=1 is the
# stated size.
# ---------------------------------------------------------------------------

def c1_tiny_prefill(device="cpu") -> Tuple[AttnBatch, SteerBatch]:
    """1 sequence of 256 tokens, 8 q = 8 kv heads, d 64, fp32 N(0,1), seed 0."""
    gen = torch.Generator().manual_seed(0)
    L = 256
    b = build_paged("c1_tiny_prefill", [L], [L], 8, 8, 64, torch.float32, 1.0, gen,
                    probe_heads=list(range(8)), query_sel=[(L - 1, L)], key_spans=[[(16, 64)]],
                    shuffle=False, poison=False, device=device, seed=0)
    hidden = _randn((L, 512), gen, torch.float32, 1.0, "cpu").to(device)
    vec = _randn((512,), gen, torch.float32, 1.0, "cpu").to(device)
    mask = torch.zeros(L, dtype=torch.uint8)
    mask[200:256] = 1
    return b, SteerBatch("c1_steer", hidden, vec, 4.0, mask.to(device))


def c2_prefill_8b(device="cpu", peaked: bool = False, shrink: int = 1) -> AttnBatch:
    """16 ragged prefills, lens U[512,2048], 32 q / 8 kv heads, d 128, bf16, seed 1."""
    gen = torch.Generator().manual_seed(1)
    nseq = max(1, 16 // (1 if shrink == 1 else min(shrink, 4)))
    lens = [max(9, L // shrink) for L in _randint(512, 2048, 16, gen)][:nseq]
    # permutation is drawn inside build_paged; heads and spans are drawn first from a
    # forked generator so the documented order (lengths, permutation, heads, spans) holds
    nblk = sum((L + BLOCK_SIZE - 1) // BLOCK_SIZE for L in lens)
    perm = torch.randperm(max(1, int(math.ceil(nblk * 1.25))), generator=gen)
    heads = _distinct_heads(12, 32, gen)
    spans = []
    for L in lens:
        ln = min(L, max(1, _randint(64, 256, 1, gen)[0] // shrink))
        st = _randint(0, L - ln, 1, gen)[0]
        spans.append([(st, st + ln)])
    qsel = [(L - 8, L) for L in lens]
    std = 1.0 if peaked else 128 ** -0.5
    return build_paged("c2_prefill_8b" + ("_peaked" if peaked else ""), lens, lens, 32, 8, 128,
                       torch.bfloat16, std, gen, heads, qsel, spans, device=device, seed=1,
                       block_perm=perm)


def c3_decode_8b(device="cpu", peaked: bool = False, shrink: int = 1) -> AttnBatch:
    """256 decodes, ctx U[1024,8192], 32/8 heads, d 128, bf16, all heads probed, seed 2."""
    gen = torch.Generator().manual_seed(2)
    nseq = max(2, 256 // shrink)
    lens = [max(2, L // shrink) for L in _randint(1024, 8192, 256, gen)][:nseq]
    nblk = sum((L + BLOCK_SIZE - 1) // BLOCK_SIZE for L in lens)
    perm = torch.randperm(max(1, int(math.ceil(nblk * 1.25))), generator=gen)
    heads = list(range(32))
    spans = [[(0, min(L, max(1, I // shrink)))] for L, I in zip(lens, _randint(32, 512, 256, gen))]
    qsel = [(0, 1)] * nseq
    std = 1.0 if peaked else 128 ** -0.5
    return build_paged("c3_decode_8b" + ("_peaked" if peaked else ""), lens, [1] * nseq, 32, 8, 128,
                       torch.bfloat16, std, gen, heads, qsel, spans, device=device, seed=2,
                       block_perm=perm)


def c4_long_prefill_70b(device="cpu", peaked: bool = False, shrink: int = 1) -> AttnBatch:
    """1 sequence of 32768 tokens, 64 q / 8 kv heads, d 128, bf16, seed 3.

    Four disjoint 1024-token spans at tile-unaligned starts (a retrieved-document
    layout), queries = the last 32 tokens.
    """
    gen = torch.Generator().manual_seed(3)
    L = 32768 // shrink
    nblk = (L + BLOCK_SIZE - 1) // BLOCK_SIZE
    perm = torch.randperm(int(math.ceil(nblk * 1.25)), generator=gen)
    heads = _distinct_heads(16, 64, gen)
    starts = [4099, 10247, 16411, 22541]
    spans = [[(s // shrink, s // shrink + 1024 // shrink) for s in starts]]
    qsel = [(L - 32, L)]
    std = 1.0 if peaked else 128 ** -0.5
    return build_paged("c4_long_prefill_70b" + ("_peaked" if peaked else ""), [L], [L], 64, 8, 128,
                       torch.bfloat16, std, gen, heads, qsel, spans, device=device, seed=3,
                       block_perm=perm)


def c5_mixed(device="cpu", peaked: bool = False, shrink: int = 1,
             prior_context: bool = False) -> Tuple[AttnBatch, SteerBatch]:
    """64 decodes (ctx 4096) then 4 prefill chunks of 2048 tokens, 32/8 heads, bf16, seed 4.

    ``prior_context`` gives the parity-only variant whose prefill chunks sit on
    2048 tokens of earlier context (L = 4096, n = 2048).
    """
    gen = torch.Generator().manual_seed(4)
    nd = max(2, 64 // shrink)
    ctx, chunk = 4096 // shrink, 2048 // shrink
    lens = [ctx] * nd + [chunk * (2 if prior_context else 1)] * 4
    qlens = [1] * nd + [chunk] * 4
    nblk = sum((L + BLOCK_SIZE - 1) // BLOCK_SIZE for L in lens)
    perm = torch.randperm(int(math.ceil(nblk * 1.25)), generator=gen)
    heads = _distinct_heads(8, 32, gen)
    spans = [[(0, max(1, 256 // shrink))] for _ in lens]
    qsel = [(n - 1, n) for n in qlens]
    std = 1.0 if peaked else 128 ** -0.5
    b = build_paged("c5_mixed" + ("_prior" if prior_context else "") + ("_peaked" if peaked else ""),
                    lens, qlens, 32, 8, 128, torch.bfloat16, std, gen, heads, qsel, spans,
                    device=device, seed=4, block_perm=perm)
    # hidden has 192 padding rows past the batch's 8256 tokens; they are never steered
    T = (8448 // shrink) if shrink > 1 else 8448
    T = max(T, b.total_q)
    D = 4096 if shrink == 1 else max(64, 4096 // shrink)
    gs = gen
    if str(device) != "cpu":
        gs = torch.Generator(device=device)
        gs.manual_seed(int(torch.randint(0, 2**31 - 1, (1,), generator=gen)))
    hidden = _randn((T, D), gs, torch.bfloat16, 1.0, device)
    v = torch.randn(D, generator=gen, dtype=torch.float32)
    vec = (v / v.norm()).to(torch.bfloat16).to(device)
    mask = torch.zeros(T, dtype=torch.uint8)
    mask[nd: b.total_q] = 1
    return b, SteerBatch("c5_steer", hidden, vec, 8.0, mask.to(device))


def c6_reranker(device="cpu", peaked: bool = False, shrink: int = 1, num_prompts: int = 4) -> AttnBatch:
    """Re-ranking prompts: a 64-token preamble, 40..100 documents of 64..256 tokens, a 32-token
    question; one span per document, the question rows selected, 8 probed heads; 32 q / 8 kv
    heads, d 128, bf16, seed 5.  Fresh prefill (L = n).  Spans beyond a prompt's document count
    are empty."""
    gen = torch.Generator().manual_seed(5)
    lens, spans = [], []
    for _ in range(num_prompts):
        ndoc = max(2, _randint(40, 100, 1, gen)[0] // shrink)
        pos = max(1, 64 // shrink)
        sp = []
        for dl in _randint(64, 256, ndoc, gen):
            dl = max(1, dl // shrink)
            sp.append((pos, pos + dl))
            pos += dl
        spans.append(sp)
        lens.append(pos + 32)
    nblk = sum((L + BLOCK_SIZE - 1) // BLOCK_SIZE for L in lens)
    perm = torch.randperm(max(1, int(math.ceil(nblk * 1.25))), generator=gen)
    heads = _distinct_heads(8, 32, gen)
    qsel = [(L - 32, L) for L in lens]
    std = 1.0 if peaked else 128 ** -0.5
    return build_paged("c6_reranker" + ("_peaked" if peaked else ""), lens, lens, 32, 8, 128, torch.bfloat16, std,
                       gen, heads, qsel, spans, max_sel_q=32, device=device, seed=5, block_perm=perm)


def random_batch(
    seed: int,
    seq_lens: Sequence[int],
    q_lens: Sequence[int],
    num_q_heads: int = 8,
    num_kv_heads: int = 2,
    head_dim: int = 128,
    dtype: torch.dtype = torch.bfloat16,
    std: float = 1.0,
    num_probe_heads: int = 3,
    max_sel_q: int = 4,
    max_spans: int = 2,
    block_size: int = BLOCK_SIZE,
    shuffle: bool = True,
    poison: bool = True,
    device="cpu",
    scale: Optional[float] = None,
    wild_spans: bool = True,
) -> AttnBatch:
    """General ragged batch for parity and edge-case tests.

    Spans are drawn so that some are empty, some reach past the causal horizon or
    the sequence end, some start below zero and some overlap (``wild_spans``).
    """
    gen = torch.Generator().manual_seed(seed)
    nblk = sum((int(L) + block_size - 1) // block_size for L in seq_lens)
    perm = None
    if shuffle:
        perm = torch.randperm(max(1, int(math.ceil(nblk * 1.25))), generator=gen)
    heads = _distinct_heads(min(num_probe_heads, num_q_heads), num_q_heads, gen)
    qsel, spans = [], []
    for L, n in zip(seq_lens, q_lens):
        if n == 0:
            qsel.append((0, 0))
        else:
            cnt = min(n, _randint(0, max_sel_q, 1, gen)[0])
            b = _randint(0, n - cnt, 1, gen)[0]
            qsel.append((b, b + cnt))
        sp = []
        for r in range(max_spans):
            lo = -4 if wild_spans else 0
            hi = L + 4 if wild_spans else L
            a, e = sorted(_randint(lo, max(lo, hi), 2, gen))
            if wild_spans and _randint(0, 5, 1, gen)[0] == 0:
                a, e = e, a  # start >= end: empty
            sp.append((a, e))
        spans.append(sp)
    return build_paged(f"random_{seed}", list(seq_lens), list(q_lens), num_q_heads, num_kv_heads,
                       head_dim, dtype, std, gen, heads, qsel, spans, max_sel_q=max_sel_q,
                       max_spans=max_spans, block_size=block_size, shuffle=shuffle, poison=poison,
                       device=device, seed=seed, block_perm=perm, scale=scale)


def steer_batch(seed: int, T: int, D: int, dtype: torch.dtype, alpha: float,
                mask_frac: float = 0.5, device="cpu") -> SteerBatch:
    gen = torch.Generator().manual_seed(seed)
    mask = (torch.rand(T, generator=gen) < mask_frac).to(torch.uint8)
    hidden = _randn((T, D), gen, dtype, 1.0, "cpu").to(device)
    vec = _randn((D,), gen, dtype, 1.0, "cpu").to(device)
    return SteerBatch(f"steer_{seed}", hidden, vec, float(alpha), mask.to(device))
