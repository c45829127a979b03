"""Reference for the compact q/k capture (TEST INFRASTRUCTURE ONLY; no code shared with the GPU
library).  Section 2.1 (qkv_hook): per hooked layer the hook keeps the queries (last token or all
tokens) and all keys, split per batch item.  Here: explicit loops and single-element copies, so
the result is the definition written out; values are copied, never computed."""
from typing import Sequence, Tuple

import torch


def capture_qk(q, k_cache, block_table, seq_lens, cu_q_lens, probe_heads, max_sel_q, query_sel,
               capture_kv_heads) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (q_out [num_seqs, P, NQ, d], k_out [total_k, KH, d], cu_k_lens [num_seqs + 1])."""
    q, k_cache = q.cpu(), k_cache.cpu()
    table = block_table.cpu().tolist()
    lens = seq_lens.cpu().tolist()
    cu = cu_q_lens.cpu().tolist()
    heads = probe_heads.cpu().tolist()
    qsel = query_sel.cpu().tolist()
    kvh = capture_kv_heads.cpu().tolist()
    num_seqs = len(lens)
    B, d = k_cache.shape[2], k_cache.shape[3]
    cu_k = [0]
    for L in lens:
        cu_k.append(cu_k[-1] + L)
    q_out = torch.zeros((num_seqs, len(heads), max_sel_q, d), dtype=q.dtype)
    k_out = torch.zeros((cu_k[-1], len(kvh), d), dtype=k_cache.dtype)   # the cache's elements as they are (bytes of an 8-bit cache)
    for i in range(num_seqs):
        n = cu[i + 1] - cu[i]
        for p, h in enumerate(heads):
            for tt in range(max_sel_q):
                t = qsel[i][0] + tt
                if 0 <= t < qsel[i][1] and t < n:
                    q_out[i, p, tt] = q[cu[i] + t, h]
        for j in range(lens[i]):
            blk = table[i][j // B]
            for c, g in enumerate(kvh):
                k_out[cu_k[i] + j, c] = k_cache[blk, g, j % B]
    return q_out, k_out, torch.tensor(cu_k, dtype=torch.int32)


def _e4m3_table():
    """The 127 non-negative finite numbers of the 8-bit E4M3 format, by byte value 0x00 .. 0x7E,
    written out from the format's definition (bias 7, 3 mantissa bits, subnormals for E = 0)."""
    vals = []
    for byte in range(0x7F):
        E, M = byte >> 3, byte & 7
        vals.append((M / 8.0) * 2.0 ** -6 if E == 0 else (1.0 + M / 8.0) * 2.0 ** (E - 7))
    return vals


def quantize_e4m3(x: torch.Tensor, scale: float) -> torch.Tensor:
    """Bytes of an 8-bit E4M3 cache for the fp32 / bf16 values `x` under one scale:
    y = x / scale as a correctly rounded fp32 quotient, clamped to [-448, 448] (the format has no
    infinities: out-of-range values saturate), then the NEAREST representable number, ties to the
    one whose last mantissa bit is 0; the sign bit is kept (so -0 and negative underflow give 0x80),
    NaN gives the NaN byte 0x7F.  Written as a search of the 127-entry table: the definition of
    round-to-nearest-even, not a bit trick."""
    table = _e4m3_table()
    # the fp64 quotient of two fp32 numbers rounded to fp32 is the correctly rounded fp32 quotient
    y = (x.double() / float(torch.tensor(scale, dtype=torch.float32))).float().double().flatten().tolist()
    out = []
    for v in y:
        if v != v:
            out.append(0x7F)
            continue
        neg = (v < 0) or (v == 0 and str(v).startswith("-"))
        a = min(abs(v), 448.0)
        best = 0
        for byte in range(1, 0x7F):
            d_new, d_best = abs(table[byte] - a), abs(table[best] - a)
            if d_new < d_best or (d_new == d_best and (byte & 1) == 0):
                best = byte
        out.append(best | (0x80 if neg else 0))
    return torch.tensor(out, dtype=torch.uint8).reshape(x.shape)


def kv_write(k_new, v_new, block_table, seq_lens, cu_q_lens, k_cache, v_cache, k_scale=None, v_scale=None):
    """Reference for writing the new tokens' K/V into the paged cache (the attention call expects
    them there): returns updated copies of (k_cache, v_cache).  Row t of sequence i goes to position
    L_i - n_i + t; plain loops, single-row copies.  With uint8 caches (8-bit E4M3) and per-kv-head
    scales the rows are quantised on the way (quantize_e4m3)."""
    k_cache, v_cache = k_cache.cpu().clone(), v_cache.cpu().clone()
    k_new, v_new = k_new.cpu(), v_new.cpu()
    if k_cache.dtype == torch.uint8:
        ks, vs = k_scale.cpu().tolist(), v_scale.cpu().tolist()
        k_new = torch.stack([quantize_e4m3(k_new[:, g].float(), ks[g]) for g in range(k_new.shape[1])], dim=1)
        v_new = torch.stack([quantize_e4m3(v_new[:, g].float(), vs[g]) for g in range(v_new.shape[1])], dim=1)
    table = block_table.cpu().tolist()
    lens = seq_lens.cpu().tolist()
    cu = cu_q_lens.cpu().tolist()
    B = k_cache.shape[2]
    for i, L in enumerate(lens):
        n = cu[i + 1] - cu[i]
        if n > L:
            continue
        for t in range(n):
            pos = L - n + t
            blk = table[i][pos // B]
            k_cache[blk, :, pos % B] = k_new[cu[i] + t]
            v_cache[blk, :, pos % B] = v_new[cu[i] + t]
    return k_cache, v_cache
