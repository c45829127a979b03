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
    k_out = torch.zeros((cu_k[-1], len(kvh), d), dtype=q.dtype)
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


def kv_write(k_new, v_new, block_table, seq_lens, cu_q_lens, k_cache, v_cache):
    """Reference for writing the new tokens' K/V into the paged cache (the attention call expects
    them there): returns updated copies of (k_cache, v_cache).  Row t of sequence i goes to position
    L_i - n_i + t; plain loops, single-row copies."""
    k_cache, v_cache = k_cache.cpu().clone(), v_cache.cpu().clone()
    k_new, v_new = k_new.cpu(), v_new.cpu()
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
