"""ctypes front end of the fp64 CPU oracle in ``hook_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg call this; the GPU library neither imports nor links it, and
nothing here touches the GPU library.  All tensors are CPU tensors; bf16 tensors
are handed to C as their raw 16-bit patterns, so the oracle sees exactly the
stored (already rounded) inputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hook_oracle.c")
_LIB = os.path.join(_HERE, "libhook_oracle.so")
_lib = None

_DT = {torch.bfloat16: 0, torch.float32: 1}


def lib_path() -> str:
    return _LIB


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        i32, dbl, vp = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        lib.hook_oracle_attn_probe.restype = i32
        lib.hook_oracle_attn_probe.argtypes = [i32] * 9 + [dbl] + [vp] * 6 + [i32, vp, i32, vp, i32, vp,
                                                                         i32, vp, vp, vp]
        lib.hook_oracle_attn_probe_kv8.restype = i32
        lib.hook_oracle_attn_probe_kv8.argtypes = [i32] * 9 + [dbl] + [vp] * 8 + [i32, vp, i32, vp, i32, vp,
                                                                             i32, vp, vp, vp]
        lib.hook_oracle_fp8_e4m3_value.restype = dbl
        lib.hook_oracle_fp8_e4m3_value.argtypes = [ctypes.c_uint8]
        lib.hook_oracle_steer.restype = i32
        lib.hook_oracle_steer.argtypes = [vp, vp, ctypes.c_float, vp, i32, i32, i32, vp]
        lib.hook_oracle_residual_steer.restype = i32
        lib.hook_oracle_residual_steer.argtypes = [vp, vp, vp, ctypes.c_float, vp, i32, i32, i32, vp]
        lib.hook_oracle_round_bf16.restype = ctypes.c_uint16
        lib.hook_oracle_round_bf16.argtypes = [dbl]
        lib.hook_oracle_num_threads.restype = i32
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().hook_oracle_num_threads())


def _cpu(t: torch.Tensor, dtype=None) -> torch.Tensor:
    t = t.detach().to("cpu")
    if dtype is not None:
        t = t.to(dtype)
    return t.contiguous()


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else ctypes.c_void_p(0)


def fp8_e4m3_value(byte: int) -> float:
    """The number an 8-bit E4M3 cache byte stands for (NaN for the one NaN pattern per sign)."""
    return float(_load().hook_oracle_fp8_e4m3_value(int(byte) & 0xFF))


def attn_probe(q, k_cache, v_cache, block_table, seq_lens, cu_q_lens, probe_heads, max_sel_q,
               query_sel, max_spans, key_spans, scale: float,
               rows: Optional[Sequence[int]] = None, k_scale=None, v_scale=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Return (out fp64 [total_q, Hq, d], mass fp64 [num_seqs, P, NQ, S]).

    ``rows`` restricts the computation to the given global query rows; other rows
    of ``out`` come back as NaN so an accidental comparison cannot pass.
    uint8 caches are 8-bit E4M3 bytes and need ``k_scale`` / ``v_scale`` ([Hkv] fp32).
    """
    lib = _load()
    q, k_cache, v_cache = _cpu(q), _cpu(k_cache), _cpu(v_cache)
    kv8 = k_cache.dtype == torch.uint8
    assert q.dtype in _DT and v_cache.dtype == k_cache.dtype and (kv8 or k_cache.dtype == q.dtype)
    if kv8:
        assert k_scale is not None and v_scale is not None
        k_scale, v_scale = _cpu(k_scale, torch.float32), _cpu(v_scale, torch.float32)
        assert k_scale.numel() == k_cache.shape[1] and v_scale.numel() == k_cache.shape[1]
    block_table = _cpu(block_table, torch.int32)
    seq_lens = _cpu(seq_lens, torch.int32)
    cu_q_lens = _cpu(cu_q_lens, torch.int32)
    probe_heads = _cpu(probe_heads, torch.int32)
    query_sel = _cpu(query_sel, torch.int32)
    key_spans = _cpu(key_spans, torch.int32)
    total_q, Hq, d = q.shape
    num_blocks, Hkv, B, d2 = k_cache.shape
    assert d2 == d and v_cache.shape == k_cache.shape
    num_seqs, max_blocks = block_table.shape
    P, NQ, S = int(probe_heads.numel()), int(max_sel_q), int(max_spans)
    out = torch.full((total_q, Hq, d), float("nan"), dtype=torch.float64)
    mass = torch.zeros((num_seqs, P, NQ, S), dtype=torch.float64)
    rows_t = None
    if rows is not None:
        rows_t = torch.tensor(list(rows), dtype=torch.int32)
    tail = (P, _ptr(probe_heads), NQ, _ptr(query_sel), S, _ptr(key_spans),
            0 if rows_t is None else int(rows_t.numel()),
            ctypes.c_void_p(rows_t.data_ptr()) if rows_t is not None else ctypes.c_void_p(0),
            _ptr(out), _ptr(mass))
    head = (num_seqs, total_q, Hq, Hkv, d, B, max_blocks, num_blocks, _DT[q.dtype], float(scale))
    if kv8:
        rc = lib.hook_oracle_attn_probe_kv8(*head, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale),
                                            _ptr(block_table), _ptr(seq_lens), _ptr(cu_q_lens), *tail)
    else:
        rc = lib.hook_oracle_attn_probe(*head, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                        _ptr(seq_lens), _ptr(cu_q_lens), *tail)
    if rc != 0:
        raise ValueError(f"hook_oracle_attn_probe rejected its arguments (code {rc})")
    return out, mass


def attn_probe_batch(b, rows: Optional[Sequence[int]] = None):
    """Same, taking any object with the batch attributes (duck-typed, nothing imported)."""
    return attn_probe(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.cu_q_lens, b.probe_heads,
                      b.max_sel_q, b.query_sel, b.max_spans, b.key_spans, b.scale, rows=rows,
                      k_scale=getattr(b, "k_scale", None), v_scale=getattr(b, "v_scale", None))


def steer(hidden: torch.Tensor, vec: torch.Tensor, alpha: float, token_mask: torch.Tensor) -> torch.Tensor:
    """Return the steered copy of ``hidden`` (input untouched), dtype preserved."""
    lib = _load()
    hidden, vec = _cpu(hidden), _cpu(vec)
    assert hidden.dtype in _DT and vec.dtype == hidden.dtype
    mask = _cpu(token_mask, torch.uint8)
    T, D = hidden.shape
    assert vec.numel() == D and mask.numel() == T
    out = torch.empty_like(hidden)
    rc = lib.hook_oracle_steer(_ptr(hidden), _ptr(vec), float(alpha), _ptr(mask), T, D, _DT[hidden.dtype],
                               _ptr(out))
    if rc != 0:
        raise ValueError(f"hook_oracle_steer rejected its arguments (code {rc})")
    return out


def residual_steer(hidden: torch.Tensor, delta: torch.Tensor, vec: torch.Tensor, alpha: float,
                   token_mask: Optional[torch.Tensor]) -> torch.Tensor:
    """hidden + delta (+ alpha * vec on masked rows), rounded once; returns a new tensor."""
    lib = _load()
    hidden, delta, vec = _cpu(hidden), _cpu(delta), _cpu(vec)
    assert hidden.dtype in _DT and vec.dtype == hidden.dtype and delta.dtype == hidden.dtype
    assert delta.shape == hidden.shape
    mask = None if token_mask is None else _cpu(token_mask, torch.uint8)
    T, D = hidden.shape
    out = torch.empty_like(hidden)
    rc = lib.hook_oracle_residual_steer(_ptr(hidden), _ptr(delta), _ptr(vec), float(alpha),
                                        None if mask is None else _ptr(mask), T, D, _DT[hidden.dtype], _ptr(out))
    if rc != 0:
        raise ValueError(f"hook_oracle_residual_steer rejected its arguments (code {rc})")
    return out


def steer_batch(s) -> torch.Tensor:
    return steer(s.hidden, s.vec, s.alpha, s.token_mask)


def round_bf16(x: float) -> int:
    """Bit pattern of x rounded to bf16 (round-to-nearest-even)."""
    return int(_load().hook_oracle_round_bf16(float(x)))
