"""ctypes front end of libhook.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
``include/hook_api.h``; torch is used for device memory and the current stream.
There is no CPU fallback: loading fails loudly if the library has not been
built (``python -m paper_2603_06588_amd.build``).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhook.so")

HOOK_OK = 0
HOOK_BF16, HOOK_F32 = 0, 1
_DT = {torch.bfloat16: HOOK_BF16, torch.float32: HOOK_F32}
EXPORTS = ["hook_attn_probe_workspace_bytes", "hook_attn_probe", "hook_attn_probe_static", "hook_attn_probe_static_capacity",
           "hook_attn_probe_device_status", "hook_attn_probe_validate", "hook_span_mass", "hook_span_mass_workspace_bytes",
           "hook_steer", "hook_residual_add_steer", "hook_kv_write", "hook_capture_qk", "hook_reduce_mass", "hook_parse_layer_heads", "hook_parse_config_json", "hook_status_string", "hook_version"]


class HookAttnProbeArgs(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32), ("total_q", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32), ("num_blocks", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("q", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p), ("cu_q_lens", ctypes.c_void_p),
        ("num_probe_heads", ctypes.c_int32), ("probe_heads", ctypes.c_void_p),
        ("max_sel_q", ctypes.c_int32), ("query_sel", ctypes.c_void_p),
        ("max_spans", ctypes.c_int32), ("key_spans", ctypes.c_void_p),
        ("out", ctypes.c_void_p), ("mass", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p), ("batch_kind", ctypes.c_int32), ("plan_mode", ctypes.c_int32),
        ("kv_dtype", ctypes.c_int32), ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
        ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p),
    ]


class HookCaptureQkArgs(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32), ("total_q", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32), ("num_blocks", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("q", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p), ("cu_q_lens", ctypes.c_void_p),
        ("num_probe_heads", ctypes.c_int32), ("probe_heads", ctypes.c_void_p),
        ("max_sel_q", ctypes.c_int32), ("query_sel", ctypes.c_void_p),
        ("num_capture_kv_heads", ctypes.c_int32), ("capture_kv_heads", ctypes.c_void_p),
        ("cu_k_lens", ctypes.c_void_p), ("total_k", ctypes.c_int32),
        ("q_out", ctypes.c_void_p), ("k_out", ctypes.c_void_p), ("stream", ctypes.c_void_p),
        ("kv_dtype", ctypes.c_int32),
    ]


class HookKvWriteArgs(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32), ("total_q", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p), ("cu_q_lens", ctypes.c_void_p),
        ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p), ("stream", ctypes.c_void_p),
        ("kv_dtype", ctypes.c_int32), ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
    ]


class HookReduceArgs(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32), ("num_probe_heads", ctypes.c_int32), ("max_sel_q", ctypes.c_int32),
        ("max_spans", ctypes.c_int32),
        ("mass", ctypes.c_void_p), ("query_sel", ctypes.c_void_p), ("cu_q_lens", ctypes.c_void_p),
        ("head_weights", ctypes.c_void_p),
        ("mode", ctypes.c_int32), ("span_a", ctypes.c_int32), ("span_b", ctypes.c_int32),
        ("accumulate", ctypes.c_int32),
        ("scores", ctypes.c_void_p), ("stream", ctypes.c_void_p),
    ]


REDUCE_SPAN_MEAN, REDUCE_RATIO_MEAN, REDUCE_RATIO_OF_SUMS = 0, 1, 2
BATCH_MIXED, BATCH_PREFILL_ONLY, BATCH_DECODE_ONLY = 0, 1, 2
KV_SAME, KV_FP8_E4M3 = 0, 1
PLAN_FRESH, PLAN_REUSE = 0, 1
(BAD_ROWS_EXCEED_CONTEXT, BAD_CONTEXT_TOO_LONG, BAD_LENGTH, BAD_BATCH_KIND, BAD_BLOCK_ID, BAD_PROBE_HEADS,
 BAD_QUERY_SEL) = 1, 2, 4, 8, 16, 32, 64


class HookError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {status_string(status)} (hook_status {int(status)})")


_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_06588_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        ap = ctypes.POINTER(HookAttnProbeArgs)
        lib.hook_attn_probe_workspace_bytes.restype = ctypes.c_size_t
        lib.hook_attn_probe_workspace_bytes.argtypes = [ap]
        lib.hook_attn_probe.restype = ctypes.c_int
        lib.hook_attn_probe.argtypes = [ap]
        lib.hook_attn_probe_static.restype = ctypes.c_int
        lib.hook_attn_probe_static.argtypes = [ap]
        lib.hook_attn_probe_static_capacity.restype = ctypes.c_size_t
        lib.hook_attn_probe_static_capacity.argtypes = []
        lib.hook_attn_probe_device_status.restype = ctypes.c_int
        lib.hook_attn_probe_device_status.argtypes = [ctypes.c_void_p, ctypes.c_void_p,
                                                      ctypes.POINTER(ctypes.c_int32)]
        lib.hook_attn_probe_validate.restype = ctypes.c_int
        lib.hook_attn_probe_validate.argtypes = [ap, ctypes.POINTER(ctypes.c_int32)]
        lib.hook_steer.restype = ctypes.c_int
        lib.hook_steer.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                   ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.hook_capture_qk.restype = ctypes.c_int
        lib.hook_capture_qk.argtypes = [ctypes.POINTER(HookCaptureQkArgs)]
        lib.hook_kv_write.restype = ctypes.c_int
        lib.hook_kv_write.argtypes = [ctypes.POINTER(HookKvWriteArgs)]
        lib.hook_span_mass_workspace_bytes.restype = ctypes.c_size_t
        lib.hook_span_mass_workspace_bytes.argtypes = [ctypes.POINTER(HookAttnProbeArgs)]
        lib.hook_span_mass.restype = ctypes.c_int
        lib.hook_span_mass.argtypes = [ctypes.POINTER(HookAttnProbeArgs)]
        lib.hook_residual_add_steer.restype = ctypes.c_int
        lib.hook_residual_add_steer.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                                ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                ctypes.c_void_p]
        lib.hook_reduce_mass.restype = ctypes.c_int
        lib.hook_reduce_mass.argtypes = [ctypes.POINTER(HookReduceArgs)]
        lib.hook_parse_layer_heads.restype = ctypes.c_int
        lib.hook_parse_layer_heads.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int32),
                                               ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                               ctypes.POINTER(ctypes.c_int32)]
        lib.hook_parse_config_json.restype = ctypes.c_int
        lib.hook_parse_config_json.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int32),
                                               ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                               ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.hook_status_string.restype = ctypes.c_char_p
        lib.hook_status_string.argtypes = [ctypes.c_int]
        lib.hook_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().hook_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().hook_version())


def _p(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None or t.numel() == 0 else t.data_ptr()


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


class AttnProbeCall:
    """A marshalled ``hook_attn_probe`` call that can be launched repeatedly.

    Holds references to every tensor it points at, the output tensors and the
    workspace, so relaunching costs one ctypes call and no allocation.
    """

    def __init__(self, q, k_cache, v_cache, block_table, seq_lens, cu_q_lens, probe_heads=None, max_sel_q=1,
                 query_sel=None, max_spans=1, key_spans=None, scale: float = 0.0, out=None, mass=None,
                 workspace=None, batch_kind: int = 0, plan_mode: int = 0, k_scale=None, v_scale=None,
                 k_new=None, v_new=None):
        lib = load_library()
        if q.dtype not in _DT:
            raise HookError(3, "hook_attn_probe (dtype)")
        dev = q.device
        self.keep = [q, k_cache, v_cache, block_table, seq_lens, cu_q_lens, probe_heads, query_sel, key_spans,
                     k_scale, v_scale, k_new, v_new]
        total_q, Hq, d = q.shape
        num_blocks, Hkv, B, _ = k_cache.shape
        num_seqs, max_blocks = block_table.shape
        P = 0 if probe_heads is None else int(probe_heads.numel())
        a = HookAttnProbeArgs()
        a.num_seqs, a.total_q, a.num_q_heads, a.num_kv_heads = num_seqs, total_q, Hq, Hkv
        a.head_dim, a.block_size, a.max_blocks_per_seq, a.num_blocks = d, B, max_blocks, num_blocks
        a.dtype, a.scale = _DT[q.dtype], float(scale)
        a.q, a.k_cache, a.v_cache = _p(q), _p(k_cache), _p(v_cache)
        a.block_table, a.seq_lens, a.cu_q_lens = _p(block_table), _p(seq_lens), _p(cu_q_lens)
        a.num_probe_heads, a.probe_heads = P, _p(probe_heads)
        a.max_sel_q, a.query_sel = int(max_sel_q), _p(query_sel)
        a.max_spans, a.key_spans = int(max_spans), _p(key_spans)
        self.out = out if out is not None else torch.empty_like(q)
        self.mass = mass if mass is not None else torch.empty((num_seqs, P, int(max_sel_q), int(max_spans)),
                                                               dtype=torch.float32, device=dev)
        a.out, a.mass = _p(self.out), _p(self.mass)
        need = int(lib.hook_attn_probe_workspace_bytes(ctypes.byref(a)))
        if workspace is None:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        self.workspace = workspace
        a.workspace, a.workspace_bytes = _p(workspace), workspace.numel()
        a.batch_kind = int(batch_kind)
        a.plan_mode = int(plan_mode)
        if k_cache.dtype == torch.uint8:      # 8-bit E4M3 bytes with one scale per kv head
            a.kv_dtype, a.k_scale, a.v_scale = KV_FP8_E4M3, _p(k_scale), _p(v_scale)
        a.k_new, a.v_new = _p(k_new), _p(v_new)
        self.args = a
        self.workspace_needed = need
        self._fn = lib.hook_attn_probe

    def launch(self, stream=None) -> None:
        self.args.stream = _stream_handle(stream)
        st = self._fn(ctypes.byref(self.args))
        if st != HOOK_OK:
            raise HookError(st, "hook_attn_probe")

    def launch_static(self, stream=None) -> None:
        """The same call on the library's own scratch array (the workspace of this object is not used)."""
        self.args.stream = _stream_handle(stream)
        st = load_library().hook_attn_probe_static(ctypes.byref(self.args))
        if st != HOOK_OK:
            raise HookError(st, "hook_attn_probe_static")

    def device_status(self, stream=None) -> int:
        bits = ctypes.c_int32(0)
        st = load_library().hook_attn_probe_device_status(self.args.workspace, _stream_handle(stream),
                                                          ctypes.byref(bits))
        if st != HOOK_OK:
            raise HookError(st, "hook_attn_probe_device_status")
        return int(bits.value)

    def validate(self, stream=None) -> int:
        """Problem bits (HOOK_BAD_*) of the device-resident contents of this call; synchronises."""
        bits = ctypes.c_int32(0)
        self.args.stream = _stream_handle(stream)
        st = load_library().hook_attn_probe_validate(ctypes.byref(self.args), ctypes.byref(bits))
        if st != HOOK_OK:
            raise HookError(st, "hook_attn_probe_validate")
        return int(bits.value)


def hook_attn_probe(q, k_cache, v_cache, block_table, seq_lens, cu_q_lens, probe_heads=None, max_sel_q=1,
                    query_sel=None, max_spans=1, key_spans=None, scale: float = 0.0,
                    stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(out, mass) of one layer's hooked attention; asynchronous on the current stream."""
    call = AttnProbeCall(q, k_cache, v_cache, block_table, seq_lens, cu_q_lens, probe_heads, max_sel_q,
                         query_sel, max_spans, key_spans, scale)
    call.launch(stream)
    return call.out, call.mass


def hook_span_mass(q, k_cache, block_table, seq_lens, cu_q_lens, probe_heads, max_sel_q, query_sel, max_spans,
                   key_spans, scale: float = 0.0, mass=None, stream=None, workspace=None,
                   use_workspace: bool = True, k_scale=None) -> torch.Tensor:
    """mass [num_seqs, P, NQ, S] for up to HOOK_MAX_SPANS_WIDE spans; computes no attention output.
    A scratch tensor lets the library split the work over the chip; it is allocated here unless
    one is passed in or use_workspace is False."""
    lib = load_library()
    total_q, Hq, d = q.shape
    num_blocks, Hkv, B, _ = k_cache.shape
    num_seqs, max_blocks = block_table.shape
    P = int(probe_heads.numel())
    if q.dtype not in _DT:
        raise HookError(3, "hook_span_mass (dtype)")
    if mass is None:
        mass = torch.empty((num_seqs, P, int(max_sel_q), int(max_spans)), dtype=torch.float32, device=q.device)
    a = HookAttnProbeArgs()
    a.num_seqs, a.total_q, a.num_q_heads, a.num_kv_heads = num_seqs, total_q, Hq, Hkv
    a.head_dim, a.block_size, a.max_blocks_per_seq, a.num_blocks = d, B, max_blocks, num_blocks
    a.dtype, a.scale = _DT[q.dtype], float(scale)
    a.q, a.k_cache = _p(q), _p(k_cache)
    a.block_table, a.seq_lens, a.cu_q_lens = _p(block_table), _p(seq_lens), _p(cu_q_lens)
    a.num_probe_heads, a.probe_heads = P, _p(probe_heads)
    a.max_sel_q, a.query_sel = int(max_sel_q), _p(query_sel)
    a.max_spans, a.key_spans = int(max_spans), _p(key_spans)
    a.mass, a.stream = _p(mass), _stream_handle(stream)
    if k_cache.dtype == torch.uint8:          # 8-bit E4M3 bytes with one scale per kv head
        a.kv_dtype, a.k_scale = KV_FP8_E4M3, _p(k_scale)
    if workspace is None and use_workspace:
        need = int(lib.hook_span_mass_workspace_bytes(ctypes.byref(a)))
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=q.device) if need else None
    if workspace is not None:
        a.workspace, a.workspace_bytes = _p(workspace), workspace.numel()
    st = lib.hook_span_mass(ctypes.byref(a))
    if st != HOOK_OK:
        raise HookError(st, "hook_span_mass")
    return mass


def hook_span_mass_batch(b, stream=None, mass=None, workspace=None, use_workspace: bool = True) -> torch.Tensor:
    return hook_span_mass(b.q, b.k_cache, b.block_table, b.seq_lens, b.cu_q_lens, b.probe_heads, b.max_sel_q,
                          b.query_sel, b.max_spans, b.key_spans, b.scale, mass, stream, workspace, use_workspace,
                          k_scale=getattr(b, "k_scale", None))


def hook_attn_probe_batch(b, stream=None, probe: bool = True):
    """Convenience for objects carrying the batch attributes (device tensors)."""
    return hook_attn_probe(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.cu_q_lens,
                           b.probe_heads if probe else None, b.max_sel_q, b.query_sel, b.max_spans,
                           b.key_spans, b.scale, stream)


def call_from_batch(b, probe: bool = True, **kw) -> AttnProbeCall:
    if getattr(b, "k_scale", None) is not None:
        kw.setdefault("k_scale", b.k_scale)
        kw.setdefault("v_scale", b.v_scale)
    return AttnProbeCall(b.q, b.k_cache, b.v_cache, b.block_table, b.seq_lens, b.cu_q_lens,
                         b.probe_heads if probe else None, b.max_sel_q, b.query_sel, b.max_spans,
                         b.key_spans, b.scale, **kw)


def hook_residual_add_steer(hidden, delta, vec, alpha: float, token_mask=None, stream=None):
    """hidden += delta (+ alpha * vec on masked rows), in place, one rounding."""
    lib = load_library()
    T, D = hidden.shape
    st = lib.hook_residual_add_steer(_p(hidden), _p(delta), _p(vec), float(alpha), _p(token_mask), T, D,
                                     _DT[hidden.dtype], _stream_handle(stream))
    if st != HOOK_OK:
        raise HookError(st, "hook_residual_add_steer")
    return hidden


def hook_kv_write(k_new, v_new, block_table, seq_lens, cu_q_lens, k_cache, v_cache, stream=None, k_scale=None,
                  v_scale=None) -> None:
    """Scatter the new tokens' K/V rows ([total_q, Hkv, d]) into the paged cache, in place (quantising
    when the cache is uint8 E4M3 bytes with per-kv-head scales)."""
    lib = load_library()
    total_q, Hkv, d = k_new.shape
    num_blocks, _, B, _ = k_cache.shape
    num_seqs, max_blocks = block_table.shape
    a = HookKvWriteArgs()
    a.num_seqs, a.total_q, a.num_kv_heads, a.head_dim = num_seqs, total_q, Hkv, d
    a.block_size, a.max_blocks_per_seq, a.num_blocks, a.dtype = B, max_blocks, num_blocks, _DT[k_new.dtype]
    a.k_new, a.v_new, a.block_table = _p(k_new), _p(v_new), _p(block_table)
    a.seq_lens, a.cu_q_lens = _p(seq_lens), _p(cu_q_lens)
    a.k_cache, a.v_cache, a.stream = _p(k_cache), _p(v_cache), _stream_handle(stream)
    if k_cache.dtype == torch.uint8:
        a.kv_dtype, a.k_scale, a.v_scale = KV_FP8_E4M3, _p(k_scale), _p(v_scale)
    st = lib.hook_kv_write(ctypes.byref(a))
    if st != HOOK_OK:
        raise HookError(st, "hook_kv_write")


def hook_capture_qk(q, k_cache, block_table, seq_lens, cu_q_lens, probe_heads, max_sel_q, query_sel,
                    capture_kv_heads, cu_k_lens, total_k: int, stream=None, q_out=None, k_out=None):
    """Gather (q_out [num_seqs, P, NQ, d], k_out [total_k, KH, d]); total_k is a host integer."""
    lib = load_library()
    total_q, Hq, d = q.shape
    num_blocks, Hkv, B, _ = k_cache.shape
    num_seqs, max_blocks = block_table.shape
    P = int(probe_heads.numel()) if probe_heads is not None else 0
    KH = int(capture_kv_heads.numel()) if capture_kv_heads is not None else 0
    if q_out is None:
        q_out = torch.empty((num_seqs, P, int(max_sel_q), d), dtype=q.dtype, device=q.device)
    if k_out is None:
        k_out = torch.empty((int(total_k), KH, d), dtype=k_cache.dtype, device=q.device)   # bytes for an 8-bit cache
    a = HookCaptureQkArgs()
    a.num_seqs, a.total_q, a.num_q_heads, a.num_kv_heads = num_seqs, total_q, Hq, Hkv
    a.head_dim, a.block_size, a.max_blocks_per_seq, a.num_blocks = d, B, max_blocks, num_blocks
    a.dtype = _DT[q.dtype]
    a.q, a.k_cache, a.block_table = _p(q), _p(k_cache), _p(block_table)
    a.seq_lens, a.cu_q_lens = _p(seq_lens), _p(cu_q_lens)
    a.num_probe_heads, a.probe_heads, a.max_sel_q, a.query_sel = P, _p(probe_heads), int(max_sel_q), _p(query_sel)
    a.num_capture_kv_heads, a.capture_kv_heads = KH, _p(capture_kv_heads)
    a.cu_k_lens, a.total_k = _p(cu_k_lens), int(total_k)
    a.q_out, a.k_out, a.stream = _p(q_out), _p(k_out), _stream_handle(stream)
    a.kv_dtype = KV_FP8_E4M3 if k_cache.dtype == torch.uint8 else KV_SAME
    st = lib.hook_capture_qk(ctypes.byref(a))
    if st != HOOK_OK:
        raise HookError(st, "hook_capture_qk")
    return q_out, k_out


def hook_reduce_mass(mass, mode: int, span_a: int = 0, span_b: int = 1, query_sel=None, cu_q_lens=None,
                     head_weights=None, scores=None, accumulate: bool = False, stream=None):
    """Reduce mass [num_seqs, P, NQ, S] to scores ([num_seqs, S] for SPAN_MEAN, else [num_seqs])."""
    lib = load_library()
    num_seqs, P, NQ, S = mass.shape
    if scores is None:
        if accumulate:
            raise ValueError("accumulate needs an existing scores tensor")
        shape = (num_seqs, S) if mode == REDUCE_SPAN_MEAN else (num_seqs,)
        scores = torch.empty(shape, dtype=torch.float32, device=mass.device)
    a = HookReduceArgs()
    a.num_seqs, a.num_probe_heads, a.max_sel_q, a.max_spans = num_seqs, P, NQ, S
    a.mass, a.query_sel, a.cu_q_lens, a.head_weights = _p(mass), _p(query_sel), _p(cu_q_lens), _p(head_weights)
    a.mode, a.span_a, a.span_b, a.accumulate = int(mode), int(span_a), int(span_b), int(bool(accumulate))
    a.scores, a.stream = _p(scores), _stream_handle(stream)
    st = lib.hook_reduce_mass(ctypes.byref(a))
    if st != HOOK_OK:
        raise HookError(st, "hook_reduce_mass")
    return scores


def parse_layer_heads(text: str):
    """'0:0,3,6;15:2' -> [(0, 0), (0, 3), (0, 6), (15, 2)] (parsed by the library)."""
    lib = load_library()
    count = ctypes.c_int32(0)
    st = lib.hook_parse_layer_heads(text.encode(), None, None, 0, ctypes.byref(count))
    if st not in (HOOK_OK, 4):
        raise HookError(st, "hook_parse_layer_heads")
    n = int(count.value)
    layers, heads = (ctypes.c_int32 * max(n, 1))(), (ctypes.c_int32 * max(n, 1))()
    st = lib.hook_parse_layer_heads(text.encode(), layers, heads, n, ctypes.byref(count))
    if st != HOOK_OK:
        raise HookError(st, "hook_parse_layer_heads")
    return [(int(layers[i]), int(heads[i])) for i in range(n)]


def parse_config_json(text: str):
    """JSON config text -> ([(layer, head), ...] in file order, hookq_mode or None)."""
    lib = load_library()
    count, mode = ctypes.c_int32(0), ctypes.c_int32(-1)
    st = lib.hook_parse_config_json(text.encode(), None, None, 0, ctypes.byref(count), ctypes.byref(mode))
    if st not in (HOOK_OK, 4):
        raise HookError(st, "hook_parse_config_json")
    n = int(count.value)
    layers, heads = (ctypes.c_int32 * max(n, 1))(), (ctypes.c_int32 * max(n, 1))()
    st = lib.hook_parse_config_json(text.encode(), layers, heads, n, ctypes.byref(count), ctypes.byref(mode))
    if st != HOOK_OK:
        raise HookError(st, "hook_parse_config_json")
    names = {0: "last_token", 1: "all_tokens"}
    return [(int(layers[i]), int(heads[i])) for i in range(n)], names.get(int(mode.value))


def probe_heads_for_layer(pairs, layer: int, device="cpu") -> torch.Tensor:
    """Sorted, de-duplicated heads of one layer as the int32 probe_heads tensor of a call."""
    hs = sorted({int(h) for (l, h) in pairs if int(l) == int(layer)})
    return torch.tensor(hs, dtype=torch.int32, device=device)


def hook_steer(hidden: torch.Tensor, vec: torch.Tensor, alpha: float, token_mask: torch.Tensor,
               stream=None) -> torch.Tensor:
    """In place: hidden[t] += alpha * vec where token_mask[t] != 0.  Returns ``hidden``."""
    lib = load_library()
    if hidden.dtype not in _DT or vec.dtype != hidden.dtype or token_mask.dtype != torch.uint8:
        raise HookError(3, "hook_steer (dtype)")
    if not (hidden.is_contiguous() and vec.is_contiguous() and token_mask.is_contiguous()):
        raise HookError(2, "hook_steer (layout)")
    T, D = hidden.shape
    if vec.numel() != D or token_mask.numel() != T:
        raise HookError(2, "hook_steer (shape)")
    st = lib.hook_steer(_p(hidden), _p(vec), float(alpha), _p(token_mask), T, D, _DT[hidden.dtype],
                        _stream_handle(stream))
    if st != HOOK_OK:
        raise HookError(st, "hook_steer")
    return hidden
