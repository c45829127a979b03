"""ctypes front end of libhook_bench.so, the measurement library (include/hook_bench.h): per-kernel
timing of the attention call and the two sustained-rate probes.  Benchmarks and the tests that
check which kernels a call launches use it; a program that only uses the method does not."""
from __future__ import annotations

import ctypes
import os

from . import binding

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhook_bench.so")
EXPORTS = ["hook_bench_attn_probe_timed", "hook_bench_attn_probe_timed_n", "hook_bench_mfma_bf16", "hook_bench_hbm_read"]
_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_06588_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        ap = ctypes.POINTER(binding.HookAttnProbeArgs)
        lib.hook_bench_attn_probe_timed.restype = ctypes.c_int
        lib.hook_bench_attn_probe_timed.argtypes = [ap, ctypes.POINTER(ctypes.c_float)]
        lib.hook_bench_attn_probe_timed_n.restype = ctypes.c_int
        lib.hook_bench_attn_probe_timed_n.argtypes = [ap, ctypes.c_int32, ctypes.POINTER(ctypes.c_float)]
        lib.hook_bench_mfma_bf16.restype = ctypes.c_int
        lib.hook_bench_mfma_bf16.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.POINTER(ctypes.c_double)]
        lib.hook_bench_hbm_read.restype = ctypes.c_int
        lib.hook_bench_hbm_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def launch_timed_n(call: "binding.AttnProbeCall", reps: int = 1, stream=None):
    """`reps` launches of a marshalled attention call back to back; mean (plan, prefill, decode,
    combine) kernel times in ms."""
    call.args.stream = binding._stream_handle(stream)
    ms = (ctypes.c_float * 4)()
    st = load_library().hook_bench_attn_probe_timed_n(ctypes.byref(call.args), int(reps), ms)
    if st != binding.HOOK_OK:
        raise binding.HookError(st, "hook_bench_attn_probe_timed_n")
    return [float(x) for x in ms]


def launch_timed(call: "binding.AttnProbeCall", stream=None):
    return launch_timed_n(call, 1, stream)


def mfma_bf16(iters: int, num_workgroups: int, sink, stream=None) -> float:
    """Launch the back-to-back MFMA probe; returns the flop count of the launch."""
    flops = ctypes.c_double(0.0)
    st = load_library().hook_bench_mfma_bf16(int(iters), int(num_workgroups), binding._p(sink),
                                             binding._stream_handle(stream), ctypes.byref(flops))
    if st != binding.HOOK_OK:
        raise binding.HookError(st, "hook_bench_mfma_bf16")
    return float(flops.value)


def hbm_read(src, sink, stream=None) -> int:
    """Launch the streaming-read probe over `src`; returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    st = load_library().hook_bench_hbm_read(binding._p(src), nbytes, binding._p(sink), binding._stream_handle(stream))
    if st != binding.HOOK_OK:
        raise binding.HookError(st, "hook_bench_hbm_read")
    return nbytes
