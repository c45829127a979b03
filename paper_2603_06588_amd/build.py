"""Builds libhook.so (the product) and libhook_bench.so (measurement aids) for gfx950 next to this
file.  hipcc cross-compiles without a GPU.  Every source is compiled to an object once, in parallel;
the product library links the product objects, the measurement library links the same objects plus
csrc/bench.hip, so the kernels it times are the product's kernels."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ = os.path.join(_HERE, "_build")
LIB = os.path.join(_HERE, "libhook.so")
BENCH_LIB = os.path.join(_HERE, "libhook_bench.so")
SOURCES = ["api.hip", "plan.hip", "prefill.hip", "prefill128.hip", "decode.hip", "attn_f32.hip", "steer.hip",
           "capture.hip", "reduce.hip", "residual_steer.hip", "span_mass.hip", "config_json.hip", "kv_write.hip",
           "validate.hip"]
BENCH_SOURCES = ["bench.hip"]
# packed fp32 instructions are switched off for every device translation unit
# only what the two headers declare is exported
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-inline-asm"]


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    _run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build_lib(verbose: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, SOURCES + BENCH_SOURCES))
    product, bench = objs[:len(SOURCES)], objs[len(SOURCES):]
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *product, "-o", LIB])
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *product, *bench, "-o", BENCH_LIB])
    if verbose:
        print("hipcc", " ".join(FLAGS), "-c csrc/*.hip ->", LIB, "and", BENCH_LIB)
    return LIB


def lib_is_stale() -> bool:
    if not (os.path.exists(LIB) and os.path.exists(BENCH_LIB)):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(BENCH_LIB))
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps += [os.path.join(os.path.dirname(_HERE), "include", h) for h in ("hook_api.h", "hook_bench.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build_lib(verbose=True))
