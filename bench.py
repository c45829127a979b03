#!/usr/bin/env python3
"""Benchmark of the hooked-attention hot path on one MI355X.

One "step" is one whole `hook_attn_probe` call (plan, prefill, decode and combine kernels)
on the 8B-shaped ragged prefill batch, inputs resident in HBM.  The same run also measures
the decode batch (HBM-bound), the long prefill, the mixed step with steering, the probing
overhead of each, and times the CPU oracle on a bounded sample.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
# HBM traffic per launch (bytes) from rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled by a 1 GiB copy
# (profiles/hbm_traffic_*.md).  Every figure is tied to the sources of the kernel it was measured on
# (sha256 over the listed files, first 16 hex digits): once a kernel changes, its figure reads null
# until the counters are taken again.
TRAFFIC = {
    # key: (bytes per launch, source files, hash of those files when the counters were taken)
    "k_prefill128/c2": (797424994, ("prefill128.hip", "hook_device.h"), "2a8a49143a6fb91c"),
    "k_prefill128/c4": (5191965184, ("prefill128.hip", "hook_device.h"), "2a8a49143a6fb91c"),
    "k_decode/c3": (4910675161, ("decode.hip", "hook_device.h"), "6a4b00fc927a5ed1"),
    "k_decode/c3_fp8": (2440025513, ("decode.hip", "hook_device.h"), "6a4b00fc927a5ed1"),
}


def _source_hash(files) -> str:
    import hashlib
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2603_06588_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def traffic_for(key: str):
    """Measured HBM bytes per launch for `key`, or None if the kernel changed since the counter run."""
    if key not in TRAFFIC:
        return None
    nbytes, files, sha = TRAFFIC[key]
    return nbytes if _source_hash(files) == sha else None


def roofline_obj(bound: str, kernel: str, per_launch: float, kernel_ms: float, traffic_key: str = ""):
    """The roofline record of one kernel: algorithmic flops (mfma) or bytes (hbm) per launch over its
    measured duration, against the published peak."""
    if bound == "mfma":
        achieved, peak, unit, name = per_launch / (kernel_ms * 1e-3) / 1e12, PEAK_BF16_MFMA_TFLOPS, "TFLOP/s", "flops_per_launch"
    else:
        achieved, peak, unit, name = per_launch / (kernel_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s", "bytes_per_launch"
    return {"bound": bound, "kernel": kernel, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
            "traffic": traffic_for(traffic_key) if traffic_key else None, "kernel_ms": kernel_ms, name: per_launch}


def causal_pairs(b) -> int:
    lens = b.seq_lens.tolist()
    qn = b.q_lens()
    tot = 0
    for L, n in zip(lens, qn):
        # rows at positions L-n .. L-1 attend to pos+1 keys
        tot += n * (L - n) + n * (n + 1) // 2
    return tot


def attn_flops(b) -> float:
    """Algorithmic flops: QK^T and PV over causal pairs only (4 * d per pair per q head)."""
    return 4.0 * b.head_dim * b.num_q_heads * causal_pairs(b)


def kv_bytes(b, decode_only: bool = True) -> float:
    """Algorithmic decode bytes: every live K and V element of every kv head once."""
    lens = b.seq_lens.tolist()
    qn = b.q_lens()
    esz = 2 if str(b.dtype).endswith("bfloat16") else 4
    if str(b.k_cache.dtype).endswith("uint8"):
        esz = 1      # 8-bit cache
    tot = 0
    for L, n in zip(lens, qn):
        if decode_only and n != 1:
            continue
        tot += L * b.num_kv_heads * b.head_dim * 2 * esz
    return float(tot)


def time_call(fn, steps: int, warmup: int):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for s, e in ev:
        s.record()
        fn()
        e.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    per = [s.elapsed_time(e) for s, e in ev]
    return {"mean_ms": sum(per) / len(per), "median_ms": statistics.median(per), "min_ms": min(per),
            "wall_ms_per_step": wall}


def time_batch(fn, steps: int, warmup: int) -> float:
    """Mean ms per call over `steps` calls queued back to back between ONE pair of events: what a
    kernel trace reports for short kernels, whose single calls mostly measure the gap between launches."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(steps):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / steps


def interleaved_overhead(call_on, call_off, steps: int, warmup: int):
    """Probe overhead: t(probing) / t(num_probe_heads = 0) - 1, runs interleaved."""
    import torch
    for _ in range(warmup):
        call_on.launch(); call_off.launch()
    torch.cuda.synchronize()
    on, off = [], []
    for _ in range(steps):
        for call, acc in ((call_on, on), (call_off, off)):
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record(); call.launch(); e.record()
            torch.cuda.synchronize()
            acc.append(s.elapsed_time(e))
    t_on, t_off = statistics.median(on), statistics.median(off)
    return {"probe_ms": t_on, "noprobe_ms": t_off, "overhead_pct": 100.0 * (t_on / t_off - 1.0)}


def kernel_times(call, steps: int):
    """Mean per-kernel durations (ms) over `steps` back-to-back calls, from HIP events recorded inside
    the library around every kernel."""
    from paper_2603_06588_amd import benchlib
    benchlib.launch_timed_n(call, max(2, steps // 5))      # bring the chip to the state of a timing loop
    ms = benchlib.launch_timed_n(call, steps)
    return dict(zip(("plan_ms", "prefill_ms", "decode_ms", "combine_ms"), ms))


def oracle_sample(b_dev, kind: str):
    """Time the CPU oracle (as it stands, never tuned) on the workload; returns (work, seconds, desc).

    The 8B-shaped prefill batch costs the oracle about 10 s on the machine's host cores, so it is run
    whole; the decode batch takes well under a second and is also run whole.
    """
    import oracle
    b = b_dev.to("cpu")
    if kind == "prefill":
        t0 = time.perf_counter()
        oracle.attn_probe_batch(b)
        dt = time.perf_counter() - t0
        return attn_flops(b), dt, f"all {b.total_q} rows x {b.num_q_heads} heads"
    t0 = time.perf_counter()
    oracle.attn_probe_batch(b)
    dt = time.perf_counter() - t0
    return kv_bytes(b), dt, f"all {b.num_seqs} sequences x {b.num_q_heads} heads"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--only", default="", help="comma list of c1,c2,c3,c4,c5,c6,d64 (default: all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-workload", default="", choices=["", "c2", "c3", "c3_fp8", "c4", "c5", "copy"],
                    help="only launch this workload --steps times (for rocprofv3 runs); prints no JSON. "
                         "'copy' runs a plain 1 GiB device copy, the known-size reference that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2603_06588_amd import benchlib, binding, build as hip_build, workloads as W
    if not (os.path.exists(hip_build.LIB) and os.path.exists(hip_build.BENCH_LIB)):
        hip_build.build_lib()
    binding.load_library()
    benchlib.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    only = set(x for x in args.only.split(",") if x) or {"c1", "c2", "c3", "c4", "c5", "c6", "d64"}
    if args.profile_workload:
        wl = args.profile_workload
        steer = None
        if wl == "copy":
            src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
            dst = torch.empty_like(src)
            for _ in range(args.warmup + args.steps):
                dst.copy_(src)
            torch.cuda.synchronize()
            print(f"profiled copy: {args.warmup + args.steps} copies of {src.numel()} bytes", file=sys.stderr)
            return 0
        kind = binding.BATCH_MIXED          # the hint bench.py's timed runs pass for the workload
        if wl == "c2":
            b, kind = W.c2_prefill_8b(device=dev), binding.BATCH_PREFILL_ONLY
        elif wl == "c3":
            b, kind = W.c3_decode_8b(device=dev), binding.BATCH_DECODE_ONLY
        elif wl == "c3_fp8":
            b, kind = W.fp8_cache_variant(W.c3_decode_8b(device=dev), 960, k_std=128 ** -0.5, v_std=128 ** -0.5), binding.BATCH_DECODE_ONLY
        elif wl == "c4":
            b, kind = W.c4_long_prefill_70b(device=dev), binding.BATCH_PREFILL_ONLY
        else:
            b, steer = W.c5_mixed(device=dev)
        call = binding.call_from_batch(b, batch_kind=kind)
        for _ in range(args.warmup + args.steps):
            call.launch()
            if steer is not None:
                binding.hook_steer(steer.hidden, steer.vec, steer.alpha, steer.token_mask)
        torch.cuda.synchronize()
        print(f"profiled {wl}: {args.warmup + args.steps} launches", file=sys.stderr)
        return 0
    K, Wm = args.steps, args.warmup
    extra = {}

    # ---- primary: 8B-shaped ragged prefill (the config the metric is quoted on) ----
    b2 = W.c2_prefill_8b(device=dev)
    # the batch is known to hold query chunks only, which the caller may say (two launches fewer)
    call2 = binding.call_from_batch(b2, batch_kind=binding.BATCH_PREFILL_ONLY)
    call2_off = binding.call_from_batch(b2, probe=False, batch_kind=binding.BATCH_PREFILL_ONLY)
    call2_nohint = binding.call_from_batch(b2)
    t2 = time_call(call2.launch, K, Wm)
    t2_nohint = time_call(call2_nohint.launch, K, Wm)
    t2 = time_call(call2.launch, K, Wm)      # timed twice, the run after the unhinted one counts (same thermal state)
    # the same call replayed from a captured graph (what a serving loop would do)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call2.launch(side)
    torch.cuda.synchronize()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2, stream=side):
        call2.launch(torch.cuda.current_stream())
    t2_graph = time_call(graph2.replay, K, Wm)
    # later layers of a model step see the same batch and can reuse the work lists: no planner launch
    call2_reuse = binding.call_from_batch(b2, batch_kind=binding.BATCH_PREFILL_ONLY, workspace=call2.workspace,
                                          plan_mode=binding.PLAN_REUSE)
    t2_reuse = time_call(call2_reuse.launch, K, Wm)
    k2 = kernel_times(call2, K)
    flops2 = attn_flops(b2)
    ov2 = interleaved_overhead(call2, call2_off, max(10, K // 2), 3)
    value = flops2 / (t2["mean_ms"] * 1e-3) / 1e12
    roofline = roofline_obj("mfma", "k_prefill128", flops2, k2["prefill_ms"], "k_prefill128/c2")
    pre_tflops = roofline["achieved"]
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        work, dt, desc = oracle_sample(b2, "prefill")
        cpu_baseline = {"value": work / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "sample": f"c2_prefill_8b: {desc}; {dt:.2f} s"}

    if "c3" in only:
        b3 = W.c3_decode_8b(device=dev)
        call3 = binding.call_from_batch(b3, batch_kind=binding.BATCH_DECODE_ONLY)
        call3_off = binding.call_from_batch(b3, probe=False, batch_kind=binding.BATCH_DECODE_ONLY)
        t3 = time_call(call3.launch, K, Wm)
        k3 = kernel_times(call3, K)
        by3 = kv_bytes(b3)
        ov3 = interleaved_overhead(call3, call3_off, max(10, K // 2), 3)
        extra["decode_c3"] = {
            "workload": "c3_decode_8b", "value": by3 / (t3["mean_ms"] * 1e-3) / 1e9, "unit": "GB/s",
            "ms_per_step": t3["mean_ms"], "median_ms": t3["median_ms"], "min_ms": t3["min_ms"], "kernels_ms": k3,
            "roofline": roofline_obj("hbm", "k_decode<128,4>", by3, k3["decode_ms"], "k_decode/c3"),
            "probe_overhead_pct": ov3["overhead_pct"],
            "workspace_mb": call3.workspace_needed / 2**20,
        }
        # the same batch over an 8-bit (E4M3) cache: half the bytes per context token
        b3q = W.fp8_cache_variant(b3, 960, k_std=128 ** -0.5, v_std=128 ** -0.5)
        call3q = binding.call_from_batch(b3q, batch_kind=binding.BATCH_DECODE_ONLY)
        t3q = time_call(call3q.launch, K, Wm)
        k3q = kernel_times(call3q, K)
        by3q = kv_bytes(b3q)
        extra["decode_c3_fp8_cache"] = {
            "workload": "c3_decode_8b with 8-bit E4M3 key/value caches (one scale per kv head)",
            "value": by3q / (t3q["mean_ms"] * 1e-3) / 1e9, "unit": "GB/s", "ms_per_step": t3q["mean_ms"],
            "kernels_ms": k3q, "speedup_vs_bf16_cache": t3["mean_ms"] / t3q["mean_ms"],
            "roofline": roofline_obj("hbm", "k_decode<128,4,fp8>", by3q, k3q["decode_ms"], "k_decode/c3_fp8")}
        del b3q, call3q
        torch.cuda.empty_cache()
        # compact q/k capture on the same batch: every key of every kv head, the probed heads' queries
        kvh = torch.arange(b3.num_kv_heads, dtype=torch.int32, device=dev)
        cu_k = torch.zeros(b3.num_seqs + 1, dtype=torch.int32, device=dev)
        cu_k[1:] = torch.cumsum(b3.seq_lens, 0)
        total_k = int(cu_k[-1])
        q_out, k_out = binding.hook_capture_qk(b3.q, b3.k_cache, b3.block_table, b3.seq_lens, b3.cu_q_lens,
                                               b3.probe_heads, b3.max_sel_q, b3.query_sel, kvh, cu_k, total_k)
        tcap = time_call(lambda: binding.hook_capture_qk(
            b3.q, b3.k_cache, b3.block_table, b3.seq_lens, b3.cu_q_lens, b3.probe_heads, b3.max_sel_q,
            b3.query_sel, kvh, cu_k, total_k, q_out=q_out, k_out=k_out), K, Wm)
        cap_bytes = 2.0 * (k_out.numel() + q_out.numel()) * k_out.element_size()   # read once + written once
        extra["capture_qk_c3"] = {
            "workload": "c3_decode_8b, all kv heads", "ms": tcap["mean_ms"],
            "roofline": roofline_obj("hbm", "k_capture_k (+ k_capture_q)", cap_bytes, tcap["mean_ms"])}
        del q_out, k_out
        if not args.no_cpu_baseline:
            work, dt, desc = oracle_sample(b3, "decode")
            extra["decode_c3"]["cpu_baseline"] = {"value": work / dt / 1e9, "unit": "GB/s",
                                                  "cores": oracle.num_threads(), "kind": "oracle",
                                                  "sample": f"c3_decode_8b: {desc}; {dt:.2f} s"}
        del b3, call3, call3_off
        torch.cuda.empty_cache()
        # a latency-bound decode step: 8 sequences of 4096 tokens, same heads; what a call costs when
        # there is too little to stream (a batch this small plans itself: decode + combine launches)
        bs = W.random_batch(7, [4096] * 8, [1] * 8, 32, 8, 128, torch.bfloat16, std=128 ** -0.5,
                            num_probe_heads=8, max_sel_q=1, max_spans=1, device=dev)
        calls = binding.call_from_batch(bs, batch_kind=binding.BATCH_DECODE_ONLY)
        ts = time_call(calls.launch, K, Wm)
        calls_reuse = binding.call_from_batch(bs, batch_kind=binding.BATCH_DECODE_ONLY, workspace=calls.workspace,
                                              plan_mode=binding.PLAN_REUSE)
        ts_reuse = time_call(calls_reuse.launch, K, Wm)
        ts_b2b = time_batch(calls.launch, 4 * K, Wm)     # calls queued back to back: what a decode loop sustains
        extra["small_decode_8x4096"] = {
            "workload": "8 decode rows at 4096 tokens of context, 32 q / 8 kv heads, d 128",
            "us_per_call": ts["mean_ms"] * 1e3, "us_per_call_plan_reused": ts_reuse["mean_ms"] * 1e3,
            "us_per_call_back_to_back": ts_b2b * 1e3,
            "kernels_ms": kernel_times(calls, K),
            "roofline": roofline_obj("hbm", "whole call back to back (k_decode + k_combine)", kv_bytes(bs), ts_b2b)}
        del bs, calls, calls_reuse
        torch.cuda.empty_cache()

    if "c2" in only:
        # one prompt on its own (the paper's detection use case: a single prompt, probed at its last token):
        # the call is bound by the longest row block's walk over the keys, not by throughput
        b1p = W.random_batch(21, [2048], [2048], 32, 8, 128, torch.bfloat16, std=128 ** -0.5, num_probe_heads=8,
                             max_sel_q=1, max_spans=2, device=dev)
        call1p = binding.call_from_batch(b1p, batch_kind=binding.BATCH_PREFILL_ONLY)
        t1p = time_batch(call1p.launch, 4 * K, Wm)
        k1p = kernel_times(call1p, K)
        extra["single_prompt_2048"] = {
            "workload": "one prefill of 2048 tokens, 32 q / 8 kv heads, d 128, 8 probed heads, last row",
            "us_per_call_back_to_back": t1p * 1e3, "kernels_ms": k1p,
            "roofline": roofline_obj("mfma", "k_prefill128", attn_flops(b1p), k1p["prefill_ms"])}
        del b1p, call1p
        torch.cuda.empty_cache()

    if "c2" in only:
        # the primary workload over 8-bit caches: query chunks gain nothing from the format (they are bound
        # by the matrix cores) and are served by the register-staged kernel; reported so the path has a number
        b2q = W.fp8_cache_variant(b2, 962, k_std=128 ** -0.5, v_std=128 ** -0.5)
        call2q = binding.call_from_batch(b2q, batch_kind=binding.BATCH_PREFILL_ONLY)
        t2q = time_call(call2q.launch, K, Wm)
        k2q = kernel_times(call2q, K)
        extra["prefill_c2_fp8_cache"] = {
            "workload": "c2_prefill_8b with 8-bit E4M3 key/value caches", "ms_per_step": t2q["mean_ms"],
            "kernels_ms": k2q,
            "roofline": roofline_obj("mfma", "k_prefill<128,fp8>", attn_flops(b2q), k2q["prefill_ms"])}
        del b2q, call2q
        torch.cuda.empty_cache()

    if "c4" in only:
        b4 = W.c4_long_prefill_70b(device=dev)
        call4 = binding.call_from_batch(b4, batch_kind=binding.BATCH_PREFILL_ONLY)
        call4_off = binding.call_from_batch(b4, probe=False, batch_kind=binding.BATCH_PREFILL_ONLY)
        k4steps = max(3, K // 6)
        t4 = time_call(call4.launch, k4steps, 1)
        k4 = kernel_times(call4, k4steps)
        fl4 = attn_flops(b4)
        ov4 = interleaved_overhead(call4, call4_off, 3, 1)
        extra["long_prefill_c4"] = {
            "workload": "c4_long_prefill_70b", "value": fl4 / (t4["mean_ms"] * 1e-3) / 1e12, "unit": "TFLOP/s",
            "ms_per_step": t4["mean_ms"], "kernels_ms": k4,
            "roofline": roofline_obj("mfma", "k_prefill128", fl4, k4["prefill_ms"], "k_prefill128/c4"),
            "probe_overhead_pct": ov4["overhead_pct"],
        }
        if not args.no_cpu_baseline:
            # the whole batch would cost the oracle minutes: all probed rows, the rows on either side of a
            # few tile boundaries and 128 seeded-random rows, for every head; scaled by causal-pair count
            n4 = b4.total_q
            g = torch.Generator().manual_seed(3)
            rows = sorted(set(range(n4 - 32, n4)) | {0, 63, 64, 255, 256, n4 // 2 - 1, n4 // 2}
                          | set(torch.randint(0, n4, (128,), generator=g).tolist()))
            b4c = b4.to("cpu")
            t0 = time.perf_counter()
            oracle.attn_probe_batch(b4c, rows=rows)
            dt = time.perf_counter() - t0
            work = 4.0 * b4.head_dim * b4.num_q_heads * sum(r + 1 for r in rows)
            extra["long_prefill_c4"]["cpu_baseline"] = {
                "value": work / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"c4_long_prefill_70b: {len(rows)} of {n4} rows x {b4.num_q_heads} heads; {dt:.2f} s; "
                          f"extrapolated whole batch {fl4 / (work / dt):.0f} s"}
            del b4c
        del b4, call4, call4_off
        torch.cuda.empty_cache()

    if "c5" in only:
        b5, s5 = W.c5_mixed(device=dev)
        call5 = binding.call_from_batch(b5)
        call5_off = binding.call_from_batch(b5, probe=False)
        hiddens = [s5.hidden.clone() for _ in range(4)]   # rotate so the 69 MB buffer is not cache-resident
        state = {"i": 0}

        def mixed_step():
            call5.launch()
            binding.hook_steer(hiddens[state["i"] % 4], s5.vec, s5.alpha, s5.token_mask)
            state["i"] += 1

        def steer_only():
            binding.hook_steer(hiddens[state["i"] % 4], s5.vec, s5.alpha, s5.token_mask)
            state["i"] += 1

        t5 = time_call(mixed_step, K, Wm)
        t5a = time_call(call5.launch, K, Wm)
        t5s = time_call(steer_only, K, Wm)
        t5s_b = time_batch(steer_only, K, Wm)
        k5 = kernel_times(call5, K)
        ov5 = interleaved_overhead(call5, call5_off, max(10, K // 2), 3)
        fl5, by5 = attn_flops(b5), kv_bytes(b5)
        steer_bytes = 2.0 * int(s5.token_mask.sum()) * s5.hidden.shape[1] * 2
        t_roof_ms = max(fl5 / (PEAK_BF16_MFMA_TFLOPS * 1e12), by5 / (PEAK_HBM_GBS * 1e9)) * 1e3
        t_sum_ms = (fl5 / (PEAK_BF16_MFMA_TFLOPS * 1e12) + by5 / (PEAK_HBM_GBS * 1e9)) * 1e3
        extra["mixed_c5"] = {
            "workload": "c5_mixed", "attn_plus_steer_ms": t5["mean_ms"], "attn_ms": t5a["mean_ms"],
            "kernels_ms": k5,
            "roofline_prefill": roofline_obj("mfma", "k_prefill128", fl5, k5["prefill_ms"]) if k5["prefill_ms"] > 0 else None,
            "roofline_decode": roofline_obj("hbm", "k_decode<128,4>", by5, k5["decode_ms"]) if k5["decode_ms"] > 0 else None,
            "roofline_max_ms": t_roof_ms, "roofline_sum_ms": t_sum_ms,
            "probe_overhead_pct": ov5["overhead_pct"],
            "steer": {"ms_single_call": t5s["mean_ms"], "ms": t5s_b, "buffers_rotated": 4,
                      "roofline": roofline_obj("hbm", "k_steer_bf16", steer_bytes, t5s_b)},
        }
        # steering folded into the residual add that writes hidden: every row read (hidden, delta) and
        # written once, the steered rows cost nothing extra
        deltas = [torch.randn_like(s5.hidden) for _ in range(4)]

        def fused_step():
            binding.hook_residual_add_steer(hiddens[state["i"] % 4], deltas[state["i"] % 4], s5.vec, s5.alpha,
                                            s5.token_mask)
            state["i"] += 1

        def unfused_step():
            hiddens[state["i"] % 4].add_(deltas[state["i"] % 4])
            binding.hook_steer(hiddens[state["i"] % 4], s5.vec, s5.alpha, s5.token_mask)
            state["i"] += 1

        # writing the step's new K/V rows into the paged cache (what the attention call expects to find)
        k_new = torch.randn((b5.total_q, b5.num_kv_heads, b5.head_dim), device=dev).to(torch.bfloat16)
        v_new = torch.randn_like(k_new)
        tkw = {"mean_ms": time_batch(lambda: binding.hook_kv_write(k_new, v_new, b5.block_table, b5.seq_lens,
                                                                   b5.cu_q_lens, b5.k_cache, b5.v_cache), K, Wm)}
        kw_bytes = 4.0 * k_new.numel() * k_new.element_size()       # K and V rows read once, written once
        extra["mixed_c5"]["kv_write"] = {"ms": tkw["mean_ms"],
                                         "roofline": roofline_obj("hbm", "k_kv_write", kw_bytes, tkw["mean_ms"])}
        # the same write done by the attention call itself (spare workgroups of its planning launch)
        call5w = binding.call_from_batch(b5, k_new=k_new, v_new=v_new)
        t5w = time_batch(call5w.launch, K, Wm)
        t5sep = time_batch(lambda: (binding.hook_kv_write(k_new, v_new, b5.block_table, b5.seq_lens, b5.cu_q_lens,
                                                          b5.k_cache, b5.v_cache), call5.launch()), K, Wm)
        extra["mixed_c5"]["kv_write"]["attn_call_back_to_back_ms"] = time_batch(call5.launch, K, Wm)
        extra["mixed_c5"]["kv_write"]["attn_call_writing_kv_ms"] = t5w
        extra["mixed_c5"]["kv_write"]["kv_write_then_attn_call_ms"] = t5sep
        del call5w
        del k_new, v_new
        t5f = {"mean_ms": time_batch(fused_step, K, Wm)}
        t5u = {"mean_ms": time_batch(unfused_step, K, Wm)}
        fused_bytes = 3.0 * s5.hidden.numel() * s5.hidden.element_size()
        extra["mixed_c5"]["residual_add_steer"] = {
            "ms": t5f["mean_ms"], "separate_add_then_steer_ms": t5u["mean_ms"], "buffers_rotated": 4,
            "roofline": roofline_obj("hbm", "k_residual_steer_bf16", fused_bytes, t5f["mean_ms"])}
        del deltas
        if not args.no_cpu_baseline:
            b5c, s5c = b5.to("cpu"), s5.to("cpu")
            t0 = time.perf_counter()
            oracle.attn_probe_batch(b5c)
            dt_a = time.perf_counter() - t0
            t0 = time.perf_counter()
            oracle.steer_batch(s5c)
            dt_s = time.perf_counter() - t0
            extra["mixed_c5"]["cpu_baseline"] = {
                "value": (dt_a + dt_s) * 1e3, "unit": "ms per step", "cores": oracle.num_threads(),
                "kind": "oracle", "sample": f"c5_mixed whole: attention {dt_a:.2f} s, steering {dt_s:.3f} s",
                "steer_gbs": steer_bytes / dt_s / 1e9}

    if "c1" in only:
        # the small fp32 case: one launch of the full-precision kernel, and the oracle on the same batch
        b1, s1 = W.c1_tiny_prefill(device=dev)
        call1 = binding.call_from_batch(b1)
        t1 = time_call(call1.launch, K, Wm)
        extra["tiny_c1"] = {"workload": "c1_tiny_prefill (fp32, 256 tokens, 8 heads, d 64)", "ms_per_step": t1["mean_ms"],
                            "gflops": attn_flops(b1) / (t1["mean_ms"] * 1e-3) / 1e9}
        if not args.no_cpu_baseline:
            b1c = b1.to("cpu")
            t0 = time.perf_counter()
            for _ in range(20):
                oracle.attn_probe_batch(b1c)
            dt = (time.perf_counter() - t0) / 20
            extra["tiny_c1"]["cpu_baseline"] = {"value": dt * 1e3, "unit": "ms per step", "cores": oracle.num_threads(),
                                                "kind": "oracle", "sample": "c1_tiny_prefill whole, mean of 20 runs"}

    if "c6" in only:
        # re-ranking shape: one span per document, question rows selected; the probe is its own pass
        b6 = W.c6_reranker(device=dev)
        call6 = binding.call_from_batch(b6, probe=False)
        mass6 = binding.hook_span_mass_batch(b6)
        ws6 = torch.empty(1 << 22, dtype=torch.uint8, device=dev)    # scratch for the split form (4 MB is plenty)
        t6a = time_call(call6.launch, max(5, K // 5), 2)
        t6p = time_call(lambda: binding.hook_span_mass_batch(b6, mass=mass6, workspace=ws6), K, Wm)
        t6s = time_call(lambda: binding.hook_span_mass_batch(b6, mass=mass6, use_workspace=False), K, Wm)
        # keys the probe pass touches: pass 1 reads [0, L) once per (probed head, 16-row block),
        # pass 2 the keys inside the spans once more
        extra["reranker_c6"] = {
            "workload": "c6_reranker: 4 prompts, 40-100 documents each, 32 question rows, 8 heads",
            "total_q": b6.total_q, "spans": b6.max_spans,
            "attention_ms": t6a["mean_ms"], "span_mass_ms": t6p["mean_ms"],
            "span_mass_without_scratch_ms": t6s["mean_ms"],
            "span_mass_overhead_pct": 100.0 * t6p["mean_ms"] / t6a["mean_ms"],
            "attention_tflops": attn_flops(b6) / (t6a["mean_ms"] * 1e-3) / 1e12}
        del b6, call6, mass6
        torch.cuda.empty_cache()

    if "d64" in only:
        # head_dim 64 (bf16): the first-generation query-chunk kernel and the d = 64 instantiation of the
        # single-row kernel, on C2- and C3-like batches, so that these paths carry a measured number too
        gl = torch.Generator().manual_seed(11)
        lens64 = [int(x) for x in torch.randint(512, 2049, (16,), generator=gl)]
        bp = W.random_batch(11, lens64, lens64, 32, 8, 64, torch.bfloat16, std=64 ** -0.5, num_probe_heads=12,
                            max_sel_q=8, max_spans=1, device=dev)
        callp = binding.call_from_batch(bp, batch_kind=binding.BATCH_PREFILL_ONLY)
        tp = time_call(callp.launch, K, Wm)
        kp = kernel_times(callp, K)
        dl = [int(x) for x in torch.randint(1024, 8193, (128,), generator=gl)]
        bd = W.random_batch(12, dl, [1] * 128, 32, 8, 64, torch.bfloat16, std=64 ** -0.5, num_probe_heads=8,
                            max_sel_q=1, max_spans=1, device=dev)
        calld = binding.call_from_batch(bd, batch_kind=binding.BATCH_DECODE_ONLY)
        td = time_call(calld.launch, K, Wm)
        kd = kernel_times(calld, K)
        extra["head_dim_64"] = {
            "prefill": {"workload": "16 ragged prefills of 512-2048 tokens, 32 q / 8 kv heads, d 64, bf16",
                        "ms_per_step": tp["mean_ms"], "kernels_ms": kp,
                        "roofline": roofline_obj("mfma", "k_prefill<64>", attn_flops(bp), kp["prefill_ms"])},
            "decode": {"workload": "128 single rows at 1024-8192 tokens of context, 32 q / 8 kv heads, d 64, bf16",
                       "ms_per_step": td["mean_ms"], "kernels_ms": kd,
                       "roofline": roofline_obj("hbm", "k_decode<64,4>", kv_bytes(bd), kd["decode_ms"])}}
        del bp, bd, callp, calld
        torch.cuda.empty_cache()

    # ---- what the chip sustains: back-to-back MFMAs and a streaming read (measured last: the MFMA
    # probe leaves the chip hot, which would tax whatever is timed right after it)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    state_f = {"flops": 0.0}

    def mfma_probe():
        state_f["flops"] = benchlib.mfma_bf16(32768, 512, sink)

    tm = time_call(mfma_probe, 3, 1)
    big = torch.empty(1 << 32, dtype=torch.uint8, device=dev).fill_(1)
    tr = time_call(lambda: benchlib.hbm_read(big, sink), 5, 2)
    sustained = {"mfma_bf16_tflops": state_f["flops"] / (tm["min_ms"] * 1e-3) / 1e12,
                 "hbm_read_gbs": big.numel() / (tr["min_ms"] * 1e-3) / 1e9,
                 "note": "measured on this box by hook_bench_mfma_bf16 / hook_bench_hbm_read (4 GiB)"}
    del big
    torch.cuda.empty_cache()

    roofline["frac_of_sustained_mfma"] = pre_tflops / sustained["mfma_bf16_tflops"]

    line = {
        "metric": "hooked_attn_prefill_tflops", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": K, "warmup": Wm, "ms_per_step": t2["mean_ms"], "median_ms": t2["median_ms"], "min_ms": t2["min_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c2_prefill_8b: 16 ragged prefills U[512,2048], 32q/8kv heads, d128, paged KV "
                               "block 16 shuffled, 12 probed heads, last 8 rows, 1 span; batch_kind=prefill_only",
                   "total_q": b2.total_q, "causal_pairs_per_head": causal_pairs(b2)},
        "kernels_ms": k2, "probe_overhead_pct": ov2["overhead_pct"],
        "launch": {"batch_kind": "prefill_only", "ms_without_hint": t2_nohint["mean_ms"],
                   "ms_graph_replay": t2_graph["mean_ms"], "ms_plan_reused": t2_reuse["mean_ms"]},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "sustained_peaks": sustained,
    }
    if "long_prefill_c4" in extra:   # the largest single-GPU prefill beside the headline batch
        line["long_prefill_c4_frac"] = extra["long_prefill_c4"]["roofline"]["frac"]
    line.update(extra)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
