/*
 * hook_bench.h - C ABI of the measurement library libhook_bench.so.
 *
 * These calls are NOT part of the method: they exist so that a benchmark can report per-kernel
 * durations and roofline fractions.  The library links the same object files as libhook.so, so
 * the kernels it times are the product's kernels; a program that only uses the method needs
 * neither this header nor that library.  Argument structs are those of hook_api.h.
 */
#ifndef HOOK_BENCH_H_
#define HOOK_BENCH_H_

#include "hook_api.h"

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default)   /* the library itself is built with hidden visibility */
#endif

/*
 * The same launches as hook_attn_probe, bracketed by HIP events on args->stream, then WAITS for
 * them.  kernel_ms (HOST pointer, 4 floats) receives the durations in milliseconds of the plan,
 * prefill, decode and combine kernels (fp32 inputs: the zero-fill and attention kernels together
 * in kernel_ms[0], the rest 0; kernels left out by batch_kind or a reused plan read 0).  Creates
 * and destroys HIP events; not for graph capture.
 */
hook_status hook_bench_attn_probe_timed(const hook_attn_probe_args* args, float* kernel_ms);

/*
 * Same, `reps` (1..4096) calls queued back to back before anything is waited for; kernel_ms
 * receives the MEAN duration of each kernel over the repetitions.  This is the steady state a
 * kernel trace of a timing loop sees (a call timed on its own starts on an idle, cooler chip).
 */
hook_status hook_bench_attn_probe_timed_n(const hook_attn_probe_args* args, int32_t reps, float* kernel_ms);

/*
 * What the chip sustains on the two resources the kernels are bound by.  Both launch one kernel
 * on `stream` and return at once; the caller times them.
 *   hook_bench_mfma_bf16  num_workgroups x 4 waves issue independent 32x32x16 bf16 MFMAs back to
 *                         back for `iters` rounds of 16; *flops (HOST) receives the flop count of
 *                         the launch.  `sink` is 4 bytes of device memory (never written in practice).
 *   hook_bench_hbm_read   streams `bytes` (multiple of 16, 16-byte aligned) from `src` once with
 *                         16-byte loads; `sink` as above.
 */
hook_status hook_bench_mfma_bf16(int32_t iters, int32_t num_workgroups, void* sink, void* stream, double* flops);
hook_status hook_bench_hbm_read(const void* src, size_t bytes, void* sink, void* stream);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* HOOK_BENCH_H_ */
