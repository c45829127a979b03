// Score reductions over the mass tensor: one wave per sequence, lanes over (probed head, row)
// pairs, fp32 sums in a fixed order (lane-strided partial sums, then a butterfly), so the
// result does not depend on anything but the inputs.
#include "../../include/hook_api.h"
#include "hook_device.h"

namespace hook {
namespace {

struct ReduceParams {
  int num_seqs, P, NQ, S, mode, span_a, span_b, accumulate;
  const float* mass;
  const int* query_sel;
  const int* cu_q_lens;
  const float* w;
  float* scores;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

__global__ __launch_bounds__(256) void k_reduce_mass(const ReduceParams p) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= p.num_seqs) return;
  int nv = p.NQ;
  if (p.query_sel) {
    const int qb = p.query_sel[2 * i];
    int qe = min(p.query_sel[2 * i + 1], qb + p.NQ);
    if (p.cu_q_lens) qe = min(qe, p.cu_q_lens[i + 1] - p.cu_q_lens[i]);
    nv = max(qe - max(qb, 0), 0);
    // slots of rows before the chunk (negative t) come first and hold zeros; they do not count
  }
  const float* m = p.mass + (size_t)i * p.P * p.NQ * p.S;
  const float inv_nv = nv > 0 ? 1.0f / (float)nv : 0.0f;
  const int skip = (p.query_sel && p.query_sel[2 * i] < 0) ? min(-p.query_sel[2 * i], p.NQ) : 0;
  const int npairs = p.P * nv;
  if (p.mode == HOOK_REDUCE_SPAN_MEAN) {
    for (int r0 = 0; r0 < p.S; r0 += kMaxSpans) {   // kMaxSpans spans at a time in registers
      float acc[kMaxSpans];
#pragma unroll
      for (int r = 0; r < kMaxSpans; ++r) acc[r] = 0.0f;
      for (int e = lane; e < npairs; e += 64) {
        const int ph = e / nv, t = skip + e - ph * nv;
        const float wp = p.w ? p.w[ph] : 1.0f / (float)p.P;
        const float* row = m + ((size_t)ph * p.NQ + t) * p.S + r0;
#pragma unroll
        for (int r = 0; r < kMaxSpans; ++r)
          if (r0 + r < p.S) acc[r] += wp * row[r];
      }
#pragma unroll
      for (int r = 0; r < kMaxSpans; ++r) {
        if (r0 + r < p.S) {
          const float v = wave_sum(acc[r]) * inv_nv;
          if (lane == 0) {
            float* dst = p.scores + (size_t)i * p.S + r0 + r;
            *dst = p.accumulate ? *dst + v : v;
          }
        }
      }
    }
    return;
  }
  float sa = 0.0f, sb = 0.0f;   // RATIO_MEAN uses sa only
  for (int e = lane; e < npairs; e += 64) {
    const int ph = e / nv, t = skip + e - ph * nv;
    const float wp = p.w ? p.w[ph] : 1.0f / (float)p.P;
    const float* row = m + ((size_t)ph * p.NQ + t) * p.S;
    const float a = row[p.span_a], b = row[p.span_b];
    if (p.mode == HOOK_REDUCE_RATIO_MEAN) {
      const float den = a + b;
      sa += den != 0.0f ? wp * (a / den) : 0.0f;
    } else {
      sa += wp * a;
      sb += wp * b;
    }
  }
  sa = wave_sum(sa);
  sb = wave_sum(sb);
  float v;
  if (p.mode == HOOK_REDUCE_RATIO_MEAN) {
    v = sa * inv_nv;
  } else {
    const float A = sa * inv_nv, B = sb * inv_nv;
    v = (A + B) != 0.0f ? A / (A + B) : 0.0f;
  }
  if (lane == 0) p.scores[i] = p.accumulate ? p.scores[i] + v : v;
}

}  // namespace
}  // namespace hook

extern "C" hook_status hook_reduce_mass(const hook_reduce_args* a) {
  using namespace hook;
  if (!a) return HOOK_ERR_NULL;
  if (a->num_seqs < 0 || a->num_probe_heads < 1 || a->max_sel_q < 1 || a->max_sel_q > HOOK_MAX_SEL_Q ||
      a->max_spans < 1 || a->max_spans > HOOK_MAX_SPANS_WIDE)
    return HOOK_ERR_SHAPE;
  if (a->mode != HOOK_REDUCE_SPAN_MEAN && a->mode != HOOK_REDUCE_RATIO_MEAN && a->mode != HOOK_REDUCE_RATIO_OF_SUMS)
    return HOOK_ERR_UNSUPPORTED;
  if (a->mode != HOOK_REDUCE_SPAN_MEAN &&
      (a->span_a < 0 || a->span_a >= a->max_spans || a->span_b < 0 || a->span_b >= a->max_spans))
    return HOOK_ERR_SHAPE;
  if (a->num_seqs == 0) return HOOK_OK;
  if (!a->mass || !a->scores) return HOOK_ERR_NULL;
  ReduceParams p{};
  p.num_seqs = a->num_seqs; p.P = a->num_probe_heads; p.NQ = a->max_sel_q; p.S = a->max_spans;
  p.mode = a->mode; p.span_a = a->span_a; p.span_b = a->span_b; p.accumulate = a->accumulate;
  p.mass = a->mass; p.query_sel = a->query_sel; p.cu_q_lens = a->cu_q_lens; p.w = a->head_weights;
  p.scores = a->scores;
  hipLaunchKernelGGL(k_reduce_mass, dim3((unsigned)((p.num_seqs + 3) / 4)), dim3(256), 0,
                     static_cast<hipStream_t>(a->stream), p);
  return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}
