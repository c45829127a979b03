// fp32 attention + probe, one wave per (query row, q head).  Full-precision inputs cannot
// go through the bf16 matrix cores without changing the result, so this path keeps every
// product and sum in fp32 on the vector ALUs: lanes take keys round-robin, each runs an
// online softmax over its keys with the output row in registers, and the 64 lane states
// are merged at the end.  It serves small full-precision batches; the bf16 kernels are the
// throughput path.
#include "hook_device.h"

namespace hook {

namespace {

template <int D>
__global__ __launch_bounds__(64) void k_attn_f32(const AttnParams p) {
  __shared__ float qs[D];
  __shared__ float red[64][D + 1];

  const int grow = blockIdx.x;   // global query row
  const int head = blockIdx.y;
  const int lane = threadIdx.x;

  // sequence of this row: largest i with cu[i] <= grow
  int lo = 0, hi = p.num_seqs;   // invariant: cu[lo] <= grow < cu[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (p.cu_q_lens[mid] <= grow) lo = mid; else hi = mid;
  }
  const int seq = lo;
  const int row0 = p.cu_q_lens[seq];
  const int n = p.cu_q_lens[seq + 1] - row0;
  int L = p.seq_lens[seq];
  const int t = grow - row0;
  // the same status bits the planner of the bf16 path records (one lane of the row's first head)
  if (head == 0 && lane == 0 && t == 0 && n > 0) {
    int bits = 0;
    if (L < 0) bits |= kStatNegative;
    else if (n > min(L, p.max_blocks * kBlock)) bits |= kStatQGtL;
    if (L > p.max_blocks * kBlock) bits |= kStatLenClamped;
    if (bits) atomicOr(&p.hdr->status, bits);
  }
  L = min(L, p.max_blocks * kBlock);
  if (t < 0 || t >= n || n > L || L <= 0) return;
  const int pos = min(L - n + t, L - 1);
  if (pos < 0) return;

  const float* const qg = static_cast<const float*>(p.q);
  const float* const kg_ = static_cast<const float*>(p.k_cache);
  const float* const vg_ = static_cast<const float*>(p.v_cache);
  const int* const bt = p.block_table + (size_t)seq * p.max_blocks;
  const int kvh = head / p.G;
  const size_t blk_stride = (size_t)p.Hkv * kBlock * D;
  const size_t head_off = (size_t)kvh * kBlock * D;

  for (int c = lane; c < D; c += 64) qs[c] = qg[((size_t)grow * p.Hq + head) * D + c];
  __syncthreads();

  int pslot = -1;
  int sp_a[kMaxSpans], sp_b[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) { sp_a[s] = 0; sp_b[s] = 0; }
  int qsel_b = 0;
  if (p.P > 0) {
    qsel_b = p.query_sel[2 * seq];
    const int qsel_e = min(p.query_sel[2 * seq + 1], qsel_b + p.NQ);
    if (t >= qsel_b && t < qsel_e) pslot = find_probe_slot(p.probe_heads, p.P, head);
    if (pslot >= 0) {
#pragma unroll
      for (int s = 0; s < kMaxSpans; ++s)
        if (s < p.S) {
          sp_a[s] = max(p.key_spans[((size_t)seq * p.S + s) * 2], 0);
          sp_b[s] = p.key_spans[((size_t)seq * p.S + s) * 2 + 1];
        }
    }
  }

  const float c = p.scale_log2;
  float m_run = -INFINITY, l_run = 0.0f;
  float am[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) am[s] = 0.0f;
  float acc[D];
#pragma unroll
  for (int e = 0; e < D; ++e) acc[e] = 0.0f;

  for (int key = lane; key <= pos; key += 64) {
    int blk = bt[key >> 4];
    blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
    const size_t off = (size_t)blk * blk_stride + head_off + (size_t)(key & 15) * D;
    const float4* kp = reinterpret_cast<const float4*>(kg_ + off);
    const float4* vp = reinterpret_cast<const float4*>(vg_ + off);
    float dot = 0.0f;
#pragma unroll
    for (int e = 0; e < D / 4; ++e) {
      const float4 kv = kp[e];
      dot = __builtin_fmaf(qs[4 * e], kv.x, dot);
      dot = __builtin_fmaf(qs[4 * e + 1], kv.y, dot);
      dot = __builtin_fmaf(qs[4 * e + 2], kv.z, dot);
      dot = __builtin_fmaf(qs[4 * e + 3], kv.w, dot);
    }
    const float tt = dot * c;
    if (tt > m_run) {
      const float alpha = fast_exp2(m_run - tt);
      m_run = tt;
      l_run *= alpha;
#pragma unroll
      for (int s = 0; s < kMaxSpans; ++s) am[s] *= alpha;
#pragma unroll
      for (int e = 0; e < D; ++e) acc[e] *= alpha;
    }
    const float pr = fast_exp2(tt - m_run);
    l_run += pr;
#pragma unroll
    for (int s = 0; s < kMaxSpans; ++s)
      if (s < p.S) am[s] += (pslot >= 0 && key >= sp_a[s] && key < sp_b[s]) ? pr : 0.0f;
#pragma unroll
    for (int e = 0; e < D / 4; ++e) {
      const float4 vv = vp[e];
      acc[4 * e] = __builtin_fmaf(pr, vv.x, acc[4 * e]);
      acc[4 * e + 1] = __builtin_fmaf(pr, vv.y, acc[4 * e + 1]);
      acc[4 * e + 2] = __builtin_fmaf(pr, vv.z, acc[4 * e + 2]);
      acc[4 * e + 3] = __builtin_fmaf(pr, vv.w, acc[4 * e + 3]);
    }
  }

  // merge the 64 lane states
  float mstar = m_run;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, off));
  const float wgt = (m_run == -INFINITY) ? 0.0f : fast_exp2(m_run - mstar);
  float l = l_run * wgt;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) l += __shfl_xor(l, off);
  const float inv = 1.0f / l;
#pragma unroll
  for (int e = 0; e < D; ++e) red[lane][e] = acc[e] * wgt;
  __syncthreads();
  float* og = static_cast<float*>(p.out) + ((size_t)grow * p.Hq + head) * D;
  for (int cidx = lane; cidx < D; cidx += 64) {
    float sum = 0.0f;
    for (int r = 0; r < 64; ++r) sum += red[r][cidx];
    og[cidx] = sum * inv;
  }
  if (pslot >= 0) {
#pragma unroll
    for (int s = 0; s < kMaxSpans; ++s) {
      if (s < p.S) {
        float a = am[s] * wgt;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);
        if (lane == 0) p.mass[(((size_t)seq * p.P + pslot) * p.NQ + (t - qsel_b)) * p.S + s] = a * inv;
      }
    }
  }
}

// clears mass and the status word of the workspace header (this path has no planner to do it)
__global__ __launch_bounds__(256) void k_zero(float* ptr, size_t n, PlanHeader* hdr) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    hdr->n_prefill = 0; hdr->n_decode = 0; hdr->chunk_keys = 0; hdr->status = 0;
  }
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) ptr[i] = 0.0f;
}

}  // namespace

hipError_t launch_attn_f32(const AttnParams& p, int D, hipStream_t st) {
  const size_t nmass = (size_t)p.num_seqs * p.P * p.NQ * p.S;
  {
    size_t blocks = (nmass + 2047) / 2048;
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_zero, dim3((unsigned)blocks), dim3(256), 0, st, p.mass, nmass, p.hdr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (p.total_q <= 0) return hipSuccess;
  const dim3 grid((unsigned)p.total_q, (unsigned)p.Hq);
  if (D == 128) hipLaunchKernelGGL(k_attn_f32<128>, grid, dim3(64), 0, st, p);
  else if (D == 64) hipLaunchKernelGGL(k_attn_f32<64>, grid, dim3(64), 0, st, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace hook
