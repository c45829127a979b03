// Residual-stream steering: hidden[t, :] += alpha * vec[:] on masked rows, in place.
// Pure HBM streaming: one workgroup per row (small workgroups keep the most independent load
// streams in flight), two 16-byte column chunks per thread requested before either is used, one
// fp32 FMA per element, hardware round-to-nearest-even back to the storage type.  Rows whose mask
// byte is zero are skipped before any access to `hidden`.
#include "hook_device.h"

namespace hook {

namespace {

constexpr int kSteerCols = 2;   // 16-byte column chunks a thread has in flight

__global__ __launch_bounds__(256) void k_steer_bf16(uint4* __restrict__ hidden, const uint4* __restrict__ vec,
                                                     float alpha, const uint8_t* __restrict__ mask, int D8) {
  const int row = blockIdx.x;
  if (mask[row] == 0) return;   // unmasked rows are neither read nor written
  uint4* const h = hidden + (size_t)row * D8;
  for (int c0 = threadIdx.x; c0 < D8; c0 += 256 * kSteerCols) {
    uint4 x[kSteerCols], v[kSteerCols];
#pragma unroll
    for (int u = 0; u < kSteerCols; ++u) {
      const int c = c0 + 256 * u;
      if (c < D8) { x[u] = h[c]; v[u] = vec[c]; }
    }
#pragma unroll
    for (int u = 0; u < kSteerCols; ++u) {
      const int c = c0 + 256 * u;
      if (c >= D8) continue;
      uint4 y;
      y.x = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v[u].x), bf16_lo(x[u].x)), __builtin_fmaf(alpha, bf16_hi(v[u].x), bf16_hi(x[u].x)));
      y.y = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v[u].y), bf16_lo(x[u].y)), __builtin_fmaf(alpha, bf16_hi(v[u].y), bf16_hi(x[u].y)));
      y.z = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v[u].z), bf16_lo(x[u].z)), __builtin_fmaf(alpha, bf16_hi(v[u].z), bf16_hi(x[u].z)));
      y.w = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v[u].w), bf16_lo(x[u].w)), __builtin_fmaf(alpha, bf16_hi(v[u].w), bf16_hi(x[u].w)));
      h[c] = y;
    }
  }
}

__global__ __launch_bounds__(256) void k_steer_f32(float4* __restrict__ hidden, const float4* __restrict__ vec,
                                                    float alpha, const uint8_t* __restrict__ mask, int D4) {
  const int row = blockIdx.x;
  if (mask[row] == 0) return;
  float4* h = hidden + (size_t)row * D4;
  for (int c = threadIdx.x; c < D4; c += 256) {
    float4 x = h[c];
    const float4 v = vec[c];
    x.x = __builtin_fmaf(alpha, v.x, x.x);
    x.y = __builtin_fmaf(alpha, v.y, x.y);
    x.z = __builtin_fmaf(alpha, v.z, x.z);
    x.w = __builtin_fmaf(alpha, v.w, x.w);
    h[c] = x;
  }
}

}  // namespace

hipError_t launch_steer(void* hidden, const void* vec, float alpha, const uint8_t* mask, int T, int D,
                        int dtype, hipStream_t st) {
  if (T <= 0 || D <= 0) return hipSuccess;
  if (dtype == 0)
    hipLaunchKernelGGL(k_steer_bf16, dim3((unsigned)T), dim3(256), 0, st, static_cast<uint4*>(hidden),
                       static_cast<const uint4*>(vec), alpha, mask, D / 8);
  else
    hipLaunchKernelGGL(k_steer_f32, dim3((unsigned)T), dim3(256), 0, st, static_cast<float4*>(hidden),
                       static_cast<const float4*>(vec), alpha, mask, D / 4);
  return hipGetLastError();
}

}  // namespace hook
