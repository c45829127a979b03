// Residual-stream steering: hidden[t, :] += alpha * vec[:] on masked rows, in place.
// Pure HBM streaming: one workgroup per row, 16-byte loads and stores, one fp32 FMA per
// element, hardware round-to-nearest-even back to the storage type.  Rows whose mask byte
// is zero are skipped before any access to `hidden`.
#include "hook_device.h"

namespace hook {

namespace {

__global__ __launch_bounds__(256) void k_steer_bf16(uint4* __restrict__ hidden, const uint4* __restrict__ vec,
                                                     float alpha, const uint8_t* __restrict__ mask, int D8) {
  const int row = blockIdx.x;
  if (mask[row] == 0) return;
  uint4* h = hidden + (size_t)row * D8;
  for (int c = threadIdx.x; c < D8; c += 256) {
    const uint4 x = h[c];
    const uint4 v = vec[c];
    uint4 y;
    y.x = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v.x), bf16_lo(x.x)), __builtin_fmaf(alpha, bf16_hi(v.x), bf16_hi(x.x)));
    y.y = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v.y), bf16_lo(x.y)), __builtin_fmaf(alpha, bf16_hi(v.y), bf16_hi(x.y)));
    y.z = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v.z), bf16_lo(x.z)), __builtin_fmaf(alpha, bf16_hi(v.z), bf16_hi(x.z)));
    y.w = pack_bf16(__builtin_fmaf(alpha, bf16_lo(v.w), bf16_lo(x.w)), __builtin_fmaf(alpha, bf16_hi(v.w), bf16_hi(x.w)));
    h[c] = y;
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
