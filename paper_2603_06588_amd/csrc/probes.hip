// Measurement aids: what this chip sustains on the two resources the kernels are bound by.
//   k_probe_mfma  every SIMD issues independent 32x32x16 bf16 MFMAs back to back (two waves
//                 per SIMD, four accumulators each) - the sustained matrix-core rate, which
//                 sits below the nominal peak because the clock drops under this load;
//   k_probe_read  a streaming read of a buffer with 16-byte non-temporal loads - the sustained
//                 HBM read bandwidth.
#include "../../include/hook_api.h"
#include "hook_device.h"

namespace hook {
namespace {

__global__ __launch_bounds__(256, 2) void k_probe_mfma(int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  // eight operand pairs of pseudo-random bf16 values in [1, 2) x 2^-7 (an integer hash of lane
  // and slot in the mantissa), so the data paths toggle the way real operands make them
  union Op { uint32_t u[4]; bf16x8 v; } a[8], b[8];
#pragma unroll
  for (int k = 0; k < 8; ++k)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t h = (uint32_t)(lane * 8 + k) * 2654435761u + (uint32_t)i * 40503u;
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      a[k].u[i] = 0x3F803F80u | (h & 0x007F007Fu);
      b[k].u[i] = 0x3C003C00u | ((h >> 7) & 0x007F007Fu);
    }
  f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int rep = 0; rep < 4; ++rep)
#pragma unroll
      for (int k = 0; k < 4; ++k)
        acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * rep + (k & 1)].v, b[2 * (k >> 1) + (rep & 1) + 4 * (rep >> 1)].v,
                                                         acc[k], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive
}

// Each workgroup takes contiguous 32 KB pieces round-robin and every thread keeps eight 16-byte
// non-temporal loads in flight: of the patterns tried (grid-stride or contiguous pieces, plain
// or non-temporal loads, 4 to 16 loads in flight) this one reads fastest on this chip.
constexpr int kReadInFlight = 8;

__global__ __launch_bounds__(256) void k_probe_read(const uint4* __restrict__ src, size_t n16, unsigned* sink) {
  constexpr size_t kPiece = 256 * kReadInFlight;   // 16-byte units per piece
  unsigned acc = 0;
  const size_t npieces = n16 / kPiece;
  for (size_t c = blockIdx.x; c < npieces; c += gridDim.x) {
    const uint4* p = src + c * kPiece + threadIdx.x;
    uint4 v[kReadInFlight];
#pragma unroll
    for (int u = 0; u < kReadInFlight; ++u) v[u] = load_stream16(&p[u * 256]);
#pragma unroll
    for (int u = 0; u < kReadInFlight; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (size_t i = npieces * kPiece + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

}  // namespace
}  // namespace hook

extern "C" {

hook_status hook_probe_mfma_bf16(int32_t iters, int32_t num_workgroups, void* sink, void* stream, double* flops) {
  if (!sink || !flops) return HOOK_ERR_NULL;
  if (iters <= 0 || num_workgroups <= 0) return HOOK_ERR_SHAPE;
  hipLaunchKernelGGL(hook::k_probe_mfma, dim3((unsigned)num_workgroups), dim3(256), 0,
                     static_cast<hipStream_t>(stream), iters, static_cast<float*>(sink));
  if (hipGetLastError() != hipSuccess) return HOOK_ERR_LAUNCH;
  // 4 waves x 16 MFMAs per iteration x 2 * 32 * 32 * 16 flops
  *flops = (double)num_workgroups * 4.0 * 16.0 * (double)iters * 32768.0;
  return HOOK_OK;
}

hook_status hook_probe_hbm_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return HOOK_ERR_NULL;
  if (bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15) != 0) return HOOK_ERR_SHAPE;
  hipLaunchKernelGGL(hook::k_probe_read, dim3(256 * 32), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), bytes / 16, static_cast<unsigned*>(sink));
  return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}

}  // extern "C"
