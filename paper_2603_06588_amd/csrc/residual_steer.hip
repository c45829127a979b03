// Steering folded into the residual add that produces the hidden state:
//   hidden[t, :] = hidden[t, :] + delta[t, :] (+ alpha * vec[:] on masked rows)
// Every row is read and written once by the add itself, so the steering costs no traffic of
// its own.  The three terms are summed in fp64 (the product alpha * vec is exact there) and
// rounded to the storage type once, round-to-nearest-even.
#include "../../include/hook_api.h"
#include "hook_device.h"

namespace hook {
namespace {

// fp64 -> bf16, one rounding to nearest even.  The value first goes to fp32 (nearest even);
// only when that lands exactly on the midpoint of two bf16 neighbours can the second step
// round the wrong way, and then the fp32 value is nudged to the side the fp64 value is on.
__device__ __forceinline__ uint32_t f64_to_bf16_bits(double x) {
  const float f = (float)x;
  uint32_t u = __float_as_uint(f);
  if ((u & 0xFFFFu) == 0x8000u) {          // rare: about one value in 65536
    const double back = (double)f;
    if (__builtin_fabs(back) > __builtin_fabs(x)) u -= 1;        // really below the midpoint
    else if (__builtin_fabs(back) < __builtin_fabs(x)) u += 1;   // really above it
  }
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// (h + d) + alpha * v for one element in fp32: u = fma(alpha, v, h + d).  `unsure` is raised unless
// rounding u to bf16 is certain to give what rounding the fp64 sum gives.  t = h + d carries at most
// half an ulp of error, the fused multiply-add (alpha * v is exact inside it) another half; unless
// the terms cancel (|u| < |t| / 2) that is at most 1.5 ulp of u, so the bf16 result can only differ
// when u lies within two fp32 ulps of the midpoint of two bf16 neighbours (low 16 bits 0x8000).
// Zero, subnormal, infinite and NaN results are left to the fp64 path as well.
__device__ __forceinline__ float steer_fast(float h, float d, float alpha, float v, bool& unsure) {
  const float t = h + d;
  const float u = __builtin_fmaf(alpha, v, t);
  const uint32_t b = __float_as_uint(u);
  // class bits: signalling / quiet NaN, -inf, -subnormal, -0, +0, +subnormal, +inf
  constexpr int kNotNormal = 0x001 | 0x002 | 0x004 | 0x010 | 0x020 | 0x040 | 0x080 | 0x200;
  unsure = unsure || (((b - 0x7FFEu) & 0xFFFFu) <= 4u) || !(__builtin_fabsf(u) >= 0.5f * __builtin_fabsf(t)) ||
           __builtin_amdgcn_classf(u, kNotNormal);
  return u;
}

constexpr int kRowsPerWg = 1;   // fp32 kernel: rows per workgroup
constexpr int kColsPerTrip = 2;  // bf16 kernel: 16-byte column chunks a thread has in flight (two streams each)

// One workgroup per row: small workgroups keep many independent load streams in flight, which
// is what this streaming kernel lives on (4, 2, 1 rows per workgroup: 47, 41, 40 us on a
// [8448, 4096] bf16 buffer).  A thread takes kColsPerTrip column chunks per trip, all loads first.
// Steered elements take the fp32 route above and fall back, pair by pair, to the fp64 sum in the
// rare cases (about one pair in ten thousand) where fp32 cannot guarantee the same rounding.
__global__ __launch_bounds__(256) void k_residual_steer_bf16(uint4* __restrict__ hidden, const uint4* __restrict__ delta,
                                                              const uint4* __restrict__ vec, float alpha,
                                                              const uint8_t* __restrict__ mask, int D8, int T) {
  const int row = blockIdx.x;
  const bool on = mask != nullptr && mask[row] != 0;
  const double a = (double)alpha;
  uint4* const hrow = hidden + (size_t)row * D8;
  const uint4* const drow = delta + (size_t)row * D8;
  for (int c0 = threadIdx.x; c0 < D8; c0 += 256 * kColsPerTrip) {
    uint4 h[kColsPerTrip], d[kColsPerTrip], v[kColsPerTrip];
#pragma unroll
    for (int u = 0; u < kColsPerTrip; ++u) {
      const int c = c0 + 256 * u;
      if (c < D8) {
        h[u] = load_stream16(&hrow[c]);
        d[u] = load_stream16(&drow[c]);
        v[u] = on ? vec[c] : make_uint4(0u, 0u, 0u, 0u);
      }
    }
#pragma unroll
    for (int u = 0; u < kColsPerTrip; ++u) {
      const int c = c0 + 256 * u;
      if (c >= D8) continue;
      const uint32_t hw[4] = {h[u].x, h[u].y, h[u].z, h[u].w};
      const uint32_t dw[4] = {d[u].x, d[u].y, d[u].z, d[u].w};
      const uint32_t vw[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
      uint32_t y[4];
      if (on) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          bool unsure = false;
          const float lo = steer_fast(bf16_lo(hw[k]), bf16_lo(dw[k]), alpha, bf16_lo(vw[k]), unsure);
          const float hi = steer_fast(bf16_hi(hw[k]), bf16_hi(dw[k]), alpha, bf16_hi(vw[k]), unsure);
          y[k] = pack_bf16(lo, hi);
          if (__builtin_expect(unsure, 0)) {   // the definition: three fp64 terms, one rounding
            const double dlo = ((double)bf16_lo(hw[k]) + (double)bf16_lo(dw[k])) + a * (double)bf16_lo(vw[k]);
            const double dhi = ((double)bf16_hi(hw[k]) + (double)bf16_hi(dw[k])) + a * (double)bf16_hi(vw[k]);
            y[k] = f64_to_bf16_bits(dlo) | (f64_to_bf16_bits(dhi) << 16);
          }
        }
      } else {
        // the sum of two bf16 values is exact in fp32 unless they are more than 2^16 apart, and
        // then the fp32 result cannot sit on a bf16 midpoint: one fp32 add, then nearest even
#pragma unroll
        for (int k = 0; k < 4; ++k)
          y[k] = pack_bf16(bf16_lo(hw[k]) + bf16_lo(dw[k]), bf16_hi(hw[k]) + bf16_hi(dw[k]));
      }
      store_stream16(&hrow[c], make_uint4(y[0], y[1], y[2], y[3]));
    }
  }
}

__global__ __launch_bounds__(256) void k_residual_steer_f32(float4* __restrict__ hidden, const float4* __restrict__ delta,
                                                             const float4* __restrict__ vec, float alpha,
                                                             const uint8_t* __restrict__ mask, int D4, int T) {
  const int row0 = blockIdx.x * kRowsPerWg;
  bool on[kRowsPerWg];
  bool any = false;
#pragma unroll
  for (int r = 0; r < kRowsPerWg; ++r) {
    on[r] = mask != nullptr && row0 + r < T && mask[row0 + r] != 0;
    any |= on[r];
  }
  const double a = (double)alpha;
  for (int c = threadIdx.x; c < D4; c += 256) {
    float4 h[kRowsPerWg], d[kRowsPerWg];
#pragma unroll
    for (int r = 0; r < kRowsPerWg; ++r)
      if (row0 + r < T) {
        h[r] = hidden[(size_t)(row0 + r) * D4 + c];
        d[r] = delta[(size_t)(row0 + r) * D4 + c];
      }
    double av[4];
    if (any) {
      const float4 v = vec[c];
      av[0] = a * (double)v.x; av[1] = a * (double)v.y; av[2] = a * (double)v.z; av[3] = a * (double)v.w;
    }
#pragma unroll
    for (int r = 0; r < kRowsPerWg; ++r) {
      if (row0 + r >= T) continue;
      float4 y;
      if (on[r]) {
        y.x = (float)(((double)h[r].x + (double)d[r].x) + av[0]);
        y.y = (float)(((double)h[r].y + (double)d[r].y) + av[1]);
        y.z = (float)(((double)h[r].z + (double)d[r].z) + av[2]);
        y.w = (float)(((double)h[r].w + (double)d[r].w) + av[3]);
      } else {
        y = make_float4(h[r].x + d[r].x, h[r].y + d[r].y, h[r].z + d[r].z, h[r].w + d[r].w);
      }
      hidden[(size_t)(row0 + r) * D4 + c] = y;
    }
  }
}

}  // namespace
}  // namespace hook

extern "C" hook_status hook_residual_add_steer(void* hidden, const void* delta, const void* vec, float alpha,
                                               const uint8_t* token_mask, int32_t num_tokens, int32_t hidden_dim,
                                               int32_t dtype, void* stream) {
  using namespace hook;
  if (num_tokens < 0 || hidden_dim < 0) return HOOK_ERR_SHAPE;
  if (dtype != HOOK_BF16 && dtype != HOOK_F32) return HOOK_ERR_UNSUPPORTED;
  const int per = dtype == HOOK_BF16 ? 8 : 4;
  if (hidden_dim % per != 0) return HOOK_ERR_UNSUPPORTED;
  if (num_tokens == 0 || hidden_dim == 0) return HOOK_OK;
  if (!hidden || !delta) return HOOK_ERR_NULL;
  const bool steer = alpha != 0.0f && token_mask != nullptr;
  if (steer && !vec) return HOOK_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(hidden) | reinterpret_cast<uintptr_t>(delta) |
       (steer ? reinterpret_cast<uintptr_t>(vec) : 0)) % 16 != 0)
    return HOOK_ERR_UNSUPPORTED;
  const int Dc = hidden_dim / per;
  const unsigned blocks = (unsigned)((num_tokens + kRowsPerWg - 1) / kRowsPerWg);   // = num_tokens
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint8_t* m = steer ? token_mask : nullptr;
  if (dtype == HOOK_BF16)
    hipLaunchKernelGGL(k_residual_steer_bf16, dim3(blocks), dim3(256), 0, st, static_cast<uint4*>(hidden),
                       static_cast<const uint4*>(delta), static_cast<const uint4*>(vec), alpha, m, Dc, num_tokens);
  else
    hipLaunchKernelGGL(k_residual_steer_f32, dim3(blocks), dim3(256), 0, st, static_cast<float4*>(hidden),
                       static_cast<const float4*>(delta), static_cast<const float4*>(vec), alpha, m, Dc, num_tokens);
  return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}
