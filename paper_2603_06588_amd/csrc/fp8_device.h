// Widening of 8-bit E4M3 cache bytes to bf16 (exact: every E4M3 number is a bf16 number), shared by
// the kernels that stage or load keys and values of an 8-bit cache through registers.
#pragma once

#include "hook_device.h"

namespace hook {

// eight E4M3 bytes (two words) -> eight bf16 values
__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(uint2 raw) {
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.x, 1.0f, false);
  const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.x, 1.0f, true);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.y, 1.0f, false);
  const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.y, 1.0f, true);
  uint4 v;
  __builtin_memcpy(&v.x, &a, 4);
  __builtin_memcpy(&v.y, &b, 4);
  __builtin_memcpy(&v.z, &c, 4);
  __builtin_memcpy(&v.w, &d, 4);
  return v;
}

}  // namespace hook
