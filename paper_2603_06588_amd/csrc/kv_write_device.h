// Device code of the cache write, shared by the stand-alone kernel (hook_kv_write) and by the
// planning kernel of the attention call, whose spare workgroups write the new tokens' rows so that
// the call needs no launch of its own for it.
#pragma once

#include "hook_device.h"

namespace hook {

constexpr int kKvRowTile = 8;    // rows of k_new / v_new per tile (16 rows: 20 us for 8256 rows, 8: 15, 4: 16.4)

// fl32(x / scale) clamped to the range of the 8-bit format (NaN stays NaN)
__device__ __forceinline__ float fp8_prescale(float x, float scale) {
  const float y = x / scale;   // correctly rounded division
  return y > 448.0f ? 448.0f : (y < -448.0f ? -448.0f : y);
}

// eight bf16 values (one 16-byte chunk) -> eight E4M3 bytes, round to nearest even
__device__ __forceinline__ uint2 quantize_chunk_e4m3(const uint4 v, float scale) {
  int lo = 0, hi = 0;
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(fp8_prescale(bf16_lo(v.x), scale), fp8_prescale(bf16_hi(v.x), scale), lo, false);
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(fp8_prescale(bf16_lo(v.y), scale), fp8_prescale(bf16_hi(v.y), scale), lo, true);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(fp8_prescale(bf16_lo(v.z), scale), fp8_prescale(bf16_hi(v.z), scale), hi, false);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(fp8_prescale(bf16_lo(v.w), scale), fp8_prescale(bf16_hi(v.w), scale), hi, true);
  return make_uint2((unsigned)lo, (unsigned)hi);
}

// One tile of kKvRowTile consecutive rows, worked on by the NT threads of a workgroup (thread index
// tid).  dst_row is kKvRowTile entries of shared memory.  One thread per row finds the row's sequence
// (binary search in cu_q_lens) and its cache slot; then every thread moves 16-byte chunks.
// Rows of invalid sequences, positions beyond the block table and block ids outside the cache are
// dropped: nothing outside the cache is ever written.
template <int NT>
__device__ __forceinline__ void kv_write_tile(const KvWriteParams& p, int tile, int tid, long long* dst_row) {
  const int rc = p.row_chunks;
  const int row0 = tile * kKvRowTile;
  __syncthreads();   // dst_row may still be read by the previous tile
  if (tid < kKvRowTile) {
    const int row = row0 + tid;
    long long r = -1;
    if (row < p.total_q) {
      // sequence of this row: largest i with cu_q_lens[i] <= row
      int lo = 0, hi = p.num_seqs;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (p.cu_q_lens[mid] <= row) lo = mid; else hi = mid;
      }
      const int first = p.cu_q_lens[lo], n = p.cu_q_lens[lo + 1] - first, L = p.seq_lens[lo];
      const int t = row - first;
      if (first >= 0 && t >= 0 && t < n && n <= L && L >= 0) {
        const int pos = L - n + t;
        if (pos < p.max_blocks * kBlock) {
          const int blk = p.block_table[(size_t)lo * p.max_blocks + (pos >> 4)];
          if ((unsigned)blk < (unsigned)p.num_blocks) r = (long long)blk * p.Hkv * kBlock + (pos & 15);
        }
      }
    }
    dst_row[tid] = r;
  }
  __syncthreads();
  const int nrow = min(kKvRowTile, p.total_q - row0);
  const int row_stride = p.Hkv * rc;            // chunks per token in k_new
  const int nchunks = nrow * row_stride;
  const uint4* ksrc = p.k_new + (size_t)row0 * row_stride;
  const uint4* vsrc = p.v_new + (size_t)row0 * row_stride;
  constexpr int kInFlight = 4;
  for (int base = tid; base < nchunks; base += NT * kInFlight) {
    uint4 kv[kInFlight], vv[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int idx = base + u * NT;
      if (idx < nchunks) { kv[u] = load_stream16(&ksrc[idx]); vv[u] = load_stream16(&vsrc[idx]); }
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int idx = base + u * NT;
      if (idx >= nchunks) continue;
      const int ts = idx / row_stride, rem = idx - ts * row_stride;
      const int g = rem / rc, cc = rem - g * rc;
      const long long r = dst_row[ts];
      if (r < 0) continue;
      const size_t d = (size_t)(r + (long long)g * kBlock) * rc + cc;   // chunk index in the cache
      if (p.kv8) {
        static_cast<uint2*>(p.k_cache)[d] = quantize_chunk_e4m3(kv[u], p.k_scale[g]);
        static_cast<uint2*>(p.v_cache)[d] = quantize_chunk_e4m3(vv[u], p.v_scale[g]);
      } else {
        static_cast<uint4*>(p.k_cache)[d] = kv[u];
        static_cast<uint4*>(p.v_cache)[d] = vv[u];
      }
    }
  }
}

}  // namespace hook
