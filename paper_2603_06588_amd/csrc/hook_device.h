// Internal declarations shared by the HIP translation units of libhook (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace hook {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 16;          // tokens per KV block
constexpr int kMaxSpans = 8;        // compile-time bound on S
constexpr int kTileKeys = 64;       // keys per prefill tile
constexpr int kWaveRows = 32;       // query rows per prefill wave
constexpr int kPartialPad = 16;     // floats after the D output values of a decode partial: m, l, a[8], pad
constexpr int kPlanBuckets = 2048;  // counting-sort buckets (tile counts) of the prefill work list
// Decode chunking rule shared by the planner (which applies it) and the host (which bounds the
// number of items it can produce): the largest chunk of 512 << k keys, up to kMaxChunkKeys, that
// still yields kDecodeFillWgs decode workgroups; 256 keys when none does.
constexpr int kChunkSizes = 5;
constexpr int kMaxChunkKeys = 512 << (kChunkSizes - 1);
constexpr int kDecodeFillWgs = 2048;
// A running maximum is only raised when a tile's maximum exceeds it by more than this many
// powers of two; exponentials then stay below 2^kLazyTau, far inside fp32 range, and the
// normaliser carries the same reference, so the result is the exact softmax.
constexpr float kLazyTau = 8.0f;

// Device-side status bits written by the plan kernel.
enum : int { kStatQGtL = 1, kStatLenClamped = 2, kStatNegative = 4, kStatHint = 8 };

struct PlanHeader {
  int n_prefill;   // prefill work items (row blocks)
  int n_decode;    // decode work items (key chunks)
  int chunk_keys;  // keys per decode work item
  int status;      // kStat* bits of the last attention call
  int problems;    // HOOK_BAD_* bits of the last hook_attn_probe_validate call (a word of its own)
  int pad[11];
};

// Work-list records.  prefill: two consecutive records per item,
// {seq, first chunk-local row, L, n} and {global row of the sequence's first query, 0, 0, 0};
// decode: one record {seq, chunk index, L, global q row}.
typedef int4 WorkItem;

// Cache write of the new tokens' rows (kv_write_device.h)
struct KvWriteParams {
  int num_seqs, total_q, Hkv, max_blocks, num_blocks;
  int row_chunks;   // 16-byte chunks per (token, kv head) row of k_new / v_new
  int kv8;          // the cache holds 8-bit E4M3 bytes: rows (bf16) are quantised on the way
  const uint4* k_new;
  const uint4* v_new;
  const int* block_table;
  const int* seq_lens;
  const int* cu_q_lens;
  void* k_cache;
  void* v_cache;
  const float* k_scale;   // [Hkv], kv8 only
  const float* v_scale;
};

struct AttnParams {
  int num_seqs, total_q, Hq, Hkv, G, max_blocks, num_blocks;
  float scale_log2;                 // softmax scale * log2(e)
  const void* q;
  const void* k_cache;
  const void* v_cache;
  const int* block_table;
  const int* seq_lens;
  const int* cu_q_lens;
  int P;
  const int* probe_heads;
  int NQ;
  const int* query_sel;
  int S;
  const int* key_spans;
  void* out;
  float* mass;
  // new tokens' key/value rows to be written into the cache before anything reads it (kvw.k_new != null)
  KvWriteParams kvw;
  // 8-bit (E4M3) key/value cache: bytes instead of `dtype` elements, one fp32 scale per kv head
  int kv8;
  const float* k_scale;
  const float* v_scale;
  // workspace carve-up
  PlanHeader* hdr;
  WorkItem* pf_items;
  int pf_cap;
  WorkItem* dec_items;              // two records per turn, longest chunks first: {seq, chunk, L, q row}, {partial slot, -, -, -}
  int dec_cap;
  int2* seq_dec;                    // per sequence {first decode item, number of chunks}
  float* partials;                  // [dec_cap, Hq, D + kPartialPad]
  int dec_parts;                    // > 0: no planner; every single-row sequence is cut into this many parts
  int plan_fresh;                   // the call promises a fully written `mass` (not a reused plan)
  int pf_self;                      // one sequence of query rows, head_dim 128: the chunk kernel plans itself
  // geometry chosen on the host from G
  int batch_kind;                   // 0 mixed, 1 no single-row sequences, 2 only single-row sequences
  int hpw;                          // q heads per prefill workgroup (4, 2 or 1)
  int rows_per_wg;                  // 32 * (4 / hpw)
  int hgroups;                      // G / hpw
  int dec_hp;                       // q heads per decode workgroup (8, 4, 2 or 1)
  int dec_hgroups;                  // G / dec_hp
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);  // v_cvt_pk_bf16_f32, round-to-nearest-even
  uint32_t u;
  __builtin_memcpy(&u, &b, 4);
  return u;
}

// 16-byte load of data that is read once and not again (K/V rows on the decode path): the
// non-temporal hint keeps the stream from displacing useful lines and measurably raises the
// sustained read rate on this chip.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte store of data that this kernel does not read again.
__device__ __forceinline__ void store_stream16(void* p, const uint4 v) {
  u32x4 x;
  x.x = v.x; x.y = v.y; x.z = v.z; x.w = v.w;
  __builtin_nontemporal_store(x, static_cast<u32x4*>(p));
}

// Index of `head` in the strictly increasing list probe_heads[0..P), or -1: a binary search, so
// the chain of dependent loads is log2(P) long (a list that is not increasing just fails to
// find some heads).
__device__ __forceinline__ int find_probe_slot(const int* probe_heads, int P, int head) {
  int lo = 0, hi = P;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (probe_heads[mid] < head) lo = mid + 1; else hi = mid;
  }
  return (lo < P && probe_heads[lo] == head) ? lo : -1;
}

// Spans of one sequence, all fetched before any is waited for (entries past S repeat the last
// span and are never used).
__device__ __forceinline__ void load_spans(const int* key_spans, int seq, int S, int (&sp_a)[kMaxSpans],
                                           int (&sp_b)[kMaxSpans]) {
  const int2* sp = reinterpret_cast<const int2*>(key_spans) + (size_t)seq * S;
  int2 v[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) v[s] = sp[min(s, S - 1)];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) {
    sp_a[s] = s < S ? max(v[s].x, 0) : 0;
    sp_b[s] = s < S ? v[s].y : 0;
  }
}

// launchers (defined next to their kernels); all return hipGetLastError() after the launch
// The dynamic-LDS limit of a kernel is an attribute per device: it is raised on the first launch
// on each device (bit per device id in `done`), from whichever host thread gets there first.
inline hipError_t raise_lds_limit_once(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  if (tracked) done.fetch_or(1ull << dev, std::memory_order_release);
  return hipSuccess;
}

// Launch grids are one-dimensional and must fit the 31-bit limit.
inline bool grid_fits(long long workgroups) { return workgroups >= 0 && workgroups <= 0x7fffffffLL; }

hipError_t launch_plan(const AttnParams& p, hipStream_t st);
hipError_t launch_kv_write(const KvWriteParams& p, hipStream_t st);
hipError_t launch_prefill(const AttnParams& p, int D, hipStream_t st);
hipError_t launch_prefill128(const AttnParams& p, hipStream_t st);
hipError_t launch_decode(const AttnParams& p, int D, hipStream_t st);
hipError_t launch_combine(const AttnParams& p, int D, hipStream_t st);
hipError_t launch_attn_f32(const AttnParams& p, int D, hipStream_t st);
hipError_t launch_steer(void* hidden, const void* vec, float alpha, const uint8_t* mask, int T, int D,
                        int dtype, hipStream_t st);

}  // namespace hook
