// Scatter of the new tokens' K and V rows into the paged cache.  A workgroup takes 16 consecutive
// rows of k_new / v_new: 16 lanes find each row's sequence (binary search in cu_q_lens) and its
// cache slot, then every thread moves 16-byte chunks, eight loads in flight.
#include "../../include/hook_api.h"
#include "hook_device.h"

namespace hook {
namespace {

struct KvWriteParams {
  int num_seqs, total_q, Hkv, max_blocks, num_blocks, row_chunks;   // row_chunks = d * esize / 16
  const uint4* k_new;
  const uint4* v_new;
  const int* block_table;
  const int* seq_lens;
  const int* cu_q_lens;
  uint4* k_cache;
  uint4* v_cache;
};

constexpr int kRowTile = 16;
constexpr int kKvInFlight = 8;

__global__ __launch_bounds__(256) void k_kv_write(const KvWriteParams p) {
  __shared__ long long dst_row[kRowTile];   // blk * Hkv * kBlock + slot, or -1: do not write
  const int rc = p.row_chunks;
  const int row0 = blockIdx.x * kRowTile;
  if (threadIdx.x < kRowTile) {
    const int row = row0 + threadIdx.x;
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
    dst_row[threadIdx.x] = r;
  }
  __syncthreads();
  const int nrow = min(kRowTile, p.total_q - row0);
  const int row_stride = p.Hkv * rc;            // chunks per token in k_new
  const int nchunks = nrow * row_stride;
  const uint4* ksrc = p.k_new + (size_t)row0 * row_stride;
  const uint4* vsrc = p.v_new + (size_t)row0 * row_stride;
  for (int base = threadIdx.x; base < nchunks; base += 256 * (kKvInFlight / 2)) {
    uint4 kv[kKvInFlight / 2], vv[kKvInFlight / 2];
#pragma unroll
    for (int u = 0; u < kKvInFlight / 2; ++u) {
      const int idx = base + u * 256;
      if (idx < nchunks) { kv[u] = load_stream16(&ksrc[idx]); vv[u] = load_stream16(&vsrc[idx]); }
    }
#pragma unroll
    for (int u = 0; u < kKvInFlight / 2; ++u) {
      const int idx = base + u * 256;
      if (idx >= nchunks) continue;
      const int ts = idx / row_stride, rem = idx - ts * row_stride;
      const int g = rem / rc, cc = rem - g * rc;
      const long long r = dst_row[ts];
      if (r < 0) continue;
      const size_t d = (size_t)(r + (long long)g * kBlock) * rc + cc;
      p.k_cache[d] = kv[u];
      p.v_cache[d] = vv[u];
    }
  }
}

}  // namespace
}  // namespace hook

extern "C" hook_status hook_kv_write(const hook_kv_write_args* a) {
  using namespace hook;
  if (!a) return HOOK_ERR_NULL;
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_kv_heads <= 0 || a->head_dim <= 0 || a->max_blocks_per_seq <= 0 ||
      a->num_blocks <= 0)
    return HOOK_ERR_SHAPE;
  if (a->block_size != HOOK_BLOCK_SIZE) return HOOK_ERR_UNSUPPORTED;
  if (a->dtype != HOOK_BF16 && a->dtype != HOOK_F32) return HOOK_ERR_UNSUPPORTED;
  const int esize = a->dtype == HOOK_BF16 ? 2 : 4;
  if ((a->head_dim * esize) % 16 != 0 || a->max_blocks_per_seq > (1 << 26)) return HOOK_ERR_UNSUPPORTED;
  if (a->num_seqs == 0 || a->total_q == 0) return HOOK_OK;
  if (!a->k_new || !a->v_new || !a->block_table || !a->seq_lens || !a->cu_q_lens || !a->k_cache || !a->v_cache)
    return HOOK_ERR_NULL;
  KvWriteParams p{};
  p.num_seqs = a->num_seqs; p.total_q = a->total_q; p.Hkv = a->num_kv_heads; p.max_blocks = a->max_blocks_per_seq;
  p.num_blocks = a->num_blocks; p.row_chunks = a->head_dim * esize / 16;
  if ((long long)kRowTile * p.Hkv * p.row_chunks > 0x7FFFFFFFll) return HOOK_ERR_UNSUPPORTED;
  p.k_new = static_cast<const uint4*>(a->k_new); p.v_new = static_cast<const uint4*>(a->v_new);
  p.block_table = a->block_table; p.seq_lens = a->seq_lens; p.cu_q_lens = a->cu_q_lens;
  p.k_cache = static_cast<uint4*>(a->k_cache); p.v_cache = static_cast<uint4*>(a->v_cache);
  hipLaunchKernelGGL(k_kv_write, dim3((unsigned)((p.total_q + kRowTile - 1) / kRowTile)), dim3(256), 0,
                     static_cast<hipStream_t>(a->stream), p);
  return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}
