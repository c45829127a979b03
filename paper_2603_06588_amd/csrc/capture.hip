// Compact q/k capture: gathers the queries of probed heads on selected rows and all keys of
// chosen kv heads from the paged cache into dense buffers.  Pure HBM streaming: 16-byte chunks,
// consecutive lanes on consecutive chunks of a (token, head) row.
#include "../../include/hook_api.h"
#include "hook_device.h"

namespace hook {
namespace {

struct CaptureParams {
  int num_seqs, total_q, Hq, Hkv, max_blocks, num_blocks;
  int row_chunks;     // 16-byte chunks per query row: d * esize / 16
  int k_row_chunks;   // 16-byte chunks per key row (fewer with an 8-bit cache)
  const uint4* q;
  const uint4* k_cache;
  const int* block_table;
  const int* seq_lens;
  const int* cu_q_lens;
  int P;
  const int* probe_heads;
  int NQ;
  const int* query_sel;
  int KH;
  const int* kv_heads;
  const int* cu_k_lens;
  int total_k;
  uint4* q_out;
  uint4* k_out;
};

// A workgroup moves kTokTile consecutive rows of k_out (all chosen heads): its first lanes find
// each token's sequence (binary search in cu_k_lens) and cache block, then every thread keeps up
// to kInFlight 16-byte loads in flight.  Destination chunks are consecutive over the whole tile;
// each source row (one token of one head) is a contiguous d-element run.
constexpr int kTokTile = 16;
constexpr int kInFlight = 8;

__global__ __launch_bounds__(256) void k_capture_k(const CaptureParams p) {
  __shared__ long long src_row[kTokTile];   // (blk * Hkv) * kBlock + slot, or -1 for a zero row
  const int rc = p.k_row_chunks;
  const int tok0 = blockIdx.x * kTokTile;
  if (threadIdx.x < kTokTile) {
    const int tok = tok0 + threadIdx.x;
    long long r = -1;
    if (tok < p.total_k) {
      // sequence of this token: largest i with cu_k_lens[i] <= tok
      int lo = 0, hi = p.num_seqs;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (p.cu_k_lens[mid] <= tok) lo = mid; else hi = mid;
      }
      const int j = tok - p.cu_k_lens[lo];
      if (j >= 0 && j < p.seq_lens[lo] && j < p.max_blocks * kBlock) {
        int blk = p.block_table[(size_t)lo * p.max_blocks + (j >> 4)];
        blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
        r = (long long)blk * p.Hkv * kBlock + (j & 15);
      }
    }
    src_row[threadIdx.x] = r;
  }
  __syncthreads();
  const int ntok = min(kTokTile, p.total_k - tok0);
  const int row_stride = p.KH * rc;            // chunks per token in k_out
  const int nchunks = ntok * row_stride;
  uint4* dst = p.k_out + (size_t)tok0 * row_stride;
  for (int base = threadIdx.x; base < nchunks; base += 256 * kInFlight) {
    uint4 v[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int idx = base + u * 256;
      v[u] = make_uint4(0, 0, 0, 0);
      if (idx < nchunks) {
        const int ts = idx / row_stride, rem = idx - ts * row_stride;
        const int c = rem / rc, cc = rem - c * rc;
        const long long r = src_row[ts];
        int g = p.kv_heads[c];
        g = ((unsigned)g < (unsigned)p.Hkv) ? g : 0;
        if (r >= 0) v[u] = load_stream16(&p.k_cache[(size_t)(r + (long long)g * kBlock) * rc + cc]);
      }
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int idx = base + u * 256;
      if (idx < nchunks) store_stream16(&dst[idx], v[u]);
    }
  }
}

// one thread per 16-byte chunk of q_out
__global__ __launch_bounds__(256) void k_capture_q(const CaptureParams p) {
  const int rc = p.row_chunks;
  const long long chunk = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = chunk / rc;                 // (i, p, tt)
  const int cc = (int)(chunk % rc);
  if (row >= (long long)p.num_seqs * p.P * p.NQ) return;
  const int tt = (int)(row % p.NQ);
  const int ps = (int)((row / p.NQ) % p.P);
  const int i = (int)(row / ((long long)p.NQ * p.P));
  const int qb = p.query_sel[2 * i], qe = p.query_sel[2 * i + 1];
  const int row0 = p.cu_q_lens[i], n = p.cu_q_lens[i + 1] - row0;
  const int t = qb + tt;
  uint4 v = make_uint4(0, 0, 0, 0);
  int h = p.probe_heads[ps];
  if (t >= 0 && t < qe && t < n && (unsigned)h < (unsigned)p.Hq && row0 >= 0 && row0 + t < p.total_q)
    v = p.q[((size_t)(row0 + t) * p.Hq + h) * rc + cc];
  p.q_out[(size_t)row * rc + cc] = v;
}

}  // namespace
}  // namespace hook

extern "C" hook_status hook_capture_qk(const hook_capture_qk_args* a) {
  using namespace hook;
  if (!a) return HOOK_ERR_NULL;
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->head_dim <= 0 ||
      a->max_blocks_per_seq <= 0 || a->num_blocks <= 0 || a->total_k < 0 || a->num_probe_heads < 0 ||
      a->num_capture_kv_heads < 0)
    return HOOK_ERR_SHAPE;
  if (a->block_size != HOOK_BLOCK_SIZE) return HOOK_ERR_UNSUPPORTED;
  if (a->dtype != HOOK_BF16 && a->dtype != HOOK_F32) return HOOK_ERR_UNSUPPORTED;
  const int esize = a->dtype == HOOK_BF16 ? 2 : 4;
  if ((a->head_dim * esize) % 16 != 0) return HOOK_ERR_UNSUPPORTED;
  if (a->kv_dtype != HOOK_KV_SAME && a->kv_dtype != HOOK_KV_FP8_E4M3) return HOOK_ERR_SHAPE;
  const int kesize = a->kv_dtype == HOOK_KV_FP8_E4M3 ? 1 : esize;
  if (a->kv_dtype == HOOK_KV_FP8_E4M3 && (a->dtype != HOOK_BF16 || a->head_dim % 16 != 0)) return HOOK_ERR_UNSUPPORTED;
  if (a->num_probe_heads > 0 && (a->max_sel_q < 1 || a->max_sel_q > HOOK_MAX_SEL_Q)) return HOOK_ERR_SHAPE;
  if (a->num_seqs == 0) return HOOK_OK;
  CaptureParams p{};
  p.num_seqs = a->num_seqs; p.total_q = a->total_q; p.Hq = a->num_q_heads; p.Hkv = a->num_kv_heads;
  p.max_blocks = a->max_blocks_per_seq; p.num_blocks = a->num_blocks;
  p.row_chunks = a->head_dim * esize / 16;
  p.k_row_chunks = a->head_dim * kesize / 16;
  p.q = static_cast<const uint4*>(a->q); p.k_cache = static_cast<const uint4*>(a->k_cache);
  p.block_table = a->block_table; p.seq_lens = a->seq_lens; p.cu_q_lens = a->cu_q_lens;
  p.P = a->num_probe_heads; p.probe_heads = a->probe_heads; p.NQ = a->max_sel_q; p.query_sel = a->query_sel;
  p.KH = a->num_capture_kv_heads; p.kv_heads = a->capture_kv_heads; p.cu_k_lens = a->cu_k_lens;
  p.total_k = a->total_k;
  p.q_out = static_cast<uint4*>(a->q_out); p.k_out = static_cast<uint4*>(a->k_out);
  hipStream_t st = static_cast<hipStream_t>(a->stream);
  // every check of both halves comes before the first launch: a rejected call writes nothing
  const bool do_q = p.P > 0, do_k = p.KH > 0 && p.total_k > 0;
  const long long chunks = (long long)p.num_seqs * p.P * p.NQ * p.row_chunks;
  if (do_q) {
    if (!a->q || !a->cu_q_lens || !a->probe_heads || !a->query_sel || !a->q_out) return HOOK_ERR_NULL;
    if (!grid_fits((chunks + 255) / 256)) return HOOK_ERR_UNSUPPORTED;
  }
  if (do_k) {
    if (!a->k_cache || !a->block_table || !a->seq_lens || !a->capture_kv_heads || !a->cu_k_lens || !a->k_out)
      return HOOK_ERR_NULL;
    if ((long long)kTokTile * p.KH * p.row_chunks > 0x7FFFFFFFll) return HOOK_ERR_UNSUPPORTED;
  }
  if (do_q) {
    hipLaunchKernelGGL(k_capture_q, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, p);
    if (hipGetLastError() != hipSuccess) return HOOK_ERR_LAUNCH;
  }
  if (do_k) {
    hipLaunchKernelGGL(k_capture_k, dim3((unsigned)((p.total_k + kTokTile - 1) / kTokTile)), dim3(256), 0, st, p);
    if (hipGetLastError() != hipSuccess) return HOOK_ERR_LAUNCH;
  }
  return HOOK_OK;
}
