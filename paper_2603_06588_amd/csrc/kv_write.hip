// Scatter of the new tokens' K and V rows into the paged cache (stand-alone launch; the attention
// call can do the same inside its planning launch).  A workgroup takes 8 consecutive rows of
// k_new / v_new; the tile code is in kv_write_device.h.
#include "../../include/hook_api.h"
#include "kv_write_device.h"

namespace hook {
namespace {

__global__ __launch_bounds__(256) void k_kv_write(const KvWriteParams p) {
  __shared__ long long dst_row[kKvRowTile];   // blk * Hkv * kBlock + slot, or -1: do not write
  kv_write_tile<256>(p, blockIdx.x, threadIdx.x, dst_row);
}

}  // namespace

hipError_t launch_kv_write(const KvWriteParams& p, hipStream_t st) {
  if (p.total_q <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_kv_write, dim3((unsigned)((p.total_q + kKvRowTile - 1) / kKvRowTile)), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace hook

extern "C" hook_status hook_kv_write(const hook_kv_write_args* a) {
  using namespace hook;
  if (!a) return HOOK_ERR_NULL;
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_kv_heads <= 0 || a->head_dim <= 0 || a->max_blocks_per_seq <= 0 ||
      a->num_blocks <= 0)
    return HOOK_ERR_SHAPE;
  if (a->block_size != HOOK_BLOCK_SIZE) return HOOK_ERR_UNSUPPORTED;
  if (a->dtype != HOOK_BF16 && a->dtype != HOOK_F32) return HOOK_ERR_UNSUPPORTED;
  if (a->kv_dtype != HOOK_KV_SAME && a->kv_dtype != HOOK_KV_FP8_E4M3) return HOOK_ERR_SHAPE;
  const bool kv8 = a->kv_dtype == HOOK_KV_FP8_E4M3;
  if (kv8 && a->dtype != HOOK_BF16) return HOOK_ERR_UNSUPPORTED;
  const int esize = a->dtype == HOOK_BF16 ? 2 : 4;
  if ((a->head_dim * esize) % 16 != 0 || a->max_blocks_per_seq > (1 << 26)) return HOOK_ERR_UNSUPPORTED;
  if (a->num_seqs == 0 || a->total_q == 0) return HOOK_OK;
  if (!a->k_new || !a->v_new || !a->block_table || !a->seq_lens || !a->cu_q_lens || !a->k_cache || !a->v_cache)
    return HOOK_ERR_NULL;
  if (kv8 && (!a->k_scale || !a->v_scale)) return HOOK_ERR_NULL;
  KvWriteParams p{};
  p.kv8 = kv8 ? 1 : 0; p.k_scale = a->k_scale; p.v_scale = a->v_scale;
  p.num_seqs = a->num_seqs; p.total_q = a->total_q; p.Hkv = a->num_kv_heads; p.max_blocks = a->max_blocks_per_seq;
  p.num_blocks = a->num_blocks; p.row_chunks = a->head_dim * esize / 16;
  if ((long long)kKvRowTile * p.Hkv * p.row_chunks > 0x7FFFFFFFll) return HOOK_ERR_UNSUPPORTED;
  p.k_new = static_cast<const uint4*>(a->k_new); p.v_new = static_cast<const uint4*>(a->v_new);
  p.block_table = a->block_table; p.seq_lens = a->seq_lens; p.cu_q_lens = a->cu_q_lens;
  p.k_cache = a->k_cache; p.v_cache = a->v_cache;
  return launch_kv_write(p, static_cast<hipStream_t>(a->stream)) == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}
