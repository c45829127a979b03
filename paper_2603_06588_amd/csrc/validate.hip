// Debug check of the device-resident contents that hook_attn_probe can only make safe, not
// verify: lengths, prefix sums, block ids of the live context, the probed-head list and the
// row selection.  One workgroup walks everything (this is not a fast path) and leaves a bit
// mask in the workspace header, which the host reads back after synchronising.
#include "../../include/hook_api.h"
#include "hook_device.h"

namespace hook {
namespace {

constexpr int kValThreads = 1024;

__global__ __launch_bounds__(kValThreads) void k_validate(const AttnParams p) {
  __shared__ int sh_bits;
  const int tid = threadIdx.x;
  if (tid == 0) sh_bits = 0;
  __syncthreads();
  int bits = 0;
  const int max_ctx = p.max_blocks * kBlock;
  for (int i = tid; i < p.num_seqs; i += kValThreads) {
    const int L = p.seq_lens[i];
    const int r0 = p.cu_q_lens[i], r1 = p.cu_q_lens[i + 1];
    const int n = r1 - r0;
    if (L < 0 || n < 0 || r0 < 0 || r1 > p.total_q) bits |= HOOK_BAD_LENGTH;
    if (L > max_ctx) bits |= HOOK_BAD_CONTEXT_TOO_LONG;
    if (n > L) bits |= HOOK_BAD_ROWS_EXCEED_CONTEXT;
    if ((p.batch_kind == HOOK_BATCH_PREFILL_ONLY && n == 1) || (p.batch_kind == HOOK_BATCH_DECODE_ONLY && n > 1))
      bits |= HOOK_BAD_BATCH_KIND;
    if (p.P > 0) {
      const int qb = p.query_sel[2 * i], qe = p.query_sel[2 * i + 1];
      // a range may reach outside the chunk (it is clipped); what loses rows is the NQ cap
      if (min(qe, n) - max(qb, 0) > 0 && min(qe, n) - qb > p.NQ) bits |= HOOK_BAD_QUERY_SEL;
    }
  }
  if (tid == 0) {
    if (p.cu_q_lens[0] != 0 || p.cu_q_lens[p.num_seqs] != p.total_q) bits |= HOOK_BAD_LENGTH;
  }
  for (int k = tid; k < p.P; k += kValThreads) {
    const int h = p.probe_heads[k];
    if (h < 0 || h >= p.Hq || (k > 0 && p.probe_heads[k - 1] >= h)) bits |= HOOK_BAD_PROBE_HEADS;
  }
  // block ids of every live cache block (a wave per sequence, lanes over its blocks)
  const int wave = tid >> 6, lane = tid & 63;
  for (int i = wave; i < p.num_seqs; i += kValThreads / 64) {
    const int L = min(max(p.seq_lens[i], 0), max_ctx);
    const int nb = (L + kBlock - 1) / kBlock;
    const int* bt = p.block_table + (size_t)i * p.max_blocks;
    for (int b = lane; b < nb; b += 64)
      if ((unsigned)bt[b] >= (unsigned)p.num_blocks) bits |= HOOK_BAD_BLOCK_ID;
  }
  if (bits) atomicOr(&sh_bits, bits);
  __syncthreads();
  if (tid == 0) p.hdr->problems = sh_bits;
}

}  // namespace
}  // namespace hook

extern "C" hook_status hook_attn_probe_validate(const hook_attn_probe_args* a, int32_t* problem_bits) {
  using namespace hook;
  if (!a || !problem_bits) return HOOK_ERR_NULL;
  *problem_bits = 0;
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 ||
      a->max_blocks_per_seq <= 0 || a->num_blocks <= 0)
    return HOOK_ERR_SHAPE;
  if (a->max_blocks_per_seq > (1 << 26)) return HOOK_ERR_UNSUPPORTED;
  if (a->batch_kind < HOOK_BATCH_MIXED || a->batch_kind > HOOK_BATCH_DECODE_ONLY) return HOOK_ERR_SHAPE;
  const int P = a->num_probe_heads;
  if (P < 0) return HOOK_ERR_SHAPE;
  if (P > 0 && (!a->probe_heads || !a->query_sel)) return HOOK_ERR_NULL;
  if (!a->block_table || !a->seq_lens || !a->cu_q_lens) return HOOK_ERR_NULL;
  if (!a->workspace || a->workspace_bytes < sizeof(PlanHeader) ||
      (reinterpret_cast<uintptr_t>(a->workspace) % 256) != 0)
    return HOOK_ERR_WORKSPACE;
  AttnParams p{};
  p.num_seqs = a->num_seqs; p.total_q = a->total_q; p.Hq = a->num_q_heads; p.Hkv = a->num_kv_heads;
  p.max_blocks = a->max_blocks_per_seq; p.num_blocks = a->num_blocks;
  p.block_table = a->block_table; p.seq_lens = a->seq_lens; p.cu_q_lens = a->cu_q_lens;
  p.P = P; p.probe_heads = a->probe_heads; p.NQ = a->max_sel_q; p.query_sel = a->query_sel;
  p.batch_kind = a->batch_kind;
  p.hdr = static_cast<PlanHeader*>(a->workspace);
  hipStream_t st = static_cast<hipStream_t>(a->stream);
  hipLaunchKernelGGL(k_validate, dim3(1), dim3(kValThreads), 0, st, p);
  if (hipGetLastError() != hipSuccess) return HOOK_ERR_LAUNCH;
  PlanHeader h{};
  if (hipMemcpyAsync(&h, a->workspace, sizeof h, hipMemcpyDeviceToHost, st) != hipSuccess) return HOOK_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return HOOK_ERR_LAUNCH;
  *problem_bits = h.problems;
  return HOOK_OK;
}
