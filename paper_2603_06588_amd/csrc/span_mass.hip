// Attention mass for MANY spans (one per document of a re-ranking prompt) on many query rows of
// a few heads: a probe-only pass that computes no attention output.  The attention call itself
// then runs with probing switched off.
//
// Workgroup = (sequence, probed head, block of 16 selected rows), 16 waves.
//   pass 1  the waves share the keys [0, pos_max] (64-key groups round-robin), each lane keeps a
//           running (max, sum) for its row over the keys it sees; merged across lanes and waves
//           into the exact softmax maximum and normaliser of each row;
//   pass 2  the spans are dealt to the waves; a wave walks the keys of its span, recomputes the
//           scores, sums exp2(s - max) per row and writes sum / normaliser.
// Every (row, span) value is produced by one wave in a fixed order: no atomics, reproducible,
// spans may overlap or be empty.  Scores are bf16 x bf16 products accumulated in fp32 on the
// matrix cores (16x16x32: 16 keys x 16 rows per instruction), exponentials and sums fp32.
#include "../../include/hook_api.h"
#include "hook_device.h"

#include <cmath>

namespace hook {
namespace {

constexpr int kSmWaves = 16;
constexpr int kSmRows = 16;     // query rows per workgroup
constexpr int kSmGroup = 4;     // 16-key tiles fetched together (independent loads in flight)

struct SpanParams {
  int num_seqs, total_q, Hq, Hkv, G, max_blocks, num_blocks;
  float scale_log2;
  const void* q;
  const void* k_cache;
  const int* block_table;
  const int* seq_lens;
  const int* cu_q_lens;
  int P;
  const int* probe_heads;
  int NQ;
  const int* query_sel;
  int S;
  const int* key_spans;
  float* mass;
};

template <int D>
struct Frag {
  static constexpr int KSTEPS = D / 32;
  uint4 k[KSTEPS];
};

// K rows of 16 keys as the A operand: lane (key slot l % 16, quarter l / 16) takes the 16-byte
// chunks 4 s + quarter of its key's row.  `key` is this lane's absolute key (already clamped
// into the sequence), looked up through the block table.
template <int D>
__device__ __forceinline__ void load_keys(const SpanParams& p, const int* bt, int g, int key, int quarter,
                                          Frag<D>& f) {
  int blk = bt[key >> 4];
  blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
  const uint4* row = static_cast<const uint4*>(p.k_cache) +
                     (((size_t)blk * p.Hkv + g) * kBlock + (key & 15)) * (D / 8);
#pragma unroll
  for (int s = 0; s < Frag<D>::KSTEPS; ++s) f.k[s] = row[4 * s + quarter];
}

template <int D>
__device__ __forceinline__ f32x4 scores(const Frag<D>& f, const bf16x8 (&qf)[D / 32]) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < D / 32; ++s) {
    bf16x8 a;
    __builtin_memcpy(&a, &f.k[s], 16);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[s], acc, 0, 0, 0);
  }
  return acc;
}

template <int D>
__global__ __launch_bounds__(kSmWaves * 64) void k_span_mass(const SpanParams p) {
  __shared__ float sh_m[kSmWaves][kSmRows];
  __shared__ float sh_l[kSmWaves][kSmRows];

  const int i = blockIdx.z, ps = blockIdx.y, rb = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, quarter = lane >> 4;

  const int Lraw = p.seq_lens[i];
  const int row0 = p.cu_q_lens[i];
  const int n = p.cu_q_lens[i + 1] - row0;
  const int L = min(Lraw, p.max_blocks * kBlock);
  if (Lraw < 0 || n <= 0 || n > L || row0 < 0 || row0 + n > p.total_q) return;   // uniform
  const int h = p.probe_heads[ps];
  if ((unsigned)h >= (unsigned)p.Hq) return;
  const int g = h / p.G;
  const int qb = p.query_sel[2 * i];
  const int qe = min(min(p.query_sel[2 * i + 1], n), qb + p.NQ);
  const int slot0 = kSmRows * rb;                 // first mass slot of this block
  const int t_lo = max(qb + slot0, 0), t_hi = min(qb + slot0 + kSmRows, qe);   // valid rows [t_lo, t_hi)
  if (t_hi <= t_lo) return;
  const int t_mine = qb + slot0 + j;
  const bool row_ok = t_mine >= t_lo && t_mine < t_hi;
  const int t = min(max(t_mine, t_lo), t_hi - 1);  // lanes without a row shadow a valid one
  const int pos = L - n + t;
  const int pos_max = L - n + t_hi - 1;

  const int* bt = p.block_table + (size_t)i * p.max_blocks;
  bf16x8 qf[D / 32];
  {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.q) +
                                                        ((size_t)(row0 + t) * p.Hq + h) * D);
#pragma unroll
    for (int s = 0; s < D / 32; ++s) qf[s] = qp[4 * s + quarter];
  }
  const float c = p.scale_log2;

  // ---- pass 1: row maximum and normaliser
  float m = -INFINITY, l = 0.0f;
  const int ntile = pos_max / 16 + 1;
  for (int b0 = wave * kSmGroup; b0 < ntile; b0 += kSmWaves * kSmGroup) {
    Frag<D> f[kSmGroup];
#pragma unroll
    for (int u = 0; u < kSmGroup; ++u) {
      const int key = min(16 * (b0 + u) + j, pos_max);
      load_keys<D>(p, bt, g, key, quarter, f[u]);
    }
#pragma unroll
    for (int u = 0; u < kSmGroup; ++u) {
      if (b0 + u >= ntile) continue;               // uniform
      const f32x4 s4 = scores<D>(f[u], qf);
      float sv[4];
      float mt = -INFINITY;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int key = 16 * (b0 + u) + 4 * quarter + r;
        sv[r] = key <= pos ? s4[r] * c : -INFINITY;
        mt = fmaxf(mt, sv[r]);
      }
      if (mt > m) {
        l *= fast_exp2(m - mt);                     // m = -inf gives 0 * l with l = 0
        m = mt;
      }
      if (m != -INFINITY) {
#pragma unroll
        for (int r = 0; r < 4; ++r) l += fast_exp2(sv[r] - m);
      }
    }
  }
  // merge the four quarters of a row, then the waves
#pragma unroll
  for (int off = 16; off <= 32; off <<= 1) {
    const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
    const float mn = fmaxf(m, mo);
    if (mn != -INFINITY) l = l * fast_exp2(m - mn) + lo * fast_exp2(mo - mn);
    m = mn;
  }
  if (quarter == 0) { sh_m[wave][j] = m; sh_l[wave][j] = l; }
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < kSmWaves; ++w) M = fmaxf(M, sh_m[w][j]);
  float Lsum = 0.0f;
#pragma unroll
  for (int w = 0; w < kSmWaves; ++w) {
    const float mw = sh_m[w][j];
    if (mw != -INFINITY) Lsum += sh_l[w][j] * fast_exp2(mw - M);
  }
  const float inv = 1.0f / Lsum;   // every valid row sees at least key 0, so Lsum >= 1 term

  // ---- pass 2: spans
  float* mrow = p.mass + (((size_t)i * p.P + ps) * p.NQ + (slot0 + j)) * p.S;
  for (int r = wave; r < p.S; r += kSmWaves) {
    const int a = max(p.key_spans[((size_t)i * p.S + r) * 2], 0);
    const int e = min(p.key_spans[((size_t)i * p.S + r) * 2 + 1], pos_max + 1);
    if (e <= a) continue;                          // uniform; mass was zero-filled
    float acc = 0.0f;
    for (int k0 = a; k0 < e; k0 += 16 * kSmGroup) {
      Frag<D> f[kSmGroup];
#pragma unroll
      for (int u = 0; u < kSmGroup; ++u) {
        const int key = min(k0 + 16 * u + j, pos_max);
        load_keys<D>(p, bt, g, key, quarter, f[u]);
      }
#pragma unroll
      for (int u = 0; u < kSmGroup; ++u) {
        if (k0 + 16 * u >= e) continue;            // uniform
        const f32x4 s4 = scores<D>(f[u], qf);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int key = k0 + 16 * u + 4 * quarter + rr;
          if (key < e && key <= pos) acc += fast_exp2(s4[rr] * c - M);
        }
      }
    }
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (quarter == 0 && row_ok) mrow[r] = acc * inv;
  }
}

__global__ __launch_bounds__(256) void k_zero_mass(float* ptr, size_t n) {
  for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < n; x += (size_t)gridDim.x * 256) ptr[x] = 0.0f;
}

}  // namespace
}  // namespace hook

extern "C" hook_status hook_span_mass(const hook_attn_probe_args* a) {
  using namespace hook;
  if (!a) return HOOK_ERR_NULL;
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 ||
      a->max_blocks_per_seq <= 0 || a->num_blocks <= 0 || a->head_dim <= 0)
    return HOOK_ERR_SHAPE;
  if (a->num_q_heads % a->num_kv_heads != 0) return HOOK_ERR_SHAPE;
  if (a->block_size != HOOK_BLOCK_SIZE || a->dtype != HOOK_BF16 || (a->head_dim != 64 && a->head_dim != 128))
    return HOOK_ERR_UNSUPPORTED;
  if (a->max_blocks_per_seq > (1 << 26)) return HOOK_ERR_UNSUPPORTED;
  const int P = a->num_probe_heads;
  if (P < 1 || P > a->num_q_heads || a->max_sel_q < 1 || a->max_spans < 1) return HOOK_ERR_SHAPE;
  if (a->max_sel_q > HOOK_MAX_SEL_Q || a->max_spans > HOOK_MAX_SPANS_WIDE) return HOOK_ERR_UNSUPPORTED;
  if (a->num_seqs > 65535 || P > 65535) return HOOK_ERR_UNSUPPORTED;
  if (!a->probe_heads || !a->query_sel || !a->key_spans || !a->mass) return HOOK_ERR_NULL;
  if (a->num_seqs == 0) return HOOK_OK;
  if (!a->q || !a->k_cache || !a->block_table || !a->seq_lens || !a->cu_q_lens) return HOOK_ERR_NULL;

  SpanParams p{};
  p.num_seqs = a->num_seqs; p.total_q = a->total_q; p.Hq = a->num_q_heads; p.Hkv = a->num_kv_heads;
  p.G = p.Hq / p.Hkv; p.max_blocks = a->max_blocks_per_seq; p.num_blocks = a->num_blocks;
  const float scale = a->scale > 0.0f ? a->scale : 1.0f / std::sqrt((float)a->head_dim);
  p.scale_log2 = scale * 1.44269504088896340736f;
  p.q = a->q; p.k_cache = a->k_cache; p.block_table = a->block_table; p.seq_lens = a->seq_lens;
  p.cu_q_lens = a->cu_q_lens; p.P = P; p.probe_heads = a->probe_heads; p.NQ = a->max_sel_q;
  p.query_sel = a->query_sel; p.S = a->max_spans; p.key_spans = a->key_spans; p.mass = a->mass;
  hipStream_t st = static_cast<hipStream_t>(a->stream);

  const size_t nmass = (size_t)p.num_seqs * p.P * p.NQ * p.S;
  size_t zb = (nmass + 2047) / 2048;
  if (zb > 2048) zb = 2048;
  hipLaunchKernelGGL(k_zero_mass, dim3((unsigned)zb), dim3(256), 0, st, p.mass, nmass);
  if (hipGetLastError() != hipSuccess) return HOOK_ERR_LAUNCH;
  const dim3 grid((unsigned)((p.NQ + kSmRows - 1) / kSmRows), (unsigned)P, (unsigned)p.num_seqs);
  if (a->head_dim == 128) hipLaunchKernelGGL(k_span_mass<128>, grid, dim3(kSmWaves * 64), 0, st, p);
  else hipLaunchKernelGGL(k_span_mass<64>, grid, dim3(kSmWaves * 64), 0, st, p);
  return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}
