// Attention mass for MANY spans (one per document of a re-ranking prompt) on many query rows of
// a few heads: a probe-only pass that computes no attention output.  The attention call itself
// then runs with probing switched off.
//
// Workgroup of the single-kernel form = (sequence, probed head, block of 16 selected rows), 16 waves.
//   pass 1  the waves share the keys [0, pos_max] (32-key groups round-robin), each lane keeps a
//           running (max, sum) for its row over the keys it sees; merged across lanes and waves
//           into the exact softmax maximum and normaliser of each row;
//   pass 2  the spans are dealt to the waves; a wave walks the keys of its span, recomputes the
//           scores, sums exp2(s - max) per row and writes sum / normaliser.
// Every (row, span) value is produced by one wave in a fixed order: no atomics, reproducible,
// spans may overlap or be empty.  Scores are bf16 x bf16 products accumulated in fp32 on the
// matrix cores (16x16x32: 16 keys x 16 rows per instruction), exponentials and sums fp32.
#include "../../include/hook_api.h"
#include "fp8_device.h"
#include "hook_device.h"

#include <cmath>

namespace hook {
namespace {

constexpr int kSmWaves = 16;
constexpr int kSmRows = 16;     // query rows per workgroup
constexpr int kSmGroup = 2;     // 16-key tiles per pipeline stage

struct SpanParams {
  int num_seqs, total_q, Hq, Hkv, G, max_blocks, num_blocks;
  float scale_log2;
  const float* k_scale;   // 8-bit cache: one fp32 scale per kv head, folded into the softmax scale
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
  float2* stats;    // split path: (max, sum) of every (sequence, probed head, row slot, key split)
  int nsplit;       // key splits of pass 1
  int sgroups;      // span groups of pass 2
  int nq_pad;       // NQ rounded up to whole 16-row blocks
};

template <int D>
struct Frag {
  static constexpr int KSTEPS = D / 32;
  uint4 k[KSTEPS];
};

// K rows of 16 keys as the A operand: lane (key slot l % 16, quarter l / 16) takes the 16-byte
// chunks 4 s + quarter of its key's row.  `key` is this lane's absolute key (already clamped
// into the sequence), looked up through the block table.
// With an 8-bit cache (KV8) the same eight dimensions are eight bytes, widened to bf16 after the load.
template <int D, bool KV8>
__device__ __forceinline__ void load_keys(const SpanParams& p, int blk, int g, int key, int quarter, Frag<D>& f) {
  blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
  const size_t row_index = ((size_t)blk * p.Hkv + g) * kBlock + (key & 15);
  if constexpr (KV8) {
    const uint2* row = static_cast<const uint2*>(p.k_cache) + row_index * (D / 8);
#pragma unroll
    for (int s = 0; s < Frag<D>::KSTEPS; ++s) f.k[s] = e4m3x8_to_bf16x8(row[4 * s + quarter]);
  } else {
    const uint4* row = static_cast<const uint4*>(p.k_cache) + row_index * (D / 8);
#pragma unroll
    for (int s = 0; s < Frag<D>::KSTEPS; ++s) f.k[s] = row[4 * s + quarter];
  }
}

template <int D>
__device__ __forceinline__ f32x4 scores(const Frag<D>& f, const bf16x8 (&qf)[D / 32]);

// A stream of key groups (kSmGroup tiles of 16 keys; group n starts at key first + n * step) run
// as a three-stage pipeline per wave: block ids two groups ahead, K rows one group ahead,
// arithmetic on the current group - so neither load latency sits on the critical path.
// `use(tile_first_key, scores[NB])` is called for every tile whose first key is below `end`; NB blocks
// of 16 query rows share every K fetch.
template <int D, int NB, bool KV8, typename F>
__device__ __forceinline__ void stream_keys(const SpanParams& p, const int* bt, int g, int j, int quarter,
                                            const bf16x8 (&qf)[NB][D / 32], int first, int step, int end, int pos_max,
                                            F&& use) {
  auto lane_key = [&](int base, int u) { return min(base + 16 * u + j, pos_max); };
  auto ids = [&](int base, int (&id)[kSmGroup]) {
#pragma unroll
    for (int u = 0; u < kSmGroup; ++u) id[u] = bt[lane_key(base, u) >> 4];
  };
  auto rows = [&](int base, const int (&id)[kSmGroup], Frag<D> (&f)[kSmGroup]) {
#pragma unroll
    for (int u = 0; u < kSmGroup; ++u) load_keys<D, KV8>(p, id[u], g, lane_key(base, u), quarter, f[u]);
  };
  auto work = [&](int base, const Frag<D> (&f)[kSmGroup]) {
#pragma unroll
    for (int u = 0; u < kSmGroup; ++u)
      if (base + 16 * u < end) {   // uniform
        f32x4 sc[NB];              // one K fetch serves the NB blocks of 16 rows
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sc[nb] = scores<D>(f[u], qf[nb]);
        use(base + 16 * u, sc);
      }
  };
  if (first >= end) return;
  // Every load below is issued unconditionally - keys are clamped into the sequence, so reading a
  // group past `end` is harmless - because the compiler can only keep loads in flight across a
  // wait when their number does not depend on the path taken.
  int idA[kSmGroup], idB[kSmGroup];
  Frag<D> fA[kSmGroup], fB[kSmGroup];
  ids(first, idA);
  rows(first, idA, fA);
  ids(first + step, idB);
  for (int base = first; base < end; base += 2 * step) {
    // fA holds (or awaits) the rows of `base`, idB the ids of base + step.  Loads return in issue
    // order, so ids are requested BEFORE the rows of the group in front of them: waiting for ids
    // then never drains rows issued after them.
    int idC[kSmGroup];
    ids(base + 2 * step, idC);
    rows(base + step, idB, fB);
    work(base, fA);
    ids(base + 3 * step, idB);
    rows(base + 2 * step, idC, fA);
    work(base + step, fB);
  }
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

template <int D, bool KV8>
__global__ __launch_bounds__(kSmWaves * 64) void k_span_mass(const SpanParams p) {
  __shared__ float sh_m[kSmWaves][kSmRows];
  __shared__ float sh_l[kSmWaves][kSmRows];

  const int i = blockIdx.z, ps = blockIdx.y, rb = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps the key loops scalar
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
  bf16x8 qf[1][D / 32];
  {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.q) +
                                                        ((size_t)(row0 + t) * p.Hq + h) * D);
#pragma unroll
    for (int s = 0; s < D / 32; ++s) qf[0][s] = qp[4 * s + quarter];
  }
  const float c = KV8 ? p.scale_log2 * p.k_scale[g] : p.scale_log2;

  // ---- pass 1: row maximum and normaliser
  float m = -INFINITY, l = 0.0f;
  const int ntile = pos_max / 16 + 1;
  stream_keys<D, 1, KV8>(p, bt, g, j, quarter, qf, 16 * kSmGroup * wave, 16 * kSmGroup * kSmWaves, 16 * ntile, pos_max,
                    [&](int key0, const f32x4 (&sc)[1]) {
    const f32x4 s4 = sc[0];
    float sv[4];
    float mt = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int key = key0 + 4 * quarter + r;
      sv[r] = key <= pos ? s4[r] * c : -INFINITY;
      mt = fmaxf(mt, sv[r]);
    }
    // branch-free update (a divergent branch between the loads would make the compiler wait for
    // every load in flight): with everything masked so far the reference is 0 and all terms vanish
    const float mn = fmaxf(m, mt);
    const float ref = (mn == -INFINITY) ? 0.0f : mn;
    l *= fast_exp2(m - ref);                        // m = -inf: l is 0 and stays 0
#pragma unroll
    for (int r = 0; r < 4; ++r) l += fast_exp2(sv[r] - ref);
    m = mn;
  });
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
    stream_keys<D, 1, KV8>(p, bt, g, j, quarter, qf, a, 16 * kSmGroup, e, pos_max, [&](int key0, const f32x4 (&sc)[1]) {
      const f32x4 s4 = sc[0];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int key = key0 + 4 * quarter + rr;
        acc += (key < e && key <= pos) ? fast_exp2(s4[rr] * c - M) : 0.0f;
      }
    });
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (quarter == 0 && row_ok) mrow[r] = acc * inv;
  }
}

// ---- the same two passes as two kernels, for callers that provide scratch memory: a single
// workgroup per row block has to pull a long sequence's keys through one CU (about 100 us per
// 10 k keys and pass); here pass 1 is split over the keys and pass 2 over the spans, so the
// work spreads over the chip.

// What both kernels need to know about their row block; false if there is nothing to do.
struct RowBlock {
  int g, h, row0, pos, pos_max, slot0;
  bool row_ok;
};

__device__ __forceinline__ bool row_block(const SpanParams& p, int i, int ps, int rb, int j, RowBlock& r) {
  const int Lraw = p.seq_lens[i];
  r.row0 = p.cu_q_lens[i];
  const int n = p.cu_q_lens[i + 1] - r.row0;
  const int L = min(Lraw, p.max_blocks * kBlock);
  if (Lraw < 0 || n <= 0 || n > L || r.row0 < 0 || r.row0 + n > p.total_q) return false;
  r.h = p.probe_heads[ps];
  if ((unsigned)r.h >= (unsigned)p.Hq) return false;
  r.g = r.h / p.G;
  const int qb = p.query_sel[2 * i];
  const int qe = min(min(p.query_sel[2 * i + 1], n), qb + p.NQ);
  r.slot0 = kSmRows * rb;
  const int t_lo = max(qb + r.slot0, 0), t_hi = min(qb + r.slot0 + kSmRows, qe);
  if (t_hi <= t_lo) return false;
  const int t_mine = qb + r.slot0 + j;
  r.row_ok = t_mine >= t_lo && t_mine < t_hi;
  const int t = min(max(t_mine, t_lo), t_hi - 1);
  r.pos = L - n + t;
  r.pos_max = L - n + t_hi - 1;
  r.row0 += t;      // global q row of this lane
  return true;
}

template <int D>
__device__ __forceinline__ void load_q(const SpanParams& p, const RowBlock& r, int quarter, bf16x8 (&qf)[D / 32]) {
  const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.q) + ((size_t)r.row0 * p.Hq + r.h) * D);
#pragma unroll
  for (int s = 0; s < D / 32; ++s) qf[s] = qp[4 * s + quarter];
}

constexpr int kSplitWaves = 4;
constexpr int kSplitBlocks = 2;   // blocks of 16 rows per workgroup: they share every K fetch

// The kSplitBlocks row blocks of workgroup column `bx`.  A block without rows shadows a block that
// has some (same loads and arithmetic, nothing written); false if no block has rows.
__device__ __forceinline__ bool row_blocks(const SpanParams& p, int i, int ps, int bx, int j,
                                           RowBlock (&r)[kSplitBlocks], bool (&has)[kSplitBlocks], int& pos_max) {
  int good = -1;
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) {
    has[nb] = row_block(p, i, ps, kSplitBlocks * bx + nb, j, r[nb]);
    if (has[nb] && good < 0) good = nb;
  }
  if (good < 0) return false;
  pos_max = 0;
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) {
    if (!has[nb]) {
      r[nb] = r[good];
      r[nb].slot0 = kSmRows * (kSplitBlocks * bx + nb);
      r[nb].row_ok = false;
    }
    pos_max = max(pos_max, r[nb].pos_max);
  }
  return true;
}

template <int D, bool KV8>
__global__ __launch_bounds__(kSplitWaves * 64) void k_span_stats(const SpanParams p) {
  __shared__ float sh_m[kSplitWaves][kSplitBlocks][kSmRows];
  __shared__ float sh_l[kSplitWaves][kSplitBlocks][kSmRows];
  // every workgroup helps zero-filling mass (the second kernel writes only entries with a row and a span)
  {
    const size_t nmass = (size_t)p.num_seqs * p.P * p.NQ * p.S;
    const size_t nthreads = (size_t)gridDim.x * gridDim.y * gridDim.z * blockDim.x;
    const size_t me = (((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
    for (size_t x = me; x < nmass; x += nthreads) p.mass[x] = 0.0f;
  }
  const int i = blockIdx.z / p.nsplit, sp = blockIdx.z % p.nsplit, ps = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane & 15, quarter = lane >> 4;
  RowBlock r[kSplitBlocks];
  bool has[kSplitBlocks];
  int pos_max;
  if (!row_blocks(p, i, ps, blockIdx.x, j, r, has, pos_max)) return;   // uniform
  const int* bt = p.block_table + (size_t)i * p.max_blocks;
  bf16x8 qf[kSplitBlocks][D / 32];
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) load_q<D>(p, r[nb], quarter, qf[nb]);
  const float c = KV8 ? p.scale_log2 * p.k_scale[r[0].g] : p.scale_log2;
  const int ntile = pos_max / 16 + 1;
  const int per = (ntile + p.nsplit - 1) / p.nsplit;           // tiles per split
  const int lo = 16 * per * sp, hi = min(16 * per * (sp + 1), 16 * ntile);
  float m[kSplitBlocks], l[kSplitBlocks];
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) { m[nb] = -INFINITY; l[nb] = 0.0f; }
  stream_keys<D, kSplitBlocks, KV8>(p, bt, r[0].g, j, quarter, qf, lo + 16 * kSmGroup * wave, 16 * kSmGroup * kSplitWaves,
                               hi, pos_max, [&](int key0, const f32x4 (&sc)[kSplitBlocks]) {
#pragma unroll
    for (int nb = 0; nb < kSplitBlocks; ++nb) {
      float sv[4];
      float mt = -INFINITY;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int key = key0 + 4 * quarter + q;
        sv[q] = key <= r[nb].pos ? sc[nb][q] * c : -INFINITY;
        mt = fmaxf(mt, sv[q]);
      }
      const float mn = fmaxf(m[nb], mt);
      const float ref = (mn == -INFINITY) ? 0.0f : mn;
      l[nb] *= fast_exp2(m[nb] - ref);
#pragma unroll
      for (int q = 0; q < 4; ++q) l[nb] += fast_exp2(sv[q] - ref);
      m[nb] = mn;
    }
  });
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) {
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float mo = __shfl_xor(m[nb], off), lo2 = __shfl_xor(l[nb], off);
      const float mn = fmaxf(m[nb], mo);
      if (mn != -INFINITY) l[nb] = l[nb] * fast_exp2(m[nb] - mn) + lo2 * fast_exp2(mo - mn);
      m[nb] = mn;
    }
    if (quarter == 0) { sh_m[wave][nb][j] = m[nb]; sh_l[wave][nb][j] = l[nb]; }
  }
  __syncthreads();
  if (threadIdx.x < kSplitBlocks * kSmRows) {
    const int nb = threadIdx.x / kSmRows, jj = threadIdx.x % kSmRows;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kSplitWaves; ++w) M = fmaxf(M, sh_m[w][nb][jj]);
    float Ls = 0.0f;
#pragma unroll
    for (int w = 0; w < kSplitWaves; ++w) {
      const float mw = sh_m[w][nb][jj];
      if (mw != -INFINITY) Ls += sh_l[w][nb][jj] * fast_exp2(mw - M);
    }
    const int slot = kSmRows * (kSplitBlocks * blockIdx.x + nb) + jj;
    if (slot < p.nq_pad) p.stats[(((size_t)i * p.P + ps) * p.nq_pad + slot) * p.nsplit + sp] = make_float2(M, Ls);
  }
}

template <int D, bool KV8>
__global__ __launch_bounds__(kSplitWaves * 64) void k_span_sums(const SpanParams p) {
  const int i = blockIdx.z / p.sgroups, sg = blockIdx.z % p.sgroups, ps = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane & 15, quarter = lane >> 4;
  RowBlock r[kSplitBlocks];
  bool has[kSplitBlocks];
  int pos_max;
  if (!row_blocks(p, i, ps, blockIdx.x, j, r, has, pos_max)) return;   // uniform
  const int* bt = p.block_table + (size_t)i * p.max_blocks;
  bf16x8 qf[kSplitBlocks][D / 32];
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) load_q<D>(p, r[nb], quarter, qf[nb]);
  const float c = KV8 ? p.scale_log2 * p.k_scale[r[0].g] : p.scale_log2;
  // each row's softmax maximum and normaliser from the key splits of the first kernel
  float M[kSplitBlocks], inv[kSplitBlocks];
#pragma unroll
  for (int nb = 0; nb < kSplitBlocks; ++nb) {
    M[nb] = 0.0f;
    inv[nb] = 0.0f;
    if (has[nb]) {   // uniform; a shadow block has no statistics of its own and writes nothing
      const float2* st = p.stats + (((size_t)i * p.P + ps) * p.nq_pad + r[nb].slot0 + j) * p.nsplit;
      float mx = -INFINITY;
      for (int sp = 0; sp < p.nsplit; ++sp) mx = fmaxf(mx, st[sp].x);
      float Lsum = 0.0f;
      for (int sp = 0; sp < p.nsplit; ++sp) {
        const float2 v = st[sp];
        if (v.x != -INFINITY) Lsum += v.y * fast_exp2(v.x - mx);
      }
      M[nb] = mx;
      inv[nb] = 1.0f / Lsum;
    }
  }
  for (int s = sg * kSplitWaves + wave; s < p.S; s += p.sgroups * kSplitWaves) {
    const int a = max(p.key_spans[((size_t)i * p.S + s) * 2], 0);
    const int e = min(p.key_spans[((size_t)i * p.S + s) * 2 + 1], pos_max + 1);
    if (e <= a) continue;                          // uniform; mass was zero-filled
    float acc[kSplitBlocks];
#pragma unroll
    for (int nb = 0; nb < kSplitBlocks; ++nb) acc[nb] = 0.0f;
    stream_keys<D, kSplitBlocks, KV8>(p, bt, r[0].g, j, quarter, qf, a, 16 * kSmGroup, e, pos_max,
                                 [&](int key0, const f32x4 (&sc)[kSplitBlocks]) {
#pragma unroll
      for (int nb = 0; nb < kSplitBlocks; ++nb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int key = key0 + 4 * quarter + q;
          acc[nb] += (key < e && key <= r[nb].pos) ? fast_exp2(sc[nb][q] * c - M[nb]) : 0.0f;
        }
    });
#pragma unroll
    for (int nb = 0; nb < kSplitBlocks; ++nb) {
      float v = acc[nb];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      if (quarter == 0 && r[nb].row_ok)
        p.mass[(((size_t)i * p.P + ps) * p.NQ + (r[nb].slot0 + j)) * p.S + s] = v * inv[nb];
    }
  }
}

// geometry of the split path from host scalars only
struct SplitGeom { int nsplit, sgroups, nq_pad; size_t bytes; bool usable; };

inline SplitGeom split_geometry(const hook_attn_probe_args* a) {
  SplitGeom g{};
  const long long max_ctx = (long long)a->max_blocks_per_seq * kBlock;
  g.nsplit = (int)((max_ctx + 2047) / 2048);
  if (g.nsplit < 1) g.nsplit = 1;
  if (g.nsplit > 16) g.nsplit = 16;
  g.sgroups = (a->max_spans + 2 * kSplitWaves - 1) / (2 * kSplitWaves);
  if (g.sgroups < 1) g.sgroups = 1;
  if (g.sgroups > 32) g.sgroups = 32;
  g.nq_pad = (a->max_sel_q + kSmRows - 1) / kSmRows * kSmRows;
  g.bytes = (size_t)a->num_seqs * a->num_probe_heads * g.nq_pad * g.nsplit * sizeof(float2);
  g.usable = (long long)a->num_seqs * g.nsplit <= 65535 && (long long)a->num_seqs * g.sgroups <= 65535;
  return g;
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
  if (a->kv_dtype != HOOK_KV_SAME && a->kv_dtype != HOOK_KV_FP8_E4M3) return HOOK_ERR_SHAPE;
  const bool kv8 = a->kv_dtype == HOOK_KV_FP8_E4M3;
  if (kv8 && !a->k_scale) return HOOK_ERR_NULL;

  SpanParams p{};
  p.k_scale = a->k_scale;
  p.num_seqs = a->num_seqs; p.total_q = a->total_q; p.Hq = a->num_q_heads; p.Hkv = a->num_kv_heads;
  p.G = p.Hq / p.Hkv; p.max_blocks = a->max_blocks_per_seq; p.num_blocks = a->num_blocks;
  const float scale = a->scale > 0.0f ? a->scale : 1.0f / std::sqrt((float)a->head_dim);
  p.scale_log2 = scale * 1.44269504088896340736f;
  p.q = a->q; p.k_cache = a->k_cache; p.block_table = a->block_table; p.seq_lens = a->seq_lens;
  p.cu_q_lens = a->cu_q_lens; p.P = P; p.probe_heads = a->probe_heads; p.NQ = a->max_sel_q;
  p.query_sel = a->query_sel; p.S = a->max_spans; p.key_spans = a->key_spans; p.mass = a->mass;
  hipStream_t st = static_cast<hipStream_t>(a->stream);

  // with enough scratch memory: pass 1 split over the keys, pass 2 over the spans
  const SplitGeom geo = split_geometry(a);
  if (geo.usable && a->workspace && a->workspace_bytes >= geo.bytes &&
      (reinterpret_cast<uintptr_t>(a->workspace) % 8) == 0) {
    p.stats = static_cast<float2*>(a->workspace);
    p.nsplit = geo.nsplit; p.sgroups = geo.sgroups; p.nq_pad = geo.nq_pad;
    const unsigned gx = (unsigned)((geo.nq_pad / kSmRows + kSplitBlocks - 1) / kSplitBlocks);
    const dim3 ga(gx, (unsigned)P, (unsigned)(p.num_seqs * geo.nsplit)), gb(gx, (unsigned)P, (unsigned)(p.num_seqs * geo.sgroups));
    const dim3 tb(kSplitWaves * 64);
    if (a->head_dim == 128 && !kv8) {
      hipLaunchKernelGGL((k_span_stats<128, false>), ga, tb, 0, st, p);
      hipLaunchKernelGGL((k_span_sums<128, false>), gb, tb, 0, st, p);
    } else if (a->head_dim == 128) {
      hipLaunchKernelGGL((k_span_stats<128, true>), ga, tb, 0, st, p);
      hipLaunchKernelGGL((k_span_sums<128, true>), gb, tb, 0, st, p);
    } else if (!kv8) {
      hipLaunchKernelGGL((k_span_stats<64, false>), ga, tb, 0, st, p);
      hipLaunchKernelGGL((k_span_sums<64, false>), gb, tb, 0, st, p);
    } else {
      hipLaunchKernelGGL((k_span_stats<64, true>), ga, tb, 0, st, p);
      hipLaunchKernelGGL((k_span_sums<64, true>), gb, tb, 0, st, p);
    }
    return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
  }

  const size_t nmass = (size_t)p.num_seqs * p.P * p.NQ * p.S;
  size_t zb = (nmass + 2047) / 2048;
  if (zb > 2048) zb = 2048;
  hipLaunchKernelGGL(k_zero_mass, dim3((unsigned)zb), dim3(256), 0, st, p.mass, nmass);
  if (hipGetLastError() != hipSuccess) return HOOK_ERR_LAUNCH;
  const dim3 grid((unsigned)((p.NQ + kSmRows - 1) / kSmRows), (unsigned)P, (unsigned)p.num_seqs);
  const dim3 tb(kSmWaves * 64);
  if (a->head_dim == 128 && !kv8) hipLaunchKernelGGL((k_span_mass<128, false>), grid, tb, 0, st, p);
  else if (a->head_dim == 128) hipLaunchKernelGGL((k_span_mass<128, true>), grid, tb, 0, st, p);
  else if (!kv8) hipLaunchKernelGGL((k_span_mass<64, false>), grid, tb, 0, st, p);
  else hipLaunchKernelGGL((k_span_mass<64, true>), grid, tb, 0, st, p);
  return hipGetLastError() == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}

extern "C" size_t hook_span_mass_workspace_bytes(const hook_attn_probe_args* a) {
  if (!a || a->num_seqs <= 0 || a->num_probe_heads <= 0 || a->max_sel_q <= 0 || a->max_spans <= 0 ||
      a->max_blocks_per_seq <= 0)
    return 0;
  const hook::SplitGeom g = hook::split_geometry(a);
  return g.usable ? g.bytes : 0;
}
