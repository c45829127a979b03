// Tiled causal attention for query chunks (n_i >= 2), head_dim 128, bf16 MFMA.
//
// Workgroup = 4 waves = (hpw q heads of one kv head) x (4 / hpw blocks of 32 query rows),
// all sharing the K/V tiles of their kv head.  Data movement is built around two gfx950
// features:
//   * K and V tiles (64 keys x 256 B) go from the paged cache straight into LDS with
//     16-byte direct-to-LDS loads, one uniform cache block per instruction, so staging costs
//     no vector registers and almost no vector ALU work.  16-byte chunks are XOR-swizzled
//     inside each 256-byte row (K by key & 15, V by 4 * (key & 3)) so that the MFMA operand
//     reads below are free of bank conflicts although rows are unpadded;
//   * V stays in its natural [key][dim] layout and is read TRANSPOSED with
//     ds_read_b64_tr_b16, which hands each lane four consecutive keys of one output
//     dimension - the A operand of O^T = V^T P^T.
//
// Per wave the score tile is computed transposed, S^T = K Q^T (32x32x16 MFMA, keys = M,
// queries = N): lane l owns query l % 32 and 16 keys per 32-key block, so softmax row
// statistics are in-lane reductions plus one exchange between lane halves, and the
// exponentials, rounded to bf16, already form the B operand of the second MFMA.
//
// The loop is software pipelined inside each wave: while the vector ALUs run the softmax
// of tile t, the matrix cores compute the scores of tile t+1 (the two instruction streams
// are interleaved explicitly), then P V of tile t follows.  K tiles are fetched two tiles
// ahead and V tiles one tile ahead, which makes one workgroup barrier per tile sufficient
// with two LDS buffers each.
//
// Probe span sums are taken from the fp32 exponentials under the same running reference
// as the normaliser and divided by it at the end: the captured mass is the exact softmax
// mass of the row.  Waves that probe run a second instantiation of the same loop whose
// arithmetic for `out` is identical.
#include "hook_device.h"

namespace hook {

namespace {

constexpr int D = 128;
constexpr int kRowBytes = 2 * D;                   // one key row in LDS
constexpr int kTileBytes = kTileKeys * kRowBytes;  // 16 KB
constexpr int kLdsBytes = 4 * kTileBytes;          // K[2] + V[2]

typedef short v4i16 __attribute__((ext_vector_type(4)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

struct WaveCtx {
  // loop-invariant per-lane / per-wave values
  unsigned k_read_addr;   // LDS byte offset of this lane's K row with its swizzle term folded in
  unsigned v_read_addr;   // same for the transposed V reads
  int hf, qi;
  int pos;                // causal horizon of this lane's query row
  float c;                // scale * log2(e)
  int S;                  // number of spans
};

// ---- one pipelined iteration --------------------------------------------------------------
// Scur holds the raw scores of tile kt.  Computes (if NEXT) the scores of tile kt+1 into Snext,
// the softmax update of tile kt and O += P V.
template <bool MASK, bool NEXT, bool PROBE>
__device__ __forceinline__ void tile_iter(const WaveCtx& cx, const unsigned char* smem, int kt,
                                          f32x16 (&Scur)[2], f32x16 (&Snext)[2], const bf16x8 (&qf)[8],
                                          f32x16 (&O)[4], float& m_run, float& l_run, float (&am)[kMaxSpans],
                                          const int (&sp_a)[kMaxSpans], const int (&sp_b)[kMaxSpans]) {
  const int key0 = kt * kTileKeys;
  const unsigned char* kb = smem + ((kt + 1) & 1) * kTileBytes;             // K of tile kt+1
  const unsigned char* vb = smem + 2 * kTileBytes + (kt & 1) * kTileBytes;  // V of tile kt

  // -- stage 1: mask and row maximum of the current tile
  if constexpr (MASK) {
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 32 * kbk + 8 * (r >> 2) + 4 * cx.hf + (r & 3);
        if (key > cx.pos) Scur[kbk][r] = -INFINITY;
      }
  }
  float mx = Scur[0][0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, Scur[0][r]);
#pragma unroll
  for (int r = 0; r < 16; ++r) mx = fmaxf(mx, Scur[1][r]);
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float mt = mx * cx.c;
  const bool upd = mt > m_run + kLazyTau;
  if (__builtin_amdgcn_ballot_w64(upd) != 0) {
    const float alpha = upd ? fast_exp2(m_run - mt) : 1.0f;
    m_run = upd ? mt : m_run;
    l_run *= alpha;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
#pragma unroll
    for (int s = 0; s < kMaxSpans; ++s) am[s] *= alpha;
  }
  const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;

  // -- stage 2: exponentials of tile kt on the vector ALUs, scores of tile kt+1 on the matrix cores
  if constexpr (NEXT) {
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) Snext[kbk][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const unsigned a = cx.k_read_addr ^ (32u * s);
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(kb + a);
      const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(kb + a + 32 * kRowBytes);
      Snext[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[s], Snext[0], 0, 0, 0);
      Snext[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[s], Snext[1], 0, 0, 0);
    }
  }
  float tsum = 0.0f;
#pragma unroll
  for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float e = fast_exp2(__builtin_fmaf(Scur[kbk][r], cx.c, -m_safe));
      Scur[kbk][r] = e;
      tsum += e;
    }
  l_run += tsum;
  union PB { uint32_t u[4]; bf16x8 v; } pb[4];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      pb[m].u[e] = pack_bf16(Scur[m >> 1][8 * (m & 1) + 2 * e], Scur[m >> 1][8 * (m & 1) + 2 * e + 1]);
  if constexpr (NEXT) {
    // interleave: one MFMA, its two LDS reads, a slice of the vector work
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // DS read
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);  // VALU
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  if constexpr (PROBE) {
#pragma unroll
    for (int s = 0; s < kMaxSpans; ++s) {
      if (s < cx.S) {
        const int a = sp_a[s], b = sp_b[s];
        if (b > key0 && a < key0 + kTileKeys) {
          if (a <= key0 && b >= key0 + kTileKeys) {
            am[s] += tsum;  // whole tile inside the span; masked keys contributed 0
          } else {
            float acc = 0.0f;
#pragma unroll
            for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int key = key0 + 32 * kbk + 8 * (r >> 2) + 4 * cx.hf + (r & 3);
                acc += (key >= a && key < b) ? Scur[kbk][r] : 0.0f;
              }
            am[s] += acc;
          }
        }
      }
    }
  }

  // -- stage 3: O^T += V^T P^T, V read transposed from its natural layout
#pragma unroll
  for (int m = 0; m < 4; ++m) {
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      const unsigned a = (cx.v_read_addr ^ (64u * mb)) + (16 * m) * kRowBytes;
      union { v4i16 h[2]; bf16x8 v; } av;
      av.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(vb + a));
      av.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) v4i16*)(vb + a + 8 * kRowBytes));
      O[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av.v, pb[m].v, O[mb], 0, 0, 0);
    }
  }
}

template <bool PROBE>
__device__ __forceinline__ void run_tiles(const WaveCtx& cx, const unsigned char* smem, int ntiles, int n_nomask,
                                          const bf16x8 (&qf)[8], f32x16 (&O)[4], float& m_run, float& l_run,
                                          float (&am)[kMaxSpans], const int (&sp_a)[kMaxSpans],
                                          const int (&sp_b)[kMaxSpans], const int* bt, int last_blk,
                                          const char* kbase, const char* vbase, size_t blk_bytes, int num_blocks,
                                          unsigned k_goff, unsigned v_goff, int L, int w, int lane,
                                          unsigned char* smem_w) {
  // block ids of up to 64 consecutive blocks (16 tiles) live in one register per lane
  int grp = 0;
  int btv0 = bt[min(lane, last_blk)];
  int btv1 = bt[min(64 + lane, last_blk)];

  auto block_id = [&](int bidx) -> int {   // bidx uniform, already clamped to last_blk
    const int g = bidx >> 6;
    const int v = (g == grp) ? btv0 : btv1;
    int blk = __builtin_amdgcn_readlane(v, bidx & 63);
    return ((unsigned)blk < (unsigned)num_blocks) ? blk : 0;
  };
  // direct-to-LDS load of one tile (4 blocks of 16 keys): wave w fills rows 4w..4w+3 of each block
  auto issue = [&](int tile, const char* gbase, unsigned goff, unsigned char* lds_tile) {
    const int key0 = tile * kTileKeys;
    if (__builtin_expect(key0 + kTileKeys <= L, 1)) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int blk = block_id(4 * tile + j);
        const char* src = gbase + (size_t)blk * blk_bytes;
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src + goff), LDS_PTR(lds_tile + (16 * j + 4 * w) * kRowBytes),
                                         16, 0, 0);
      }
    } else {
      // the tile reaches past the last token: rows beyond it re-read the last valid row of
      // the last block - finite data that the causal mask hides and that P = 0 multiplies -
      // never the stale tail of a block or a block the sequence does not own
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int bidx = min(4 * tile + j, last_blk);
        const int blk = block_id(bidx);
        const char* src = gbase + (size_t)blk * blk_bytes;
        const int r = 4 * w + (lane >> 4);
        const int rmax = L - 1 - 16 * bidx;              // >= 0 because bidx <= last_blk
        const unsigned off = goff - (unsigned)(r - min(r, rmax)) * kRowBytes;
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src + off), LDS_PTR(lds_tile + (16 * j + 4 * w) * kRowBytes),
                                         16, 0, 0);
      }
    }
  };
  unsigned char* const Kbuf = smem_w;
  unsigned char* const Vbuf = smem_w + 2 * kTileBytes;

  f32x16 S0[2], S1[2];

  issue(0, kbase, k_goff, Kbuf);
  issue(0, vbase, v_goff, Vbuf);
  if (ntiles > 1) issue(1, kbase, k_goff, Kbuf + kTileBytes);
  wait_vmem();
  __syncthreads();
  // scores of tile 0
#pragma unroll
  for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
    for (int r = 0; r < 16; ++r) S0[kbk][r] = 0.0f;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const unsigned a = cx.k_read_addr ^ (32u * s);
    const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(smem + a);
    const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(smem + a + 32 * kRowBytes);
    S0[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[s], S0[0], 0, 0, 0);
    S0[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[s], S0[1], 0, 0, 0);
  }

  auto top = [&](int kt) {
    wait_vmem();
    __syncthreads();
    // rotate the block-id registers when the K prefetch (two tiles ahead) enters a new group
    if (((kt + 2) >> 4) > grp + 1) {
      grp += 1;
      btv0 = btv1;
      btv1 = bt[min(64 * (grp + 1) + lane, last_blk)];
    }
    if (kt + 2 < ntiles) issue(kt + 2, kbase, k_goff, Kbuf + (kt & 1) * kTileBytes);
    if (kt + 1 < ntiles) issue(kt + 1, vbase, v_goff, Vbuf + ((kt + 1) & 1) * kTileBytes);
  };

  int kt = 0;
  const int end_nomask = min(n_nomask, ntiles - 1);
  // unmasked tiles, two per trip so the score registers ping-pong without copies
  while (kt + 2 <= end_nomask) {
    top(kt);
    tile_iter<false, true, PROBE>(cx, smem, kt, S0, S1, qf, O, m_run, l_run, am, sp_a, sp_b);
    top(kt + 1);
    tile_iter<false, true, PROBE>(cx, smem, kt + 1, S1, S0, qf, O, m_run, l_run, am, sp_a, sp_b);
    kt += 2;
  }
  if (kt < end_nomask) {
    top(kt);
    tile_iter<false, true, PROBE>(cx, smem, kt, S0, S1, qf, O, m_run, l_run, am, sp_a, sp_b);
    S0[0] = S1[0]; S0[1] = S1[1];
    kt += 1;
  }
  // masked tiles that still have a successor
  while (kt < ntiles - 1) {
    top(kt);
    tile_iter<true, true, PROBE>(cx, smem, kt, S0, S1, qf, O, m_run, l_run, am, sp_a, sp_b);
    S0[0] = S1[0]; S0[1] = S1[1];
    kt += 1;
  }
  // last tile
  top(kt);
  tile_iter<true, false, PROBE>(cx, smem, kt, S0, S1, qf, O, m_run, l_run, am, sp_a, sp_b);
}

__global__ __launch_bounds__(256, 2) void k_prefill128(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int bid = blockIdx.x;
  const int kvh = bid % p.Hkv;
  const int rest = bid / p.Hkv;
  const int hg = rest % p.hgroups;
  const int item = rest / p.hgroups;
  if (item >= p.hdr->n_prefill) return;
  const WorkItem it = p.pf_items[item];
  const int seq = it.x, row0 = it.y, L = it.z, n = it.w;
  const int qbase = p.cu_q_lens[seq];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hh = w % p.hpw, rb = w / p.hpw;
  const int head = kvh * p.G + hg * p.hpw + hh;
  const int wrow0 = row0 + rb * kWaveRows;
  const bool wave_active = wrow0 < n;
  const int qi = lane & 31, hf = lane >> 5;
  const int t = max(min(wrow0 + qi, n - 1), 0);
  const int wave_pos_min = L - n + min(wrow0, n - 1);
  const int wg_pos_max = L - n + min(row0 + p.rows_per_wg, n) - 1;
  const int ntiles = wg_pos_max / kTileKeys + 1;
  const int n_nomask = (wave_pos_min + 1) / kTileKeys;   // tiles whose last key is within every row's horizon

  WaveCtx cx;
  cx.hf = hf;
  cx.qi = qi;
  cx.pos = L - n + t;
  cx.c = p.scale_log2;
  cx.S = p.S;
  // K reads: lane (row qi [+32], half hf) reads logical chunk 2s + hf, stored at chunk ^ (row & 15)
  cx.k_read_addr = (unsigned)qi * kRowBytes | ((unsigned)((hf ^ (qi & 15)) & 15) << 4);
  {
    // transposed V reads: within a 16-lane group lane s supplies row (s >> 2) and 8-byte piece (s & 3)
    const int g = lane >> 4, s16 = lane & 15;
    const int hfv = g >> 1, ddhalf = g & 1;
    const unsigned rowc = (unsigned)(4 * hfv + (s16 >> 2)) * kRowBytes;
    const unsigned lowc = (unsigned)(2 * ddhalf + ((s16 & 3) >> 1)) * 16 + (unsigned)(s16 & 1) * 8;
    const unsigned xorc = (unsigned)(s16 >> 2) * 64;
    cx.v_read_addr = rowc | lowc | xorc;
  }

  const __bf16* const qg = static_cast<const __bf16*>(p.q);
  const int* const bt = p.block_table + (size_t)seq * p.max_blocks;
  const size_t blk_bytes = (size_t)p.Hkv * kBlock * D * 2;
  const char* const kbase = static_cast<const char*>(p.k_cache) + (size_t)kvh * kBlock * D * 2;
  const char* const vbase = static_cast<const char*>(p.v_cache) + (size_t)kvh * kBlock * D * 2;
  const int last_blk = (L - 1) >> 4;

  // per-lane source offsets of the direct-to-LDS loads: LDS slot (row r, physical chunk pc)
  // receives logical chunk pc ^ swizzle(r)
  const int r = 4 * w + (lane >> 4), pc = lane & 15;
  const unsigned k_goff = (unsigned)r * kRowBytes + (unsigned)(pc ^ (r & 15)) * 16;
  const unsigned v_goff = (unsigned)r * kRowBytes + (unsigned)(pc ^ ((r & 3) << 2)) * 16;

  bf16x8 qf[8];
  {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(qg + ((size_t)(qbase + t) * p.Hq + head) * D + 8 * hf);
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = qp[2 * s];
  }

  int pslot = -1, qsel_b = 0, qsel_e = 0;
  int sp_a[kMaxSpans], sp_b[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) { sp_a[s] = 0; sp_b[s] = 0; }
  if (p.P > 0) {
    pslot = find_probe_slot(p.probe_heads, p.P, head);
    qsel_b = p.query_sel[2 * seq];
    qsel_e = min(p.query_sel[2 * seq + 1], qsel_b + p.NQ);
#pragma unroll
    for (int s = 0; s < kMaxSpans; ++s)
      if (s < p.S) {
        sp_a[s] = max(p.key_spans[((size_t)seq * p.S + s) * 2], 0);
        sp_b[s] = p.key_spans[((size_t)seq * p.S + s) * 2 + 1];
      }
  }
  const bool wave_probe = wave_active && pslot >= 0 && qsel_b < min(wrow0 + kWaveRows, n) && qsel_e > wrow0;

  f32x16 O[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int rr = 0; rr < 16; ++rr) O[mb][rr] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  float am[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) am[s] = 0.0f;

  if (wave_probe)
    run_tiles<true>(cx, smem, ntiles, n_nomask, qf, O, m_run, l_run, am, sp_a, sp_b, bt, last_blk, kbase, vbase,
                    blk_bytes, p.num_blocks, k_goff, v_goff, L, w, lane, smem);
  else
    run_tiles<false>(cx, smem, ntiles, n_nomask, qf, O, m_run, l_run, am, sp_a, sp_b, bt, last_blk, kbase, vbase,
                     blk_bytes, p.num_blocks, k_goff, v_goff, L, w, lane, smem);

  // epilogue: normalise, transpose through LDS (K buffers, 16-byte chunks swizzled by row), coalesced stores
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  __syncthreads();
  unsigned char* const ot = smem + w * (kWaveRows * kRowBytes);
  if (wave_active) {
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        uint2 v;
        v.x = pack_bf16(O[mb][4 * g4] * inv, O[mb][4 * g4 + 1] * inv);
        v.y = pack_bf16(O[mb][4 * g4 + 2] * inv, O[mb][4 * g4 + 3] * inv);
        const int ch = 4 * mb + g4;
        *reinterpret_cast<uint2*>(ot + qi * kRowBytes + ((ch ^ (qi & 15)) << 4) + 8 * hf) = v;
      }
  }
  __syncthreads();
  if (wave_active) {
    __bf16* const og = static_cast<__bf16*>(p.out);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int rr = (lane >> 4) + 4 * j;
      const int ch = lane & 15;
      const int tr = wrow0 + rr;
      if (tr < n) {
        const uint4 v = *reinterpret_cast<const uint4*>(ot + rr * kRowBytes + ((ch ^ (rr & 15)) << 4));
        *reinterpret_cast<uint4*>(og + ((size_t)(qbase + tr) * p.Hq + head) * D + 8 * ch) = v;
      }
    }
    if (wave_probe) {
#pragma unroll
      for (int s = 0; s < kMaxSpans; ++s) {
        if (s < p.S) {
          const float a_tot = am[s] + __shfl_xor(am[s], 32);
          const int tr = wrow0 + qi;
          if (hf == 0 && tr < n && tr >= qsel_b && tr < qsel_e)
            p.mass[(((size_t)seq * p.P + pslot) * p.NQ + (tr - qsel_b)) * p.S + s] = a_tot * inv;
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_prefill128(const AttnParams& p, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_prefill128),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const long long grid = (long long)p.pf_cap * p.Hkv * p.hgroups;
  if (grid <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_prefill128, dim3((unsigned)grid), dim3(256), kLdsBytes, st, p);
  return hipGetLastError();
}

}  // namespace hook
