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

// 16-byte direct-to-LDS load: lane i's data lands at lds + 16 * i.  Written as assembly so
// that its completion is tracked only by the explicit vmcnt wait at the top of each
// iteration; the compiler would otherwise make every later LDS read wait for the load.
__device__ __forceinline__ void dma16(const void* base, unsigned voff, const void* lds) {
  const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) const void*)lds;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}

// The same load with its address arithmetic folded in: m0 is written first, and the two scalar
// adds that form the global address (base + 64-bit block offset) fill the wait state that an m0
// write needs before the load that uses it.
__device__ __forceinline__ void dma16_at(unsigned base_lo, unsigned base_hi, unsigned off_lo, unsigned off_hi,
                                         unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\t"
               "s_add_u32 s98, %1, %3\n\t"
               "s_addc_u32 s99, %2, %4\n\t"
               "global_load_lds_dwordx4 %5, s[98:99]"
               :: "s"(lds_addr), "s"(base_lo), "s"(base_hi), "s"(off_lo), "s"(off_hi), "v"(voff)
               : "memory", "m0", "s98", "s99", "scc");
}

struct WaveCtx {
  // loop-invariant per-lane / per-wave values
  unsigned k_read_addr;   // LDS byte offset of this lane's K row with its swizzle term folded in
  unsigned v_read_addr;   // same for the transposed V reads
  int hf, qi;
  int pos;                // causal horizon of this lane's query row
  float c;                // scale * log2(e)
  int S;                  // number of spans
  // direct-to-LDS staging
  const char* kbase;      // k_cache + kv-head offset
  const char* vbase;
  unsigned kb_lo, kb_hi, vb_lo, vb_hi;   // the same two addresses as 32-bit halves
  unsigned lds_base;      // LDS address of the K/V buffers
  unsigned lds_row0;      // byte offset of this wave's first row inside a 16-key block of a tile
  unsigned blk_units;     // 256-byte units per cache block (all kv heads)
  unsigned blk_bytes;     // bytes per cache block (all kv heads)
  unsigned k_gchunk, v_gchunk;  // per-lane byte offset of the (swizzled) 16-byte chunk inside a row
  unsigned k_off;         // k_gchunk + this lane's row offset inside a block (loop invariant)
  unsigned v_row_off;     // this lane's row offset inside a block
  int L, last_blk, w, lane;
};

// lane l and lane l ^ 32 hold the two key halves of one query: maximum over both (one swap between
// the lane halves instead of a round trip through LDS)
__device__ __forceinline__ float half_max(float mx) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// mask (optional) and row maximum of a raw score tile; both lane halves end up with the same value
template <bool MASK>
__device__ __forceinline__ float tile_max(const WaveCtx& cx, int key0, f32x16 (&S)[2]) {
  if constexpr (MASK) {
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 32 * kbk + 8 * (r >> 2) + 4 * cx.hf + (r & 3);
        if (key > cx.pos) S[kbk][r] = -INFINITY;
      }
  }
  float m0 = fmaxf(S[0][0], S[0][1]), m1 = fmaxf(S[1][0], S[1][1]);
#pragma unroll
  for (int r = 2; r < 16; r += 2) {
    m0 = fmaxf(m0, fmaxf(S[0][r], S[0][r + 1]));
    m1 = fmaxf(m1, fmaxf(S[1][r], S[1][r + 1]));
  }
  return half_max(fmaxf(m0, m1));
}

// Block ids of 64 consecutive blocks (16 tiles) live in one register per lane; two registers
// cover the group being consumed and the next one.
struct BlockIds {
  int grp;
  int cur, nxt;
};

__device__ __forceinline__ int load_ids(const int* bt, int first, int lane, int last_blk, int num_blocks) {
  const int blk = bt[min(first + lane, last_blk)];
  return ((unsigned)blk < (unsigned)num_blocks) ? blk : 0;
}

// One direct-to-LDS load: block j of a K or V tile; wave w fills rows 4w..4w+3 of the block.
// Rows past the last token re-read the last valid row of the last block - finite data that
// the causal mask hides and that P = 0 multiplies - never the stale tail of a block or a
// block the sequence does not own.
//
// That row clamp is needed for V only (0 * NaN would poison the output).  A K row past the last
// token may hold anything: it only produces scores of keys beyond every row's horizon, and
// those are overwritten with -inf before use; the row still lies inside a block the sequence
// owns.  So K is fetched with a loop-invariant per-lane offset.
template <bool CLAMP_ROWS>
__device__ __forceinline__ void issue_block(const WaveCtx& cx, int tile, int j, const char* gbase, unsigned gchunk,
                                            unsigned long long boff, unsigned char* lds_tile) {
  const int r = 4 * cx.w + (cx.lane >> 4);
  unsigned off;
  if constexpr (CLAMP_ROWS) {
    const int bidx = min(4 * tile + j, cx.last_blk);
    const int rmax = cx.L - 1 - 16 * bidx;             // >= 0 because bidx <= last_blk
    off = gchunk + ((unsigned)min(r, rmax) << 8);
  } else {
    off = gchunk + ((unsigned)r << 8);
  }
  dma16(gbase + boff, off, lds_tile + (16 * j + 4 * cx.w) * kRowBytes);
}

__device__ __forceinline__ unsigned long long block_offset(const WaveCtx& cx, int sel, int tile, int j) {
  const int bidx = min(4 * tile + j, cx.last_blk);      // same 64-block group as block 4 * tile
  const unsigned blk = (unsigned)__builtin_amdgcn_readlane(sel, bidx & 63);
  return (unsigned long long)blk * cx.blk_bytes;
}

__device__ __forceinline__ bf16x8 read_k(const WaveCtx& cx, const unsigned char* kb, int s, int kbk) {
  const unsigned a = cx.k_read_addr ^ (32u * s);
  return *reinterpret_cast<const bf16x8*>(kb + a + kbk * 32 * kRowBytes);
}

__device__ __forceinline__ bf16x8 read_vt(const WaveCtx& cx, const unsigned char* vb, int m, int mb) {
  const unsigned a = (cx.v_read_addr ^ (64u * mb)) + (16 * m) * kRowBytes;
  union { v4i16 h[2]; bf16x8 v; } av;
  av.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(vb + a));
  av.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) v4i16*)(vb + a + 8 * kRowBytes));
  return av.v;
}

__device__ __forceinline__ void qk_tile(const WaveCtx& cx, const unsigned char* kb, const bf16x8 (&qf)[8],
                                        f32x16 (&S)[2]) {
#pragma unroll
  for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
    for (int r = 0; r < 16; ++r) S[kbk][r] = 0.0f;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_k(cx, kb, s, 0), qf[s], S[0], 0, 0, 0);
    S[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_k(cx, kb, s, 1), qf[s], S[1], 0, 0, 0);
  }
}

// ---- one pipelined iteration --------------------------------------------------------------
// On entry Scur holds the raw (already masked) scores of tile kt and mx_cur their row maximum.
//   stage B  raise the running reference if needed (rare);
//   stage C  exponentials of tile kt on the vector ALUs while the matrix cores compute the
//            scores of tile kt+1 into Snext (8 slices: 2 MFMAs + 4 exponentials each);
//   stage D  O += P V of tile kt on the matrix cores while the scalar/vector units issue the
//            direct-to-LDS loads of V(kt+1) and K(kt+2) and reduce the row maximum of tile
//            kt+1 (16 slices: 1 MFMA + one piece of the other work each); V^T operands are
//            requested two MFMAs ahead of their use (the first two during stage C).
// The slices are fenced so the instruction streams stay interleaved as written.  Loads are
// issued unconditionally with the tile index clamped to the last tile: the buffers they land
// in are free by then and are never read again.
// Returns the row maximum of tile kt+1.
template <bool MASKNEXT, bool NEXT, bool PROBE>
__device__ __forceinline__ float tile_iter(const WaveCtx& cx, unsigned char* smem, int kt, int ntiles,
                                           BlockIds& ids, const int* bt, int num_blocks,
                                           unsigned long long (&boff_next)[4],
                                           f32x16 (&Scur)[2], float mx_cur, f32x16 (&Snext)[2],
                                           const bf16x8 (&qf)[8], f32x16 (&O)[4], float& m_run, float& l_run,
                                           float (&am)[kMaxSpans], const int (&sp_a)[kMaxSpans],
                                           const int (&sp_b)[kMaxSpans]) {
  const int key0 = kt * kTileKeys;
  unsigned char* const Kbuf = smem;
  unsigned char* const Vbuf = smem + 2 * kTileBytes;
  const unsigned char* kb = Kbuf + ((kt + 1) & 1) * kTileBytes;  // K of tile kt+1
  const unsigned char* vb = Vbuf + (kt & 1) * kTileBytes;        // V of tile kt

  // K(kt+1) and V(kt) were issued one iteration ago; after the barrier every wave has also
  // finished reading the buffers that the loads issued below will overwrite
  wait_vmem();
  __syncthreads();

  // -- stage B
  const float mt = mx_cur * cx.c;
  const bool upd = mt > m_run + kLazyTau;
  if (__builtin_amdgcn_ballot_w64(upd) != 0) {
    const float alpha = upd ? fast_exp2(m_run - mt) : 1.0f;
    m_run = upd ? mt : m_run;
    l_run *= alpha;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
    if constexpr (PROBE) {
#pragma unroll
      for (int s = 0; s < kMaxSpans; ++s) am[s] *= alpha;
    }
  }
  const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;
  // block-id registers: the K prefetch (two tiles ahead) may enter a new group of 64 blocks
  const int tk = min(kt + 2, ntiles - 1), tv = min(kt + 1, ntiles - 1);
  if ((tk >> 4) > ids.grp + 1) {
    ids.grp += 1;
    ids.cur = ids.nxt;
    ids.nxt = load_ids(bt, 64 * (ids.grp + 1), cx.lane, cx.last_blk, num_blocks);
  }
  const int sel = ((tk >> 4) == ids.grp) ? ids.cur : ids.nxt;
  __builtin_amdgcn_sched_barrier(0);

  // -- stage C
  float tsum = 0.0f;
  union PB { uint32_t u[4]; bf16x8 v; } pb[4];
  bf16x8 va[3];   // ring of V^T operands: requested two matrix instructions ahead of their use
  {
    bf16x8 ka[2][2];
    if constexpr (NEXT) {
      ka[0][0] = read_k(cx, kb, 0, 0);
      ka[0][1] = read_k(cx, kb, 0, 1);
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if constexpr (NEXT) {
        if (s < 7) {
          ka[(s + 1) & 1][0] = read_k(cx, kb, s + 1, 0);
          ka[(s + 1) & 1][1] = read_k(cx, kb, s + 1, 1);
          __builtin_amdgcn_sched_barrier(0);   // requested a whole slice before their use
        }
        if (s == 0) {
          const f32x16 z = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
          Snext[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0][0], qf[0], z, 0, 0, 0);
          Snext[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0][1], qf[0], z, 0, 0, 0);
        } else {
          Snext[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s & 1][0], qf[s], Snext[0], 0, 0, 0);
          Snext[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s & 1][1], qf[s], Snext[1], 0, 0, 0);
        }
      }
      // the first V^T operands of the P V stage are requested here, two slices before their use
      if (s == 6) va[0] = read_vt(cx, vb, 0, 0);
      if (s == 7) va[1] = read_vt(cx, vb, 0, 1);
      // exponentials of elements 4s .. 4s+3 of the current tile
      const int kbk = s >> 2, r0 = 4 * (s & 3);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float ex = fast_exp2(__builtin_fmaf(Scur[kbk][r0 + e], cx.c, -m_safe));
        Scur[kbk][r0 + e] = ex;
        tsum += ex;
      }
      const int m = 2 * kbk + ((s & 3) >> 1);
      pb[m].u[2 * (s & 1)] = pack_bf16(Scur[kbk][r0], Scur[kbk][r0 + 1]);
      pb[m].u[2 * (s & 1) + 1] = pack_bf16(Scur[kbk][r0 + 2], Scur[kbk][r0 + 3]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  l_run += tsum;

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
    __builtin_amdgcn_sched_barrier(0);
  }

  // -- stage D
  float mx_acc = -INFINITY;   // running maximum of the next tile's scores
  if constexpr (NEXT && MASKNEXT) {
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + kTileKeys + 32 * kbk + 8 * (r >> 2) + 4 * cx.hf + (r & 3);
        if (key > cx.pos) Snext[kbk][r] = -INFINITY;
      }
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_setprio(2);   // the matrix-core-bound stage wins issue arbitration over the other wave
  const unsigned lds_v = cx.lds_base + (2 + ((kt + 1) & 1)) * kTileBytes + cx.lds_row0;   // V(kt+1)
  const unsigned lds_k = cx.lds_base + (kt & 1) * kTileBytes + cx.lds_row0;               // K(kt+2)
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int m = i >> 2, mb = i & 3;
    if (i + 2 < 16) va[(i + 2) % 3] = read_vt(cx, vb, (i + 2) >> 2, (i + 2) & 3);
    __builtin_amdgcn_sched_barrier(0);
    O[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[i % 3], pb[m].v, O[mb], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (i < 8) {
      if constexpr (NEXT) {   // the last tile of an item has nothing left to fetch
        if (i < 4) {
          // V(kt+1): block offsets were computed when K(kt+1) was issued
          unsigned off = cx.v_gchunk + cx.v_row_off;
          if constexpr (MASKNEXT) {   // only a tile that needs the causal mask can reach past the last token
            const int bidx = min(4 * tv + i, cx.last_blk);
            const int rmax = cx.L - 1 - 16 * bidx;
            off = cx.v_gchunk + ((unsigned)min(4 * cx.w + (cx.lane >> 4), rmax) << 8);
          }
          dma16_at(cx.vb_lo, cx.vb_hi, (unsigned)boff_next[i], (unsigned)(boff_next[i] >> 32), off,
                   lds_v + 16 * i * kRowBytes);
        } else {
          const int j = i - 4;
          boff_next[j] = block_offset(cx, sel, tk, j);
          dma16_at(cx.kb_lo, cx.kb_hi, (unsigned)boff_next[j], (unsigned)(boff_next[j] >> 32), cx.k_off,
                   lds_k + 16 * j * kRowBytes);
        }
      }
    } else if constexpr (NEXT) {
      const int q = i - 8;   // scores 4q .. 4q+3 of the next tile
      const int kbk = q >> 2, r0 = 4 * (q & 3);
      // three-operand maxima written out (fmaxf() would first canonicalise every score with a v_max
      // of its own), both in one statement so that nothing is put between them
      asm volatile("v_max3_f32 %0, %0, %1, %2\n\tv_max3_f32 %0, %0, %3, %4"
                   : "+v"(mx_acc)
                   : "v"(Snext[kbk][r0]), "v"(Snext[kbk][r0 + 1]), "v"(Snext[kbk][r0 + 2]), "v"(Snext[kbk][r0 + 3]));
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_setprio(0);
  float mx_next = 0.0f;
  if constexpr (NEXT) {
    mx_next = half_max(mx_acc);
  }
  return mx_next;
}

template <bool PROBE>
__device__ __forceinline__ void run_tiles(const WaveCtx& cx, unsigned char* smem, int ntiles, int n_nomask,
                                          const bf16x8 (&qf)[8], f32x16 (&O)[4], float& m_run, float& l_run,
                                          float (&am)[kMaxSpans], const int (&sp_a)[kMaxSpans],
                                          const int (&sp_b)[kMaxSpans], const int* bt, int num_blocks) {
  BlockIds ids;
  ids.grp = 0;
  ids.cur = load_ids(bt, 0, cx.lane, cx.last_blk, num_blocks);
  ids.nxt = load_ids(bt, 64, cx.lane, cx.last_blk, num_blocks);
  unsigned char* const Kbuf = smem;
  unsigned char* const Vbuf = smem + 2 * kTileBytes;

  f32x16 S0[2], S1[2];
  unsigned long long boff[4];

  // prologue: K(0), V(0), K(1) in flight, then the scores of tile 0
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    boff[j] = block_offset(cx, ids.cur, 0, j);
    issue_block<false>(cx, 0, j, cx.kbase, cx.k_gchunk, boff[j], Kbuf);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) issue_block<true>(cx, 0, j, cx.vbase, cx.v_gchunk, boff[j], Vbuf);
  if (ntiles > 1) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      boff[j] = block_offset(cx, ids.cur, 1, j);
      issue_block<false>(cx, 1, j, cx.kbase, cx.k_gchunk, boff[j], Kbuf + kTileBytes);
    }
  }
  // only K(0) has to have landed for the first scores; V(0) and K(1) are waited for at the
  // top of the first iteration.  Loads complete in issue order, so it is enough to let the 8
  // (4 when there is no second tile) younger ones stay in flight.
  if (ntiles > 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  __syncthreads();
  qk_tile(cx, Kbuf, qf, S0);
  float mx = (n_nomask > 0) ? tile_max<false>(cx, 0, S0) : tile_max<true>(cx, 0, S0);

  // tile kt+1 needs no mask while kt+1 < n_nomask
  int kt = 0;
  const int end_nomask = min(n_nomask - 1, ntiles - 1);
  // two tiles per trip so the score registers ping-pong without copies
  while (kt + 2 <= end_nomask) {
    mx = tile_iter<false, true, PROBE>(cx, smem, kt, ntiles, ids, bt, num_blocks, boff, S0, mx, S1, qf, O, m_run,
                                       l_run, am, sp_a, sp_b);
    mx = tile_iter<false, true, PROBE>(cx, smem, kt + 1, ntiles, ids, bt, num_blocks, boff, S1, mx, S0, qf, O,
                                       m_run, l_run, am, sp_a, sp_b);
    kt += 2;
  }
  if (kt < end_nomask) {
    mx = tile_iter<false, true, PROBE>(cx, smem, kt, ntiles, ids, bt, num_blocks, boff, S0, mx, S1, qf, O, m_run,
                                       l_run, am, sp_a, sp_b);
    S0[0] = S1[0]; S0[1] = S1[1];
    kt += 1;
  }
  // tiles whose successor needs the causal mask
  while (kt < ntiles - 1) {
    mx = tile_iter<true, true, PROBE>(cx, smem, kt, ntiles, ids, bt, num_blocks, boff, S0, mx, S1, qf, O, m_run,
                                      l_run, am, sp_a, sp_b);
    S0[0] = S1[0]; S0[1] = S1[1];
    kt += 1;
  }
  // last tile
  (void)tile_iter<true, false, PROBE>(cx, smem, kt, ntiles, ids, bt, num_blocks, boff, S0, mx, S1, qf, O, m_run,
                                      l_run, am, sp_a, sp_b);
}

// One work item: rows [row0, row0 + rows_per_wg) of sequence `seq` (context L, n rows, first q row
// qbase) for the heads of (kvh, hg).  ZERO_REST (self-planned call only): the wave that owns a probed
// head in the item of row 0 also writes zeros to that head's `mass` slots that hold no row, so that
// every entry of `mass` is written exactly once without a planner's zero-fill.
template <bool ZERO_REST>
__device__ __forceinline__ void prefill128_item(const AttnParams& p, unsigned char* smem, int kvh, int hg, int seq,
                                                int row0, int L, int n, int qbase) {
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
  cx.blk_bytes = (unsigned)p.Hkv * kBlock * D * 2;
  cx.kbase = static_cast<const char*>(p.k_cache) + (size_t)kvh * kBlock * D * 2;
  cx.vbase = static_cast<const char*>(p.v_cache) + (size_t)kvh * kBlock * D * 2;
  cx.L = L;
  cx.last_blk = (L - 1) >> 4;
  cx.w = w;
  cx.lane = lane;

  // per-lane source offsets of the direct-to-LDS loads: LDS slot (row r, physical chunk pc)
  // receives logical chunk pc ^ swizzle(r)
  const int r = 4 * w + (lane >> 4), pc = lane & 15;
  cx.k_gchunk = (unsigned)(pc ^ (r & 15)) * 16;
  cx.v_gchunk = (unsigned)(pc ^ ((r & 3) << 2)) * 16;
  cx.k_off = cx.k_gchunk + ((unsigned)r << 8);
  cx.v_row_off = (unsigned)r << 8;
  cx.kb_lo = (unsigned)(size_t)cx.kbase; cx.kb_hi = (unsigned)((size_t)cx.kbase >> 32);
  cx.vb_lo = (unsigned)(size_t)cx.vbase; cx.vb_hi = (unsigned)((size_t)cx.vbase >> 32);
  cx.lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) const void*)smem;
  cx.lds_row0 = (unsigned)(4 * w) * kRowBytes;

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
    load_spans(p.key_spans, seq, p.S, sp_a, sp_b);
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
    run_tiles<true>(cx, smem, ntiles, n_nomask, qf, O, m_run, l_run, am, sp_a, sp_b, bt, p.num_blocks);
  else
    run_tiles<false>(cx, smem, ntiles, n_nomask, qf, O, m_run, l_run, am, sp_a, sp_b, bt, p.num_blocks);

  // epilogue: normalise, transpose through LDS (K buffers, 16-byte chunks swizzled by row), coalesced stores
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  wait_vmem();   // the clamped prefetches of the last iterations must have landed before LDS is reused
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
  if constexpr (ZERO_REST) {
    if (row0 == 0 && rb == 0 && pslot >= 0 && p.plan_fresh) {
      const int lo = max(qsel_b, 0), hi = min(qsel_e, n);     // slots lo - qsel_b .. hi - qsel_b - 1 hold rows
      for (int e = lane; e < p.NQ * p.S; e += 64) {
        const int tr = qsel_b + e / p.S;
        if (tr < lo || tr >= hi) p.mass[((size_t)seq * p.P + pslot) * p.NQ * p.S + e] = 0.0f;
      }
    }
  }
}

// PLANNED: the work item comes from the planner's list.  Otherwise the call holds ONE sequence and
// plans itself (no planning launch, which is a sixth of a 2048-token prompt's call): the row blocks are
// taken last block first (longest first), workgroup 0 writes the status word, and `mass` is written
// entry by entry by the waves that own the entries.  All stores sit behind the body, so that the loads
// of the batch description stay scalar loads.
template <bool PLANNED>
__global__ __launch_bounds__(256, 2) void k_prefill128(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int bid = blockIdx.x;
  const int kvh = bid % p.Hkv;
  const int rest = bid / p.Hkv;
  const int hg = rest % p.hgroups;
  const int item = rest / p.hgroups;
  if constexpr (PLANNED) {
    // the grid covers the whole item capacity, so both records can be fetched together with
    // the item count instead of after it
    const WorkItem it = p.pf_items[2 * item];
    const int qbase = p.pf_items[2 * item + 1].x;
    if (item >= p.hdr->n_prefill) return;
    prefill128_item<false>(p, smem, kvh, hg, it.x, it.y, it.z, it.w, qbase);
  } else {
    const int max_ctx = p.max_blocks * kBlock;
    const int Lraw = p.seq_lens[0], qbase = p.cu_q_lens[0], n = p.cu_q_lens[1] - qbase;
    const int L = min(Lraw, max_ctx);
    int status = 0;
    bool valid = false;
    if (Lraw < 0 || n < 0) status = kStatNegative;
    else {
      if (Lraw > max_ctx) status |= kStatLenClamped;
      if (n > L) status |= kStatQGtL;
      else if (qbase < 0 || qbase + n > p.total_q) status |= kStatNegative;
      else if (n == 1) status |= kStatHint;      // a single row in a call promised to hold chunks: dropped
      else valid = n >= 2;
    }
    const int nitems = valid ? (n + p.rows_per_wg - 1) / p.rows_per_wg : 0;
    if (item < nitems)
      prefill128_item<true>(p, smem, kvh, hg, 0, (nitems - 1 - item) * p.rows_per_wg, L, n, qbase);
    if (bid == 0) {
      if (threadIdx.x == 0) { p.hdr->n_prefill = nitems; p.hdr->n_decode = 0; p.hdr->chunk_keys = 0; p.hdr->status = status; }
      if (!valid && p.plan_fresh)     // nothing ran: every entry of `mass` is zero
        for (int e = threadIdx.x; e < p.P * p.NQ * p.S; e += 256) p.mass[e] = 0.0f;
    }
  }
}

}  // namespace

hipError_t launch_prefill128(const AttnParams& p, hipStream_t st) {
  static std::atomic<unsigned long long> configured{0}, configured_self{0};
  const long long grid = (long long)p.pf_cap * p.Hkv * p.hgroups;
  if (grid <= 0) return hipSuccess;
  if (!grid_fits(grid)) return hipErrorInvalidValue;
  if (p.pf_self) {
    const hipError_t e = raise_lds_limit_once(reinterpret_cast<const void*>(&k_prefill128<false>), kLdsBytes, configured_self);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_prefill128<false>, dim3((unsigned)grid), dim3(256), kLdsBytes, st, p);
    return hipGetLastError();
  }
  const hipError_t e = raise_lds_limit_once(reinterpret_cast<const void*>(&k_prefill128<true>), kLdsBytes, configured);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_prefill128<true>, dim3((unsigned)grid), dim3(256), kLdsBytes, st, p);
  return hipGetLastError();
}

}  // namespace hook
