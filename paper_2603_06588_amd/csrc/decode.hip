// Split-key decode attention (one query row per sequence) and the kernel that merges the
// per-chunk partial results.
//
// The path is bound by HBM: every live K and V element of a kv head is read exactly once
// and shared by the HP query heads of its group.  A workgroup owns one (sequence, key chunk,
// kv head); each of its 4 waves streams a contiguous run of 16-key cache blocks straight
// from global memory into registers (16-byte loads, one block ahead):
//   - the K block is the A operand of S^T = K Q^T (16x16x32 bf16 MFMA, keys = M, heads = N),
//     whose accumulator gives lane (head j, key group kq) the scores of 4 keys;
//   - every (head, key group) lane runs its own online softmax over the keys it sees, so
//     the loop has no cross-lane reduction; exponentials are handed to the lanes that hold
//     the matching V rows with a lane shuffle, and P V is plain fp32 FMAs on V in its
//     natural layout;
//   - the key-group streams of a wave, the waves of a workgroup and finally the chunks of a
//     sequence are merged with the usual (max, sum) weights; probe span sums ride along with
//     the normaliser in every merge.
#include "hook_device.h"

namespace hook {

namespace {

template <int D>
struct DecodeCfg {
  static constexpr int KSTEPS = D / 32;        // MFMA k-steps
  static constexpr int CHV = D / 8;            // 16-byte chunks per V row
  static constexpr int VK = 64 / CHV;          // V key groups per block (lanes / chunks)
  static constexpr int KPL = kBlock / VK;      // keys per V lane per block (4 or 2)
  static constexpr int PSTR = D + kPartialPad; // floats per partial record
};

// 8-bit cache: two fp8 values of one 16-bit half of `w` as bf16 (exact: 3 mantissa bits)
__device__ __forceinline__ uint32_t fp8x2_to_bf16x2(uint32_t w, bool upper_half) {
  bf16x2 v;
  if (upper_half) v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);
  else v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
  uint32_t u;
  __builtin_memcpy(&u, &v, 4);
  return u;
}

// KV8: the caches hold 8-bit E4M3 bytes ([num_blocks, Hkv, 16, D] bytes), one fp32 scale per kv head.
// The key scale is folded into the softmax scale and the value scale into the partial output, so
// the loop differs from the 16-bit one only in its loads and conversions: a block is half as many
// bytes, so loads run two blocks ahead instead of one to keep as many bytes in flight.
// The keys [kstart, kend) of one sequence for one (kv head, head group): four waves split the cache
// blocks, merge in LDS and leave one partial record per head in slot `item`.
template <int D, int HP, bool KV8>
__device__ __forceinline__ void decode_range(const AttnParams& p, float (&red)[4][HP][DecodeCfg<D>::PSTR], int tid, int lane,
                                             int w, int kvh, int head0, int seq, int qrow, int kstart, int kend,
                                             int item) {
  using C = DecodeCfg<D>;
  constexpr int NW = 4;
  const int nblk = (kend - kstart + kBlock - 1) / kBlock;
  const int bpw = (nblk + NW - 1) / NW;
  const int b0 = min(w * bpw, nblk), b1 = min(b0 + bpw, nblk);

  const __bf16* const qg = static_cast<const __bf16*>(p.q);
  const __bf16* const kg_ = static_cast<const __bf16*>(p.k_cache);
  const __bf16* const vg_ = static_cast<const __bf16*>(p.v_cache);
  const unsigned char* const kg8 = static_cast<const unsigned char*>(p.k_cache);
  const unsigned char* const vg8 = static_cast<const unsigned char*>(p.v_cache);
  const int* const bt = p.block_table + (size_t)seq * p.max_blocks;
  const size_t blk_stride = (size_t)p.Hkv * kBlock * D;   // in elements (bytes for the 8-bit cache)
  const size_t head_off = (size_t)kvh * kBlock * D;

  // score-lane role: head j = lane % 16 (real if j < HP), key group kq = lane / 16
  const int j = lane & 15, kq = lane >> 4;
  // value-lane role: key group vk, 16-byte chunk ch; its keys KPL*vk .. KPL*vk+KPL-1 all
  // belong to score key group (KPL*vk)/4
  const int vk = lane / C::CHV, ch = lane % C::CHV;
  const int src_base = 16 * ((C::KPL * vk) >> 2);     // lane of head 0 in the matching score group

  bf16x8 qf[C::KSTEPS];
#pragma unroll
  for (int s = 0; s < C::KSTEPS; ++s) {
    uint4 v = make_uint4(0, 0, 0, 0);
    // the contraction may take the dimensions in any order as long as both operands agree: with the
    // 8-bit cache a lane's key bytes are the 16-byte piece (s / 2) of its row, so k-step s covers
    // dimensions 64 (s / 2) + 16 kq + 8 (s % 2) + 0..7 instead of 32 s + 8 kq + 0..7
    const int dim0 = KV8 ? 64 * (s >> 1) + 16 * kq + 8 * (s & 1) : 32 * s + 8 * kq;
    if (j < HP)
      v = *reinterpret_cast<const uint4*>(qg + ((size_t)qrow * p.Hq + head0 + j) * D + dim0);
    __builtin_memcpy(&qf[s], &v, 16);
  }

  // probe set-up: per score lane (its head), spans uniform
  int sp_a[kMaxSpans], sp_b[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) { sp_a[s] = 0; sp_b[s] = 0; }
  bool any_probe = false;
  bool lane_probe = false;
  if (p.P > 0) {
    // the single row t = 0 is selected when begin <= 0 < min(end, begin + NQ); its slot is -begin
    const int qb = p.query_sel[2 * seq], qe = min(p.query_sel[2 * seq + 1], qb + p.NQ);
    any_probe = (qb <= 0 && qe > 0);
    if (any_probe) {
      // is head0 + h probed?  The list is read 64 entries at a time, one per lane, and matched
      // with a ballot, so the answer costs one load instead of a search per head
      for (int i0 = 0; i0 < p.P; i0 += 64) {
        const int ph = (i0 + lane < p.P) ? p.probe_heads[i0 + lane] : -1;
#pragma unroll
        for (int h = 0; h < HP; ++h) {
          const bool hit = __builtin_amdgcn_ballot_w64(ph == head0 + h) != 0;
          if (j == h) lane_probe = lane_probe || hit;
        }
      }
      load_spans(p.key_spans, seq, p.S, sp_a, sp_b);
    }
  }

  float m_run = -INFINITY, l_run = 0.0f;
  float am[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) am[s] = 0.0f;
  float acc[HP][8];
#pragma unroll
  for (int h = 0; h < HP; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;
  const float c = KV8 ? p.scale_log2 * p.k_scale[kvh] : p.scale_log2;

  constexpr int kRing = KV8 ? 3 : 2;                       // blocks in registers
  constexpr int kKr = KV8 ? C::KSTEPS / 2 : C::KSTEPS;     // 16-byte K pieces per lane and block
  uint4 kr[kRing][kKr];
  uint4 vr[kRing][C::KPL];                                 // 8-bit cache: only .x, .y are used

  auto load_block = [&](int b, uint4 (&kd)[kKr], uint4 (&vd)[C::KPL]) {
    const int jb = (kstart >> 4) + b;                   // block index inside the sequence
    int blk = bt[jb];
    blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
    const int key_k = jb * kBlock + j;                  // this lane's key as a score-lane
    const bool ok_k = key_k < kend;
    if constexpr (KV8) {
      const unsigned char* kb = kg8 + (size_t)blk * blk_stride + head_off;
      const unsigned char* vb = vg8 + (size_t)blk * blk_stride + head_off;
#pragma unroll
      for (int h = 0; h < kKr; ++h) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ok_k) v = load_stream16(kb + (size_t)j * D + 64 * h + 16 * kq);
        kd[h] = v;
      }
#pragma unroll
      for (int i = 0; i < C::KPL; ++i) {
        const int kl = C::KPL * vk + i;
        uint2 v = make_uint2(0, 0);
        if (jb * kBlock + kl < kend) v = *reinterpret_cast<const uint2*>(vb + (size_t)kl * D + 8 * ch);
        vd[i] = make_uint4(v.x, v.y, 0, 0);
      }
    } else {
      const __bf16* kb = kg_ + (size_t)blk * blk_stride + head_off;
      const __bf16* vb = vg_ + (size_t)blk * blk_stride + head_off;
#pragma unroll
      for (int s = 0; s < C::KSTEPS; ++s) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ok_k) v = load_stream16(kb + (size_t)j * D + 32 * s + 8 * kq);
        kd[s] = v;
      }
#pragma unroll
      for (int i = 0; i < C::KPL; ++i) {
        const int kl = C::KPL * vk + i;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (jb * kBlock + kl < kend) v = load_stream16(vb + (size_t)kl * D + 8 * ch);
        vd[i] = v;
      }
    }
  };

  auto compute_block = [&](int b, const uint4 (&kd)[kKr], const uint4 (&vd)[C::KPL]) {
    const int key0 = kstart + b * kBlock;
    f32x4 sacc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s) {
      bf16x8 a;
      if constexpr (KV8) {
        // bytes 8 (s % 2) .. 8 (s % 2) + 7 of piece s / 2
        const uint32_t w0 = (s & 1) ? kd[s >> 1].z : kd[s >> 1].x;
        const uint32_t w1 = (s & 1) ? kd[s >> 1].w : kd[s >> 1].y;
        const uint4 cv = make_uint4(fp8x2_to_bf16x2(w0, false), fp8x2_to_bf16x2(w0, true),
                                    fp8x2_to_bf16x2(w1, false), fp8x2_to_bf16x2(w1, true));
        __builtin_memcpy(&a, &cv, 16);
      } else {
        __builtin_memcpy(&a, &kd[s], 16);
      }
      sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[s], sacc, 0, 0, 0);
    }
    // lane (j, kq): sacc[r] = score of head j with key key0 + 4 kq + r
    float tt[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      tt[r] = sacc[r] * c;
      if (key0 + 4 * kq + r >= kend) tt[r] = -INFINITY;
    }
    const float bm = fmaxf(fmaxf(tt[0], tt[1]), fmaxf(tt[2], tt[3]));
    const bool upd = bm > m_run + kLazyTau;
    if (__builtin_amdgcn_ballot_w64(upd) != 0) {
      const float alpha = upd ? fast_exp2(m_run - bm) : 1.0f;
      m_run = upd ? bm : m_run;
      l_run *= alpha;
#pragma unroll
      for (int s = 0; s < kMaxSpans; ++s) am[s] *= alpha;
#pragma unroll
      for (int h = 0; h < HP; ++h) {
        const float ah = __shfl(alpha, src_base + h);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] *= ah;
      }
    }
    const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;
    float pr[4];
    float psum = 0.0f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      pr[r] = fast_exp2(tt[r] - m_safe);
      psum += pr[r];
    }
    l_run += psum;
    if (any_probe) {
#pragma unroll
      for (int s = 0; s < kMaxSpans; ++s) {
        if (s < p.S) {
          const int a = sp_a[s], bnd = sp_b[s];
          if (bnd > key0 && a < key0 + kBlock) {
            float add = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int key = key0 + 4 * kq + r;
              add += (key >= a && key < bnd) ? pr[r] : 0.0f;
            }
            am[s] += lane_probe ? add : 0.0f;
          }
        }
      }
    }
    // P V on the value lanes
#pragma unroll
    for (int i = 0; i < C::KPL; ++i) {
      float vf[8];
      if constexpr (KV8) {
        const f32x2 a0 = __builtin_amdgcn_cvt_pk_f32_fp8(vd[i].x, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8(vd[i].x, true);
        const f32x2 a2 = __builtin_amdgcn_cvt_pk_f32_fp8(vd[i].y, false), a3 = __builtin_amdgcn_cvt_pk_f32_fp8(vd[i].y, true);
        vf[0] = a0[0]; vf[1] = a0[1]; vf[2] = a1[0]; vf[3] = a1[1];
        vf[4] = a2[0]; vf[5] = a2[1]; vf[6] = a3[0]; vf[7] = a3[1];
      } else {
        vf[0] = bf16_lo(vd[i].x); vf[1] = bf16_hi(vd[i].x);
        vf[2] = bf16_lo(vd[i].y); vf[3] = bf16_hi(vd[i].y);
        vf[4] = bf16_lo(vd[i].z); vf[5] = bf16_hi(vd[i].z);
        vf[6] = bf16_lo(vd[i].w); vf[7] = bf16_hi(vd[i].w);
      }
#pragma unroll
      for (int h = 0; h < HP; ++h) {
        float ph;
        if constexpr (C::KPL == 4) {
          ph = __shfl(pr[i], src_base + h);
        } else {
          const float lo = __shfl(pr[i], src_base + h);
          const float hi = __shfl(pr[2 + i], src_base + h);
          ph = (vk & 1) ? hi : lo;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = __builtin_fmaf(ph, vf[e], acc[h][e]);
      }
    }
  };

  if constexpr (KV8) {
    // stream this wave's blocks, two blocks of loads in flight ahead of the arithmetic
    if (b0 < b1) load_block(b0, kr[0], vr[0]);
    if (b0 + 1 < b1) load_block(b0 + 1, kr[1], vr[1]);
    for (int b = b0; b < b1; b += 3) {
      if (b + 2 < b1) load_block(b + 2, kr[2], vr[2]);
      compute_block(b, kr[0], vr[0]);
      if (b + 1 < b1) {
        if (b + 3 < b1) load_block(b + 3, kr[0], vr[0]);
        compute_block(b + 1, kr[1], vr[1]);
      }
      if (b + 2 < b1) {
        if (b + 4 < b1) load_block(b + 4, kr[1], vr[1]);
        compute_block(b + 2, kr[2], vr[2]);
      }
    }
  } else {
    // stream this wave's blocks, one block of loads in flight ahead of the arithmetic
    if (b0 < b1) load_block(b0, kr[0], vr[0]);
    for (int b = b0; b < b1; b += 2) {
      if (b + 1 < b1) load_block(b + 1, kr[1], vr[1]);
      compute_block(b, kr[0], vr[0]);
      if (b + 1 < b1) {
        if (b + 2 < b1) load_block(b + 2, kr[0], vr[0]);
        compute_block(b + 1, kr[1], vr[1]);
      }
    }
  }

  // merge the key-group streams of this wave
  float m_w = fmaxf(m_run, __shfl_xor(m_run, 16));
  m_w = fmaxf(m_w, __shfl_xor(m_w, 32));
  const float wgt = (m_run == -INFINITY) ? 0.0f : fast_exp2(m_run - m_w);
  float l_w = l_run * wgt;
  l_w += __shfl_xor(l_w, 16);
  l_w += __shfl_xor(l_w, 32);
  float am_w[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) {
    float v = am[s] * wgt;
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    am_w[s] = v;
  }
#pragma unroll
  for (int h = 0; h < HP; ++h) {
    const float wh = __shfl(wgt, src_base + h);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[h][e] * wh;
      if constexpr (C::VK == 8) v += __shfl_xor(v, 8);
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      acc[h][e] = v;
    }
  }
  // lanes with vk == 0 hold o[h][8 ch + e]; score lanes with kq == 0 hold (m, l, a) of head j
  if (vk == 0) {
#pragma unroll
    for (int h = 0; h < HP; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) red[w][h][8 * ch + e] = acc[h][e];
  }
  if (kq == 0 && j < HP) {
    red[w][j][D] = m_w;
    red[w][j][D + 1] = l_w;
#pragma unroll
    for (int s = 0; s < kMaxSpans; ++s) red[w][j][D + 2 + s] = am_w[s];
  }
  __syncthreads();

  // merge the 4 waves and write one partial record per head
  const float vscale = KV8 ? p.v_scale[kvh] : 1.0f;
  for (int idx = tid; idx < HP * C::PSTR; idx += 256) {
    const int h = idx / C::PSTR, col = idx % C::PSTR;
    float mm = red[0][h][D];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) mm = fmaxf(mm, red[ww][h][D]);
    float out = 0.0f;
    if (col == D) {
      out = mm;
    } else if (col < D + 2 + kMaxSpans) {
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) {
        const float mw = red[ww][h][D];
        const float e = (mw == -INFINITY) ? 0.0f : fast_exp2(mw - mm);
        out += e * red[ww][h][col];
      }
      if (KV8 && col < D) out *= vscale;
    }
    p.partials[((size_t)item * p.Hq + head0 + h) * C::PSTR + col] = out;
  }
}

// SELF: the variant for batches of few single rows, where the planning launch is a large part of
// the call.  Every sequence is cut into the same number of parts (p.dec_parts, chosen on the host so
// that the grid fills the chip and the records fit the workspace) and a workgroup works out its own
// part from the sequence length, so no planner runs: part 0 of a sequence also zero-fills the
// sequence's `mass` entries and tells the merge kernel how many records to expect, and workgroup 0
// writes the status word.
template <int D, int HP, bool KV8, bool SELF>
__global__ __launch_bounds__(256) void k_decode(const AttnParams p) {
  using C = DecodeCfg<D>;
  constexpr int NW = 4;
  __shared__ float red[NW][HP][C::PSTR];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bid = blockIdx.x;
  const int kvh = bid % p.Hkv;
  const int rest = bid / p.Hkv;
  const int hg = rest % p.dec_hgroups;
  const int turn = rest / p.dec_hgroups;
  const int head0 = kvh * p.G + hg * HP;
  int seq, L, qrow, kstart, kend, item;
  bool active = true;
  // what this workgroup owes besides its part (SELF only; stores, so kept behind every load of the
  // batch description: a store ahead of them would turn those scalar loads into vector loads)
  bool owes_seq = false;      // zero-fill the sequence's `mass` entries of its heads, announce the record count
  int n_records = 0;
  auto settle = [&]() {
    if constexpr (SELF) {
      if (owes_seq) {
        // (a reusing call keeps its promise of writing selected rows only; the merge kernel fills
        // the selected entries in afterwards)
        if (p.P > 0 && p.plan_fresh) {
          const int per = p.NQ * p.S;
          for (int ps = 0; ps < p.P; ++ps) {
            const int ph = p.probe_heads[ps];
            if (ph >= head0 && ph < head0 + HP)
              for (int e = tid; e < per; e += 256) p.mass[((size_t)seq * p.P + ps) * per + e] = 0.0f;
          }
        }
        if (kvh == 0 && hg == 0 && tid == 0) p.seq_dec[seq] = make_int2(seq * p.dec_parts, n_records);
      }
      if (bid == 0) {   // the status word a planner would have written: one pass over the batch
        __shared__ int sh_status;
        if (tid == 0) sh_status = 0;
        __syncthreads();
        const int max_ctx = p.max_blocks * kBlock;
        int bits = 0;
        for (int i = tid; i < p.num_seqs; i += 256) {
          const int Li = p.seq_lens[i], r0 = p.cu_q_lens[i], ni = p.cu_q_lens[i + 1] - r0;
          if (Li < 0 || ni < 0) { bits |= kStatNegative; continue; }
          if (Li > max_ctx) bits |= kStatLenClamped;
          if (ni > min(Li, max_ctx)) bits |= kStatQGtL;
          else if (r0 < 0 || r0 + ni > p.total_q) bits |= kStatNegative;
          else if (ni > 1) bits |= kStatHint;   // a row block in a batch promised to hold single rows
        }
        if (bits) atomicOr(&sh_status, bits);
        __syncthreads();
        if (tid == 0) { p.hdr->n_prefill = 0; p.hdr->n_decode = 0; p.hdr->chunk_keys = 0; p.hdr->status = sh_status; }
      }
    }
  };
  if constexpr (SELF) {
    const int P = p.dec_parts;
    seq = turn / P;
    const int part = turn - seq * P;
    const int Lraw = p.seq_lens[seq];
    qrow = p.cu_q_lens[seq];
    const int n = p.cu_q_lens[seq + 1] - qrow;
    L = min(Lraw, p.max_blocks * kBlock);
    const bool valid = Lraw >= 0 && n == 1 && L >= 1 && qrow >= 0 && qrow < p.total_q;
    const int nblk_seq = valid ? (L + kBlock - 1) / kBlock : 0;
    const int bpp = (nblk_seq + P - 1) / P;          // cache blocks per part
    owes_seq = part == 0;
    n_records = valid ? (nblk_seq + bpp - 1) / bpp : 0;
    active = valid && part * bpp < nblk_seq;   // uniform over the workgroup
    // (all of this is uniform over the workgroup; saying so keeps it out of the vector registers)
    kstart = __builtin_amdgcn_readfirstlane(part * bpp * kBlock);
    kend = __builtin_amdgcn_readfirstlane(min(L, kstart + bpp * kBlock));
    qrow = __builtin_amdgcn_readfirstlane(qrow);
    seq = __builtin_amdgcn_readfirstlane(seq);
    item = turn;
  } else {
    // the grid covers the whole item capacity, so the turn's records (longest chunks first) can be
    // fetched together with the item count instead of after it
    const WorkItem it = p.dec_items[2 * turn];
    const int slot = p.dec_items[2 * turn + 1].x;
    if (turn >= p.hdr->n_decode) return;
    // the clamp only matters if the planner's capacity bound were ever violated
    item = min(max(slot, 0), p.dec_cap - 1);
    seq = it.x; L = it.z; qrow = it.w;
    const int CH = p.hdr->chunk_keys;
    kstart = it.y * CH;
    kend = min(L, kstart + CH);
  }

  if (active) decode_range<D, HP, KV8>(p, red, tid, lane, w, kvh, head0, seq, qrow, kstart, kend, item);
  settle();
}

// One workgroup per (sequence, 4 q heads): wave = head, lane = output columns.
template <int D>
__global__ __launch_bounds__(256) void k_combine(const AttnParams p) {
  using C = DecodeCfg<D>;
  const int seq = blockIdx.x;
  const int2 sd = p.seq_dec[seq];
  if (sd.y <= 0) return;
  const int lane = threadIdx.x & 63;
  const int head = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (head >= p.Hq) return;
  const float* rec0 = p.partials + ((size_t)sd.x * p.Hq + head) * C::PSTR;
  const size_t rstride = (size_t)p.Hq * C::PSTR;

  // The records were written by other workgroups, possibly under another L2, so every first touch
  // pays a trip to memory: the chunks' (max, sum) pairs are fetched one per lane in one go, and the
  // accumulation below keeps four records in flight instead of walking them one by one.
  float mstar = -INFINITY;
  for (int c0 = 0; c0 < sd.y && sd.y > 1; c0 += 64) {
    const float mc = (c0 + lane < sd.y) ? rec0[(size_t)(c0 + lane) * rstride + D] : -INFINITY;
    mstar = fmaxf(mstar, mc);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, off));
  float l = 0.0f;
  float o[D / 64];
#pragma unroll
  for (int e = 0; e < D / 64; ++e) o[e] = 0.0f;
  float a = 0.0f;  // lane s < S merges span s
  if (sd.y == 1) {   // a single chunk needs no weights: its record is the result up to the division
    l = rec0[D + 1];
#pragma unroll
    for (int e = 0; e < D / 64; ++e) o[e] = rec0[lane + 64 * e];
    if (lane < kMaxSpans) a = rec0[D + 2 + lane];
  }
  for (int c0 = 0; c0 < sd.y && sd.y > 1; c0 += 64) {
    // lane c holds the weight of chunk c0 + c
    float wl = 0.0f, wgt_mine = 0.0f;
    if (c0 + lane < sd.y) {
      const float* rec = rec0 + (size_t)(c0 + lane) * rstride;
      const float mc = rec[D];
      wgt_mine = (mc == -INFINITY) ? 0.0f : fast_exp2(mc - mstar);
      wl = wgt_mine * rec[D + 1];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wl += __shfl_xor(wl, off);
    l += wl;
    const int nc = min(64, sd.y - c0);
    int c = 0;
    for (; c + 4 <= nc; c += 4) {
      float v[4][D / 64], sp[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float* rec = rec0 + (size_t)(c0 + c + u) * rstride;
#pragma unroll
        for (int e = 0; e < D / 64; ++e) v[u][e] = rec[lane + 64 * e];
        sp[u] = (lane < kMaxSpans) ? rec[D + 2 + lane] : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float wg = __shfl(wgt_mine, c + u);
#pragma unroll
        for (int e = 0; e < D / 64; ++e) o[e] += wg * v[u][e];
        a += wg * sp[u];
      }
    }
    for (; c < nc; ++c) {
      const float* rec = rec0 + (size_t)(c0 + c) * rstride;
      const float wg = __shfl(wgt_mine, c);
#pragma unroll
      for (int e = 0; e < D / 64; ++e) o[e] += wg * rec[lane + 64 * e];
      if (lane < kMaxSpans) a += wg * rec[D + 2 + lane];
    }
  }
  const float inv = 1.0f / l;
  const int qrow = p.cu_q_lens[seq];
  __bf16* og = static_cast<__bf16*>(p.out) + ((size_t)qrow * p.Hq + head) * D;
#pragma unroll
  for (int e = 0; e < D / 64; ++e) og[lane + 64 * e] = (__bf16)(o[e] * inv);
  if (p.P > 0 && lane < p.S) {
    const int qb = p.query_sel[2 * seq], qe = min(p.query_sel[2 * seq + 1], qb + p.NQ);
    if (qb <= 0 && qe > 0) {   // row t = 0 sits in slot t - begin, as on every other path
      const int pslot = find_probe_slot(p.probe_heads, p.P, head);
      if (pslot >= 0) p.mass[(((size_t)seq * p.P + pslot) * p.NQ + (-qb)) * p.S + lane] = a * inv;
    }
  }
}

template <int D, int HP>
hipError_t launch_decode_dh(const AttnParams& p, hipStream_t st) {
  const long long grid = (long long)p.dec_cap * p.Hkv * p.dec_hgroups;
  if (grid <= 0) return hipSuccess;
  if (!grid_fits(grid)) return hipErrorInvalidValue;
  if (p.dec_parts > 0) {   // self-planned: the grid is exact
    const long long sgrid = (long long)p.num_seqs * p.dec_parts * p.Hkv * p.dec_hgroups;
    if (p.kv8) hipLaunchKernelGGL((k_decode<D, HP, true, true>), dim3((unsigned)sgrid), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((k_decode<D, HP, false, true>), dim3((unsigned)sgrid), dim3(256), 0, st, p);
    return hipGetLastError();
  }
  if (p.kv8) hipLaunchKernelGGL((k_decode<D, HP, true, false>), dim3((unsigned)grid), dim3(256), 0, st, p);
  else hipLaunchKernelGGL((k_decode<D, HP, false, false>), dim3((unsigned)grid), dim3(256), 0, st, p);
  return hipGetLastError();
}

template <int D>
hipError_t launch_decode_d(const AttnParams& p, hipStream_t st) {
  switch (p.dec_hp) {
    case 8: return launch_decode_dh<D, 8>(p, st);
    case 4: return launch_decode_dh<D, 4>(p, st);
    case 2: return launch_decode_dh<D, 2>(p, st);
    case 1: return launch_decode_dh<D, 1>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_decode(const AttnParams& p, int D, hipStream_t st) {
  if (D == 128) return launch_decode_d<128>(p, st);
  if (D == 64) return launch_decode_d<64>(p, st);
  return hipErrorInvalidValue;
}

hipError_t launch_combine(const AttnParams& p, int D, hipStream_t st) {
  if (p.dec_cap <= 0 || p.num_seqs <= 0) return hipSuccess;
  const dim3 grid((unsigned)p.num_seqs, (unsigned)((p.Hq + 3) / 4));
  if (D == 128) hipLaunchKernelGGL(k_combine<128>, grid, dim3(256), 0, st, p);
  else if (D == 64) hipLaunchKernelGGL(k_combine<64>, grid, dim3(256), 0, st, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace hook
