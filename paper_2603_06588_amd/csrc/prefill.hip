// Tiled causal attention for query chunks (n_i >= 2) over the paged KV cache, bf16 MFMA.
//
// Workgroup = 4 waves = (hpw q heads of one kv head) x (4 / hpw blocks of 32 query rows).
// Key tiles of 64 are staged once per workgroup in LDS (double buffered) and shared by all
// waves: K row-major, V transposed (keys contiguous) so both feed the MFMA A operand with
// 16-byte LDS reads.
//
// Per wave the score tile is computed TRANSPOSED, S^T = K Q^T (32x32x16 MFMA, keys = M,
// queries = N).  In the accumulator layout lane l then owns query l % 32 and 16 keys per
// 32-key block, so the softmax row statistics are in-lane reductions plus one exchange
// between lane halves, and the exponentials, rounded to bf16, are already laid out as the
// B operand of O^T = V^T P^T without touching LDS.  Probe span sums are accumulated from
// the fp32 exponentials under the same running reference as the normaliser and divided by
// it at the end, so the captured mass is the exact softmax mass.
//
// KV8: the caches hold 8-bit E4M3 bytes with one fp32 scale per kv head.  Tiles are staged through
// registers here, so the bytes are widened to bf16 (exactly: every E4M3 number is a bf16 number) on
// their way into LDS and the loop itself does not change; the key scale is folded into the softmax
// scale and the value scale into the final normalisation of `out`.  This is what serves query chunks
// over an 8-bit cache for both head dimensions (the direct-to-LDS kernel for head_dim 128 cannot
// convert on the way).
#include "fp8_device.h"
#include "hook_device.h"

namespace hook {

namespace {

template <int D>
struct PrefillCfg {
  static constexpr int KSTR = D + 8;          // LDS K row stride in elements (16-byte pad)
  static constexpr int VSTR = kTileKeys + 8;  // LDS V^T row stride in elements
  static constexpr int CHK = D / 8;           // 16-byte chunks per K/V row
  static constexpr int KPASS = CHK / 4;       // K staging passes (256 threads, 64 keys)
  static constexpr int KEYS_PER_PASS = 256 / CHK;
  static constexpr int KSTEPS = D / 16;       // MFMA k-steps of S^T = K Q^T
  static constexpr int MB = D / 32;           // 32-row blocks of O^T
  static constexpr int KS_ELEMS = kTileKeys * KSTR;
  static constexpr int VT_ELEMS = D * VSTR;
  static constexpr size_t LDS_BYTES = 2 * (size_t)(KS_ELEMS + VT_ELEMS) * 2;
};

// position (in elements) of 4-key group kg (0..15) inside a V^T row: the order in which the
// score accumulator hands keys to the second MFMA (see the file comment)
__device__ __forceinline__ int vt_group_pos(int kg) {
  return 16 * (kg >> 2) + 8 * (kg & 1) + 4 * ((kg >> 1) & 1);
}

template <int D, bool KV8>
__global__ __launch_bounds__(256, 2) void k_prefill(const AttnParams p) {
  using C = PrefillCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __bf16* const Ks = reinterpret_cast<__bf16*>(smem_raw);   // [2][64][KSTR]
  __bf16* const Vt = Ks + 2 * C::KS_ELEMS;                   // [2][D][VSTR]

  const int bid = blockIdx.x;
  const int kvh = bid % p.Hkv;
  const int rest = bid / p.Hkv;
  const int hg = rest % p.hgroups;
  const int item = rest / p.hgroups;
  // the grid covers the whole item capacity, so both records can be fetched together with
  // the item count instead of after it
  const WorkItem it = p.pf_items[2 * item];
  const int qbase = p.pf_items[2 * item + 1].x;
  if (item >= p.hdr->n_prefill) return;
  const int seq = it.x, row0 = it.y, L = it.z, n = it.w;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hh = w % p.hpw, rb = w / p.hpw;
  const int head = kvh * p.G + hg * p.hpw + hh;
  const int wrow0 = row0 + rb * kWaveRows;
  const bool wave_active = wrow0 < n;
  const int qi = lane & 31, hf = lane >> 5;
  const int t = max(min(wrow0 + qi, n - 1), 0);
  const int pos = L - n + t;                                   // this lane's causal horizon
  const int wave_pos_min = L - n + min(wrow0, n - 1);
  const int wave_pos_max = L - n + min(wrow0 + kWaveRows, n) - 1;
  const int wg_pos_max = L - n + min(row0 + p.rows_per_wg, n) - 1;
  const int ntiles = wg_pos_max / kTileKeys + 1;

  const __bf16* const qg = static_cast<const __bf16*>(p.q);
  const __bf16* const kg_ = static_cast<const __bf16*>(p.k_cache);
  const __bf16* const vg_ = static_cast<const __bf16*>(p.v_cache);
  const unsigned char* const kg8 = static_cast<const unsigned char*>(p.k_cache);
  const unsigned char* const vg8 = static_cast<const unsigned char*>(p.v_cache);
  const int* const bt = p.block_table + (size_t)seq * p.max_blocks;
  const size_t blk_stride = (size_t)p.Hkv * kBlock * D;        // elements per block
  const size_t head_off = (size_t)kvh * kBlock * D;

  // Q^T fragments: lane (query qi, half hf) holds q[16 s + 8 hf .. +7] for every k-step s
  bf16x8 qf[C::KSTEPS];
  {
    const bf16x8* qp = reinterpret_cast<const bf16x8*>(qg + ((size_t)(qbase + t) * p.Hq + head) * D + 8 * hf);
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s) qf[s] = qp[2 * s];
  }

  // probe set-up (wave-uniform)
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

  // staging thread roles
  const int k_key = tid / C::CHK, k_ch = tid % C::CHK;          // + KEYS_PER_PASS * pass
  const bool v_thread = tid < 16 * C::CHK;
  const int v_dc = 4 * w + (lane & 3);                           // 8-wide column chunk of V
  const int v_kg = lane >> 2;                                    // 4-key group inside the tile
  const int v_pos = vt_group_pos(v_kg);

  uint4 kreg[C::KPASS];
  uint4 vreg[4];

  auto load_tile = [&](int kt) {
    const int key0 = kt * kTileKeys;
#pragma unroll
    for (int j = 0; j < C::KPASS; ++j) {
      const int key = key0 + k_key + C::KEYS_PER_PASS * j;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (key < L) {
        int blk = bt[key >> 4];
        blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
        const size_t off = (size_t)blk * blk_stride + head_off + (size_t)(key & 15) * D + 8 * k_ch;   // in elements
        if constexpr (KV8) v = e4m3x8_to_bf16x8(*reinterpret_cast<const uint2*>(kg8 + off));
        else v = *reinterpret_cast<const uint4*>(kg_ + off);
      }
      kreg[j] = v;
    }
    if (v_thread) {
      const int kbase = key0 + 4 * v_kg;
      int blk = 0;
      if (kbase < L) {
        blk = bt[kbase >> 4];
        blk = ((unsigned)blk < (unsigned)p.num_blocks) ? blk : 0;
      }
      const size_t voff = (size_t)blk * blk_stride + head_off + (size_t)(kbase & 15) * D + 8 * v_dc;   // in elements
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (kbase + i < L) {
          if constexpr (KV8) v = e4m3x8_to_bf16x8(*reinterpret_cast<const uint2*>(vg8 + voff + (size_t)i * D));
          else v = *reinterpret_cast<const uint4*>(vg_ + voff + (size_t)i * D);
        }
        vreg[i] = v;
      }
    }
  };

  auto store_tile = [&](int buf) {
    __bf16* ks = Ks + buf * C::KS_ELEMS;
#pragma unroll
    for (int j = 0; j < C::KPASS; ++j)
      *reinterpret_cast<uint4*>(ks + (k_key + C::KEYS_PER_PASS * j) * C::KSTR + 8 * k_ch) = kreg[j];
    if (v_thread) {
      __bf16* vt = Vt + buf * C::VT_ELEMS + (8 * v_dc) * C::VSTR + v_pos;
      const uint32_t a[4][4] = {{vreg[0].x, vreg[0].y, vreg[0].z, vreg[0].w},
                                {vreg[1].x, vreg[1].y, vreg[1].z, vreg[1].w},
                                {vreg[2].x, vreg[2].y, vreg[2].z, vreg[2].w},
                                {vreg[3].x, vreg[3].y, vreg[3].z, vreg[3].w}};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        // 4 keys x columns (2c, 2c+1): low halves -> row 2c, high halves -> row 2c+1
        uint2 lo, hi;
        lo.x = __builtin_amdgcn_perm(a[1][c], a[0][c], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(a[3][c], a[2][c], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(a[1][c], a[0][c], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(a[3][c], a[2][c], 0x07060302u);
        *reinterpret_cast<uint2*>(vt + (2 * c) * C::VSTR) = lo;
        *reinterpret_cast<uint2*>(vt + (2 * c + 1) * C::VSTR) = hi;
      }
    }
  };

  // running state: lane (query qi, half hf) holds partial sums over its half of the keys
  f32x16 O[C::MB];
#pragma unroll
  for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[mb][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  float am[kMaxSpans];
#pragma unroll
  for (int s = 0; s < kMaxSpans; ++s) am[s] = 0.0f;
  const float c = KV8 ? p.scale_log2 * p.k_scale[kvh] : p.scale_log2;

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int kt = 0; kt < ntiles; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < ntiles;
    if (more) load_tile(kt + 1);

    const int key0 = kt * kTileKeys;
    if (wave_active && key0 <= wave_pos_max) {
      const __bf16* ks = Ks + buf * C::KS_ELEMS;
      const __bf16* vt = Vt + buf * C::VT_ELEMS;
      f32x16 S[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[kb][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < C::KSTEPS; ++s) {
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(ks + qi * C::KSTR + 16 * s + 8 * hf);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(ks + (32 + qi) * C::KSTR + 16 * s + 8 * hf);
        S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[s], S[0], 0, 0, 0);
        S[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[s], S[1], 0, 0, 0);
      }
      // causal mask (also hides the zero-filled keys past L): only tiles that reach past
      // the smallest horizon in this wave need it
      if (key0 + kTileKeys - 1 > wave_pos_min) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (key > pos) S[kb][r] = -INFINITY;
          }
      }
      float mx = S[0][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[0][r]);
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[1][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mt = mx * c;
      const bool upd = mt > m_run + kLazyTau;
      if (__builtin_amdgcn_ballot_w64(upd) != 0) {
        const float alpha = upd ? fast_exp2(m_run - mt) : 1.0f;
        m_run = upd ? mt : m_run;
        l_run *= alpha;
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
#pragma unroll
        for (int s = 0; s < kMaxSpans; ++s) am[s] *= alpha;
      }
      const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;
      float tsum = 0.0f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = fast_exp2(__builtin_fmaf(S[kb][r], c, -m_safe));
          S[kb][r] = e;
          tsum += e;
        }
      l_run += tsum;

      if (wave_probe) {
#pragma unroll
        for (int s = 0; s < kMaxSpans; ++s) {
          if (s < p.S) {
            const int a = sp_a[s], b = sp_b[s];
            if (b > key0 && a < key0 + kTileKeys) {
              if (a <= key0 && b >= key0 + kTileKeys) {
                am[s] += tsum;  // whole tile inside the span; masked keys contributed 0
              } else {
                float acc = 0.0f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                  for (int r = 0; r < 16; ++r) {
                    const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * hf + (r & 3);
                    acc += (key >= a && key < b) ? S[kb][r] : 0.0f;
                  }
                am[s] += acc;
              }
            }
          }
        }
      }

      // P^T as bf16 B operands, then O^T += V^T P^T
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int kb = m >> 1, r0 = 8 * (m & 1);
        union { uint32_t u[4]; bf16x8 v; } pb;
#pragma unroll
        for (int e = 0; e < 4; ++e) pb.u[e] = pack_bf16(S[kb][r0 + 2 * e], S[kb][r0 + 2 * e + 1]);
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
          const bf16x8 av = *reinterpret_cast<const bf16x8*>(vt + (32 * mb + qi) * C::VSTR + 16 * m + 8 * hf);
          O[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb.v, O[mb], 0, 0, 0);
        }
      }
    }

    if (more) store_tile(buf ^ 1);
    __syncthreads();
  }

  // epilogue: normalise, transpose through LDS (the K buffers are free now), coalesced stores
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv_l = 1.0f / l_tot;
  const float inv = KV8 ? inv_l * p.v_scale[kvh] : inv_l;     // `out` carries the value scale, `mass` does not
  __bf16* const ot = Ks + w * (kWaveRows * C::KSTR);
  if (wave_active) {
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        uint2 v;
        v.x = pack_bf16(O[mb][4 * g4] * inv, O[mb][4 * g4 + 1] * inv);
        v.y = pack_bf16(O[mb][4 * g4 + 2] * inv, O[mb][4 * g4 + 3] * inv);
        *reinterpret_cast<uint2*>(ot + qi * C::KSTR + 32 * mb + 8 * g4 + 4 * hf) = v;
      }
  }
  __syncthreads();
  if (wave_active) {
    __bf16* const og = static_cast<__bf16*>(p.out);
    constexpr int ROWS_PER_IT = 64 / C::CHK;
#pragma unroll
    for (int j = 0; j < kWaveRows / ROWS_PER_IT; ++j) {
      const int r = lane / C::CHK + ROWS_PER_IT * j;
      const int ch = lane % C::CHK;
      const int tr = wrow0 + r;
      if (tr < n) {
        const uint4 v = *reinterpret_cast<const uint4*>(ot + r * C::KSTR + 8 * ch);
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
            p.mass[(((size_t)seq * p.P + pslot) * p.NQ + (tr - qsel_b)) * p.S + s] = a_tot * inv_l;
        }
      }
    }
  }
}

template <int D, bool KV8>
hipError_t launch_prefill_d(const AttnParams& p, hipStream_t st) {
  using C = PrefillCfg<D>;
  static std::atomic<unsigned long long> configured{0};
  const hipError_t e = raise_lds_limit_once(reinterpret_cast<const void*>(&k_prefill<D, KV8>), (int)C::LDS_BYTES, configured);
  if (e != hipSuccess) return e;
  const long long grid = (long long)p.pf_cap * p.Hkv * p.hgroups;
  if (grid <= 0) return hipSuccess;
  if (!grid_fits(grid)) return hipErrorInvalidValue;
  hipLaunchKernelGGL((k_prefill<D, KV8>), dim3((unsigned)grid), dim3(256), C::LDS_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill(const AttnParams& p, int D, hipStream_t st) {
  if (p.kv8) {   // 8-bit caches: the register-staged kernel, which widens the bytes on their way into LDS
    if (D == 128) return launch_prefill_d<128, true>(p, st);
    if (D == 64) return launch_prefill_d<64, true>(p, st);
    return hipErrorInvalidValue;
  }
  if (D == 128) return launch_prefill128(p, st);
  if (D == 64) return launch_prefill_d<64, false>(p, st);
  return hipErrorInvalidValue;
}

}  // namespace hook
