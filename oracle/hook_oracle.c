/*
 * CPU oracle for the hooked-attention path.  TEST INFRASTRUCTURE ONLY: it is
 * called from the tests, the smoke check and the benchmark's CPU-baseline leg,
 * never from the product path, and it shares no code with the GPU library.
 *
 * What it computes is the plain definition, in fp64, with an explicit two-pass
 * softmax and explicit span sums:
 *
 *   - the paper's analyzer recomputes the attention of the configured
 *     [layer, head] pairs from captured queries and all keys (Section 2.2,
 *     "recompute selective attentions"), for the last token or for all tokens
 *     (Section 2, "hookq_mode"), and aggregates it over token ranges given per
 *     prompt (Section 2.2, "input_range": instruction range and data range);
 *   - the attention output itself is what the engine's attention module returns
 *     and must stay intact under passive programming (Section 1, passive
 *     programming; Section 2.1, execute_model pass-through);
 *   - activation steering adds a steering vector to a layer's activations
 *     (Section 1, "Model Steering"; Section 3, activation steering demo).
 *
 * The paper prints no formula for attention; the reading taken here is scaled
 * dot-product attention with a causal mask, softmax over keys, grouped-query
 * heads in contiguous groups (kv head = q head / (Hq / Hkv)), half-open spans
 * clipped to the causal horizon [0, pos].
 *
 * Pins (tests/test_oracle_pins.py): brute force on tiny inputs, row sums equal
 * one, closed form for Q = 0, dominant-key limit, torch fp64 softmax(QK^T)V on
 * un-paged tensors, paging permutation invariance, chunked-prefill positions,
 * GQA replication, steering special cases; for the 8-bit cache: the 256-entry
 * decoding table against a library's, and equality with the 16-bit path on caches
 * whose dequantised values bf16 holds exactly.  Every function below is pinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1, ORACLE_FP8_E4M3 = 2 };

int hook_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * One byte of an 8-bit floating-point cache -> double, exactly.  The format is the 8-bit
 * "E4M3" interchange format (1 sign, 4 exponent, 3 mantissa bits, bias 7, no infinities, the one
 * NaN pattern S.1111.111): value = (-1)^S * 2^(E-7) * (1 + M/8) for E > 0 and
 * (-1)^S * 2^-6 * M/8 for E = 0.
 */
static double load_fp8_e4m3(uint8_t b) {
  const int sign = b >> 7, E = (b >> 3) & 15, M = b & 7;
  double v;
  if (E == 15 && M == 7) return NAN;
  if (E == 0) v = ldexp((double)M / 8.0, -6);
  else v = ldexp(1.0 + (double)M / 8.0, E - 7);
  return sign ? -v : v;
}

/* Exposed so a test can pin the 256-entry decoding table on its own. */
double hook_oracle_fp8_e4m3_value(uint8_t b) { return load_fp8_e4m3(b); }

/* Stored element -> double, exactly (bf16 is the top half of an IEEE float). */
static double load_elem(const void* base, size_t idx, int dtype) {
  if (dtype == ORACLE_F32) return (double)((const float*)base)[idx];
  if (dtype == ORACLE_FP8_E4M3) return load_fp8_e4m3(((const uint8_t*)base)[idx]);
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* double -> bf16 with one round-to-nearest-even step (no intermediate float rounding). */
static uint16_t double_to_bf16_rne(double x) {
  uint16_t sign = signbit(x) ? 0x8000u : 0u;
  if (isnan(x)) return (uint16_t)(sign | 0x7FC0u);
  double a = fabs(x);
  if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
  if (a == 0.0) return sign;
  int e;
  (void)frexp(a, &e);          /* a = m * 2^e, m in [0.5, 1)  => unbiased exponent e-1 */
  int ue = e - 1;
  if (ue < -126) ue = -126;    /* subnormal range shares the quantum of the smallest normal */
  double quantum = ldexp(1.0, ue - 7);
  double r = nearbyint(a / quantum) * quantum; /* exact scaling; ties to even */
  if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
  float f = (float)r;          /* exact: r has at most 8 significant bits */
  uint32_t bits;
  memcpy(&bits, &f, sizeof bits);
  return (uint16_t)(sign | (uint16_t)(bits >> 16));
}

/*
 * Attention output and span masses.
 *
 * For sequence i, chunk-local query row t in [0, n_i), absolute position
 * pos = L_i - n_i + t, q head h, kv head g = h / (Hq / Hkv):
 *   K[j] = k_cache[block_table[i, j / B], g, j % B, :]  (V likewise), j = 0..pos
 *   s_j  = scale * <q[t,h,:], K[j]>
 *   p_j  = exp(s_j - max s) / sum_j exp(s_j - max s)
 *   out[t,h,:] = sum_j p_j V[j]
 *   mass[i, p, t - begin, r] = sum of p_j over j in [max(a,0), min(b, pos+1))
 *     for probed head h = probe_heads[p], begin <= t < end, span r = [a, b).
 *
 * rows == NULL: all rows.  Otherwise only the listed global row indices are
 * computed (their `out` rows and, if selected, their masses); everything else
 * in `out` is left untouched.  `mass` is zero-filled first.
 * Returns 0, or a negative code for malformed arguments.
 */
static int attn_probe_impl(
    int num_seqs, int total_q, int Hq, int Hkv, int d, int B, int max_blocks, int num_blocks,
    int dtype, double scale,
    const void* q, const void* k_cache, const void* v_cache,
    const int32_t* block_table, const int32_t* seq_lens, const int32_t* cu_q_lens,
    int P, const int32_t* probe_heads, int NQ, const int32_t* query_sel, int S, const int32_t* key_spans,
    int n_rows, const int32_t* rows,
    int kv_dtype, const float* k_scale, const float* v_scale,
    double* out, double* mass) {
  if (Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || B <= 0) return -1;
  if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return -2;
  if (kv_dtype != dtype && kv_dtype != ORACLE_FP8_E4M3) return -2;
  const int G = Hq / Hkv;
  if (mass && P > 0) memset(mass, 0, sizeof(double) * (size_t)num_seqs * P * NQ * S);
  int bad = 0;

  /* row filter as a byte map over global rows */
  unsigned char* want = NULL;
  if (rows) {
    want = (unsigned char*)calloc((size_t)(total_q > 0 ? total_q : 1), 1);
    for (int r = 0; r < n_rows; ++r)
      if (rows[r] >= 0 && rows[r] < total_q) want[rows[r]] = 1;
  }

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < num_seqs; ++i) {
    for (int g = 0; g < Hkv; ++g) {
      const int L = seq_lens[i];
      const int row0 = cu_q_lens[i];
      const int n = cu_q_lens[i + 1] - row0;
      if (n <= 0 || L <= 0) continue;
      if (n > L) { bad = 1; continue; }
      int any = (want == NULL);
      for (int t = 0; t < n && !any; ++t) any = want[row0 + t];
      if (!any) continue;

      /* step 1: gather this sequence's keys and values of kv head g through the block table */
      double* Kd = (double*)malloc(sizeof(double) * (size_t)L * d);
      double* Vd = (double*)malloc(sizeof(double) * (size_t)L * d);
      double* s = (double*)malloc(sizeof(double) * (size_t)L);
      double* qd = (double*)malloc(sizeof(double) * (size_t)d);
      double* od = (double*)malloc(sizeof(double) * (size_t)d);
      int ok = 1;
      for (int j = 0; j < L; ++j) {
        const int blk = block_table[(size_t)i * max_blocks + j / B];
        if (blk < 0 || blk >= num_blocks) { ok = 0; break; }
        const size_t base = (((size_t)blk * Hkv + g) * B + (size_t)(j % B)) * d;
        for (int c = 0; c < d; ++c) {
          Kd[(size_t)j * d + c] = load_elem(k_cache, base + c, kv_dtype);
          Vd[(size_t)j * d + c] = load_elem(v_cache, base + c, kv_dtype);
          /* a quantised cache stores value / scale: one scale per kv head */
          if (k_scale) Kd[(size_t)j * d + c] *= (double)k_scale[g];
          if (v_scale) Vd[(size_t)j * d + c] *= (double)v_scale[g];
        }
      }
      if (!ok) { bad = 1; free(Kd); free(Vd); free(s); free(qd); free(od); continue; }

      for (int t = 0; t < n; ++t) {
        if (want && !want[row0 + t]) continue;
        const int pos = L - n + t;
        for (int hh = 0; hh < G; ++hh) {
          const int h = g * G + hh;
          const size_t qbase = ((size_t)(row0 + t) * Hq + h) * d;
          /* step 2: scores */
          for (int c = 0; c < d; ++c) qd[c] = load_elem(q, qbase + c, dtype);
          double smax = -INFINITY;
          for (int j = 0; j <= pos; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += qd[c] * Kd[(size_t)j * d + c];
            s[j] = scale * acc;
            if (s[j] > smax) smax = s[j];
          }
          /* step 3: two-pass softmax */
          double denom = 0.0;
          for (int j = 0; j <= pos; ++j) { s[j] = exp(s[j] - smax); denom += s[j]; }
          for (int j = 0; j <= pos; ++j) s[j] /= denom;
          /* step 4: output */
          for (int c = 0; c < d; ++c) od[c] = 0.0;
          for (int j = 0; j <= pos; ++j)
            for (int c = 0; c < d; ++c) od[c] += s[j] * Vd[(size_t)j * d + c];
          for (int c = 0; c < d; ++c) out[qbase + c] = od[c];
          /* step 5: span masses for probed heads and selected rows */
          if (mass && P > 0) {
            const int qb = query_sel[2 * i], qe = query_sel[2 * i + 1];
            if (t >= qb && t < qe && t - qb < NQ) {
              for (int p = 0; p < P; ++p) {
                if (probe_heads[p] != h) continue;
                for (int r = 0; r < S; ++r) {
                  int a = key_spans[((size_t)i * S + r) * 2];
                  int b = key_spans[((size_t)i * S + r) * 2 + 1];
                  if (a < 0) a = 0;
                  if (b > pos + 1) b = pos + 1;
                  double m = 0.0;
                  for (int j = a; j < b; ++j) m += s[j];
                  mass[(((size_t)i * P + p) * NQ + (t - qb)) * S + r] = m;
                }
              }
            }
          }
        }
      }
      free(Kd); free(Vd); free(s); free(qd); free(od);
    }
  }
  free(want);
  return bad ? -3 : 0;
}

int hook_oracle_attn_probe(
    int num_seqs, int total_q, int Hq, int Hkv, int d, int B, int max_blocks, int num_blocks,
    int dtype, double scale,
    const void* q, const void* k_cache, const void* v_cache,
    const int32_t* block_table, const int32_t* seq_lens, const int32_t* cu_q_lens,
    int P, const int32_t* probe_heads, int NQ, const int32_t* query_sel, int S, const int32_t* key_spans,
    int n_rows, const int32_t* rows,
    double* out, double* mass) {
  return attn_probe_impl(num_seqs, total_q, Hq, Hkv, d, B, max_blocks, num_blocks, dtype, scale, q, k_cache, v_cache,
                         block_table, seq_lens, cu_q_lens, P, probe_heads, NQ, query_sel, S, key_spans, n_rows, rows,
                         dtype, NULL, NULL, out, mass);
}

/*
 * The same definition over an 8-bit (E4M3) key/value cache: every cache byte is first turned back
 * into the number it stands for, K[j][c] = value(byte) * k_scale[g] (V alike, one fp32 scale per kv
 * head), then everything is as above.  q keeps its own dtype.  This is the "dequantise, then the
 * plain definition" reading of a quantised cache; the paper does not discuss cache precision.
 */
int hook_oracle_attn_probe_kv8(
    int num_seqs, int total_q, int Hq, int Hkv, int d, int B, int max_blocks, int num_blocks,
    int dtype, double scale,
    const void* q, const void* k_cache, const void* v_cache, const float* k_scale, const float* v_scale,
    const int32_t* block_table, const int32_t* seq_lens, const int32_t* cu_q_lens,
    int P, const int32_t* probe_heads, int NQ, const int32_t* query_sel, int S, const int32_t* key_spans,
    int n_rows, const int32_t* rows,
    double* out, double* mass) {
  if (!k_scale || !v_scale) return -1;
  return attn_probe_impl(num_seqs, total_q, Hq, Hkv, d, B, max_blocks, num_blocks, dtype, scale, q, k_cache, v_cache,
                         block_table, seq_lens, cu_q_lens, P, probe_heads, NQ, query_sel, S, key_spans, n_rows, rows,
                         ORACLE_FP8_E4M3, k_scale, v_scale, out, mass);
}

/*
 * Steering: hidden_out[t,:] = round_to_dtype((double)hidden[t,:] + (double)alpha * (double)vec[:])
 * for rows with token_mask[t] != 0 (round-to-nearest-even, one rounding);
 * all other rows are copied bit for bit.
 */
int hook_oracle_steer(const void* hidden, const void* vec, float alpha, const uint8_t* token_mask,
                      int T, int D, int dtype, void* hidden_out) {
  if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return -2;
  const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
  for (int t = 0; t < T; ++t) {
    const size_t base = (size_t)t * D;
    if (!token_mask[t]) {
      memcpy((char*)hidden_out + base * esz, (const char*)hidden + base * esz, (size_t)D * esz);
      continue;
    }
    for (int c = 0; c < D; ++c) {
      double r = load_elem(hidden, base + c, dtype) + (double)alpha * load_elem(vec, (size_t)c, dtype);
      if (dtype == ORACLE_F32) ((float*)hidden_out)[base + c] = (float)r;
      else ((uint16_t*)hidden_out)[base + c] = double_to_bf16_rne(r);
    }
  }
  return 0;
}

/*
 * Steering folded into the residual add that writes the hidden state (the "next" fused form):
 * out[t,:] = round_to_dtype((double)hidden[t,:] + (double)delta[t,:] [+ (double)alpha * (double)vec[:]])
 * with the bracket on rows whose token_mask byte is non-zero; one rounding, nearest-even.
 * token_mask may be null (no row is steered).
 */
int hook_oracle_residual_steer(const void* hidden, const void* delta, const void* vec, float alpha,
                               const uint8_t* token_mask, int T, int D, int dtype, void* hidden_out) {
  if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return -2;
  for (int t = 0; t < T; ++t) {
    const size_t base = (size_t)t * D;
    const int on = token_mask && token_mask[t] && alpha != 0.0f;
    for (int c = 0; c < D; ++c) {
      double r = load_elem(hidden, base + c, dtype) + load_elem(delta, base + c, dtype);
      if (on) r += (double)alpha * load_elem(vec, (size_t)c, dtype);
      if (dtype == ORACLE_F32) ((float*)hidden_out)[base + c] = (float)r;
      else ((uint16_t*)hidden_out)[base + c] = double_to_bf16_rne(r);
    }
  }
  return 0;
}

/* Exposed so a test can pin the rounding step on its own. */
uint16_t hook_oracle_round_bf16(double x) { return double_to_bf16_rne(x); }
