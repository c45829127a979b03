/*
 * Drives the CPU oracle (oracle/hook_oracle.c, compiled into this program) under
 * AddressSanitizer and UndefinedBehaviorSanitizer.  The oracle indexes through a block table
 * and allocates per (sequence, kv head); this run makes every such access on ragged paged
 * inputs whose buffers are exactly as large as the shapes say, so an access one element too far
 * is reported.  It also checks the results against what the mathematics fixes (rows sum to one,
 * uniform attention for q = 0), so the sanitised build is known to compute, not just to run.
 *
 * Built and run by tests/test_oracle_sanitized.py; exit status 0 and a final "ok" mean clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int hook_oracle_attn_probe(int num_seqs, int total_q, int Hq, int Hkv, int d, int B, int max_blocks, int num_blocks,
                           int dtype, double scale, const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* block_table, const int32_t* seq_lens, const int32_t* cu_q_lens, int P,
                           const int32_t* probe_heads, int NQ, const int32_t* query_sel, int S,
                           const int32_t* key_spans, int n_rows, const int32_t* rows, double* out, double* mass);
int hook_oracle_attn_probe_kv8(int num_seqs, int total_q, int Hq, int Hkv, int d, int B, int max_blocks, int num_blocks,
                               int dtype, double scale, const void* q, const void* k_cache, const void* v_cache,
                               const float* k_scale, const float* v_scale, const int32_t* block_table,
                               const int32_t* seq_lens, const int32_t* cu_q_lens, int P, const int32_t* probe_heads,
                               int NQ, const int32_t* query_sel, int S, const int32_t* key_spans, int n_rows,
                               const int32_t* rows, double* out, double* mass);
double hook_oracle_fp8_e4m3_value(uint8_t byte);
int hook_oracle_steer(const void* hidden, const void* vec, float alpha, const uint8_t* token_mask, int T, int D,
                      int dtype, void* hidden_out);
int hook_oracle_residual_steer(const void* hidden, const void* delta, const void* vec, float alpha,
                               const uint8_t* token_mask, int T, int D, int dtype, void* hidden_out);
uint16_t hook_oracle_round_bf16(double x);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) {   /* xorshift, uniform in [-1, 1) */
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { printf("FAIL: " __VA_ARGS__); printf("\n"); ++failures; } } while (0)

enum { NSEQ = 4, HQ = 4, HKV = 2, D = 8, B = 16, P = 2, NQ = 5, S = 4 };

static void run_attention(int dtype, int zero_q) {
  const int lens[NSEQ] = {37, 5, 64, 0}, qn[NSEQ] = {37, 1, 20, 0};
  int cu[NSEQ + 1] = {0};
  int nblk_needed = 0, max_blocks = 0;
  for (int i = 0; i < NSEQ; ++i) {
    cu[i + 1] = cu[i] + qn[i];
    const int nb = (lens[i] + B - 1) / B;
    nblk_needed += nb;
    if (nb > max_blocks) max_blocks = nb;
  }
  const int total_q = cu[NSEQ], num_blocks = nblk_needed + 3;
  const size_t esz = dtype == 0 ? 2 : 4;
  const size_t nq = (size_t)total_q * HQ * D, nkv = (size_t)num_blocks * HKV * B * D;
  void* q = malloc(nq * esz);
  void* k = malloc(nkv * esz);
  void* v = malloc(nkv * esz);
  for (size_t e = 0; e < nq; ++e) {
    const double x = zero_q ? 0.0 : rnd();
    if (dtype == 0) ((uint16_t*)q)[e] = hook_oracle_round_bf16(x); else ((float*)q)[e] = (float)x;
  }
  for (size_t e = 0; e < nkv; ++e) {
    const double x = rnd(), y = rnd();
    if (dtype == 0) { ((uint16_t*)k)[e] = hook_oracle_round_bf16(x); ((uint16_t*)v)[e] = hook_oracle_round_bf16(y); }
    else { ((float*)k)[e] = (float)x; ((float*)v)[e] = (float)y; }
  }
  /* block table: live entries take the pool's blocks in reverse order, dead entries an id far outside */
  int32_t* table = malloc(sizeof(int32_t) * (size_t)NSEQ * max_blocks);
  int next = num_blocks - 1;
  for (int i = 0; i < NSEQ; ++i)
    for (int b = 0; b < max_blocks; ++b)
      table[i * max_blocks + b] = b < (lens[i] + B - 1) / B ? next-- : 0x7FFFFFF0;
  const int32_t heads[P] = {1, 2};
  /* row ranges: ordinary, beginning before the chunk, reaching past it, empty */
  const int32_t sel[NSEQ * 2] = {33, 37, -2, 1, 18, 40, 0, 0};
  int32_t spans[NSEQ * S * 2];
  for (int i = 0; i < NSEQ; ++i) {
    const int32_t sp[S * 2] = {0, lens[i], -3, 7, lens[i] - 2, lens[i] + 9, 6, 2};   /* whole, clipped low, clipped high, empty */
    memcpy(spans + i * S * 2, sp, sizeof sp);
  }
  double* out = malloc(sizeof(double) * nq);
  double* mass = malloc(sizeof(double) * (size_t)NSEQ * P * NQ * S);
  for (size_t e = 0; e < nq; ++e) out[e] = NAN;
  int rc = hook_oracle_attn_probe(NSEQ, total_q, HQ, HKV, D, B, max_blocks, num_blocks, dtype, 0.25, q, k, v, table,
                                  lens, cu, P, heads, NQ, sel, S, spans, 0, NULL, out, mass);
  CHECK(rc == 0, "attn_probe returned %d (dtype %d)", rc, dtype);
  for (size_t e = 0; e < nq; ++e) CHECK(isfinite(out[e]), "out[%zu] not finite", e);
  for (int i = 0; i < NSEQ; ++i)
    for (int p = 0; p < P; ++p)
      for (int slot = 0; slot < NQ; ++slot) {
        const int t = sel[2 * i] + slot;
        const int live = t >= 0 && t < sel[2 * i + 1] && t < qn[i];
        const double* m = mass + (((size_t)i * P + p) * NQ + slot) * S;
        if (!live) { for (int r = 0; r < S; ++r) CHECK(m[r] == 0.0, "seq %d slot %d span %d should be empty", i, slot, r); continue; }
        const int pos = lens[i] - qn[i] + t;
        CHECK(fabs(m[0] - 1.0) < 1e-12, "seq %d slot %d: whole-context mass %.17g", i, slot, m[0]);
        CHECK(m[3] == 0.0, "empty span has mass");
        if (zero_q) {   /* uniform attention: |span intersected with [0, pos]| / (pos + 1) */
          const int hi1 = 7 < pos + 1 ? 7 : pos + 1;
          CHECK(fabs(m[1] - (double)hi1 / (pos + 1)) < 1e-12, "seq %d slot %d: clipped-low span %.17g", i, slot, m[1]);
          int lo2 = lens[i] - 2; if (lo2 < 0) lo2 = 0;
          const int cnt2 = pos + 1 - lo2 > 0 ? pos + 1 - lo2 : 0;
          CHECK(fabs(m[2] - (double)cnt2 / (pos + 1)) < 1e-12, "seq %d slot %d: clipped-high span %.17g", i, slot, m[2]);
        }
      }
  /* a row subset: the listed rows agree with the full run, the others are left alone */
  double* out2 = malloc(sizeof(double) * nq);
  for (size_t e = 0; e < nq; ++e) out2[e] = -7.0;
  const int32_t rows[4] = {0, 36, 37, total_q - 1};
  rc = hook_oracle_attn_probe(NSEQ, total_q, HQ, HKV, D, B, max_blocks, num_blocks, dtype, 0.25, q, k, v, table, lens,
                              cu, P, heads, NQ, sel, S, spans, 4, rows, out2, mass);
  CHECK(rc == 0, "row subset returned %d", rc);
  for (int r = 0; r < total_q; ++r) {
    int listed = 0;
    for (int u = 0; u < 4; ++u) listed |= rows[u] == r;
    for (int e = 0; e < HQ * D; ++e) {
      const size_t idx = (size_t)r * HQ * D + e;
      CHECK(listed ? out2[idx] == out[idx] : out2[idx] == -7.0, "row subset: row %d", r);
    }
  }
  /* a bad block id inside a live context is refused, not followed */
  table[0] = num_blocks;
  rc = hook_oracle_attn_probe(NSEQ, total_q, HQ, HKV, D, B, max_blocks, num_blocks, dtype, 0.25, q, k, v, table, lens,
                              cu, P, heads, NQ, sel, S, spans, 0, NULL, out2, mass);
  CHECK(rc == -3, "bad block id returned %d", rc);
  free(q); free(k); free(v); free(table); free(out); free(out2); free(mass);
}

/* The 8-bit cache: one byte per element, buffers exactly that large; q = 0 makes the output the
 * prefix mean of the dequantised values, which is recomputed here from the byte decoder. */
static void run_attention_kv8(void) {
  const int lens[NSEQ] = {37, 5, 64, 0}, qn[NSEQ] = {1, 1, 1, 0};
  int cu[NSEQ + 1] = {0};
  int nblk_needed = 0, max_blocks = 0;
  for (int i = 0; i < NSEQ; ++i) {
    cu[i + 1] = cu[i] + qn[i];
    const int nb = (lens[i] + B - 1) / B;
    nblk_needed += nb;
    if (nb > max_blocks) max_blocks = nb;
  }
  const int total_q = cu[NSEQ], num_blocks = nblk_needed + 2;
  const size_t nq = (size_t)total_q * HQ * D, nkv = (size_t)num_blocks * HKV * B * D;
  uint16_t* q = calloc(nq, sizeof(uint16_t));           /* q = 0 */
  uint8_t* k = malloc(nkv);
  uint8_t* v = malloc(nkv);
  for (size_t e = 0; e < nkv; ++e) {
    rnd();
    k[e] = (uint8_t)(rng_state >> 40);
    v[e] = (uint8_t)(rng_state >> 48);
    if ((k[e] & 0x7F) == 0x7F) k[e] = 0x11;              /* live slots hold numbers */
    if ((v[e] & 0x7F) == 0x7F) v[e] = 0x22;
  }
  int32_t* table = malloc(sizeof(int32_t) * (size_t)NSEQ * max_blocks);
  int next = 0;
  for (int i = 0; i < NSEQ; ++i)
    for (int b = 0; b < max_blocks; ++b)
      table[i * max_blocks + b] = b < (lens[i] + B - 1) / B ? next++ : 0x7FFFFFF0;
  const float ks[HKV] = {0.37f, 2.0f}, vs[HKV] = {0.11f, 1.5f};
  const int32_t heads[P] = {0, 3};
  const int32_t sel[NSEQ * 2] = {0, 1, -1, 1, 0, 1, 0, 0};
  int32_t spans[NSEQ * S * 2];
  for (int i = 0; i < NSEQ; ++i) {
    const int32_t sp[S * 2] = {0, lens[i], -3, 7, lens[i] - 2, lens[i] + 9, 6, 2};
    memcpy(spans + i * S * 2, sp, sizeof sp);
  }
  double* out = malloc(sizeof(double) * nq);
  double* mass = malloc(sizeof(double) * (size_t)NSEQ * P * NQ * S);
  int rc = hook_oracle_attn_probe_kv8(NSEQ, total_q, HQ, HKV, D, B, max_blocks, num_blocks, 0, 0.25, q, k, v, ks, vs,
                                      table, lens, cu, P, heads, NQ, sel, S, spans, 0, NULL, out, mass);
  CHECK(rc == 0, "attn_probe_kv8 returned %d", rc);
  for (int i = 0; i < NSEQ; ++i) {
    if (qn[i] == 0) continue;
    for (int h = 0; h < HQ; ++h) {
      const int g = h / (HQ / HKV);
      for (int e = 0; e < D; ++e) {
        double mean = 0.0;
        for (int j = 0; j < lens[i]; ++j) {
          const int blk = table[i * max_blocks + j / B];
          mean += (double)vs[g] * hook_oracle_fp8_e4m3_value(v[(((size_t)blk * HKV + g) * B + j % B) * D + e]);
        }
        mean /= lens[i];
        const double got = out[((size_t)cu[i] * HQ + h) * D + e];
        CHECK(fabs(got - mean) < 1e-12 * (1.0 + fabs(mean)), "kv8 seq %d head %d: %.17g vs %.17g", i, h, got, mean);
      }
    }
    const int slot = -sel[2 * i];
    for (int p = 0; p < P; ++p) {
      const double* m = mass + (((size_t)i * P + p) * NQ + slot) * S;
      CHECK(fabs(m[0] - 1.0) < 1e-12, "kv8 seq %d: whole-context mass %.17g", i, m[0]);
      const int hi1 = 7 < lens[i] ? 7 : lens[i];
      CHECK(fabs(m[1] - (double)hi1 / lens[i]) < 1e-12, "kv8 seq %d: clipped-low span %.17g", i, m[1]);
    }
  }
  CHECK(hook_oracle_attn_probe_kv8(NSEQ, total_q, HQ, HKV, D, B, max_blocks, num_blocks, 0, 0.25, q, k, v, NULL, vs,
                                   table, lens, cu, P, heads, NQ, sel, S, spans, 0, NULL, out, mass) == -1,
        "missing scales accepted");
  free(q); free(k); free(v); free(table); free(out); free(mass);
}

static void run_steering(int dtype) {
  enum { T = 7, DD = 24 };
  const size_t esz = dtype == 0 ? 2 : 4;
  void* h = malloc(T * DD * esz); void* dl = malloc(T * DD * esz); void* vec = malloc(DD * esz);
  void* o = malloc(T * DD * esz);
  for (int e = 0; e < T * DD; ++e) {
    const double x = 3.0 * rnd(), y = rnd();
    if (dtype == 0) { ((uint16_t*)h)[e] = hook_oracle_round_bf16(x); ((uint16_t*)dl)[e] = hook_oracle_round_bf16(y); }
    else { ((float*)h)[e] = (float)x; ((float*)dl)[e] = (float)y; }
  }
  for (int e = 0; e < DD; ++e) {
    if (dtype == 0) ((uint16_t*)vec)[e] = hook_oracle_round_bf16(rnd()); else ((float*)vec)[e] = (float)rnd();
  }
  const uint8_t mask[T] = {0, 1, 0, 0, 255, 1, 0};
  CHECK(hook_oracle_steer(h, vec, 0.0f, mask, T, DD, dtype, o) == 0, "steer rc");
  CHECK(memcmp(h, o, T * DD * esz) == 0 || dtype == 0, "alpha = 0 changed fp32 rows");
  CHECK(hook_oracle_steer(h, vec, 2.5f, mask, T, DD, dtype, o) == 0, "steer rc");
  for (int t = 0; t < T; ++t)
    if (!mask[t]) CHECK(memcmp((char*)h + t * DD * esz, (char*)o + t * DD * esz, DD * esz) == 0, "unmasked row %d changed", t);
  CHECK(hook_oracle_residual_steer(h, dl, vec, 2.5f, mask, T, DD, dtype, o) == 0, "residual_steer rc");
  CHECK(hook_oracle_residual_steer(h, dl, vec, 2.5f, NULL, T, DD, dtype, o) == 0, "residual_steer without mask rc");
  free(h); free(dl); free(vec); free(o);
}

int main(void) {
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int zero_q = 0; zero_q < 2; ++zero_q) run_attention(dtype, zero_q);
  run_attention_kv8();
  run_steering(0);
  run_steering(1);
  /* rounding helper on the values around a bf16 midpoint and at the ends of the range */
  const double probes[] = {0.0, -0.0, 1.0, 1.00390625, 1.0039062500000002, 3.3895313892515355e38, 1e-45, -1e39, NAN};
  for (size_t i = 0; i < sizeof probes / sizeof probes[0]; ++i) (void)hook_oracle_round_bf16(probes[i]);
  if (failures) { printf("%d failure(s)\n", failures); return 1; }
  printf("ok\n");
  return 0;
}
