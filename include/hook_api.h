/*
 * hook_api.h - C ABI of the hooked paged-attention library for MI355X (gfx950).
 *
 * Two operations, both asynchronous on a caller-supplied HIP stream:
 *
 *   hook_attn_probe  causal grouped-query attention forward over a paged KV
 *                    cache which, for configured heads, also returns the softmax
 *                    attention mass that chosen query rows place on chosen key
 *                    spans.  This is the statistic the paper's passive
 *                    programming obtains by saving q and all k of the configured
 *                    [layer, head] pairs and recomputing attention afterwards
 *                    (Section 2.1 worker hook; Section 2.2 analyzer, "recompute
 *                    selective attentions" and the per-prompt token ranges of
 *                    `input_range`), here reduced inside the attention kernel so
 *                    that neither q/k copies nor the probability matrix reach
 *                    memory.  The attention output is unaffected by probing
 *                    (Section 1: passive programming keeps generation intact).
 *
 *   hook_steer       residual-stream steering, hidden[t,:] += alpha * vec[:] on
 *                    masked tokens (Section 1, "Model Steering": a steering
 *                    vector injected into a layer's activations).
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer unless stated otherwise.  The
 *     caller owns all buffers; the library allocates no device memory, keeps no
 *     state between calls and never synchronises the stream.  The host reads only
 *     the scalar fields, so a call is a fixed sequence of kernel launches.
 *   - Inputs are read-only.  The only writes are `out`, `mass`, `workspace`
 *     (hook_attn_probe) and `hidden` (hook_steer).
 *   - Errors are returned as hook_status; nothing is launched or written when a
 *     call is rejected.  Contents of device arrays (block ids, lengths) cannot be
 *     checked without a sync: block ids outside [0, num_blocks) are clamped so a
 *     bad table cannot fault, lengths beyond the table are clamped, and the
 *     condition is recorded in the workspace (see hook_attn_probe_device_status;
 *     hook_attn_probe_validate checks the contents on request).
 *   - One call covers one layer; [layer, head] lists (Section 2, config example)
 *     are split per layer by the caller.
 */
#ifndef HOOK_API_H_
#define HOOK_API_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default)   /* the library itself is built with hidden visibility */
#endif

typedef enum {
  HOOK_OK = 0,
  HOOK_ERR_NULL = 1,         /* a required pointer is null */
  HOOK_ERR_SHAPE = 2,        /* negative / inconsistent sizes */
  HOOK_ERR_UNSUPPORTED = 3,  /* dtype, head_dim, block_size or limits not supported */
  HOOK_ERR_WORKSPACE = 4,    /* workspace missing, misaligned or too small */
  HOOK_ERR_LAUNCH = 5        /* the HIP runtime refused a launch */
} hook_status;

typedef enum { HOOK_BF16 = 0, HOOK_F32 = 1 } hook_dtype;

/*
 * Element type of the key/value caches when it differs from `dtype` (a quantised cache).
 * HOOK_KV_FP8_E4M3: one byte per element in the 8-bit E4M3 format (1 sign, 4 exponent, 3 mantissa
 * bits, bias 7, no infinities, NaN = S.1111.111); the element a byte stands for is its value times
 * the fp32 scale of its kv head: K[j][c] = value(k_cache byte) * k_scale[g], V alike with v_scale.
 * Needs HOOK_BF16 queries; the cache layout stays [num_blocks, Hkv, B, d] with one byte per
 * element.  Any batch is served: single rows stream the bytes as they are (the bandwidth-bound
 * case the format pays for), query chunks widen them to bf16 on their way into local memory, so a
 * chunked prefill can run on the same cache.  hook_span_mass takes it as well (k_scale).  The paper does not
 * discuss cache precision; this is the usual serving option of halving the bytes a decode step
 * streams.
 */
typedef enum { HOOK_KV_SAME = 0, HOOK_KV_FP8_E4M3 = 1 } hook_kv_dtype;

/*
 * Composition of a batch, as far as the caller knows it.  The library never reads the sequence
 * lengths on the host, so without a hint every call launches both the kernel for query chunks
 * (n_i >= 2) and the pair for single rows (n_i == 1), one of which may find nothing to do.
 * With a hint the launches that cannot have work are left out (two of four for a prefill-only
 * batch).  A sequence that contradicts the hint is NOT computed: its rows of `out` stay untouched,
 * its `mass` entries are zero and bit 3 of the device status word is set.
 * A small HOOK_BATCH_DECODE_ONLY batch (HOOK_BF16, at most 512 (sequence, kv head, head group)
 * triples, i.e. up to 64 sequences at 8 kv heads) plans itself: every sequence is cut into the same
 * number of parts, the workgroups read the lengths themselves and the planning launch is left out
 * (two launches instead of three).  Results are the same to rounding order; the status word is
 * written as always.  A HOOK_BATCH_PREFILL_ONLY call that holds ONE sequence (a single prompt;
 * HOOK_BF16, head_dim 128) needs no planning launch either: the chunk kernel works out its row
 * blocks itself, with results bit for bit those of the planned call.
 */
typedef enum hook_batch_kind {
  HOOK_BATCH_MIXED = 0,         /* anything (default) */
  HOOK_BATCH_PREFILL_ONLY = 1,  /* every n_i is 0 or >= 2 */
  HOOK_BATCH_DECODE_ONLY = 2    /* every n_i is 0 or 1 */
} hook_batch_kind;

/*
 * The work lists in the workspace depend only on the batch description (seq_lens, cu_q_lens, the
 * shape fields and batch_kind), not on q, the caches or the probe arguments, and every layer of a
 * model step sees the same batch.  HOOK_PLAN_REUSE tells a call that the workspace still holds the
 * lists a HOOK_PLAN_FRESH call wrote for exactly this batch: the planning kernel is left out.
 * Because that kernel is also what zero-fills `mass`, a reusing call writes only the entries of
 * valid selected rows and leaves every other entry of `mass` as it is (give it a zeroed buffer
 * once; those entries are never written afterwards).  Reusing lists of a different batch is a
 * caller error that is not detected.
 */
typedef enum hook_plan_mode {
  HOOK_PLAN_FRESH = 0,   /* plan this call (default) */
  HOOK_PLAN_REUSE = 1    /* the workspace holds the plan of the same batch */
} hook_plan_mode;

#define HOOK_MAX_SPANS 8      /* S: key spans per sequence (hook_attn_probe) */
#define HOOK_MAX_SPANS_WIDE 1024  /* S for hook_span_mass and hook_reduce_mass */
#define HOOK_MAX_SEL_Q 65536  /* NQ: selected query rows per sequence */
#define HOOK_BLOCK_SIZE 16    /* tokens per KV-cache block */

/*
 * Arguments of hook_attn_probe.
 *
 * Shapes: Hq = num_q_heads, Hkv = num_kv_heads (Hq % Hkv == 0; q head h reads kv
 * head h / (Hq / Hkv)), d = head_dim (64 or 128, both dtypes),
 * B = block_size (must be 16).
 *
 * Sequence i has L_i = seq_lens[i] tokens of context INCLUDING its n_i new
 * tokens, whose keys/values are already in the cache.  Its query rows are rows
 * cu_q_lens[i] .. cu_q_lens[i+1]-1 of `q`; chunk-local row t sits at absolute
 * position pos = L_i - n_i + t and attends to keys 0..pos.  n_i = 0 is allowed
 * (the sequence is skipped); n_i > L_i is invalid.
 *
 * Key j of sequence i, kv head g lives at
 *   k_cache[block_table[i, j / B], g, j % B, :]      (v_cache likewise).
 *
 * Probe: for p in [0, P), head probe_heads[p]; for chunk-local rows t in
 * [query_sel[i,0], query_sel[i,1]) (at most max_sel_q rows); for span r with
 * [a, b) = key_spans[i, r, :] in absolute key positions:
 *   mass[i, p, t - query_sel[i,0], r] = sum of softmax probabilities of row t
 *                                       over keys max(a,0) .. min(b, pos+1)-1.
 * Entries with no selected row or an empty span (a >= b after clipping) are 0.
 * Spans may overlap; they are independent.
 *
 * query_sel[i] is any half-open range of chunk-local row numbers.  It is clipped to the rows
 * the chunk has, [0, n_i), and to max_sel_q slots: the rows that count are
 *   t in [max(begin, 0), min(end, n_i, begin + max_sel_q)),
 * and row t ALWAYS lands in slot t - begin.  So begin < 0 is valid (a range written relative to
 * a longer prompt of which this chunk holds the tail): the first -begin slots stay 0.  end <=
 * begin selects nothing.  Every kernel (query chunks, single rows, hook_span_mass,
 * hook_capture_qk) and hook_reduce_mass follow this one rule.
 */
typedef struct hook_attn_probe_args {
  /* shapes (host scalars) */
  int32_t num_seqs;
  int32_t total_q;             /* rows of q = cu_q_lens[num_seqs] */
  int32_t num_q_heads;
  int32_t num_kv_heads;
  int32_t head_dim;
  int32_t block_size;
  int32_t max_blocks_per_seq;  /* row length of block_table; bounds every L_i by max_blocks_per_seq * B */
  int32_t num_blocks;          /* blocks in k_cache / v_cache */
  int32_t dtype;               /* hook_dtype of q, k_cache, v_cache, out */
  float   scale;               /* softmax scale; <= 0 selects 1/sqrt(head_dim) */

  /* inputs (device, borrowed) */
  const void*    q;            /* [total_q, Hq, d], sequences back to back */
  const void*    k_cache;      /* [num_blocks, Hkv, B, d] */
  const void*    v_cache;      /* [num_blocks, Hkv, B, d] */
  const int32_t* block_table;  /* [num_seqs, max_blocks_per_seq] */
  const int32_t* seq_lens;     /* [num_seqs] */
  const int32_t* cu_q_lens;    /* [num_seqs + 1], cu_q_lens[0] = 0 */

  /* probe (num_probe_heads == 0 disables probing; the arrays may then be null) */
  int32_t        num_probe_heads;  /* P <= Hq */
  const int32_t* probe_heads;      /* [P] q-head indices, strictly increasing */
  int32_t        max_sel_q;        /* NQ, 1..HOOK_MAX_SEL_Q */
  const int32_t* query_sel;        /* [num_seqs, 2] */
  int32_t        max_spans;        /* S, 1..HOOK_MAX_SPANS */
  const int32_t* key_spans;        /* [num_seqs, S, 2] */

  /* outputs (device, caller-allocated) */
  void*  out;                  /* [total_q, Hq, d], dtype as q; rows of skipped sequences untouched */
  float* mass;                 /* [num_seqs, P, NQ, S] fp32; fully written (zeros where unused) by a
                                  HOOK_PLAN_FRESH call; a HOOK_PLAN_REUSE call writes only the entries
                                  of selected rows (see hook_plan_mode) */

  /* scratch (device, caller-allocated, 256-byte aligned) and stream */
  void*  workspace;
  size_t workspace_bytes;      /* >= hook_attn_probe_workspace_bytes(args) */
  void*  stream;               /* hipStream_t; null = the default stream */

  /* what the caller knows about the batch (it built cu_q_lens on the host); 0 is always valid */
  int32_t batch_kind;          /* hook_batch_kind */
  int32_t plan_mode;           /* hook_plan_mode */

  /* quantised key/value cache (all zero / null: the caches hold `dtype` elements) */
  int32_t      kv_dtype;       /* hook_kv_dtype */
  const float* k_scale;        /* [Hkv] fp32, device: key element = stored value * k_scale[g] */
  const float* v_scale;        /* [Hkv] fp32, device */

  /* optional: the new tokens' keys and values, [total_q, Hkv, d] of `dtype`, device.  When both are
     given the call first writes them into k_cache / v_cache at positions L_i - n_i + t (exactly what
     hook_kv_write does, quantising for an 8-bit cache) and only then reads the caches - inside the
     planning launch where the call has one, else in a launch of its own ahead of the attention
     kernels: the one place where the call writes through k_cache / v_cache. */
  const void*  k_new;
  const void*  v_new;
} hook_attn_probe_args;

/*
 * Bytes of workspace hook_attn_probe needs for these shapes.  Reads only the
 * scalar shape fields (num_seqs, total_q, head counts, head_dim,
 * max_blocks_per_seq, max_spans, dtype); returns 0 if they are unsupported.
 */
size_t hook_attn_probe_workspace_bytes(const hook_attn_probe_args* args);

/*
 * Launches the attention + probe kernels on args->stream and returns without
 * waiting.  Sequences with one query row take a split-key decode path whose
 * partial results are merged by a combine kernel; longer chunks take the tiled
 * prefill path; both may be mixed in one call.  Results are deterministic: the
 * same inputs (batch_kind included: a hint may change how single rows are split,
 * which changes the order of the sums) give bit-identical `out` and `mass` on
 * every call, for any physical block permutation, and `out` does not depend on
 * the probe arguments.
 * HOOK_F32 inputs take one full-precision kernel that needs no work lists: batch_kind and plan_mode
 * are ignored for them (every valid sequence is computed and `mass` is zero-filled on every call);
 * the status word is written as for bf16 (bits 0-2).
 */
hook_status hook_attn_probe(const hook_attn_probe_args* args);

/*
 * hook_attn_probe for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  The same
 * launches with the same results bit for bit, but the work lists and decode partial results live
 * in a fixed array of HOOK_STATIC_SCRATCH_BYTES that is part of the library's device image (every
 * GPU the library runs on holds its own copy until the process ends).  args->workspace and
 * args->workspace_bytes are ignored; inputs and outputs are still the caller's.  The call makes no
 * allocation of any kind (no hipMalloc / hipFree, no events, no host containers).
 *   - A batch whose hook_attn_probe_workspace_bytes() exceeds HOOK_STATIC_SCRATCH_BYTES is
 *     refused with HOOK_ERR_WORKSPACE before anything is launched (the five reference batches,
 *     up to 256 decode rows of 8192 tokens or one 32768-row prefill, need under 10 MB).
 *   - All calls on one GPU share the one array: calls that may overlap in time (different streams,
 *     different host threads) race on it.  Serialise them, or give the overlapping ones a
 *     workspace of their own through hook_attn_probe.
 *   - The array keeps what the last call left.  Nothing in it needs to start at zero: a
 *     HOOK_PLAN_FRESH call rewrites every word it later reads; HOOK_PLAN_REUSE reuses the lists
 *     of the previous static call on this GPU and is valid only if that call was for this batch.
 *   - hook_attn_probe_device_status cannot reach the array; use hook_attn_probe to debug.
 *   - The first call on a GPU asks the runtime for the array's address on that GPU (once, kept per
 *     device); make that call outside graph capture, as any warm-up call does.
 */
#define HOOK_STATIC_SCRATCH_BYTES (16u << 20)
hook_status hook_attn_probe_static(const hook_attn_probe_args* args);

/* HOOK_STATIC_SCRATCH_BYTES of the library that is loaded (host only). */
size_t hook_attn_probe_static_capacity(void);

/*
 * Debug aid: copies the device-side status word of the last hook_attn_probe
 * call that used `workspace` back to the host (this SYNCHRONISES the stream).
 * *status_bits: bit 0 = some n_i > L_i (sequence skipped), bit 1 = some L_i
 * exceeded max_blocks_per_seq * B (clamped), bit 2 = negative length, bit 3 = a sequence
 * contradicted batch_kind (not computed).
 */
hook_status hook_attn_probe_device_status(const void* workspace, void* stream, int32_t* status_bits);

/*
 * Debug aid: checks, on the device, the array CONTENTS that hook_attn_probe cannot verify
 * without a sync and therefore only makes safe (the conventions at the top of this file), and
 * returns what it found in *problem_bits (0 = nothing).  Reads the same argument struct; uses
 * one word of the first 64 bytes of `workspace` (256-byte aligned; a word of its own, so the
 * status word that hook_attn_probe_device_status reads is left alone); launches one small kernel
 * on `stream` and SYNCHRONISES it.  Not a fast path: one
 * workgroup walks every length, every block id of the live contexts, the probed-head list and
 * the row selections.  q, k_cache, v_cache, key_spans, out and mass are not touched.
 */
typedef enum hook_problem {
  HOOK_BAD_ROWS_EXCEED_CONTEXT = 1,  /* some n_i > L_i                                        */
  HOOK_BAD_CONTEXT_TOO_LONG = 2,     /* some L_i > max_blocks_per_seq * block_size            */
  HOOK_BAD_LENGTH = 4,               /* negative L_i or n_i, cu_q_lens not 0 ... total_q      */
  HOOK_BAD_BATCH_KIND = 8,           /* a sequence contradicts batch_kind                     */
  HOOK_BAD_BLOCK_ID = 16,            /* a block id of a live context outside [0, num_blocks)  */
  HOOK_BAD_PROBE_HEADS = 32,         /* probe_heads not strictly increasing or out of range   */
  HOOK_BAD_QUERY_SEL = 64            /* a query_sel range whose rows inside the chunk do not all fit
                                        max_sel_q slots (slot = t - begin): rows are dropped.  A
                                        range that merely reaches outside [0, n_i) is clipped and
                                        is not reported                                        */
} hook_problem;

hook_status hook_attn_probe_validate(const hook_attn_probe_args* args, int32_t* problem_bits);

/*
 * hidden[t, :] += alpha * vec[:] for every row t with token_mask[t] != 0,
 * computed as one fp32 fused multiply-add per element and rounded to the storage
 * dtype with round-to-nearest-even.  Rows with token_mask[t] == 0 are neither
 * read nor written.  alpha == 0 returns HOOK_OK without launching, so the buffer
 * stays bit-identical (signed zeros and NaN payloads included).
 *   hidden      [num_tokens, hidden_dim], in place, device
 *   vec         [hidden_dim], dtype of hidden, device
 *   token_mask  [num_tokens] bytes, device
 * hidden_dim must be a multiple of 8 (bf16) or 4 (f32).
 */
hook_status hook_steer(void* hidden, const void* vec, float alpha, const uint8_t* token_mask,
                       int32_t num_tokens, int32_t hidden_dim, int32_t dtype, void* stream);

/*
 * Steering folded into the residual add that produces the hidden state (the producer of the
 * activations that Section 1 "Model Steering" / Section 3 modify), so the steered rows cost
 * no memory traffic of their own:
 *   hidden[t, :] = hidden[t, :] + delta[t, :]                          for every row t
 *                  + alpha * vec[:]   on rows with token_mask[t] != 0
 * The terms are added in fp64 (alpha * vec is exact there) and rounded ONCE to the storage
 * dtype, round-to-nearest-even.  token_mask may be null and alpha may be 0: then this is the
 * plain residual add (vec is not read).
 *   hidden      [num_tokens, hidden_dim], in place, device
 *   delta       [num_tokens, hidden_dim], dtype of hidden, device, read only
 *   vec         [hidden_dim], dtype of hidden, device
 *   token_mask  [num_tokens] bytes, device, or null
 * hidden_dim must be a multiple of 8 (bf16) or 4 (f32); hidden, delta, vec 16-byte aligned.
 */
hook_status hook_residual_add_steer(void* hidden, const void* delta, const void* vec, float alpha,
                                    const uint8_t* token_mask, int32_t num_tokens, int32_t hidden_dim,
                                    int32_t dtype, void* stream);

/*
 * Compact q/k capture: the literal output of the paper's passive hook (Section 2.1, qkv_hook:
 * per hooked layer the queries of the last token or of all tokens and ALL keys, split per
 * batch item), gathered on the device into dense buffers instead of being copied out whole.
 *   q_out[i, p, t - query_sel[i,0], :] = q[cu_q_lens[i] + t, probe_heads[p], :]
 *       for t in [query_sel[i,0], query_sel[i,1]) (at most max_sel_q rows, chunk-local);
 *       entries without a selected row are zero-filled.
 *   k_out[cu_k_lens[i] + j, c, :] = k_cache[block_table[i, j / B], capture_kv_heads[c], j % B, :]
 *       for j in [0, L_i): the keys of the chosen kv heads, sequences back to back.
 * All arrays are DEVICE pointers, caller-owned; cu_k_lens holds the prefix sums of seq_lens
 * (cu_k_lens[num_seqs] = total_k, which the host needs anyway to size k_out).  Pure data
 * movement: outputs are bit-identical to the inputs they copy (the keys of an 8-bit cache as its
 * bytes, see kv_dtype).  Asynchronous on `stream`.
 * Block ids outside [0, num_blocks) are clamped as in hook_attn_probe.
 */
typedef struct hook_capture_qk_args {
  int32_t num_seqs, total_q, num_q_heads, num_kv_heads, head_dim, block_size;
  int32_t max_blocks_per_seq, num_blocks, dtype;
  const void*    q;                 /* [total_q, Hq, d] */
  const void*    k_cache;           /* [num_blocks, Hkv, B, d] */
  const int32_t* block_table;       /* [num_seqs, max_blocks_per_seq] */
  const int32_t* seq_lens;          /* [num_seqs] */
  const int32_t* cu_q_lens;         /* [num_seqs + 1] */
  int32_t        num_probe_heads;   /* P (0: no q capture) */
  const int32_t* probe_heads;       /* [P] */
  int32_t        max_sel_q;         /* NQ */
  const int32_t* query_sel;         /* [num_seqs, 2] */
  int32_t        num_capture_kv_heads;  /* KH (0: no k capture) */
  const int32_t* capture_kv_heads;  /* [KH] kv head indices */
  const int32_t* cu_k_lens;         /* [num_seqs + 1] */
  int32_t        total_k;
  void* q_out;                      /* [num_seqs, P, NQ, d] */
  void* k_out;                      /* [total_k, KH, d] */
  void* stream;
  int32_t kv_dtype;                 /* hook_kv_dtype of k_cache; with HOOK_KV_FP8_E4M3 k_out holds the
                                       cache's bytes as they are ([total_k, KH, d] bytes; the caller has
                                       the scales) */
} hook_capture_qk_args;

hook_status hook_capture_qk(const hook_capture_qk_args* args);

/*
 * Writes the keys and values of the new tokens into the paged cache, which hook_attn_probe expects
 * to find there (it takes no separate new-token K/V): for sequence i and chunk-local row t,
 *   pos = L_i - n_i + t,
 *   k_cache[block_table[i, pos / B], g, pos % B, :] = k_new[cu_q_lens[i] + t, g, :]   for every kv head g
 * and likewise for v.  Pure data movement (bit-identical copies), asynchronous on `stream`.
 * Sequences with n_i > L_i, negative lengths or rows outside [0, total_q) are skipped; a block id
 * outside [0, num_blocks) or a position beyond max_blocks_per_seq * B drops that token's write
 * (nothing outside the cache is ever written).  Two sequences must not own the same block.
 *   k_new, v_new   [total_q, Hkv, d], dtype `dtype`, device
 * With kv_dtype = HOOK_KV_FP8_E4M3 the rows (bf16) are quantised on the way: stored byte = the E4M3
 * number nearest to fl32(x / scale[g]) clamped to [-448, 448] (the format has no infinities), ties to
 * the even mantissa, sign kept, NaN -> NaN; the inverse of the dequantisation hook_attn_probe applies.
 * hook_attn_probe can do this write itself (its k_new / v_new fields) and save the launch.
 */
typedef struct hook_kv_write_args {
  int32_t num_seqs, total_q, num_kv_heads, head_dim, block_size, max_blocks_per_seq, num_blocks;
  int32_t dtype;
  const void*    k_new;
  const void*    v_new;
  const int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* cu_q_lens;
  void*          k_cache;
  void*          v_cache;
  void*          stream;
  /* quantising write into an 8-bit cache (all zero / null: the cache holds `dtype` elements) */
  int32_t        kv_dtype;     /* hook_kv_dtype; HOOK_KV_FP8_E4M3 needs dtype = HOOK_BF16 */
  const float*   k_scale;      /* [Hkv] fp32, device */
  const float*   v_scale;      /* [Hkv] fp32, device */
} hook_kv_write_args;

hook_status hook_kv_write(const hook_kv_write_args* args);

/*
 * Attention mass for many spans: the re-ranking shape of Section 3 (selective attention-based
 * retrieval: attention from the query tokens of selected heads onto each document gives the
 * document's relevance), i.e. tens to hundreds of spans x many query rows x a few heads.
 * Takes the SAME argument struct as hook_attn_probe and writes the same
 *   mass[i, p, t - query_sel[i,0], r]
 * (identical definition, clipping and zero fill), but
 *   - max_spans may be up to HOOK_MAX_SPANS_WIDE,
 *   - no attention output is computed: out and v_cache are ignored (run hook_attn_probe with
 *     num_probe_heads = 0 for the output),
 *   - workspace is optional scratch: with at least hook_span_mass_workspace_bytes(args) bytes (8-byte
 *     aligned) the two passes run as two kernels split over keys and spans and use the whole chip;
 *     without it one workgroup per (sequence, head, 16 rows) does everything (same results to
 *     rounding, several times slower on long sequences),
 *   - only HOOK_BF16 inputs are supported (HOOK_ERR_UNSUPPORTED otherwise); the key cache may be
 *     8-bit (kv_dtype, k_scale; v_scale is not read),
 * Two passes over the keys of each (sequence, probed head, 16-row block): exact softmax maximum
 * and normaliser first, then the span sums; no atomics, results reproducible bit for bit.
 * A content-free calibration prompt is a second call; hook_reduce_mass with negated weights
 * subtracts it.
 */
hook_status hook_span_mass(const hook_attn_probe_args* args);

/* Scratch bytes that let hook_span_mass take its split path (0: not available for these shapes). */
size_t hook_span_mass_workspace_bytes(const hook_attn_probe_args* args);

/*
 * Score reductions over the mass tensor of one hook_attn_probe call (Section 2.2, analyzer:
 * the captured attention is aggregated over the token ranges of each prompt and reduced to a
 * score; Section 2, config file: the reduction is an average or a weighted sum; Section 3:
 * focus score of the important heads on the instruction, per-document relevance for the
 * re-ranker).  The paper elides the formula, so the reading is a choice of the caller:
 *   HOOK_REDUCE_SPAN_MEAN      scores[i, r] = sum_p w_p * mean_t mass[i, p, t, r]        [num_seqs, S]
 *   HOOK_REDUCE_RATIO_MEAN     scores[i] = sum_p w_p * mean_t a / (a + b)                [num_seqs]
 *   HOOK_REDUCE_RATIO_OF_SUMS  scores[i] = A / (A + B), A = sum_p w_p * mean_t a, B alike [num_seqs]
 * with a = mass[i, p, t, span_a], b = mass[i, p, t, span_b]; a ratio whose denominator is 0
 * counts as 0.  mean_t runs over the slots that hold a row the probe call selected for sequence
 * i, i.e. slots t - begin for t in [max(begin, 0), min(end, n_i, begin + NQ)) with [begin, end)
 * = query_sel[i] (leading slots of a negative begin hold no row and do not count), or over all
 * NQ slots when query_sel is null; a sequence without selected rows scores 0.  w_p is
 * head_weights[p], or 1 / P (the average) when head_weights is null.  With accumulate != 0
 * the result is added to `scores` instead of stored, which sums layers (one call each, the
 * layer weight folded into head_weights) and subtracts a calibration pass (negated weights).
 * Sums run in fp32 in a fixed order, so results are reproducible bit for bit.
 * All arrays are DEVICE pointers, caller-owned; asynchronous on `stream`.
 */
typedef enum hook_reduce_mode {
  HOOK_REDUCE_SPAN_MEAN = 0,
  HOOK_REDUCE_RATIO_MEAN = 1,
  HOOK_REDUCE_RATIO_OF_SUMS = 2
} hook_reduce_mode;

typedef struct hook_reduce_args {
  int32_t num_seqs, num_probe_heads, max_sel_q, max_spans;   /* shape of mass: [num_seqs, P, NQ, S] */
  const float*   mass;
  const int32_t* query_sel;       /* [num_seqs, 2] as passed to the probe call, or null */
  const int32_t* cu_q_lens;       /* [num_seqs + 1] as passed to the probe call, or null (then rows are
                                     limited by query_sel and NQ only) */
  const float*   head_weights;    /* [P] or null */
  int32_t        mode;            /* hook_reduce_mode */
  int32_t        span_a, span_b;  /* ratio modes only: indices in [0, S) */
  int32_t        accumulate;
  float*         scores;          /* [num_seqs, S] (SPAN_MEAN) or [num_seqs] */
  void*          stream;
} hook_reduce_args;

hook_status hook_reduce_mass(const hook_reduce_args* args);

/*
 * Host helper: parses the layer/heads string of the paper's worker configuration
 * (Section 2.1, `_parse_layer_heads`: '0:0,3,6;15:2' means layer 0 heads 0, 3, 6 and layer 15
 * head 2) into (layer, head) pairs in the order written.  All pointers are HOST pointers.
 *   text      NUL-terminated string; blanks around numbers and empty ';' parts are ignored
 *   layers, heads   arrays of `capacity` entries (may be null when capacity is 0)
 *   *count    receives the number of pairs in the string, also when it exceeds `capacity`
 * Returns HOOK_ERR_SHAPE for a malformed string (missing ':', empty head list, non-digits,
 * values above 2^30) and HOOK_ERR_WORKSPACE when the pairs do not fit `capacity` (the first
 * `capacity` pairs are written).  One hook_attn_probe call covers one layer: the caller passes
 * the heads of that layer, sorted, as probe_heads.
 */
hook_status hook_parse_layer_heads(const char* text, int32_t* layers, int32_t* heads, int32_t capacity,
                                   int32_t* count);

/*
 * Host helper: reads the JSON configuration file of the hook (Section 2, config file example:
 * "params"/"important_heads" lists the [layer, head] pairs to analyse, "hookq"/"hookq_mode"
 * says whether the query of the last token or of all tokens is wanted).  Everything else in
 * the document is skipped.  All pointers are HOST pointers.
 *   text         NUL-terminated JSON text whose top level is an object
 *   layers, heads, capacity, *count   as for hook_parse_layer_heads, pairs in file order
 *   *hookq_mode  0 = "last_token", 1 = "all_tokens", -1 = key absent
 * Returns HOOK_ERR_SHAPE for malformed JSON, a pair that is not two non-negative integers, or an
 * unknown mode string; HOOK_ERR_WORKSPACE when the pairs do not fit.  query_sel of a call is
 * [n_i - 1, n_i) for mode 0 and [0, n_i) for mode 1.
 */
hook_status hook_parse_config_json(const char* text, int32_t* layers, int32_t* heads, int32_t capacity,
                                   int32_t* count, int32_t* hookq_mode);

const char* hook_status_string(hook_status status);
int hook_version(void);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* HOOK_API_H_ */
