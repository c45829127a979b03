// Host side of the C ABI declared in include/hook_api.h: argument checks, workspace
// carve-up and the fixed launch sequence.  No device memory is allocated here and the
// stream is never synchronised (except in the explicit debug status call).
#include "../../include/hook_api.h"
#include "hook_device.h"

#include <cmath>

namespace {

using namespace hook;

constexpr size_t kAlign = 256;
// A batch of single rows with at most this many (sequence, kv head, head group) triples plans
// itself: every sequence is cut into the same number of parts and the planning launch, a quarter
// of such a call, is left out.  Larger batches keep the planner, which balances ragged lengths.
constexpr long long kSelfPlanMaxTriples = 512;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t off_hdr, off_pf, off_dec, off_seq, off_part, total;
  int pf_cap, dec_cap, hpw, rows_per_wg, hgroups, dec_hp, dec_hgroups;
};

bool shapes_supported(const hook_attn_probe_args* a) {
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0) return false;
  if (a->max_blocks_per_seq <= 0 || a->num_blocks <= 0) return false;
  if (a->num_q_heads % a->num_kv_heads != 0) return false;
  if (a->block_size != HOOK_BLOCK_SIZE) return false;
  if (a->dtype != HOOK_BF16 && a->dtype != HOOK_F32) return false;
  if (a->head_dim != 64 && a->head_dim != 128) return false;
  if (a->max_blocks_per_seq > (1 << 26)) return false;
  return true;
}

// Upper bound on the number of decode items the planner can produce, from host scalars only.
// The planner takes the largest chunk size c in {512, 1024, ..., kMaxChunkKeys} whose item count
// still gives kDecodeFillWgs workgroups, else 256 keys.  Halving a chunk at most doubles a
// sequence's item count, so whenever the next larger size was refused (fewer than kDecodeFillWgs
// workgroups, i.e. at most (kDecodeFillWgs - 1) / wg_per_item items) the chosen size yields at most
// twice that; and the largest size yields at most one item per kMaxChunkKeys keys of the longest
// context the block table allows.  (The 256-key tiling of every context is a bound as well.)
int decode_item_bound(long long num_decode_seqs, long long max_context, int wg_per_item) {
  const long long refused = 2 * ((kDecodeFillWgs - 1) / wg_per_item);
  const long long largest = num_decode_seqs * ((max_context + kMaxChunkKeys - 1) / kMaxChunkKeys);
  const long long finest = num_decode_seqs * ((max_context + 255) / 256);
  long long cap = refused > largest ? refused : largest;
  if (cap > finest) cap = finest;
  if (cap > (1ll << 30)) cap = 1ll << 30;
  return (int)cap;
}

Layout make_layout(const hook_attn_probe_args* a) {
  Layout l{};
  const int G = a->num_q_heads / a->num_kv_heads;
  l.hpw = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  l.rows_per_wg = kWaveRows * (4 / l.hpw);
  l.hgroups = G / l.hpw;
  l.dec_hp = (G % 8 == 0) ? 8 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  l.dec_hgroups = G / l.dec_hp;
  if (a->dtype == HOOK_BF16) {
    l.pf_cap = a->total_q / l.rows_per_wg + a->num_seqs;
    l.dec_cap = decode_item_bound(a->num_seqs < a->total_q ? a->num_seqs : a->total_q,
                                  (long long)a->max_blocks_per_seq * kBlock, a->num_kv_heads * l.dec_hgroups);
  }
  size_t off = 0;
  l.off_hdr = off;  off = align_up(off + sizeof(PlanHeader));
  l.off_pf = off;   off = align_up(off + 2 * sizeof(WorkItem) * (size_t)l.pf_cap);
  l.off_dec = off;  off = align_up(off + 2 * sizeof(WorkItem) * (size_t)l.dec_cap);
  l.off_seq = off;  off = align_up(off + sizeof(int2) * (size_t)(a->num_seqs > 0 ? a->num_seqs : 1));
  l.off_part = off;
  off = align_up(off + sizeof(float) * (size_t)l.dec_cap * a->num_q_heads * (a->head_dim + kPartialPad));
  l.total = off;
  return l;
}

// Parts per sequence of a self-planned batch of single rows, 0 where the planner is kept.  As many
// parts as give one resident round of workgroups (256 compute units times the 3 workgroups each
// holds, 2 for groups of 8 heads): measured on 4-32 sequences of 1-64 k tokens this beats both
// fewer and more (a second, partial round costs more than its finer balance gains).  The records
// of part j of sequence i sit in slot i * parts + j, so the slot capacity of the workspace bounds
// the count as well.
int self_plan_parts(const hook_attn_probe_args* a, const Layout& l) {
  if (a->dtype != HOOK_BF16 || a->batch_kind != HOOK_BATCH_DECODE_ONLY || a->num_seqs <= 0) return 0;
  const long long triples = (long long)a->num_seqs * a->num_kv_heads * l.dec_hgroups;
  if (triples > kSelfPlanMaxTriples) return 0;
  const long long one_round = 256 * (l.dec_hp == 8 ? 2 : 3);
  long long parts = (one_round + triples - 1) / triples;
  if (parts > l.dec_cap / a->num_seqs) parts = l.dec_cap / a->num_seqs;
  return (int)parts;
}

}  // namespace

extern "C" {

size_t hook_attn_probe_workspace_bytes(const hook_attn_probe_args* a) {
  if (!a || !shapes_supported(a)) return 0;
  return make_layout(a).total;
}

}  // extern "C"

namespace hook {
// Validates, carves the workspace and launches.  With `ev` (5 events) the launches are
// bracketed by event records so a profiling caller can read per-kernel durations (used by the
// separate measurement library, which links these objects; not part of the exported ABI).
// Everything about a call that the host can check without its workspace.  HOOK_OK with *nothing_to_do
// set means a valid call that has no work (no sequences or no rows).
__attribute__((visibility("hidden"))) hook_status check_attn_probe_args(const hook_attn_probe_args* a, bool* nothing_to_do) {
  *nothing_to_do = false;
  if (!a) return HOOK_ERR_NULL;
  if (a->num_seqs < 0 || a->total_q < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 ||
      a->max_blocks_per_seq <= 0 || a->num_blocks <= 0 || a->head_dim <= 0)
    return HOOK_ERR_SHAPE;
  if (a->num_q_heads % a->num_kv_heads != 0) return HOOK_ERR_SHAPE;
  if (!shapes_supported(a)) return HOOK_ERR_UNSUPPORTED;
  if (a->batch_kind < HOOK_BATCH_MIXED || a->batch_kind > HOOK_BATCH_DECODE_ONLY) return HOOK_ERR_SHAPE;
  if (a->plan_mode != HOOK_PLAN_FRESH && a->plan_mode != HOOK_PLAN_REUSE) return HOOK_ERR_SHAPE;
  const int P = a->num_probe_heads;
  if (P < 0 || P > a->num_q_heads) return HOOK_ERR_SHAPE;
  if (P > 0) {
    if (a->max_sel_q < 1 || a->max_spans < 1) return HOOK_ERR_SHAPE;
    if (a->max_sel_q > HOOK_MAX_SEL_Q || a->max_spans > HOOK_MAX_SPANS) return HOOK_ERR_UNSUPPORTED;
    if (!a->probe_heads || !a->query_sel || !a->key_spans || !a->mass) return HOOK_ERR_NULL;
  }
  if (a->kv_dtype != HOOK_KV_SAME && a->kv_dtype != HOOK_KV_FP8_E4M3) return HOOK_ERR_SHAPE;
  const bool kv8 = a->kv_dtype == HOOK_KV_FP8_E4M3;
  // the 8-bit cache goes with bf16 queries
  if (kv8 && a->dtype != HOOK_BF16) return HOOK_ERR_UNSUPPORTED;
  if (a->num_seqs == 0 || a->total_q == 0) { *nothing_to_do = true; return HOOK_OK; }
  if (!a->q || !a->k_cache || !a->v_cache || !a->block_table || !a->seq_lens || !a->cu_q_lens || !a->out)
    return HOOK_ERR_NULL;
  if (kv8 && (!a->k_scale || !a->v_scale)) return HOOK_ERR_NULL;
  if ((a->k_new == nullptr) != (a->v_new == nullptr)) return HOOK_ERR_NULL;
  return HOOK_OK;
}

__attribute__((visibility("hidden"))) hook_status run_attn_probe(const hook_attn_probe_args* a, hipEvent_t* ev,
                                                                 void* workspace, size_t workspace_bytes) {
  bool nothing_to_do = false;
  const hook_status checked = check_attn_probe_args(a, &nothing_to_do);
  if (checked != HOOK_OK || nothing_to_do) return checked;
  const int P = a->num_probe_heads;
  const bool kv8 = a->kv_dtype == HOOK_KV_FP8_E4M3;
  const Layout l = make_layout(a);
  // one-dimensional launch grids over the item capacities
  if (a->dtype == HOOK_BF16 &&
      (!grid_fits((long long)l.pf_cap * a->num_kv_heads * l.hgroups) ||
       !grid_fits((long long)l.dec_cap * a->num_kv_heads * l.dec_hgroups)))
    return HOOK_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < l.total || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
    return HOOK_ERR_WORKSPACE;

  AttnParams p{};
  p.num_seqs = a->num_seqs;
  p.total_q = a->total_q;
  p.Hq = a->num_q_heads;
  p.Hkv = a->num_kv_heads;
  p.G = p.Hq / p.Hkv;
  p.max_blocks = a->max_blocks_per_seq;
  p.num_blocks = a->num_blocks;
  const float scale = a->scale > 0.0f ? a->scale : 1.0f / std::sqrt((float)a->head_dim);
  p.scale_log2 = scale * 1.44269504088896340736f;
  p.q = a->q; p.k_cache = a->k_cache; p.v_cache = a->v_cache;
  p.block_table = a->block_table; p.seq_lens = a->seq_lens; p.cu_q_lens = a->cu_q_lens;
  p.P = P;
  p.probe_heads = a->probe_heads;
  p.NQ = P > 0 ? a->max_sel_q : 0;
  p.query_sel = a->query_sel;
  p.S = P > 0 ? a->max_spans : 0;
  p.key_spans = a->key_spans;
  p.out = a->out;
  p.mass = a->mass;
  p.kv8 = kv8 ? 1 : 0;
  p.k_scale = a->k_scale;
  p.v_scale = a->v_scale;
  const bool writes_kv = a->k_new != nullptr;
  if (writes_kv) {
    const int esize = a->dtype == HOOK_BF16 ? 2 : 4;
    KvWriteParams& w = p.kvw;
    w.num_seqs = a->num_seqs; w.total_q = a->total_q; w.Hkv = a->num_kv_heads; w.max_blocks = a->max_blocks_per_seq;
    w.num_blocks = a->num_blocks; w.row_chunks = a->head_dim * esize / 16; w.kv8 = p.kv8;
    w.k_new = static_cast<const uint4*>(a->k_new); w.v_new = static_cast<const uint4*>(a->v_new);
    w.block_table = a->block_table; w.seq_lens = a->seq_lens; w.cu_q_lens = a->cu_q_lens;
    w.k_cache = const_cast<void*>(a->k_cache); w.v_cache = const_cast<void*>(a->v_cache);
    w.k_scale = a->k_scale; w.v_scale = a->v_scale;
  }
  char* ws = static_cast<char*>(workspace);
  p.hdr = reinterpret_cast<PlanHeader*>(ws + l.off_hdr);
  p.pf_items = reinterpret_cast<WorkItem*>(ws + l.off_pf);
  p.pf_cap = l.pf_cap;
  p.dec_items = reinterpret_cast<WorkItem*>(ws + l.off_dec);
  p.dec_cap = l.dec_cap;
  p.seq_dec = reinterpret_cast<int2*>(ws + l.off_seq);
  p.partials = reinterpret_cast<float*>(ws + l.off_part);
  p.hpw = l.hpw; p.rows_per_wg = l.rows_per_wg; p.hgroups = l.hgroups;
  p.dec_hp = l.dec_hp; p.dec_hgroups = l.dec_hgroups;
  p.batch_kind = a->batch_kind;
  p.dec_parts = self_plan_parts(a, l);
  // a single prompt on its own needs no planner either (head_dim 128: the kernel that can plan for itself)
  p.pf_self = a->dtype == HOOK_BF16 && a->head_dim == 128 && !kv8 && a->batch_kind == HOOK_BATCH_PREFILL_ONLY &&
              a->num_seqs == 1;
  p.plan_fresh = a->plan_mode == HOOK_PLAN_FRESH;

  hipStream_t st = static_cast<hipStream_t>(a->stream);
  auto mark = [&](int i) { return !ev || hipEventRecord(ev[i], st) == hipSuccess; };
  if (!mark(0)) return HOOK_ERR_LAUNCH;
  // the planning launch carries the cache write; where there is no such launch it gets its own
  if (writes_kv && (a->dtype == HOOK_F32 || a->plan_mode == HOOK_PLAN_REUSE || p.dec_parts > 0 || p.pf_self) &&
      launch_kv_write(p.kvw, st) != hipSuccess)
    return HOOK_ERR_LAUNCH;
  if (a->dtype == HOOK_F32) {
    if (launch_attn_f32(p, a->head_dim, st) != hipSuccess) return HOOK_ERR_LAUNCH;
    for (int i = 1; i < 5; ++i)
      if (!mark(i)) return HOOK_ERR_LAUNCH;
    return HOOK_OK;
  }
  // a reusing call finds the work lists of the same batch in the workspace; a self-planned batch
  // of single rows needs none
  if ((a->plan_mode == HOOK_PLAN_FRESH && p.dec_parts == 0 && !p.pf_self && launch_plan(p, st) != hipSuccess) || !mark(1))
    return HOOK_ERR_LAUNCH;
  const bool chunks = a->batch_kind != HOOK_BATCH_DECODE_ONLY, singles = a->batch_kind != HOOK_BATCH_PREFILL_ONLY;
  if ((chunks && launch_prefill(p, a->head_dim, st) != hipSuccess) || !mark(2)) return HOOK_ERR_LAUNCH;
  if ((singles && launch_decode(p, a->head_dim, st) != hipSuccess) || !mark(3)) return HOOK_ERR_LAUNCH;
  if ((singles && launch_combine(p, a->head_dim, st) != hipSuccess) || !mark(4)) return HOOK_ERR_LAUNCH;
  return HOOK_OK;
}
}  // namespace hook

using hook::run_attn_probe;

extern "C" {

hook_status hook_attn_probe(const hook_attn_probe_args* a) {
  return a ? run_attn_probe(a, nullptr, a->workspace, a->workspace_bytes) : HOOK_ERR_NULL;
}

// ---- the same call on the library's own scratch memory ---------------------------------------
// Work lists and decode partials live in a fixed array in device memory instead of a caller
// workspace, so the call needs nothing allocated by anybody.  Every GPU holds its own copy of the
// array at its own address; the host learns that address once per device.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[HOOK_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // zero-initialised: address of `scratch` on each device

// Device address of `scratch` on the current device (null on failure).  The array's name is a
// host-side handle, not an address: only the pointer returned here may be given to kernels.
void* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // racing threads store the same value
  return ptr;
}
}  // namespace

size_t hook_attn_probe_static_capacity(void) { return (size_t)HOOK_STATIC_SCRATCH_BYTES; }

hook_status hook_attn_probe_static(const hook_attn_probe_args* a) {
  // the argument and size checks come first, so that a call that is refused never touches the device
  bool nothing_to_do = false;
  const hook_status checked = hook::check_attn_probe_args(a, &nothing_to_do);
  if (checked != HOOK_OK || nothing_to_do) return checked;
  if (make_layout(a).total > (size_t)HOOK_STATIC_SCRATCH_BYTES) return HOOK_ERR_WORKSPACE;
  void* ws = scratch_on_current_device();
  if (!ws) return HOOK_ERR_LAUNCH;
  return run_attn_probe(a, nullptr, ws, (size_t)HOOK_STATIC_SCRATCH_BYTES);
}


hook_status hook_attn_probe_device_status(const void* workspace, void* stream, int32_t* status_bits) {
  if (!workspace || !status_bits) return HOOK_ERR_NULL;
  PlanHeader h{};
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&h, workspace, sizeof h, hipMemcpyDeviceToHost, st) != hipSuccess) return HOOK_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return HOOK_ERR_LAUNCH;
  *status_bits = h.status;
  return HOOK_OK;
}

hook_status hook_steer(void* hidden, const void* vec, float alpha, const uint8_t* token_mask,
                       int32_t num_tokens, int32_t hidden_dim, int32_t dtype, void* stream) {
  if (num_tokens < 0 || hidden_dim < 0) return HOOK_ERR_SHAPE;
  if (dtype != HOOK_BF16 && dtype != HOOK_F32) return HOOK_ERR_UNSUPPORTED;
  if (hidden_dim % (dtype == HOOK_BF16 ? 8 : 4) != 0) return HOOK_ERR_UNSUPPORTED;
  if (num_tokens == 0 || hidden_dim == 0) return HOOK_OK;
  if (!hidden || !vec || !token_mask) return HOOK_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(hidden) | reinterpret_cast<uintptr_t>(vec)) % 16 != 0) return HOOK_ERR_UNSUPPORTED;
  if (alpha == 0.0f) return HOOK_OK;
  return launch_steer(hidden, vec, alpha, token_mask, num_tokens, hidden_dim, dtype,
                      static_cast<hipStream_t>(stream)) == hipSuccess ? HOOK_OK : HOOK_ERR_LAUNCH;
}

hook_status hook_parse_layer_heads(const char* text, int32_t* layers, int32_t* heads, int32_t capacity,
                                   int32_t* count) {
  if (!text || !count || capacity < 0 || (capacity > 0 && (!layers || !heads))) return HOOK_ERR_NULL;
  *count = 0;
  const char* c = text;
  auto skip_blank = [&]() { while (*c == ' ' || *c == '\t' || *c == '\n' || *c == '\r') ++c; };
  auto number = [&](int32_t* out) -> bool {   // blanks, digits, blanks
    skip_blank();
    if (*c < '0' || *c > '9') return false;
    long long v = 0;
    while (*c >= '0' && *c <= '9') {
      v = v * 10 + (*c - '0');
      if (v > (1ll << 30)) return false;
      ++c;
    }
    skip_blank();
    *out = (int32_t)v;
    return true;
  };
  int32_t n = 0;
  for (;;) {
    skip_blank();
    if (*c == '\0') break;
    if (*c == ';') { ++c; continue; }          // empty part
    int32_t layer = 0;
    if (!number(&layer) || *c != ':') return HOOK_ERR_SHAPE;
    ++c;
    int32_t in_part = 0;
    for (;;) {
      int32_t head = 0;
      if (!number(&head)) return HOOK_ERR_SHAPE;
      if (n < capacity) { layers[n] = layer; heads[n] = head; }
      ++n;
      ++in_part;
      if (*c == ',') { ++c; continue; }
      break;
    }
    if (in_part == 0) return HOOK_ERR_SHAPE;
    if (*c == ';') { ++c; continue; }
    if (*c == '\0') break;
    return HOOK_ERR_SHAPE;
  }
  *count = n;
  return n > capacity ? HOOK_ERR_WORKSPACE : HOOK_OK;
}

const char* hook_status_string(hook_status s) {
  switch (s) {
    case HOOK_OK: return "ok";
    case HOOK_ERR_NULL: return "null pointer";
    case HOOK_ERR_SHAPE: return "inconsistent shape";
    case HOOK_ERR_UNSUPPORTED: return "unsupported configuration";
    case HOOK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case HOOK_ERR_LAUNCH: return "kernel launch failed";
  }
  return "unknown status";
}

int hook_version(void) { return 2; }

}  // extern "C"
