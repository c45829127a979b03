// Device-side planner: reads the ragged batch description and writes the work lists the
// attention kernels index with blockIdx.  Keeping this on the device means the host never
// needs the sequence lengths, so a call is a fixed launch sequence.
//
//   prefill items  one per (sequence with n_i >= 2, block of rows_per_wg query rows), ordered
//                  by decreasing number of key tiles (longest first) with a counting sort;
//   decode items   one per (sequence with n_i == 1, chunk of chunk_keys keys); the chunk size
//                  (256..8192) is the largest that still gives the decode grid enough workgroups
//                  to fill the chip; they are processed longest first.
// The same launch zero-fills `mass`.
#include "kv_write_device.h"

namespace hook {

namespace {

constexpr int kPlanThreads = 1024;
constexpr int kListCap = 1024;   // queued prefill sequences
constexpr int kDecBuckets = kMaxChunkKeys / kBlock;   // longest decode chunk in cache blocks

struct SeqInfo { int L, n, row0, kind; };  // kind: 0 skip, 1 prefill, 2 decode

__device__ __forceinline__ SeqInfo read_seq(const AttnParams& p, int i, int* status) {
  SeqInfo s;
  s.L = p.seq_lens[i];
  s.row0 = p.cu_q_lens[i];
  s.n = p.cu_q_lens[i + 1] - s.row0;
  s.kind = 0;
  const int max_ctx = p.max_blocks * kBlock;
  if (s.L < 0 || s.n < 0) { *status |= kStatNegative; return s; }
  if (s.L > max_ctx) { *status |= kStatLenClamped; s.L = max_ctx; }
  if (s.n > s.L) { *status |= kStatQGtL; return s; }
  if (s.row0 < 0 || s.row0 + s.n > p.total_q) { *status |= kStatNegative; return s; }
  if (s.n == 0) return s;
  s.kind = (s.n == 1) ? 2 : 1;
  // a sequence the caller's hint rules out: its kernels are not launched, so it is dropped here
  if ((p.batch_kind == 1 && s.kind == 2) || (p.batch_kind == 2 && s.kind == 1)) {
    *status |= kStatHint;
    s.kind = 0;
  }
  return s;
}

__global__ __launch_bounds__(kPlanThreads) void k_plan(const AttnParams p) {
  const int tid = threadIdx.x;
  // every block helps clearing mass
  const size_t nmass = (size_t)p.num_seqs * p.P * p.NQ * p.S;
  for (size_t i = (size_t)blockIdx.x * kPlanThreads + tid; i < nmass; i += (size_t)gridDim.x * kPlanThreads)
    p.mass[i] = 0.0f;
  if (blockIdx.x != 0) {
    // the spare blocks also write the new tokens' key/value rows into the cache, if the call brings
    // them: the attention kernels are launched after this one, so they find the cache complete
    // (a block works on four tiles of rows at a time, one per group of 256 threads; the trip count
    // is the same for every group because the tile code synchronises the whole block)
    if (p.kvw.k_new != nullptr) {
      constexpr int kGroups = kPlanThreads / 256;
      __shared__ long long dst_row[kGroups][kKvRowTile];
      const int ntiles = (p.kvw.total_q + kKvRowTile - 1) / kKvRowTile;
      const int group = tid >> 8;
      for (int t0 = (blockIdx.x - 1) * kGroups; t0 < ntiles; t0 += (gridDim.x - 1) * kGroups)
        kv_write_tile<256>(p.kvw, t0 + group, tid & 255, dst_row[group]);
    }
    return;
  }

  __shared__ int hist[kPlanBuckets];
  __shared__ int sh_cnt[kChunkSizes];   // number of decode chunks for each candidate size
  __shared__ int sh_status;
  __shared__ int sh_dec_next;
  __shared__ int sh_dec_total;   // decode items actually written
  __shared__ int sh_nlist;
  __shared__ int sh_list[kListCap];
  __shared__ int4 sh_list_info[kListCap];   // {L, n, row0, -} of the queued sequences: read once
  __shared__ int dhist[kDecBuckets + 1];   // decode items by length in cache blocks (<= 2048 / 16)
  __shared__ int sh_wsum[kPlanThreads / 64];

  for (int b = tid; b < kPlanBuckets; b += kPlanThreads) hist[b] = 0;
  if (tid < kChunkSizes) sh_cnt[tid] = 0;
  if (tid == 0) sh_status = 0;
  if (tid <= kDecBuckets) dhist[tid] = 0;
  if (tid == 0) { sh_dec_next = 0; sh_nlist = 0; sh_dec_total = 0; }
  __syncthreads();

  // pass 1: histogram of prefill items by tile count, decode chunk counts per candidate size
  // Decode sequences are handled one per thread.  Prefill sequences are queued (up to
  // kListCap; the overflow is handled by the thread that found it) and then taken one per
  // wave with the lanes spread over the row blocks, so a single long sequence does not loop
  // in one thread.
  const int wave = tid >> 6, lane = tid & 63;
  constexpr int kWaves = kPlanThreads / 64;
  int status = 0;
  int cnt[kChunkSizes];
#pragma unroll
  for (int k = 0; k < kChunkSizes; ++k) cnt[k] = 0;
  SeqInfo my_s;               // the thread's first sequence, kept for the later passes
  my_s.L = my_s.n = my_s.row0 = my_s.kind = 0;
  for (int i = tid; i < p.num_seqs; i += kPlanThreads) {
    const SeqInfo s = read_seq(p, i, &status);
    if (i == tid) my_s = s;
    if (s.kind == 1) {
      const int pos = atomicAdd(&sh_nlist, 1);
      if (pos < kListCap) {
        sh_list[pos] = i;
        sh_list_info[pos] = make_int4(s.L, s.n, s.row0, 0);
      } else {
        for (int r0 = 0; r0 < s.n; r0 += p.rows_per_wg) {
          const int last = min(r0 + p.rows_per_wg, s.n) - 1;
          const int tiles = (s.L - s.n + last) / kTileKeys + 1;
          atomicAdd(&hist[min(tiles, kPlanBuckets - 1)], 1);
        }
      }
    } else if (s.kind == 2) {
#pragma unroll
      for (int k = 0; k < kChunkSizes; ++k) cnt[k] += (s.L + (512 << k) - 1) / (512 << k);
    }
  }
  // one atomic per wave and counter: lanes hitting one LDS address are served one at a time
#pragma unroll
  for (int k = 0; k < kChunkSizes; ++k) {
    int v = cnt[k];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    if (lane == 0 && v) atomicAdd(&sh_cnt[k], v);
  }
  if (status) atomicOr(&sh_status, status);
  __syncthreads();
  const int nlist = min(sh_nlist, kListCap);
  for (int k = wave; k < nlist; k += kWaves) {
    const int4 info = sh_list_info[k];
    SeqInfo s;
    s.L = info.x; s.n = info.y; s.row0 = info.z; s.kind = 1;
    for (int r0 = lane * p.rows_per_wg; r0 < s.n; r0 += 64 * p.rows_per_wg) {
      const int last = min(r0 + p.rows_per_wg, s.n) - 1;
      const int tiles = (s.L - s.n + last) / kTileKeys + 1;
      atomicAdd(&hist[min(tiles, kPlanBuckets - 1)], 1);
    }
  }
  __syncthreads();

  // descending exclusive offsets: bucket b starts after all items of the buckets above it.  Every
  // thread owns two neighbouring buckets; a wave scan plus the wave totals give the offsets with
  // two barriers.  A batch without query chunks skips it.
  static_assert(kPlanBuckets == 2 * kPlanThreads, "two buckets per planner thread");
  int n_prefill = 0;
  if (sh_nlist > 0) {   // uniform
    const int hi = kPlanBuckets - 1 - 2 * tid, lo = hi - 1;   // this thread's buckets, longest first
    const int c_hi = hist[hi], c_lo = hist[lo];
    int inc = c_hi + c_lo;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(inc, off);
      if (lane >= off) inc += t;
    }
    if (lane == 63) sh_wsum[wave] = inc;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const int v = sh_wsum[w];
      before += (w < wave) ? v : 0;
      n_prefill += v;
    }
    const int start = before + inc - (c_hi + c_lo);
    hist[hi] = start;            // running cursors of the scatter pass
    hist[lo] = start + c_hi;
  }
  // chunk size: every workgroup pays a few microseconds of start-up and merge, so long chunks
  // stream best; take the largest candidate that still yields at least 2048 decode workgroups
  // (8 per CU), else 256 keys
  const int wg_per_item = p.Hkv * p.dec_hgroups;
  int chunk = 256;
#pragma unroll
  for (int k = 0; k < kChunkSizes; ++k)
    if ((long long)sh_cnt[k] * wg_per_item >= kDecodeFillWgs) chunk = 512 << k;
  __syncthreads();

  // pass 2: scatter.  What the ordering pass below needs about a thread's first sequence stays
  // in registers (batches of up to kPlanThreads sequences never re-read anything).
  int2 my_sd = make_int2(0, 0);
  // the trip count is uniform so that the lanes of a wave can pool their requests: one atomic per
  // wave for the item range and one for the bucket of full chunks (lanes hitting one LDS address
  // are served one at a time)
  for (int i0 = 0; i0 < p.num_seqs; i0 += kPlanThreads) {
    const int i = i0 + tid;
    SeqInfo s;
    s.L = s.n = s.row0 = s.kind = 0;
    if (i < p.num_seqs) {
      int dummy = 0;
      s = (i == tid) ? my_s : read_seq(p, i, &dummy);
    }
    const int nch = (s.kind == 2) ? (s.L + chunk - 1) / chunk : 0;
    int inc = nch;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(inc, off);
      if (lane >= off) inc += t;
    }
    int wbase = 0;
    if (lane == 63 && inc > 0) wbase = atomicAdd(&sh_dec_next, inc);
    wbase = __shfl(wbase, 63);
    const int base = wbase + inc - nch;
    int2 sd = make_int2(0, 0);
    if (nch > 0 && base + nch <= p.dec_cap) {
      sd = make_int2(base, nch);
      atomicAdd(&dhist[(s.L - (nch - 1) * chunk + kBlock - 1) / kBlock], 1);
    }
    // every chunk but the last is full
    int full = sd.y > 1 ? sd.y - 1 : 0;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) full += __shfl_xor(full, off);
    if (lane == 0 && full > 0) atomicAdd(&dhist[chunk / kBlock], full);
    if (i < p.num_seqs) p.seq_dec[i] = sd;
    if (i == tid) my_sd = sd;
  }
  auto scatter_rows = [&](int i, const SeqInfo& s, int first, int step) {
    for (int r0 = first * p.rows_per_wg; r0 < s.n; r0 += step * p.rows_per_wg) {
      const int last = min(r0 + p.rows_per_wg, s.n) - 1;
      const int tiles = (s.L - s.n + last) / kTileKeys + 1;
      const int slot = atomicAdd(&hist[min(tiles, kPlanBuckets - 1)], 1);
      if (slot < p.pf_cap) {
        p.pf_items[2 * slot] = make_int4(i, r0, s.L, s.n);
        p.pf_items[2 * slot + 1] = make_int4(s.row0, 0, 0, 0);
      }
    }
  };
  for (int k = wave; k < nlist; k += kWaves) {
    const int4 info = sh_list_info[k];
    SeqInfo s;
    s.L = info.x; s.n = info.y; s.row0 = info.z; s.kind = 1;
    scatter_rows(sh_list[k], s, lane, 64);
  }
  if (sh_nlist > kListCap) {   // sequences that did not fit the queue
    for (int i = tid; i < p.num_seqs; i += kPlanThreads) {
      int dummy = 0;
      const SeqInfo s = read_seq(p, i, &dummy);
      if (s.kind != 1) continue;
      bool queued = false;
      for (int k = 0; k < kListCap && !queued; ++k) queued = (sh_list[k] == i);
      if (!queued) scatter_rows(i, s, 0, 1);
    }
  }
  __syncthreads();
  // processing order of the decode items: by decreasing length, so that the short last chunks
  // of the sequences fill the end of the launch instead of being scattered through it
  const bool any_decode = sh_dec_next > 0;   // uniform
  if (any_decode && tid < 64) {   // exclusive offsets in descending bucket order: lanes take runs of buckets, then a wave scan
    constexpr int kPer = (kDecBuckets + 1 + 63) / 64;
    int loc[kPer];
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const int b = kDecBuckets - (tid * kPer + k);
      loc[k] = b >= 0 ? dhist[b] : 0;
      sum += loc[k];
    }
    int inc = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(inc, off);
      if (tid >= off) inc += t;
    }
    int run = inc - sum;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const int b = kDecBuckets - (tid * kPer + k);
      if (b >= 0) { dhist[b] = run; run += loc[k]; }
    }
    if (tid == 63) sh_dec_total = inc;
  }
  __syncthreads();
  if (any_decode) {
    for (int i0 = 0; i0 < p.num_seqs; i0 += kPlanThreads) {
      const int i = i0 + tid;
      int2 sd = make_int2(0, 0);
      int L = 0, qrow = 0;
      if (i == tid) {
        sd = my_sd;
        L = my_s.L;
        qrow = my_s.row0;
      } else if (i < p.num_seqs) {
        sd = p.seq_dec[i];   // written by this same thread above
        if (sd.y > 0) {
          int dummy = 0;
          const SeqInfo s = read_seq(p, i, &dummy);
          L = s.L;
          qrow = s.row0;
        }
      }
      // the full chunks of all lanes share one bucket: one cursor update per wave
      const int full = sd.y > 1 ? sd.y - 1 : 0;
      int inc = full;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
      }
      int wbase = 0;
      if (lane == 63 && inc > 0) wbase = atomicAdd(&dhist[chunk / kBlock], inc);
      wbase = __shfl(wbase, 63);
      const int pos = wbase + inc - full;
      // a turn's records: what the workgroup needs to start, and the slot of its partial result
      auto put = [&](int turn, int c) {
        p.dec_items[2 * turn] = make_int4(i, c, L, qrow);
        p.dec_items[2 * turn + 1] = make_int4(sd.x + c, 0, 0, 0);
      };
      for (int c = 0; c < full; ++c) put(pos + c, c);
      if (sd.y > 0) {
        const int len = L - (sd.y - 1) * chunk;
        put(atomicAdd(&dhist[(len + kBlock - 1) / kBlock], 1), sd.y - 1);
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    p.hdr->n_prefill = min(n_prefill, p.pf_cap);
    p.hdr->n_decode = sh_dec_total;
    p.hdr->chunk_keys = chunk;
    p.hdr->status = sh_status;
  }
}

}  // namespace

hipError_t launch_plan(const AttnParams& p, hipStream_t st) {
  const size_t nmass = (size_t)p.num_seqs * p.P * p.NQ * p.S;
  int blocks = 1 + (int)((nmass + 8 * kPlanThreads - 1) / (8 * kPlanThreads));
  if (blocks > 64) blocks = 64;
  if (p.kvw.k_new != nullptr) {   // one spare block per four tiles of rows to write, up to two per CU
    const int tiles = (p.kvw.total_q + kKvRowTile - 1) / kKvRowTile;
    const int groups = (tiles + kPlanThreads / 256 - 1) / (kPlanThreads / 256);
    const int want = 1 + (groups < 512 ? groups : 512);
    if (want > blocks) blocks = want;
  }
  hipLaunchKernelGGL(k_plan, dim3(blocks), dim3(kPlanThreads), 0, st, p);
  return hipGetLastError();
}

}  // namespace hook
