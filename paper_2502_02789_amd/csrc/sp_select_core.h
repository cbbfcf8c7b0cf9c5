// Pieces of the chunk selection shared by sp_select.hip and the fused short-prompt kernel
// (sp_fused.hip): the kernel-side argument view, the order-preserving keys, and the single-sequence
// top-k + compaction done by one workgroup (Sec. 3.2.3 of arXiv 2502.02789: Top-K chunks, keep
// rate = ratio of chunks; equal scores go to the lower chunk index).
#pragma once

// the k formula below must stay a separate multiply and subtract (for every includer)
#pragma clang fp contract(off)

#include "sp_common.h"

namespace sp {

struct SelDev {
  int B;
  int T;
  int chunk, radius;
  double keep_rate;
  int64_t capacity;
  const int32_t* cu;
  const float* scores;
  int32_t* kept_idx;
  int32_t* cu_keep;
  float* chunk_scores_out;
  int32_t* cu_chunks;   // [B+1]
  int32_t* seq_keep;    // [B]
  double* cs;           // [max_chunks]
  int32_t* chunk_off;   // [max_chunks]: offset of the chunk's first token inside its sequence's kept list, or -1
};

// NaN, decided on the bit pattern (device code is compiled on the assumption that there are none)
__device__ __forceinline__ bool is_nan_bits(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  return (u & 0x7ff0000000000000ull) == 0x7ff0000000000000ull && (u & 0x000fffffffffffffull) != 0;
}

// monotone map double -> uint64 (larger value <-> larger key)
__device__ __forceinline__ uint64_t order_key(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// Inclusive prefix sum over the 64 lanes of a wave; *total gets the wave's sum.  Inside each row
// of 16 lanes by DPP row shifts (lanes shifted in from outside the row contribute zero), the
// three row totals that lie below a lane through scalar registers: no LDS round trips.
__device__ __forceinline__ int wave_inclusive_scan(int v, int* total) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);  // row_shr:8
  const int r0 = __builtin_amdgcn_readlane(v, 15), r1 = __builtin_amdgcn_readlane(v, 31);
  const int r2 = __builtin_amdgcn_readlane(v, 47), r3 = __builtin_amdgcn_readlane(v, 63);
  const int lane = threadIdx.x & 63;
  *total = r0 + r1 + r2 + r3;
  return v + (lane >= 16 ? r0 : 0) + (lane >= 32 ? r1 : 0) + (lane >= 48 ? r2 : 0);
}

// exclusive prefix sum over the 1024 threads of the workgroup (the 16 wave totals go through
// `sh`): two barriers
__device__ __forceinline__ int block_exclusive_scan_1024(int v, int* sh, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int wave_total;
  const int incl = wave_inclusive_scan(v, &wave_total);
  if (lane == kWave - 1) sh[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int s = sh[w];
    all += s;
    before += (w < wave) ? s : 0;
  }
  *total = all;
  __syncthreads();  // `sh` may be written again
  return before + incl - v;
}

// The bucket holding the need-th largest of the keys still in play: the highest bucket whose
// count, added to the counts above it, reaches `need`.  Done by a whole wave (four buckets per
// lane, suffix sums by shuffles); every lane gets the bucket and how many keys of that bucket are
// still needed.
__device__ __forceinline__ void find_bucket(const int* hist, int need, int* bucket_out, int* need_left) {
  const int lane = threadIdx.x & 63;
  int h[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) h[u] = hist[4 * lane + u];
  const int own = h[0] + h[1] + h[2] + h[3];
  int all;
  const int upto = wave_inclusive_scan(own, &all);
  const int suffix = all - upto + own;  // counts of this lane's buckets and of all higher lanes'
  int above = suffix - own;
  int bucket = -1, left = 0;
  if (above < need && need <= suffix) {  // exactly one lane: the keys still in play number at least `need`
    bucket = 4 * lane;
#pragma unroll
    for (int u = 3; u >= 0; --u) {
      if (above + h[u] >= need) { bucket = 4 * lane + u; break; }
      above += h[u];
    }
    left = need - above;
  }
  const int src = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)__ballot(bucket >= 0)) - 1);
  *bucket_out = __builtin_amdgcn_readlane(bucket, src);
  *need_left = __builtin_amdgcn_readlane(left, src);
}

// Radix select over 64-bit keys, eight bits a pass from the top: afterwards `prefix` is the k-th
// largest key and `need` says how many keys equal to it are among the k largest.  key_at(j) gives
// key j of n.  Call with all 1024 threads; `hist` has room for 3 x 256 counters.  One barrier per
// pass: the counters of pass i live in hist[i % 3], the next pass's are cleared meanwhile (their
// last readers finished two barriers ago), and every wave finds the bucket for itself.
template <typename KeyAt>
__device__ __forceinline__ void radix_select_kth(KeyAt key_at, int n, int k, int* hist, uint64_t* prefix_out, int* need_out) {
  const int t = threadIdx.x;
  if (t < 256) hist[t] = 0;
  __syncthreads();
  uint64_t prefix = 0;
  int need = k;
#pragma unroll 1
  for (int i = 0; i < 8; ++i) {
    int* cur = hist + (i % 3) * 256;
    int* nxt = hist + ((i + 1) % 3) * 256;
    if (t < 256) nxt[t] = 0;
    const int shift = (7 - i) * 8;
    const uint64_t himask = (i == 0) ? 0ull : (~0ull << (shift + 8));
    for (int j = t; j < n; j += 1024) {
      const uint64_t key = key_at(j);
      const bool in_play = (key & himask) == prefix;
      const int digit = (int)((key >> shift) & 255u);
      // Scores of one prompt share their sign and most exponent bits, so in the upper passes a
      // whole wave lands in one counter, and 64 additions to one LDS word are done one after
      // the other: where the wave's digits all agree, one lane adds the count.
      const unsigned long long mask = __ballot(in_play);
      if (mask == 0) continue;
      const int leader = __builtin_amdgcn_readfirstlane(__ffsll(mask) - 1);
      const int first = __builtin_amdgcn_readlane(digit, leader);
      if (__ballot(in_play && digit != first) == 0) {
        if ((t & 63) == leader) atomicAdd(&cur[first], __popcll(mask));
      } else if (in_play) {
        atomicAdd(&cur[digit], 1);
      }
    }
    __syncthreads();
    int bucket;
    find_bucket(cur, need, &bucket, &need);
    prefix |= (uint64_t)bucket << shift;
  }
  *prefix_out = prefix;
  *need_out = need;
}

// Single sequence with at most kSingleMaxChunks chunks: top-k, compaction and the kept-index
// list in one workgroup and one launch.  Above kCountMaxChunks chunks the k-th largest key is
// found by the same 8-pass radix select as in select_kernel, on keys held in LDS; ties at the
// threshold go to the lower chunk indices by an ordered scan; kept tokens are written straight away.
constexpr int kSingleMaxChunks = 2048;
constexpr int kCountMaxChunks = 256;  // up to here the chunks are ranked by counting instead
// `cs`: the chunk scores (global or LDS memory); `keys`: LDS room for kSingleMaxChunks 64-bit keys.
// Call with all 1024 threads of the workgroup.
__device__ __forceinline__ void select_emit_single(const SelDev& p, const double* cs, uint64_t* keys) {
  __shared__ int hist[3 * 256];
  __shared__ int sh[16];
  const int t = threadIdx.x;
  const int M = p.T;
  const int n = (M + p.chunk - 1) / p.chunk;
  if (t == 0) p.cu_keep[0] = 0;
  if (n == 0) {
    if (t == 0) p.cu_keep[1] = 0;
    return;
  }
  const double scaled = p.keep_rate * (double)n;
  const double kd = ceil(scaled - 1e-9);
  const int k = (int)fmin((double)n, fmax(1.0, kd));
  int bad = 0;
  for (int j = t; j < n; j += 1024) {
    const double v = cs[j];
    bad |= is_nan_bits(v) ? 1 : 0;
    keys[j] = order_key(v);
  }
  if (__syncthreads_or(bad)) {  // invalid scores: reported in band, nothing kept
    if (t == 0) p.cu_keep[1] = -1;
    return;
  }

  if (n <= kCountMaxChunks) {
    // Few chunks: thread t ranks chunk t by counting the chunks that come before it in the order
    // (larger score, or equal score and lower index); the k first are kept.  All chunks but the
    // last have the same length, so a kept token's place follows from the number of kept chunks
    // before its own: no scan, two barriers.
    __shared__ uint64_t kept_mask[kCountMaxChunks / 64];
    bool keep = false;
    if (t < n) {
      const uint64_t mine = keys[t];
      int rank = 0;
#pragma unroll 8
      for (int j = 0; j < n; ++j) {
        const uint64_t other = keys[j];
        rank += (other > mine || (other == mine && j < t)) ? 1 : 0;
      }
      keep = rank < k;
    }
    const uint64_t ballot = __ballot(keep);
    if (t < kCountMaxChunks && (t & 63) == 0) kept_mask[t >> 6] = ballot;
    __syncthreads();
    for (int i = t; i < M; i += 1024) {
      const int c = i / p.chunk, w = c >> 6;
      const uint64_t word = kept_mask[w];
      if (!((word >> (c & 63)) & 1ull)) continue;
      int before = __popcll(word & ((1ull << (c & 63)) - 1ull));
      for (int x = 0; x < w; ++x) before += __popcll(kept_mask[x]);
      const int64_t pos = (int64_t)before * p.chunk + (i - c * p.chunk);
      if (pos < p.capacity) p.kept_idx[pos] = i;
    }
    if (t == 0) {
      int kept_chunks = 0;
      for (int x = 0; x < kCountMaxChunks / 64; ++x) kept_chunks += __popcll(kept_mask[x]);
      const bool last_kept = (kept_mask[(n - 1) >> 6] >> ((n - 1) & 63)) & 1ull;
      p.cu_keep[1] = (int32_t)((int64_t)kept_chunks * p.chunk - (last_kept ? (int64_t)n * p.chunk - M : 0));
    }
    return;
  }

  uint64_t prefix;
  int need;
  radix_select_kth([&](int j) { return keys[j]; }, n, k, hist, &prefix, &need);

  // ordered pass: thread t owns chunks [j0, j1) in index order
  const int per = (n + 1023) / 1024;
  const int j0 = min(n, t * per), j1 = min(n, j0 + per);
  int eq = 0;
  for (int j = j0; j < j1; ++j) eq += (keys[j] == prefix) ? 1 : 0;
  int total_eq;
  int eq_rank = block_exclusive_scan_1024(eq, sh, &total_eq);
  int tokens = 0;
  {
    int r = eq_rank;
    for (int j = j0; j < j1; ++j) {
      const uint64_t key = keys[j];
      const bool keep = key > prefix || (key == prefix && r++ < need);
      if (keep) tokens += min(p.chunk, M - j * p.chunk);
    }
  }
  int total_tokens;
  int off = block_exclusive_scan_1024(tokens, sh, &total_tokens);
  // Kept chunks by rank: all kept chunks but possibly the very last are full, so a chunk that
  // starts at token offset `off` of the kept list is kept chunk number off / chunk ...
  __shared__ unsigned short kept_list[kSingleMaxChunks];
  for (int j = j0; j < j1; ++j) {
    const uint64_t key = keys[j];
    const bool keep = key > prefix || (key == prefix && eq_rank++ < need);
    if (!keep) continue;
    kept_list[off / p.chunk] = (unsigned short)j;
    off += min(p.chunk, M - j * p.chunk);
  }
  __syncthreads();
  // ... and the kept tokens are written by all threads, a token each
  const int64_t n_write = min((int64_t)total_tokens, p.capacity);
  for (int64_t pos = t; pos < n_write; pos += 1024) {
    const int q = (int)(pos / p.chunk);
    p.kept_idx[pos] = (int)kept_list[q] * p.chunk + (int)(pos - (int64_t)q * p.chunk);
  }
  if (t == 0) p.cu_keep[1] = total_tokens;
}


}  // namespace sp
