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

__device__ __forceinline__ int block_exclusive_scan_1024(int v, int* sh, int* total) {
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const int add = (t >= off) ? sh[t - off] : 0;
    __syncthreads();
    sh[t] += add;
    __syncthreads();
  }
  const int incl = sh[t];
  *total = sh[1023];
  __syncthreads();
  return incl - v;
}

// The bucket holding the need-th largest of the keys still in play: the highest bucket whose
// count, added to the counts above it, reaches `need`.  One wave, four buckets per lane, suffix
// sums by shuffles.  Call with threads 0..63; writes *bucket and *need_left.
__device__ __forceinline__ void find_bucket(const int* hist, int need, int t, int* bucket_out, int* need_left) {
  int h[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) h[u] = hist[4 * t + u];
  const int own = h[0] + h[1] + h[2] + h[3];
  int suffix = own;  // counts of this lane's buckets and of all higher lanes'
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int v = __shfl_down(suffix, off, kWave);
    if (t + off < kWave) suffix += v;
  }
  int above = suffix - own;
  if (above < need && need <= suffix) {  // exactly one lane: the keys still in play number at least `need`
    int bucket = 4 * t;
#pragma unroll
    for (int u = 3; u >= 0; --u) {
      if (above + h[u] >= need) { bucket = 4 * t + u; break; }
      above += h[u];
    }
    *bucket_out = bucket;
    *need_left = need - above;
  }
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
  __shared__ int hist[256];
  __shared__ int sh[1024];
  __shared__ int s_bucket, s_need;
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

  uint64_t prefix = 0;
  int need = k;
  for (int pass = 7; pass >= 0; --pass) {
    if (t < 256) hist[t] = 0;
    __syncthreads();
    const int shift = pass * 8;
    const uint64_t himask = (pass == 7) ? 0ull : (~0ull << (shift + 8));
    for (int j = t; j < n; j += 1024) {
      const uint64_t key = keys[j];
      if ((key & himask) == prefix) atomicAdd(&hist[(int)((key >> shift) & 255u)], 1);
    }
    __syncthreads();
    if (t < kWave) find_bucket(hist, need, t, &s_bucket, &s_need);
    __syncthreads();
    prefix |= (uint64_t)s_bucket << shift;
    need = s_need;
    __syncthreads();
  }

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
  for (int j = j0; j < j1; ++j) {
    const uint64_t key = keys[j];
    const bool keep = key > prefix || (key == prefix && eq_rank++ < need);
    if (!keep) continue;
    const int len = min(p.chunk, M - j * p.chunk);
    for (int r = 0; r < len; ++r)
      if ((int64_t)off + r < p.capacity) p.kept_idx[off + r] = j * p.chunk + r;
    off += len;
  }
  if (t == 0) p.cu_keep[1] = total_tokens;
}


}  // namespace sp
