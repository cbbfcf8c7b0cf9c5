// sp_pool_select: 1-D average pooling, chunk means, top-k chunks with a lower-index
// tie-break, and ordered compaction of the kept tokens (Sec. 3.2.3 and Algorithm 1,
// chunk_select_from_smoothed_attention, of arXiv 2502.02789; keep rate = ratio of
// chunks, Sec. 4.1).
//
// All arithmetic is fp64 on the fp32 input scores, summed in index order with adds and
// divides only, so the chunk scores (and therefore the kept set) do not depend on how the
// work is split over lanes.  Top-k is an 8-pass radix select on order-preserving 64-bit
// keys followed by an ordered scan that resolves equal scores to the lower chunk index.
#include <mutex>

// the k formula below must stay a separate multiply and subtract
#pragma clang fp contract(off)

#include "sp_select_core.h"

namespace sp {

__global__ __launch_bounds__(1024) void chunk_table_kernel(const SelDev p) {
  block_prefix_table(p.B, [&](int b) { return (p.cu[b + 1] - p.cu[b] + p.chunk - 1) / p.chunk; }, p.cu_chunks);
}

__device__ __forceinline__ double shfl_f64(double v, int src) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl(lo, src, kWave);
  hi = __shfl(hi, src, kWave);
  return __hiloint2double(hi, lo);
}

// One wave serves a group of 64/chunk consecutive chunks (one chunk when chunk >= 64).
// Lanes pool one token each; every lane then adds its chunk's pooled values in token order.
template <bool SINGLE>  // SINGLE: one sequence of T tokens, no chunk table
__global__ __launch_bounds__(256) void pool_chunk_kernel(const SelDev p) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n_chunks = SINGLE ? (p.T + p.chunk - 1) / p.chunk : p.cu_chunks[p.B];
  const bool wide = p.chunk >= kWave;
  const int cpw = wide ? 1 : kWave / p.chunk;          // chunks per wave
  const int seg_len = wide ? kWave : p.chunk;          // tokens of a chunk handled per step
  const int n_seg = (p.chunk + seg_len - 1) / seg_len;
  const int n_groups = (n_chunks + cpw - 1) / cpw;
  const int q = wide ? 0 : lane / p.chunk;             // chunk of the group this lane serves
  const int t_in = lane - q * seg_len;
  for (int grp = blockIdx.x * 4 + wave; grp < n_groups; grp += gridDim.x * 4) {
    const int j = grp * cpw + q;
    const bool live = (q < cpw) && (j < n_chunks);
    int lo = 0, hi = 0, s0 = 0, s1 = 0;
    if (live) {
      if (SINGLE) {
        hi = p.T;
        s0 = j * p.chunk;
      } else {
        const int b = upper_segment(p.cu_chunks, p.B, j);
        lo = p.cu[b];
        hi = p.cu[b + 1];
        s0 = lo + (j - p.cu_chunks[b]) * p.chunk;
      }
      s1 = min(s0 + p.chunk, hi);
    }
    double tot = 0.0;
    for (int seg = 0; seg < n_seg; ++seg) {
      const int i = s0 + seg * seg_len + t_in;
      double pooled = 0.0;
      if (live && i < s1) {
        const int a = max(lo, i - p.radius), e = min(hi - 1, i + p.radius);
        double sum = 0.0;
        for (int x = a; x <= e; ++x) sum += (double)p.scores[x];
        pooled = sum / (double)(e - a + 1);
      }
      const int base = q * seg_len;
      const int have = min(seg_len, s1 - (s0 + seg * seg_len));  // tokens of this chunk in this step
      for (int t = 0; t < seg_len; ++t) {                         // uniform trip count
        const double v = shfl_f64(pooled, base + t);
        if (t < have) tot += v;
      }
    }
    if (live && t_in == 0) {
      const double mean = tot / (double)(s1 - s0);
      p.cs[j] = mean;
      if (p.chunk_scores_out) p.chunk_scores_out[j] = (float)mean;
    }
  }
}

// One workgroup per sequence.
__global__ __launch_bounds__(1024) void select_kernel(const SelDev p) {
  __shared__ int hist[3 * 256];
  __shared__ int sh[16];
  const int b = blockIdx.x, t = threadIdx.x;
  const int c0 = p.cu_chunks[b];
  const int n = p.cu_chunks[b + 1] - c0;
  const int lo = p.cu[b], hi = p.cu[b + 1];
  if (n == 0) {
    if (t == 0) p.seq_keep[b] = 0;
    return;
  }
  const double scaled = p.keep_rate * (double)n;
  const double kd = ceil(scaled - 1e-9);
  const int k = (int)fmin((double)n, fmax(1.0, kd));
  const double* cs = p.cs + c0;

  // invalid scores (NaN: the scorer's mark for "a device-side wait expired") are reported in band:
  // a negative count here turns every cu_keep entry after the first into -1
  {
    int bad = 0;
    for (int j = t; j < n; j += 1024) bad |= is_nan_bits(cs[j]) ? 1 : 0;
    if (__syncthreads_or(bad)) {
      for (int j = t; j < n; j += 1024) p.chunk_off[c0 + j] = -1;
      if (t == 0) p.seq_keep[b] = -1;
      return;
    }
  }

  // radix select: after the loop `prefix` is the key of the k-th largest chunk score and
  // `need` is how many chunks with exactly that score are still to be taken
  uint64_t prefix;
  int need;
  radix_select_kth([&](int j) { return order_key(cs[j]); }, n, k, hist, &prefix, &need);

  // ordered pass: thread t owns chunks [j0, j1) in index order
  const int per = (n + 1023) / 1024;
  const int j0 = min(n, t * per), j1 = min(n, j0 + per);
  int eq = 0;
  for (int j = j0; j < j1; ++j) eq += (order_key(cs[j]) == prefix) ? 1 : 0;
  int total_eq;
  int eq_rank = block_exclusive_scan_1024(eq, sh, &total_eq);
  int tokens = 0;
  {
    int r = eq_rank;
    for (int j = j0; j < j1; ++j) {
      const uint64_t key = order_key(cs[j]);
      const bool keep = key > prefix || (key == prefix && r++ < need);
      if (keep) tokens += min(p.chunk, (hi - lo) - j * p.chunk);
    }
  }
  int total_tokens;
  int off = block_exclusive_scan_1024(tokens, sh, &total_tokens);
  for (int j = j0; j < j1; ++j) {
    const uint64_t key = order_key(cs[j]);
    const bool keep = key > prefix || (key == prefix && eq_rank++ < need);
    p.chunk_off[c0 + j] = keep ? off : -1;
    if (keep) off += min(p.chunk, (hi - lo) - j * p.chunk);
  }
  if (t == 0) p.seq_keep[b] = total_tokens;
}

__global__ __launch_bounds__(1024) void select_emit_single_kernel(const SelDev p) {
  __shared__ uint64_t keys[kSingleMaxChunks];
  select_emit_single(p, p.cs, keys);
}

__global__ __launch_bounds__(1024) void cu_keep_kernel(const SelDev p) {
  int bad = 0;
  for (int b = threadIdx.x; b < p.B; b += 1024) bad |= p.seq_keep[b] < 0 ? 1 : 0;
  bad = __syncthreads_or(bad);
  block_prefix_table(p.B, [&](int b) { return max(p.seq_keep[b], 0); }, p.cu_keep);
  if (bad)  // some sequence had invalid scores: no keep set is handed on
    for (int b = 1 + threadIdx.x; b <= p.B; b += 1024) p.cu_keep[b] = -1;
}

// one thread per prompt token: if its chunk is kept, write its flat index to its slot
__global__ __launch_bounds__(256) void emit_kernel(const SelDev p) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= p.T || p.cu_keep[p.B] < 0) return;
  const int b = upper_segment(p.cu, p.B, i);
  const int in_seq = i - p.cu[b];
  const int j = in_seq / p.chunk;
  const int off = p.chunk_off[p.cu_chunks[b] + j];
  if (off < 0) return;
  const int64_t slot = (int64_t)p.cu_keep[b] + off + (in_seq - j * p.chunk);
  if (slot < p.capacity) p.kept_idx[slot] = i;
}

static bool select_shape_ok(const sp_pool_select_args* a) {
  if (a->B < 1 || a->T < 0 || a->T >= (int64_t)INT32_MAX) return false;
  if (a->chunk < 1 || a->pool_window < 1 || (a->pool_window & 1) == 0) return false;
  if (!finite_f64(a->keep_rate) || a->keep_rate <= 0.0 || a->keep_rate > 1.0) return false;
  return true;
}
static size_t select_max_chunks(const sp_pool_select_args* a) { return (size_t)(a->T / a->chunk) + a->B; }

}  // namespace sp

extern "C" int64_t sp_keep_upper_bound(int32_t B, const int32_t* h_seqlens, int32_t chunk, double keep_rate) {
  if (B < 0 || (B > 0 && !h_seqlens) || chunk < 1 || !sp::finite_f64(keep_rate) || keep_rate <= 0.0 || keep_rate > 1.0)
    return -1;
  int64_t total = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t M = h_seqlens[b];
    if (M < 0) return -1;
    if (M == 0) continue;
    const int64_t n = (M + chunk - 1) / chunk;
    const double scaled = keep_rate * (double)n;
    int64_t k = (int64_t)ceil(scaled - 1e-9);
    k = k < 1 ? 1 : (k > n ? n : k);
    const int64_t toks = k * chunk;
    total += toks < M ? toks : M;
  }
  return total;
}

extern "C" size_t sp_pool_select_workspace_bytes(const sp_pool_select_args* a) {
  if (!a || !sp::select_shape_ok(a)) return 0;
  const size_t mc = sp::select_max_chunks(a);
  return sp::align_up(4 * ((size_t)a->B + 1), 256) + sp::align_up(4 * (size_t)a->B, 256) +
         sp::align_up(8 * mc, 256) + sp::align_up(4 * mc, 256);
}

namespace sp {

// argument checks shared by the two entry points (everything but the scratch space)
static sp_status check_select_args(const sp_pool_select_args* a) {
  if (!a) return SP_ENULL;
  if (!select_shape_ok(a)) return SP_EINVAL;
  if (!a->d_cu_seqlens || !a->d_scores || !a->d_kept_idx || !a->d_cu_keep) return SP_ENULL;
  if (a->kept_capacity < 0) return SP_EINVAL;
  return SP_OK;
}

// enqueue the selection with `scratch` (device memory, 256-byte aligned, at least
// sp_pool_select_workspace_bytes(a) bytes) as the kernels' scratch space
static sp_status run_pool_select(const sp_pool_select_args* a, void* scratch, hipStream_t stream) {
  const size_t mc = select_max_chunks(a);
  SelDev p;
  p.B = a->B; p.T = (int)a->T; p.chunk = a->chunk; p.radius = (a->pool_window - 1) / 2;
  p.keep_rate = a->keep_rate; p.capacity = a->kept_capacity;
  p.cu = a->d_cu_seqlens; p.scores = a->d_scores; p.kept_idx = a->d_kept_idx; p.cu_keep = a->d_cu_keep;
  p.chunk_scores_out = a->d_chunk_scores;
  char* ws = static_cast<char*>(scratch);
  p.cu_chunks = reinterpret_cast<int32_t*>(ws); ws += align_up(4 * ((size_t)a->B + 1), 256);
  p.seq_keep = reinterpret_cast<int32_t*>(ws);  ws += align_up(4 * (size_t)a->B, 256);
  p.cs = reinterpret_cast<double*>(ws);         ws += align_up(8 * mc, 256);
  p.chunk_off = reinterpret_cast<int32_t*>(ws);

  const int cpw = a->chunk >= kWave ? 1 : kWave / a->chunk;
  const size_t groups = (mc + cpw - 1) / cpw;
  const int pool_blocks = (int)std::min<size_t>((groups + 3) / 4, 65535);
  if (a->B == 1 && (a->T + a->chunk - 1) / a->chunk <= kSingleMaxChunks) {
    // one sequence (its length is T, known here): no chunk table, no cross-sequence scan
    hipLaunchKernelGGL(pool_chunk_kernel<true>, dim3(std::max(pool_blocks, 1)), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(select_emit_single_kernel, dim3(1), dim3(1024), 0, stream, p);
    return launch_status();
  }
  hipLaunchKernelGGL(chunk_table_kernel, dim3(1), dim3(1024), 0, stream, p);
  hipLaunchKernelGGL(pool_chunk_kernel<false>, dim3(std::max(pool_blocks, 1)), dim3(256), 0, stream, p);
  hipLaunchKernelGGL(select_kernel, dim3(a->B), dim3(1024), 0, stream, p);
  hipLaunchKernelGGL(cu_keep_kernel, dim3(1), dim3(1024), 0, stream, p);
  if (a->T > 0)
    hipLaunchKernelGGL(emit_kernel, dim3((unsigned)((a->T + 255) / 256)), dim3(256), 0, stream, p);
  return launch_status();
}

}  // namespace sp

extern "C" sp_status sp_pool_select(const sp_pool_select_args* a, void* hip_stream) {
  using namespace sp;
  const sp_status st = check_select_args(a);
  if (st != SP_OK) return st;
  if (!a->d_workspace || a->workspace_bytes < sp_pool_select_workspace_bytes(a)) return SP_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(a->d_workspace) & 255u) return SP_EALIGN;
  return run_pool_select(a, a->d_workspace, static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------------------------------------------
// the variant for callers that cannot allocate: scratch space inside the library's image
// ---------------------------------------------------------------------------------------
// One copy per GPU (each device that loads the library's code object gets its own), alive until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[SP_STATIC_SCRATCH_BYTES];

namespace sp {

// device address of `scratch` on the current GPU, looked up once per device
static void* static_scratch_address() {
  static std::mutex mu;
  static void* address[kMaxDevices] = {};
  std::lock_guard<std::mutex> lock(mu);
  const int slot = current_device();
  if (!address[slot]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    address[slot] = ptr;
  }
  return address[slot];
}

}  // namespace sp

extern "C" sp_status sp_pool_select_static(const sp_pool_select_args* a, void* hip_stream) {
  using namespace sp;
  const sp_status st = check_select_args(a);
  if (st != SP_OK) return st;
  if (a->B > SP_STATIC_MAX_SEQS || select_max_chunks(a) > (size_t)SP_STATIC_MAX_CHUNKS) return SP_EUNSUPPORTED;
  static_assert(256 * ((4 * ((size_t)SP_STATIC_MAX_SEQS + 1) + 255) / 256) + 256 * ((4 * (size_t)SP_STATIC_MAX_SEQS + 255) / 256) +
                        12 * (size_t)SP_STATIC_MAX_CHUNKS + 512 <= SP_STATIC_SCRATCH_BYTES,
                "the static scratch must hold the largest workspace the limits allow");
  if (sp_pool_select_workspace_bytes(a) > SP_STATIC_SCRATCH_BYTES) return SP_EUNSUPPORTED;
  void* ptr = static_scratch_address();
  if (!ptr) return SP_ELAUNCH;
  // nothing in the scratch has to start at zero: every word the kernels read was written earlier
  // in the same call (chunk table, chunk scores, per-chunk offsets, per-sequence counts)
  return run_pool_select(a, ptr, static_cast<hipStream_t>(hip_stream));
}
