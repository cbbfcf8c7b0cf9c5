// sp_score_pool_select: scoring and chunk selection of ONE SHORT prompt in a single launch.
//
// For a prompt of a few thousand tokens the separate calls are bound by their launches (about
// eight kernels for half a megabyte of keys), not by any throughput.  Here one workgroup does
// everything the two calls do: logits, row softmax over the prompt, max over heads (and layers),
// mean over the valid queries (Sec. 3.2 equation and Sec. 3.2.2 of arXiv 2502.02789), then the
// average pooling, chunk means, top-k chunks and compaction of Sec. 3.2.3 -- the paper's
// variants without look-ahead (Sec. 4.3) on short contexts are exactly this case.
//
// One thread owns up to kKeysPerThread keys.  Per (layer, KV head): the thread's logits against
// the KV head's R = (H / H_kv) * N query rows stay in registers, the rows' (max, sum exp) are
// reduced over the workgroup, and the thread turns its logits into log-probabilities and folds
// them into its own running [key][query] maxima (registers again).  Nothing but the final scores
// ever leaves the workgroup.  Plain fp32 FMAs: at these sizes the matrix cores would change
// nothing.  The selection then runs on the scores in LDS with the same arithmetic, in the same
// order, as sp_pool_select (fp64, index order), so both paths keep the same tokens.
#include "sp_score_internal.h"
#include "sp_select_core.h"

namespace sp {

constexpr int kFusedThreads = 1024;
constexpr int kFusedMaxKeys = 2048;
constexpr int kKeysPerThread = kFusedMaxKeys / kFusedThreads;  // 2
constexpr int kFusedMaxRows = 8;                               // query rows per KV head: (H / H_kv) * N

struct FusedDev {
  int M, L, N, H, H_kv, G, d, layer_reduce;
  float scale;
  int64_t ts, hs;  // token / head stride of the K cache, elements
  const uint16_t* q;
  const int32_t* n_valid;
  float* scores;
  float* lse_out;
  SelDev sel;
  const uint16_t* k[SP_MAX_LAYERS];
};

// sum and max over the workgroup of R per-thread values each; results land in out_m[r], out_z[r]
// (LDS) for every thread to read after the call
template <int R>
__device__ __forceinline__ void block_row_stats(const float (&m)[R], const float (&z)[R], float* red_m, float* red_z,
                                                float* out_m, float* out_z) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float wm = wave_max(m[r]);
    const float wz = wave_sum(m[r] == -INFINITY ? 0.f : z[r] * expf(m[r] - wm));
    if (lane == 0) { red_m[r * 16 + wave] = wm; red_z[r * 16 + wave] = wz; }
  }
  __syncthreads();
  if (threadIdx.x < R * 16) {  // 16 lanes per row
    const int r = threadIdx.x >> 4;
    float wm = red_m[threadIdx.x], wz = red_z[threadIdx.x];
    float bm = wm;
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) bm = fmaxf(bm, __shfl_xor(bm, off, 16));
    float bz = (wm == -INFINITY) ? 0.f : wz * expf(wm - bm);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) bz += __shfl_xor(bz, off, 16);
    if ((threadIdx.x & 15) == 0) { out_m[r] = bm; out_z[r] = bz; }
  }
  __syncthreads();
}

template <int D, int R>
__global__ __launch_bounds__(kFusedThreads) void fused_short_kernel(const FusedDev p) {
  __shared__ float q_lds[R * D];          // the KV head's query rows, fp32
  __shared__ float red_m[R * 16], red_z[R * 16], row_m[R], row_z[R];
  __shared__ float score_lds[kFusedMaxKeys];
  __shared__ double cs_lds[kSingleMaxChunks];
  const int tid = threadIdx.x;
  const int rows = p.G * p.N;             // <= R

  float tot[kKeysPerThread][kFusedMaxRows];  // per own key and query: running max (or per-layer sums)
#pragma unroll
  for (int kk = 0; kk < kKeysPerThread; ++kk)
#pragma unroll
    for (int n = 0; n < kFusedMaxRows; ++n) tot[kk][n] = (p.layer_reduce == SP_LAYER_MAX) ? -INFINITY : 0.f;

  for (int l = 0; l < p.L; ++l) {
    float lmax[kKeysPerThread][kFusedMaxRows];  // this layer's max over heads
#pragma unroll
    for (int kk = 0; kk < kKeysPerThread; ++kk)
#pragma unroll
      for (int n = 0; n < kFusedMaxRows; ++n) lmax[kk][n] = -INFINITY;
    for (int g = 0; g < p.H_kv; ++g) {
      // query rows r = n * G + j of this KV head -> LDS as fp32
      for (int i = tid; i < rows * D; i += kFusedThreads) {
        const int r = i / D, t = i - r * D;
        const int n = r / p.G, j = r - n * p.G;
        q_lds[i] = __uint_as_float((uint32_t)p.q[(((int64_t)l * p.N + n) * p.H + g * p.G + j) * D + t] << 16);
      }
      __syncthreads();
      float s[kKeysPerThread][R];
      float m[R], z[R];
#pragma unroll
      for (int r = 0; r < R; ++r) { m[r] = -INFINITY; z[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < kKeysPerThread; ++kk) {
        const int key = tid + kk * kFusedThreads;
        const bool valid = key < p.M;
        float acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = 0.f;
        const uint4* kp = reinterpret_cast<const uint4*>(p.k[l] + (int64_t)(valid ? key : 0) * p.ts + (int64_t)g * p.hs);
#pragma unroll 4
        for (int c = 0; c < D / 8; ++c) {
          const uint4 v = kp[c];
          const float k0 = bf16_lo(v.x), k1 = bf16_hi(v.x), k2 = bf16_lo(v.y), k3 = bf16_hi(v.y);
          const float k4 = bf16_lo(v.z), k5 = bf16_hi(v.z), k6 = bf16_lo(v.w), k7 = bf16_hi(v.w);
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const float* qr = q_lds + r * D + 8 * c;
            float a = acc[r];
            a = fmaf(qr[0], k0, a); a = fmaf(qr[1], k1, a); a = fmaf(qr[2], k2, a); a = fmaf(qr[3], k3, a);
            a = fmaf(qr[4], k4, a); a = fmaf(qr[5], k5, a); a = fmaf(qr[6], k6, a); a = fmaf(qr[7], k7, a);
            acc[r] = a;
          }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float x = (valid && r < rows) ? p.scale * acc[r] : -INFINITY;
          s[kk][r] = x;
          const float mn = fmaxf(m[r], x);
          z[r] = (mn == -INFINITY) ? 0.f : z[r] * expf(m[r] - mn) + expf(x - mn);
          m[r] = mn;
        }
      }
      block_row_stats<R>(m, z, red_m, red_z, row_m, row_z);  // (its barriers also fence q_lds for the next KV head)
      float lse[R];
#pragma unroll
      for (int r = 0; r < R; ++r) lse[r] = row_m[r] + logf(row_z[r]);
      if (p.lse_out && tid < rows) {
        const int n = tid / p.G, j = tid - n * p.G;
        p.lse_out[((int64_t)l * p.N + n) * p.H + g * p.G + j] = row_m[tid] + logf(row_z[tid]);
      }
#pragma unroll
      for (int kk = 0; kk < kKeysPerThread; ++kk)
#pragma unroll
        for (int r = 0; r < R; ++r)
          if (r < rows) {
            const int n = r / p.G;
            // (n < kFusedMaxRows because rows <= R <= kFusedMaxRows; written so that the index is a constant after unrolling)
#pragma unroll
            for (int nn = 0; nn < kFusedMaxRows; ++nn)
              if (nn == n) lmax[kk][nn] = fmaxf(lmax[kk][nn], s[kk][r] - lse[r]);
          }
    }
#pragma unroll
    for (int kk = 0; kk < kKeysPerThread; ++kk)
#pragma unroll
      for (int n = 0; n < kFusedMaxRows; ++n) {
        if (p.layer_reduce == SP_LAYER_MAX) tot[kk][n] = fmaxf(tot[kk][n], lmax[kk][n]);
        else tot[kk][n] += expf(lmax[kk][n]);
      }
  }

  int nv = p.n_valid ? p.n_valid[0] : p.N;
  nv = max(1, min(nv, p.N));
#pragma unroll
  for (int kk = 0; kk < kKeysPerThread; ++kk) {
    const int key = tid + kk * kFusedThreads;
    if (key < p.M) {
      float acc = 0.f;
#pragma unroll
      for (int n = 0; n < kFusedMaxRows; ++n)
        if (n < nv) acc += (p.layer_reduce == SP_LAYER_MAX) ? expf(tot[kk][n]) : tot[kk][n];
      const float denom = (p.layer_reduce == SP_LAYER_MAX) ? (float)nv : (float)nv * (float)p.L;
      const float sc = acc / denom;
      score_lds[key] = sc;
      p.scores[key] = sc;
    }
  }
  __syncthreads();

  // Sec. 3.2.3 on the scores in LDS; the same fp64 arithmetic in the same order as sp_pool_select
  const SelDev& sp_ = p.sel;
  const int n_chunks = (p.M + sp_.chunk - 1) / sp_.chunk;
  for (int j = tid; j < n_chunks; j += kFusedThreads) {
    const int s0 = j * sp_.chunk, s1 = min(s0 + sp_.chunk, p.M);
    double t = 0.0;
    for (int i = s0; i < s1; ++i) {  // pooled value of token i, then straight into its chunk's sum
      const int a = max(0, i - sp_.radius), e = min(p.M - 1, i + sp_.radius);
      double sum = 0.0;
      for (int x = a; x <= e; ++x) sum += (double)score_lds[x];
      t += sum / (double)(e - a + 1);
    }
    const double mean = t / (double)(s1 - s0);
    cs_lds[j] = mean;
    if (sp_.chunk_scores_out) sp_.chunk_scores_out[j] = (float)mean;
  }
  __syncthreads();
  select_emit_single(sp_, cs_lds);
}

template <int D>
static sp_status launch_fused(const FusedDev& dev, int rows, hipStream_t stream) {
  if (rows <= 1) hipLaunchKernelGGL((fused_short_kernel<D, 1>), dim3(1), dim3(kFusedThreads), 0, stream, dev);
  else if (rows <= 2) hipLaunchKernelGGL((fused_short_kernel<D, 2>), dim3(1), dim3(kFusedThreads), 0, stream, dev);
  else if (rows <= 4) hipLaunchKernelGGL((fused_short_kernel<D, 4>), dim3(1), dim3(kFusedThreads), 0, stream, dev);
  else hipLaunchKernelGGL((fused_short_kernel<D, 8>), dim3(1), dim3(kFusedThreads), 0, stream, dev);
  return launch_status();
}

}  // namespace sp

extern "C" sp_status sp_score_pool_select(const sp_score_args* a, const sp_pool_select_args* s, void* hip_stream) {
  using namespace sp;
  if (!a || !s) return SP_ENULL;
  // each half is checked as the separate calls check it (workspaces are not needed here)
  if (a->B < 1 || a->N < 1 || a->N > SP_MAX_QUERIES || a->L < 1 || a->L > SP_MAX_LAYERS) return SP_EINVAL;
  if (a->H < 1 || a->H_kv < 1 || a->H % a->H_kv != 0 || a->H / a->H_kv > 8) return SP_EINVAL;
  if (a->d != 64 && a->d != 128) return SP_EINVAL;
  if (a->T < 0 || a->T >= (int64_t)INT32_MAX) return SP_EINVAL;
  if (a->layer_reduce != SP_LAYER_MAX && a->layer_reduce != SP_LAYER_MEAN) return SP_EINVAL;
  if (!finite_f32(a->scale) || a->scale <= 0.f || !finite_f32(a->rope_theta) || a->rope_theta < 0.f) return SP_EINVAL;
  if (a->flags & ~(uint32_t)SP_SCORE_EXCLUSIVE_DEVICE) return SP_EINVAL;
  if (!a->d_q || !a->k_layers || !a->d_cu_seqlens || !a->d_scores) return SP_ENULL;
  for (int l = 0; l < a->L; ++l)
    if (!a->k_layers[l]) return SP_ENULL;
  if (a->k_token_stride < 0 || a->k_head_stride < 0) return SP_EINVAL;
  if ((a->k_token_stride & 7) || (a->k_head_stride & 7) || !aligned16(a->d_q)) return SP_EALIGN;
  for (int l = 0; l < a->L; ++l)
    if (!aligned16(a->k_layers[l])) return SP_EALIGN;
  if (s->B != a->B || s->T != a->T || s->d_scores != a->d_scores || s->d_cu_seqlens != a->d_cu_seqlens) return SP_EINVAL;
  if (s->chunk < 1 || s->pool_window < 1 || (s->pool_window & 1) == 0) return SP_EINVAL;
  if (!finite_f64(s->keep_rate) || s->keep_rate <= 0.0 || s->keep_rate > 1.0 || s->kept_capacity < 0) return SP_EINVAL;
  if (!s->d_kept_idx || !s->d_cu_keep) return SP_ENULL;
  // what one workgroup can hold
  const int rows = a->H / a->H_kv * a->N;
  if (a->B != 1 || a->T < 1 || a->T > kFusedMaxKeys || rows > kFusedMaxRows || a->rope_theta != 0.f || a->d_block_table ||
      (a->T + s->chunk - 1) / s->chunk > kSingleMaxChunks)
    return SP_EUNSUPPORTED;

  FusedDev dev;
  dev.M = (int)a->T; dev.L = a->L; dev.N = a->N; dev.H = a->H; dev.H_kv = a->H_kv; dev.G = a->H / a->H_kv; dev.d = a->d;
  dev.layer_reduce = a->layer_reduce;
  dev.scale = a->scale;
  dev.ts = a->k_token_stride; dev.hs = a->k_head_stride;
  dev.q = static_cast<const uint16_t*>(a->d_q);
  dev.n_valid = a->d_n_valid;
  dev.scores = a->d_scores;
  dev.lse_out = a->d_lse;
  for (int l = 0; l < SP_MAX_LAYERS; ++l) dev.k[l] = l < a->L ? static_cast<const uint16_t*>(a->k_layers[l]) : nullptr;
  SelDev& p = dev.sel;
  p.B = 1; p.T = (int)a->T; p.chunk = s->chunk; p.radius = (s->pool_window - 1) / 2;
  p.keep_rate = s->keep_rate; p.capacity = s->kept_capacity;
  p.cu = s->d_cu_seqlens; p.scores = s->d_scores; p.kept_idx = s->d_kept_idx; p.cu_keep = s->d_cu_keep;
  p.chunk_scores_out = s->d_chunk_scores;
  p.cu_chunks = nullptr; p.seq_keep = nullptr; p.cs = nullptr; p.chunk_off = nullptr;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  return a->d == 64 ? launch_fused<64>(dev, rows, stream) : launch_fused<128>(dev, rows, stream);
}
