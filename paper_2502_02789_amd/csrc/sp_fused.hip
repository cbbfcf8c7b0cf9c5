// sp_score_pool_select: scoring and chunk selection of ONE SHORT prompt in a single launch.
//
// For a prompt of a few thousand tokens the separate calls are bound by their launches (about
// eight kernels for half a megabyte of keys), not by any throughput.  Here one workgroup does
// everything the two calls do: logits, row softmax over the prompt, max over heads (and layers),
// mean over the valid queries (Sec. 3.2 equation and Sec. 3.2.2 of arXiv 2502.02789), then the
// average pooling, chunk means, top-k chunks and compaction of Sec. 3.2.3 -- the paper's
// variants without look-ahead (Sec. 4.3) on short contexts are exactly this case.
//
// One compute unit has to do all the arithmetic, so the logits go through the matrix cores even
// though at most 16 of the operand's columns are in use: v_mfma_f32_16x16x32_bf16 with 16 keys
// as rows and the KV head's (H / H_kv) * N query rows as columns.  Both operands come straight
// from global memory in the instruction's own layout (lane = row or column, 16 contiguous bytes
// of the head dim per lane), with no staging.  A lane therefore holds logits of ONE query row
// (lane % 16) against four keys per tile, which makes everything after the product cheap:
//   * (max, sum exp) of a softmax row: in-lane over the wave's tiles, two lane exchanges inside
//     the wave, one value per wave through LDS, 16 lanes per row for the second level -- two
//     barriers per batch of PB (layer, KV head) pairs;
//   * max over the heads of a KV group: DPP moves between neighbouring lanes;
//   * max / mean over layers: in-lane; mean over the valid queries: one DPP sum at the end.
// Nothing but the final scores ever leaves the workgroup.  The selection then runs on the scores
// in LDS with the same arithmetic, in the same order, as sp_pool_select (fp64, index order), so
// both paths keep the same tokens.
#include "sp_lds.h"
#include "sp_score_internal.h"
#include "sp_select_core.h"

namespace sp {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kFusedThreads = 1024;
constexpr int kFusedWaves = kFusedThreads / 64;
constexpr int kFusedMaxKeys = 2048;
constexpr int kFusedMaxRows = 16;  // query rows per KV head: (H / H_kv) * N, the columns of one MFMA

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

// the value of another lane of the same row of 16 lanes (DPP control word CTRL)
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}
struct OpMax { static __device__ __forceinline__ float f(float a, float b) { return fmaxf(a, b); } };
struct OpAdd { static __device__ __forceinline__ float f(float a, float b) { return a + b; } };
// Reduction over aligned groups of `lanes` (1, 2, 4, 8 or 16) lanes; every lane of the group gets
// the result.  Lane ^ 1, lane ^ 2 inside the quad, then the mirrored half row and the mirrored row.
template <class Op>
__device__ __forceinline__ float group_reduce(float v, int lanes) {
  if (lanes >= 2) v = Op::f(v, dpp_f32<0xB1>(v));
  if (lanes >= 4) v = Op::f(v, dpp_f32<0x4E>(v));
  if (lanes >= 8) v = Op::f(v, dpp_f32<0x141>(v));
  if (lanes >= 16) v = Op::f(v, dpp_f32<0x140>(v));
  return v;
}

template <int D, int KK>  // KK: 64-key blocks per wave (1: up to 1024 keys, 2: up to 2048)
__global__ __launch_bounds__(kFusedThreads) void fused_short_kernel(const FusedDev p) {
  constexpr int TPW = 4 * KK;  // 16-key tiles per wave
  constexpr int PB = 2 / KK;   // (layer, KV head) pairs per batch: PB * TPW * 4 logits per lane
  constexpr int KS = D / 32;   // MFMA steps along the head dim
  static_assert(PB * 16 * 16 <= kFusedThreads, "16 lanes per softmax row in the second level");
  __shared__ double wide[kFusedMaxKeys];  // first the pooled scores, then (as 64-bit keys) the selection's keys
  static_assert(kFusedMaxKeys >= kSingleMaxChunks, "the selection's keys reuse the pooled scores' room");
  __shared__ float red_m[PB * 16 * kFusedWaves], red_z[PB * 16 * kFusedWaves], row_m[PB * 16], row_z[PB * 16];
  __shared__ float score_lds[kFusedMaxKeys];
  __shared__ double cs_lds[kSingleMaxChunks];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, kg = lane >> 4;  // operand row / column; 8-element group of the head dim
  const int rows = p.G * p.N;               // <= 16; query row r = (query) * G + (head of the group)
  const int pairs = p.L * p.H_kv;
  const float scale2 = p.scale * 1.44269504088896341f;  // logits in units of ln 2
  const int tile0 = wave * TPW;             // the wave's keys: tiles tile0 .. tile0 + TPW - 1
  // logit c[t][j] of this lane: query row n, key (tile0 + t) * 16 + 4 * kg + j
  auto key_of = [&](int t, int j) { return (tile0 + t) * 16 + 4 * kg + j; };

  float tot[TPW][4], lmax[TPW][4];  // over the layers / this layer's max over heads
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      tot[t][j] = (p.layer_reduce == SP_LAYER_MAX) ? -INFINITY : 0.f;
      lmax[t][j] = -INFINITY;
    }

  for (int b0 = 0; b0 < pairs; b0 += PB) {
    f32x4 c[PB][TPW];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int pair = b0 + pb;
#pragma unroll
      for (int t = 0; t < TPW; ++t) c[pb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (pair >= pairs) continue;
      const int l = pair / p.H_kv, g = pair - l * p.H_kv;
      bf16x8 qv[KS];  // column n of the query operand (zero beyond the last query row)
      {
        const int nn = n < rows ? n : 0;
        const int nq = nn / p.G, j = nn - nq * p.G;
        const uint16_t* qp = p.q + (((int64_t)l * p.N + nq) * p.H + g * p.G + j) * D + 8 * kg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          uint4 v = *reinterpret_cast<const uint4*>(qp + 32 * ks);
          if (n >= rows) v = make_uint4(0, 0, 0, 0);
          qv[ks] = __builtin_bit_cast(bf16x8, v);
        }
      }
      // Four tiles at a time: all their loads first (rows past the end of the prompt read the
      // last key again and are masked below), so that one round trip covers the group.
      const uint16_t* kbase = p.k[l] + (int64_t)g * p.hs + 8 * kg;
#pragma unroll
      for (int t0 = 0; t0 < TPW; t0 += 4) {
        uint4 kv[4][KS];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int row = min((tile0 + t0 + t) * 16 + n, p.M - 1);
          const uint16_t* kp = kbase + (int64_t)row * p.ts;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) kv[t][ks] = *reinterpret_cast<const uint4*>(kp + 32 * ks);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            c[pb][t0 + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kv[t][ks]), qv[ks], c[pb][t0 + t], 0, 0, 0);
      }
      // base-2 logits from here on: exp2 is one instruction
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) c[pb][t][j] = key_of(t, j) < p.M ? scale2 * c[pb][t][j] : -INFINITY;
    }

    // (max, sum exp) of the batch's PB * 16 softmax rows over the workgroup
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      float wm = -INFINITY;
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) wm = fmaxf(wm, c[pb][t][j]);
      wm = fmaxf(wm, __shfl_xor(wm, 16));
      wm = fmaxf(wm, __shfl_xor(wm, 32));
      float wz = 0.f;
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) wz += (wm == -INFINITY) ? 0.f : exp2f(c[pb][t][j] - wm);
      wz += __shfl_xor(wz, 16);
      wz += __shfl_xor(wz, 32);
      if (lane < 16) { red_m[(pb * 16 + lane) * kFusedWaves + wave] = wm; red_z[(pb * 16 + lane) * kFusedWaves + wave] = wz; }
    }
    __syncthreads();
    if (tid < PB * 16 * kFusedWaves) {  // 16 lanes per row, one per wave's pair of values
      const float wm = red_m[tid], wz = red_z[tid];
      const float bm = group_reduce<OpMax>(wm, 16);
      const float bz = group_reduce<OpAdd>((wm == -INFINITY) ? 0.f : wz * exp2f(wm - bm), 16);
      if ((tid & 15) == 0) { row_m[tid >> 4] = bm; row_z[tid >> 4] = bz; }
    }
    __syncthreads();

#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int pair = b0 + pb;
      if (pair >= pairs) continue;
      const int l = pair / p.H_kv, g = pair - l * p.H_kv;
      const float lse = row_m[pb * 16 + n] + log2f(row_z[pb * 16 + n]);  // base 2
      if (p.lse_out && tid < rows) {
        const int nq = tid / p.G, j = tid - nq * p.G;
        p.lse_out[((int64_t)l * p.N + nq) * p.H + g * p.G + j] = 0.69314718055994531f * lse;
      }
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          lmax[t][j] = fmaxf(lmax[t][j], group_reduce<OpMax>(c[pb][t][j] - lse, p.G));  // over the group's heads
      if (g == p.H_kv - 1) {  // the layer is complete
#pragma unroll
        for (int t = 0; t < TPW; ++t)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (p.layer_reduce == SP_LAYER_MAX) tot[t][j] = fmaxf(tot[t][j], lmax[t][j]);
            else tot[t][j] += exp2f(lmax[t][j]);
            lmax[t][j] = -INFINITY;
          }
      }
    }
  }

  // mean over the valid queries: the lanes of a query's first head carry its value
  int nv = p.n_valid ? p.n_valid[0] : p.N;
  nv = max(1, min(nv, p.N));
  const bool counts = n < rows && n % p.G == 0 && n / p.G < nv;
  const float inv_denom = 1.f / ((p.layer_reduce == SP_LAYER_MAX) ? (float)nv : (float)nv * (float)p.L);
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float mine = (p.layer_reduce == SP_LAYER_MAX) ? exp2f(tot[t][j]) : tot[t][j];
      const float sc = group_reduce<OpAdd>(counts ? mine : 0.f, 16) * inv_denom;
      const int key = key_of(t, j);
      if (n == 0 && key < p.M) {
        score_lds[key] = sc;
        p.scores[key] = sc;
      }
    }
  __syncthreads();

  // Sec. 3.2.3 on the scores in LDS; the same fp64 arithmetic in the same order as sp_pool_select
  const SelDev& sp_ = p.sel;
  for (int i = tid; i < p.M; i += kFusedThreads) {
    const int a = max(0, i - sp_.radius), e = min(p.M - 1, i + sp_.radius);
    double sum = 0.0;
    for (int x = a; x <= e; ++x) sum += (double)score_lds[x];
    wide[i] = sum / (double)(e - a + 1);
  }
  __syncthreads();
  const int n_chunks = (p.M + sp_.chunk - 1) / sp_.chunk;
  for (int j = tid; j < n_chunks; j += kFusedThreads) {
    const int s0 = j * sp_.chunk, s1 = min(s0 + sp_.chunk, p.M);
    double t = 0.0;
    for (int x = s0; x < s1; ++x) t += wide[x];
    const double mean = t / (double)(s1 - s0);
    cs_lds[j] = mean;
    if (sp_.chunk_scores_out) sp_.chunk_scores_out[j] = (float)mean;
  }
  __syncthreads();
  select_emit_single(sp_, cs_lds, reinterpret_cast<uint64_t*>(wide));
}

template <int D>
static sp_status launch_fused(const FusedDev& dev, hipStream_t stream) {
  if (dev.M <= kFusedThreads) hipLaunchKernelGGL((fused_short_kernel<D, 1>), dim3(1), dim3(kFusedThreads), 0, stream, dev);
  else hipLaunchKernelGGL((fused_short_kernel<D, 2>), dim3(1), dim3(kFusedThreads), 0, stream, dev);
  return launch_status();
}

}  // namespace sp

extern "C" sp_status sp_score_pool_select(const sp_score_args* a, const sp_pool_select_args* s, void* hip_stream) {
  using namespace sp;
  if (!a || !s) return SP_ENULL;
  // each half is checked as the separate calls check it (workspaces are not needed here)
  if (a->B < 1 || a->N < 1 || a->N > SP_MAX_QUERIES || a->L < 1 || a->L > SP_MAX_LAYERS) return SP_EINVAL;
  if (a->H < 1 || a->H_kv < 1 || a->H % a->H_kv != 0) return SP_EINVAL;
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
  const int G = a->H / a->H_kv, rows = G * a->N;
  if ((G & (G - 1)) != 0) return SP_EUNSUPPORTED;  // the heads of a KV group sit in an aligned run of lanes
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
  return a->d == 64 ? launch_fused<64>(dev, stream) : launch_fused<128>(dev, stream);
}
