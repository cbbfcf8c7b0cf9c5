// sp_score_pool_select: scoring and chunk selection of ONE SHORT prompt in a single launch.
//
// For a prompt of a few thousand tokens the separate calls are bound by their launches (about
// eight kernels for half a megabyte of keys), not by any throughput.  Here one launch does
// everything the two calls do: logits, row softmax over the prompt, max over heads (and layers),
// mean over the valid queries (Sec. 3.2 equation and Sec. 3.2.2 of arXiv 2502.02789), then the
// average pooling, chunk means, top-k chunks and compaction of Sec. 3.2.3 -- the paper's
// variants without look-ahead (Sec. 4.3) on short contexts are exactly this case.
//
// Two phases, joined without any waiting:
//   1. One workgroup per 64 keys; wave w takes the 16-key tile w % 4 of it and every fourth
//      (layer, KV head) pair.  v_mfma_f32_16x16x32_bf16 with the 16 keys as rows and the KV
//      head's (H / H_kv) * N query rows as columns, both operands straight from global memory in
//      the instruction's own layout.  The wave writes its base-2 logits and, per softmax row,
//      the (max, sum exp2) of its 16 keys to the workspace.
//   2. Every workgroup then counts itself in; the one that arrives LAST (whichever it is: nobody
//      waits for anybody, so nothing depends on which workgroups run together) finds all of phase 1
//      in the workspace and finishes alone: row log-sum-exps from the tile partials, per key the
//      max over heads / max or mean over layers / mean over the valid queries, and then the
//      selection on the scores in LDS with the same arithmetic, in the same order, as
//      sp_pool_select (fp64, index order), so both paths keep the same tokens.
// One workgroup alone is several times slower at phase 1 (one compute unit's load path and ALUs
// against sixteen or more), and phase 2 on compact rows wastes no lanes on the operand's unused
// columns.
#include "sp_lds.h"
#include "sp_score_internal.h"
#include "sp_select_core.h"

namespace sp {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kFusedThreads = 1024;
constexpr int kFusedMaxKeys = 2048;
constexpr int kFusedMaxRows = 16;         // query rows per KV head: (H / H_kv) * N, the columns of one MFMA
constexpr int kFusedMaxSoftmaxRows = 4096;  // L * H * N: their log-sum-exps are held in LDS in phase 2

// arrivals of the call in flight; the finishing workgroup puts it back to zero
static __device__ unsigned int fused_arrivals;

struct FusedDev {
  int M, L, N, H, H_kv, G, d, layer_reduce;
  int M_pad;       // keys rounded up to whole workgroups (64)
  float scale;
  int64_t ts, hs;  // token / head stride of the K cache, elements
  const uint16_t* q;
  const int32_t* n_valid;
  float* scores;
  float* lse_out;
  float* logit2;   // workspace [L * H_kv][rows][M_pad]: base-2 logits
  float* part_m;   // workspace [L * H_kv][rows][M_pad / 16]: max of a tile's logits
  float* part_z;   //           ... and the sum of exp2(logit - that max)
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
// Reduction over aligned groups of 16 lanes; every lane of the group gets the result.
// Lane ^ 1, lane ^ 2 inside the quad, then the mirrored half row and the mirrored row.
template <class Op>
__device__ __forceinline__ float reduce16(float v) {
  v = Op::f(v, dpp_f32<0xB1>(v));
  v = Op::f(v, dpp_f32<0x4E>(v));
  v = Op::f(v, dpp_f32<0x141>(v));
  v = Op::f(v, dpp_f32<0x140>(v));
  return v;
}

__device__ __forceinline__ void store_f32_agent(float* dst, float v) { store32_agent(dst, __float_as_uint(v)); }

template <int D>
__global__ __launch_bounds__(kFusedThreads) void fused_short_kernel(const FusedDev p) {
  constexpr int KS = D / 32;  // MFMA steps along the head dim
  __shared__ double wide[kFusedMaxKeys];  // first the pooled scores, then (as 64-bit keys) the selection's keys
  static_assert(kFusedMaxKeys >= kSingleMaxChunks, "the selection's keys reuse the pooled scores' room");
  __shared__ float score_lds[kFusedMaxKeys];
  // the softmax rows' log-sum-exps, later the chunk scores
  __shared__ __align__(16) unsigned char lse_or_cs[kSingleMaxChunks * sizeof(double)];
  static_assert(kFusedMaxSoftmaxRows * sizeof(float) <= sizeof(lse_or_cs), "the log-sum-exps must fit");
  __shared__ unsigned int ticket;
  __shared__ unsigned short item_tab[kFusedMaxSoftmaxRows];  // phase 2b's order of softmax rows, with marks
  constexpr int kRowMask = 0x0fff, kLayerEnds = 0x4000, kQueryEnds = 0x8000;
  static_assert(kFusedMaxSoftmaxRows <= kRowMask + 1, "a row number must fit under the marks");
  float* lse_lds = reinterpret_cast<float*>(lse_or_cs);
  double* cs_lds = reinterpret_cast<double*>(lse_or_cs);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rows = p.G * p.N;  // <= 16; query row r = (query) * G + (head of the group)
  const int pairs = p.L * p.H_kv;
  const int tiles = p.M_pad >> 4;
  const float scale2 = p.scale * 1.44269504088896341f;  // logits in units of ln 2: exp2 is one instruction

  // ---- phase 1: logits and tile partials of 64 keys ----
  {
    const int n = lane & 15, kg = lane >> 4;  // operand row / column; 8-element group of the head dim
    const int tile = blockIdx.x * 4 + (wave & 3);
    const int key0 = tile * 16 + 4 * kg;      // the lane's logits: query row n, keys key0 .. key0 + 3
    const int krow = min(tile * 16 + n, p.M - 1);  // rows past the end read the last key again; masked below
    for (int pair = wave >> 2; pair < pairs; pair += 4) {
      const int l = pair / p.H_kv, g = pair - l * p.H_kv;
      const int nn = n < rows ? n : 0;
      const int nq = nn / p.G, j = nn - nq * p.G;
      const uint16_t* qp = p.q + (((int64_t)l * p.N + nq) * p.H + g * p.G + j) * D + 8 * kg;
      const uint16_t* kp = p.k[l] + (int64_t)g * p.hs + (int64_t)krow * p.ts + 8 * kg;
      uint4 qv[KS], kv[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        qv[ks] = *reinterpret_cast<const uint4*>(qp + 32 * ks);
        kv[ks] = *reinterpret_cast<const uint4*>(kp + 32 * ks);
      }
      f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (n >= rows) qv[ks] = make_uint4(0, 0, 0, 0);  // columns beyond the last query row
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kv[ks]), __builtin_bit_cast(bf16x8, qv[ks]), c, 0, 0, 0);
      }
      float m = -INFINITY;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        c[jj] = key0 + jj < p.M ? scale2 * c[jj] : -INFINITY;
        m = fmaxf(m, c[jj]);
      }
      m = fmaxf(m, __shfl_xor(m, 16));
      m = fmaxf(m, __shfl_xor(m, 32));  // -inf for a tile wholly past the end of the prompt
      float z = 0.f;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) z += (m == -INFINITY) ? 0.f : exp2f(c[jj] - m);
      z += __shfl_xor(z, 16);
      z += __shfl_xor(z, 32);
      if (n < rows) {
        const int64_t row = (int64_t)pair * rows + n;
        store128_agent(p.logit2 + row * p.M_pad + key0, u32x4{__float_as_uint(c[0]), __float_as_uint(c[1]), __float_as_uint(c[2]), __float_as_uint(c[3])});
        if (kg == 0) {
          store_f32_agent(p.part_m + row * tiles + tile, m);
          store_f32_agent(p.part_z + row * tiles + tile, z);
        }
      }
    }
  }

  // ---- count in; all but the last to arrive are done ----
  wait_vmcnt<0>();  // this thread's workspace stores have been performed
  __syncthreads();
  if (tid == 0) ticket = atomicAdd(&fused_arrivals, 1u);
  __syncthreads();
  if (ticket != gridDim.x - 1) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // nothing read below may come from before the count
  if (tid == 0) __hip_atomic_store(&fused_arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // Reads of what other workgroups wrote cost a trip to memory each (microseconds): the first
  // logits phase 2b needs are requested now, so that they travel together with 2a's partials.
  int nv = p.n_valid ? p.n_valid[0] : p.N;
  nv = max(1, min(nv, p.N));
  const int heads_total = p.L * p.H;   // head f of all layers: softmax row (f / G) * rows + nq * G + f % G
  const int items = nv * heads_total;  // per key, item i: query i / heads_total, head i % heads_total
  // (divisions are dear: each item's row and its end-of-layer / end-of-query marks are tabulated once)
  for (int i = tid; i < items; i += kFusedThreads) {
    const int nq = i / heads_total, f = i - nq * heads_total;
    const int row = (f / p.G) * rows + nq * p.G + f % p.G;
    item_tab[i] = (unsigned short)(row | ((f + 1) % p.H == 0 ? kLayerEnds : 0) | (f + 1 == heads_total ? kQueryEnds : 0));
  }
  __syncthreads();
  constexpr int kAhead = 16;
  float ahead[kAhead];
#pragma unroll
  for (int u = 0; u < kAhead; ++u)
    ahead[u] = p.logit2[(int64_t)(item_tab[min(u, items - 1)] & kRowMask) * p.M_pad + min(tid, p.M - 1)];

  // ---- phase 2a: row log-sum-exps (base 2) from the tile partials, 16 lanes per row ----
  const int softmax_rows = pairs * rows;
  constexpr int kPartsPerLane = kFusedMaxKeys / 16 / 16;  // a row's tiles, dealt to 16 lanes
  for (int r0 = 0; r0 < softmax_rows; r0 += kFusedThreads / 16) {
    const int row = r0 + (tid >> 4), sub = tid & 15;
    const bool live = row < softmax_rows;
    float pm[kPartsPerLane], pz[kPartsPerLane];  // all loads first: one round trip
#pragma unroll
    for (int u = 0; u < kPartsPerLane; ++u) {
      const int x = sub + 16 * u;
      const bool has = live && x < tiles;
      const int64_t at = has ? (int64_t)row * tiles + x : 0;
      pm[u] = p.part_m[at];
      pz[u] = p.part_z[at];
      if (!has) { pm[u] = -INFINITY; pz[u] = 0.f; }
    }
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < kPartsPerLane; ++u) m = fmaxf(m, pm[u]);
    m = reduce16<OpMax>(m);  // finite for a live row: its first tile has a key
    float z = 0.f;
#pragma unroll
    for (int u = 0; u < kPartsPerLane; ++u) z += (pm[u] == -INFINITY) ? 0.f : pz[u] * exp2f(pm[u] - m);
    z = reduce16<OpAdd>(z);
    if (live && sub == 0) {
      const float lse2 = m + log2f(z);
      lse_lds[row] = lse2;
      if (p.lse_out) {
        const int pair = row / rows, r = row - pair * rows;
        const int l = pair / p.H_kv, g = pair - l * p.H_kv, nq = r / p.G, j = r - nq * p.G;
        p.lse_out[((int64_t)l * p.N + nq) * p.H + g * p.G + j] = 0.69314718055994531f * lse2;
      }
    }
  }
  __syncthreads();

  // ---- phase 2b: the scores, one key per thread at a time ----
  const float denom = (p.layer_reduce == SP_LAYER_MAX) ? (float)nv : (float)nv * (float)p.L;
  for (int key = tid; key < p.M; key += kFusedThreads) {
    float acc = 0.f;
    float over_layers = (p.layer_reduce == SP_LAYER_MAX) ? -INFINITY : 0.f;
    float lm = -INFINITY;  // max over the layer's heads of log2 p
    for (int i0 = 0; i0 < items; i0 += kAhead) {
      float v[kAhead];
      if (i0 == 0 && key == tid) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) v[u] = ahead[u];
      } else {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) v[u] = p.logit2[(int64_t)(item_tab[min(i0 + u, items - 1)] & kRowMask) * p.M_pad + key];
      }
      int entry[kAhead];
      float lse[kAhead];  // (no branches here: the table and log-sum-exp reads go out together)
#pragma unroll
      for (int u = 0; u < kAhead; ++u) entry[u] = item_tab[min(i0 + u, items - 1)];
#pragma unroll
      for (int u = 0; u < kAhead; ++u) lse[u] = lse_lds[entry[u] & kRowMask];
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        if (i0 + u >= items) entry[u] = 0, v[u] = -INFINITY;
        lm = fmaxf(lm, v[u] - lse[u]);
        if (entry[u] & kLayerEnds) {
          if (p.layer_reduce == SP_LAYER_MAX) over_layers = fmaxf(over_layers, lm);
          else over_layers += exp2f(lm);
          lm = -INFINITY;
        }
        if (entry[u] & kQueryEnds) {
          acc += (p.layer_reduce == SP_LAYER_MAX) ? exp2f(over_layers) : over_layers;
          over_layers = (p.layer_reduce == SP_LAYER_MAX) ? -INFINITY : 0.f;
        }
      }
    }
    const float sc = acc / denom;
    score_lds[key] = sc;
    p.scores[key] = sc;
  }
  __syncthreads();

  // ---- phase 2c: Sec. 3.2.3 on the scores in LDS; the same fp64 arithmetic in the same order as sp_pool_select ----
  const SelDev& sp_ = p.sel;
  for (int i = tid; i < p.M; i += kFusedThreads) {
    const int a = max(0, i - sp_.radius), e = min(p.M - 1, i + sp_.radius);
    double sum = 0.0;
#pragma unroll 8
    for (int x = a; x <= e; ++x) sum += (double)score_lds[x];
    wide[i] = sum / (double)(e - a + 1);
  }
  __syncthreads();
  const int n_chunks = (p.M + sp_.chunk - 1) / sp_.chunk;
  for (int j = tid; j < n_chunks; j += kFusedThreads) {
    const int s0 = j * sp_.chunk, s1 = min(s0 + sp_.chunk, p.M);
    double t = 0.0;
#pragma unroll 8
    for (int x = s0; x < s1; ++x) t += wide[x];
    const double mean = t / (double)(s1 - s0);
    cs_lds[j] = mean;
    if (sp_.chunk_scores_out) sp_.chunk_scores_out[j] = (float)mean;
  }
  __syncthreads();
  select_emit_single(sp_, cs_lds, reinterpret_cast<uint64_t*>(wide));
}

static bool fused_shape_ok(const sp_score_args* a) {
  if (a->B != 1 || a->T < 1 || a->T > kFusedMaxKeys || a->rope_theta != 0.f || a->d_block_table || a->k_dtype != SP_K_BF16) return false;
  if (a->H_kv < 1 || a->H % a->H_kv != 0 || (a->d != 64 && a->d != 128)) return false;
  const int G = a->H / a->H_kv;
  if (G * a->N > kFusedMaxRows || (int64_t)a->L * a->H * a->N > kFusedMaxSoftmaxRows) return false;
  return true;
}

size_t fused_workspace_bytes(const sp_score_args* a) {
  if (!fused_shape_ok(a)) return 0;
  const size_t m_pad = ((size_t)a->T + 63) / 64 * 64;
  const size_t softmax_rows = (size_t)a->L * a->H * a->N;
  return align_up(softmax_rows * m_pad * sizeof(float), 256) + 2 * align_up(softmax_rows * (m_pad / 16) * sizeof(float), 256);
}

}  // namespace sp

extern "C" sp_status sp_score_pool_select(const sp_score_args* a, const sp_pool_select_args* s, void* hip_stream) {
  using namespace sp;
  if (!a || !s) return SP_ENULL;
  // each half is checked as the separate calls check it (the selection's workspace is not needed here)
  if (a->B < 1 || a->N < 1 || a->N > SP_MAX_QUERIES || a->L < 1 || a->L > SP_MAX_LAYERS) return SP_EINVAL;
  if (a->H < 1 || a->H_kv < 1 || a->H % a->H_kv != 0) return SP_EINVAL;
  if (a->d != 64 && a->d != 128) return SP_EINVAL;
  if (a->T < 0 || a->T >= (int64_t)INT32_MAX) return SP_EINVAL;
  if (a->layer_reduce != SP_LAYER_MAX && a->layer_reduce != SP_LAYER_MEAN) return SP_EINVAL;
  if (!finite_f32(a->scale) || a->scale <= 0.f || !finite_f32(a->rope_theta) || a->rope_theta < 0.f) return SP_EINVAL;
  if (a->flags & ~(uint32_t)(SP_SCORE_EXCLUSIVE_DEVICE | SP_SCORE_WORKSPACE_KEPT)) return SP_EINVAL;
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
  // what the single launch covers
  if (!fused_shape_ok(a) || (a->T + s->chunk - 1) / s->chunk > kSingleMaxChunks) return SP_EUNSUPPORTED;
  const size_t need = fused_workspace_bytes(a);
  if (!a->d_workspace || a->workspace_bytes < need) return SP_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(a->d_workspace) & 255u) return SP_EALIGN;

  FusedDev dev;
  dev.M = (int)a->T; dev.L = a->L; dev.N = a->N; dev.H = a->H; dev.H_kv = a->H_kv; dev.G = a->H / a->H_kv; dev.d = a->d;
  dev.layer_reduce = a->layer_reduce;
  dev.scale = a->scale;
  dev.ts = a->k_token_stride; dev.hs = a->k_head_stride;
  dev.q = static_cast<const uint16_t*>(a->d_q);
  dev.n_valid = a->d_n_valid;
  dev.scores = a->d_scores;
  dev.lse_out = a->d_lse;
  dev.M_pad = (dev.M + 63) / 64 * 64;
  {
    const size_t softmax_rows = (size_t)a->L * a->H * a->N;
    char* ws = static_cast<char*>(a->d_workspace);
    dev.logit2 = reinterpret_cast<float*>(ws);
    ws += align_up(softmax_rows * dev.M_pad * sizeof(float), 256);
    dev.part_m = reinterpret_cast<float*>(ws);
    ws += align_up(softmax_rows * (dev.M_pad / 16) * sizeof(float), 256);
    dev.part_z = reinterpret_cast<float*>(ws);
  }
  for (int l = 0; l < SP_MAX_LAYERS; ++l) dev.k[l] = l < a->L ? static_cast<const uint16_t*>(a->k_layers[l]) : nullptr;
  SelDev& p = dev.sel;
  p.B = 1; p.T = (int)a->T; p.chunk = s->chunk; p.radius = (s->pool_window - 1) / 2;
  p.keep_rate = s->keep_rate; p.capacity = s->kept_capacity;
  p.cu = s->d_cu_seqlens; p.scores = s->d_scores; p.kept_idx = s->d_kept_idx; p.cu_keep = s->d_cu_keep;
  p.chunk_scores_out = s->d_chunk_scores;
  p.cu_chunks = nullptr; p.seq_keep = nullptr; p.cs = nullptr; p.chunk_off = nullptr;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const dim3 grid(dev.M_pad / 64), block(kFusedThreads);
  if (a->d == 64) hipLaunchKernelGGL((fused_short_kernel<64>), grid, block, 0, stream, dev);
  else hipLaunchKernelGGL((fused_short_kernel<128>), grid, block, 0, stream, dev);
  return launch_status();
}
