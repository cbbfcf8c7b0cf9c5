// sp_score: attention scores of the stored queries against the K cache, row softmax over
// the prompt keys (Sec. 3.2 equation of arXiv 2502.02789) and the max/mean aggregation
// over heads, layers and queries (Sec. 3.2.2).
//
// This file holds the argument checks, the dispatcher and the GENERAL kernels, which accept
// every shape the header allows (ragged batches, any G = H/H_kv <= 8, N <= 16, d in {64,128}).
// They read the K cache twice (once for the row statistics, once for the probabilities) and
// use plain fp32 FMAs.  The single-pass MFMA kernel for one long prompt lives in
// sp_score_stream.hip, the two-pass MFMA kernels for ragged batches in sp_score_tiled.hip; the
// dispatcher takes the first of the three that fits the shape.
#include "sp_common.h"
#include "sp_score_internal.h"

namespace sp {

constexpr int kTileKeys = 64;  // keys per tile of the general kernels (one per lane)

// ---------------------------------------------------------------------------------------
// tile table: tile_cu[b] = number of 64-key tiles in sequences before b
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void tile_table_kernel(int B, const int32_t* __restrict__ cu,
                                                          int32_t* __restrict__ tile_cu) {
  block_prefix_table(B, [&](int b) { return (cu[b + 1] - cu[b] + kTileKeys - 1) / kTileKeys; }, tile_cu);
}

// Rotary encoding of one un-rotated row held in registers: pair (t, t + D/2) turns by the
// angle whose (cos, sin) is rope_row[t]; results are rounded as a bf16 cache would hold them.
template <int D>
__device__ __forceinline__ void rope_row_inplace(float (&kf)[D], const float2* __restrict__ rope_row) {
#pragma unroll
  for (int t = 0; t < D / 2; ++t) {
    const float2 cs = rope_row[t];
    const float2 turned = rope_turn(kf[t], kf[t + D / 2], cs);
    kf[t] = turned.x;
    kf[t + D / 2] = turned.y;
  }
}

// (cos, sin) of pos * theta^(-2t/d) for every position and pair; the angle is formed in fp64
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ table, int64_t n, int half,
                                                          double log2_theta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int t = (int)(i % half);
  const double pos = (double)(i / half);
  table[i] = rope_cos_sin(pos, t, half, log2_theta);
}

// rotated copy of the un-rotated queries [L, B, N, H, d]; one thread per (row, pair)
__global__ __launch_bounds__(256) void rope_q_kernel(const uint16_t* __restrict__ q_raw, uint16_t* __restrict__ q_rot,
                                                      const int32_t* __restrict__ q_pos, int B, int N, int H, int half,
                                                      int64_t n, double log2_theta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int t = (int)(i % half);
  const int64_t row = i / half;               // ((l * B + b) * N + nq) * H + h
  const int nq = (int)((row / H) % N);
  const int b = (int)((row / ((int64_t)H * N)) % B);
  const float2 cs = rope_cos_sin((double)q_pos[b * N + nq], t, half, log2_theta);
  const uint16_t* src = q_raw + row * 2 * half;
  const float lo = __uint_as_float((uint32_t)src[t] << 16), hi = __uint_as_float((uint32_t)src[t + half] << 16);
  const float2 turned = rope_turn(lo, hi, cs);
  q_rot[row * 2 * half + t] = (uint16_t)(__float_as_uint(turned.x) >> 16);
  q_rot[row * 2 * half + t + half] = (uint16_t)(__float_as_uint(turned.y) >> 16);
}

template <int D>
__device__ __forceinline__ void load_k_row(const uint16_t* __restrict__ kp, bool valid, float (&kf)[D]) {
  const uint4* p4 = reinterpret_cast<const uint4*>(kp);
#pragma unroll
  for (int c = 0; c < D / 8; ++c) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (valid) v = p4[c];
    kf[8 * c + 0] = bf16_lo(v.x); kf[8 * c + 1] = bf16_hi(v.x);
    kf[8 * c + 2] = bf16_lo(v.y); kf[8 * c + 3] = bf16_hi(v.y);
    kf[8 * c + 4] = bf16_lo(v.z); kf[8 * c + 5] = bf16_hi(v.z);
    kf[8 * c + 6] = bf16_lo(v.w); kf[8 * c + 7] = bf16_hi(v.w);
  }
}

// the same from an 8-bit cache (OCP E4M3 codes, one byte per element): decoded exactly to fp32
template <int D>
__device__ __forceinline__ void load_k_row_fp8(const unsigned char* __restrict__ kp, bool valid, float (&kf)[D]) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  const uint4* p4 = reinterpret_cast<const uint4*>(kp);
#pragma unroll
  for (int c = 0; c < D / 16; ++c) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (valid) v = p4[c];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[j], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[j], true);
      kf[16 * c + 4 * j + 0] = lo[0]; kf[16 * c + 4 * j + 1] = lo[1];
      kf[16 * c + 4 * j + 2] = hi[0]; kf[16 * c + 4 * j + 3] = hi[1];
    }
  }
}
// row `off` (in elements) of layer l, either storage; scale of (layer, KV head) for an 8-bit cache
template <int D>
__device__ __forceinline__ void load_key(const ScoreDev& p, int l, int64_t off, bool valid, float (&kf)[D]) {
  if (p.k_fp8) load_k_row_fp8<D>(reinterpret_cast<const unsigned char*>(p.k[l]) + off, valid, kf);
  else load_k_row<D>(p.k[l] + off, valid, kf);
}
__device__ __forceinline__ float key_scale(const ScoreDev& p, int l, int g) {
  return (p.k_fp8 && p.k_scale) ? p.scale * p.k_scale[l * p.H_kv + g] : p.scale;
}

// element offset of key `key` of sequence b (first token seq0) inside a layer, KV head 0
__device__ __forceinline__ int64_t key_row_offset(const ScoreDev& p, int b, int seq0, int key) {
  if (!p.block_table) return (int64_t)(seq0 + key) * p.k_token_stride;
  const int page = p.block_table[(int64_t)b * p.blocks_per_seq + (key >> p.lg_page)];
  return (int64_t)page * p.k_page_stride + (int64_t)(key & ((1 << p.lg_page) - 1)) * p.k_token_stride;
}

// <q row, k row> with the q row at a wave-uniform address
template <int D>
__device__ __forceinline__ float dot_row(const uint16_t* __restrict__ qp, const float (&kf)[D]) {
  const uint4* q4 = reinterpret_cast<const uint4*>(qp);
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
  for (int c = 0; c < D / 8; ++c) {
    const uint4 v = q4[c];
    a0 = fmaf(bf16_lo(v.x), kf[8 * c + 0], a0); a1 = fmaf(bf16_hi(v.x), kf[8 * c + 1], a1);
    a2 = fmaf(bf16_lo(v.y), kf[8 * c + 2], a2); a3 = fmaf(bf16_hi(v.y), kf[8 * c + 3], a3);
    a0 = fmaf(bf16_lo(v.z), kf[8 * c + 4], a0); a1 = fmaf(bf16_hi(v.z), kf[8 * c + 5], a1);
    a2 = fmaf(bf16_lo(v.w), kf[8 * c + 6], a2); a3 = fmaf(bf16_hi(v.w), kf[8 * c + 7], a3);
  }
  return (a0 + a1) + (a2 + a3);
}

// ---------------------------------------------------------------------------------------
// pass 1: per (tile, kv head, layer) the partial (max, sum exp) of every query row
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void lse_partial_kernel(const ScoreDev p) {
  const int tile = blockIdx.x;
  const int n_tiles = p.tile_cu[p.B];
  if (tile >= n_tiles) return;
  const int g = blockIdx.y, l = blockIdx.z;
  const int lane = threadIdx.x;
  const int b = upper_segment(p.tile_cu, p.B, tile);
  const int seq0 = p.cu[b];
  const int M = p.cu[b + 1] - seq0;
  const int key = (tile - p.tile_cu[b]) * kTileKeys + lane;
  const bool valid = key < M;
  float kf[D];
  load_key<D>(p, l, key_row_offset(p, b, seq0, valid ? key : 0) + (int64_t)g * p.k_head_stride, valid, kf);
  if (p.rope) rope_row_inplace<D>(kf, p.rope + (int64_t)(valid ? key : 0) * (D / 2));
  const float scale = key_scale(p, l, g);
  for (int n = 0; n < p.N; ++n) {
    for (int j = 0; j < p.G; ++j) {
      const int h = g * p.G + j;
      const uint16_t* qp = p.q + ((((int64_t)l * p.B + b) * p.N + n) * p.H + h) * D;
      const float s = valid ? scale * dot_row<D>(qp, kf) : -INFINITY;
      const float m = wave_max(s);                       // finite: lane 0 of a tile is always valid
      const float e = valid ? expf(s - m) : 0.f;
      const float z = wave_sum(e);
      if (lane == 0) p.part[((int64_t)(l * p.N + n) * p.H + h) * p.max_tiles + tile] = make_float2(m, z);
    }
  }
}

// ---------------------------------------------------------------------------------------
// pass 1b: combine the tile partials of a row into its log-sum-exp
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void lse_combine_kernel(const ScoreDev p) {
  const int row = blockIdx.x;  // ((l*B + b)*N + n)*H + h
  const int lane = threadIdx.x;
  const int h = row % p.H;
  const int n = (row / p.H) % p.N;
  const int b = (row / (p.H * p.N)) % p.B;
  const int l = row / (p.H * p.N * p.B);
  const int t0 = p.tile_cu[b], t1 = p.tile_cu[b + 1];
  const float2* part = p.part + ((int64_t)(l * p.N + n) * p.H + h) * p.max_tiles;
  float m = -INFINITY, z = 0.f;
  for (int t = t0 + lane; t < t1; t += kWave) {
    const float2 v = part[t];
    const float mn = fmaxf(m, v.x);
    z = z * expf(m - mn) + v.y * expf(v.x - mn);  // first step: z = 0 * exp(-inf) = 0
    m = mn;
  }
  const float mw = wave_max(m);
  const float zw = wave_sum(m == -INFINITY ? 0.f : z * expf(m - mw));
  if (lane == 0) {
    const float lse = (t1 > t0) ? mw + logf(zw) : 0.f;
    p.ws_lse[row] = lse;
    if (p.lse_out) p.lse_out[row] = lse;
  }
}

// ---------------------------------------------------------------------------------------
// pass 2: probabilities, max over heads, max/mean over layers, mean over valid queries
// one block = one 64-key tile; its 4 waves split the KV heads
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void score_accum_kernel(const ScoreDev p) {
  __shared__ float red[2][4][SP_MAX_QUERIES][kWave];
  const int tile = blockIdx.x;
  const int n_tiles = p.tile_cu[p.B];
  if (tile >= n_tiles) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int b = upper_segment(p.tile_cu, p.B, tile);
  const int seq0 = p.cu[b];
  const int M = p.cu[b + 1] - seq0;
  const int key = (tile - p.tile_cu[b]) * kTileKeys + lane;
  const bool valid = key < M;
  const int64_t tok = seq0 + (valid ? key : 0);
  const int64_t row_off = key_row_offset(p, b, seq0, valid ? key : 0);

  float tot[SP_MAX_QUERIES];
#pragma unroll
  for (int n = 0; n < SP_MAX_QUERIES; ++n) tot[n] = (p.layer_reduce == SP_LAYER_MAX) ? -INFINITY : 0.f;

  for (int l = 0; l < p.L; ++l) {
    float nmax[SP_MAX_QUERIES];
#pragma unroll
    for (int n = 0; n < SP_MAX_QUERIES; ++n) nmax[n] = -INFINITY;
    for (int g = wave; g < p.H_kv; g += 4) {
      float kf[D];
      load_key<D>(p, l, row_off + (int64_t)g * p.k_head_stride, valid, kf);
      if (p.rope) rope_row_inplace<D>(kf, p.rope + (int64_t)(valid ? key : 0) * (D / 2));
      const float scale = key_scale(p, l, g);
#pragma unroll
      for (int n = 0; n < SP_MAX_QUERIES; ++n) {
        if (n < p.N) {
          float mx = nmax[n];
          for (int j = 0; j < p.G; ++j) {
            const int h = g * p.G + j;
            const int64_t row = (((int64_t)l * p.B + b) * p.N + n) * p.H + h;
            const float s = scale * dot_row<D>(p.q + row * D, kf);
            mx = fmaxf(mx, s - p.ws_lse[row]);
          }
          nmax[n] = mx;
        }
      }
    }
    const int buf = l & 1;
#pragma unroll
    for (int n = 0; n < SP_MAX_QUERIES; ++n)
      if (n < p.N) red[buf][wave][n][lane] = nmax[n];
    __syncthreads();  // one barrier per layer: the buffers alternate
#pragma unroll
    for (int n = 0; n < SP_MAX_QUERIES; ++n) {
      if (n < p.N) {
        const float x = fmaxf(fmaxf(red[buf][0][n][lane], red[buf][1][n][lane]),
                              fmaxf(red[buf][2][n][lane], red[buf][3][n][lane]));
        if (p.layer_reduce == SP_LAYER_MAX) tot[n] = fmaxf(tot[n], x);
        else tot[n] += expf(x);
      }
    }
  }
  if (wave == 0 && valid) {
    int nv = p.n_valid ? p.n_valid[b] : p.N;
    nv = max(1, min(nv, p.N));
    float acc = 0.f;
#pragma unroll
    for (int n = 0; n < SP_MAX_QUERIES; ++n)
      if (n < nv) acc += (p.layer_reduce == SP_LAYER_MAX) ? expf(tot[n]) : tot[n];
    const float denom = (p.layer_reduce == SP_LAYER_MAX) ? (float)nv : (float)nv * (float)p.L;
    p.scores[tok] = acc / denom;
  }
}

// the status words (and, for the team kernel's layout, its epoch: sp_score_check then looks at word 1)
__global__ void clear_word_kernel(uint32_t* word) { word[0] = word[1] = word[2] = word[3] = 0; }

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static bool shape_ok(const sp_score_args* a) {
  if (a->B < 1 || a->N < 1 || a->N > SP_MAX_QUERIES || a->L < 1 || a->L > SP_MAX_LAYERS) return false;
  if (a->H < 1 || a->H_kv < 1 || a->H % a->H_kv != 0 || a->H / a->H_kv > 8) return false;
  if (a->d != 64 && a->d != 128) return false;
  if (a->T < 0 || a->T >= (int64_t)INT32_MAX) return false;
  if ((int64_t)a->L * a->B * a->N * a->H >= (int64_t)INT32_MAX) return false;
  if (a->layer_reduce != SP_LAYER_MAX && a->layer_reduce != SP_LAYER_MEAN) return false;
  if (a->k_dtype != SP_K_BF16 && a->k_dtype != SP_K_FP8_E4M3) return false;
  return true;
}

static int general_max_tiles(const sp_score_args* a) { return (int)(a->T / kTileKeys) + a->B; }

// the single-pass kernels are taken only on the caller's promise of an otherwise idle device
bool single_pass_wanted(const sp_score_args* a) {
  // Few query rows per KV head and a prompt short enough for the batch kernel, which keeps a sequence's logits
  // on chip and needs no exchange between workgroups: measured faster than the all-workgroup kernel up to 8K
  // keys (one query, 32 layers, head dim 128; us): 2K keys 38 against 135, 4K 57 against 137, 8K 127 against 159.
  if (tiled_supported(a) && seq_supported(a)) return false;
  return (a->flags & SP_SCORE_EXCLUSIVE_DEVICE) != 0 && (team_supported(a) || stream_supported(a));
}
// where the single-pass kernel that sp_score would pick keeps its "a wait expired" word
static size_t single_pass_status_offset(const sp_score_args* a) {
  return team_supported(a) ? team_status_offset(a) : stream_status_offset(a);
}

size_t general_workspace_bytes(const sp_score_args* a, bool with_tiled) {
  size_t bytes = align_up(sizeof(int32_t) * ((size_t)a->B + 1), 256);
  bytes += align_up(sizeof(float) * (size_t)a->L * a->B * a->N * a->H, 256);
  bytes += align_up(sizeof(float2) * (size_t)a->L * a->N * a->H * general_max_tiles(a), 256);
  if (a->rope_theta > 0.f) {  // (cos, sin) table for positions 0..T-1 and a rotated copy of the queries
    bytes += align_up(sizeof(float2) * (size_t)a->T * (a->d / 2), 256);
    bytes += align_up(sizeof(uint16_t) * (size_t)a->L * a->B * a->N * a->H * a->d, 256);
  }
  if (with_tiled) bytes += tiled_extra_workspace_bytes(a);
  return bytes;
}

void launch_lse_combine(const ScoreDev& p, hipStream_t stream) {
  hipLaunchKernelGGL(lse_combine_kernel, dim3(p.L * p.B * p.N * p.H), dim3(64), 0, stream, p);
}

// these paths have no bounded waits: leave "no wait expired" where sp_score_check looks
static void clear_stream_status(const sp_score_args* a, hipStream_t stream) {
  const size_t status_off = single_pass_wanted(a) ? single_pass_status_offset(a) : 0;
  if (status_off)
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, stream,
                       reinterpret_cast<uint32_t*>(static_cast<char*>(a->d_workspace) + status_off));
}

sp_status general_score(const sp_score_args* a, hipStream_t stream, bool allow_mfma) {
  ScoreDev p;
  fill_score_dev(a, &p);
  p.max_tiles = general_max_tiles(a);
  char* ws = static_cast<char*>(a->d_workspace);
  p.tile_cu = reinterpret_cast<int32_t*>(ws);
  ws += align_up(sizeof(int32_t) * ((size_t)a->B + 1), 256);
  p.ws_lse = reinterpret_cast<float*>(ws);
  ws += align_up(sizeof(float) * (size_t)a->L * a->B * a->N * a->H, 256);
  p.part = reinterpret_cast<float2*>(ws);
  ws += align_up(sizeof(float2) * (size_t)a->L * a->N * a->H * general_max_tiles(a), 256);
  if (a->rope_theta > 0.f) {
    float2* table = reinterpret_cast<float2*>(ws);
    ws += align_up(sizeof(float2) * (size_t)a->T * (a->d / 2), 256);
    uint16_t* q_rot = reinterpret_cast<uint16_t*>(ws);
    ws += align_up(sizeof(uint16_t) * (size_t)a->L * a->B * a->N * a->H * a->d, 256);
    const double log2_theta = std::log2((double)a->rope_theta);
    const int half = a->d / 2;
    const int64_t n_tab = a->T * half;
    if (n_tab > 0 && !(allow_mfma && tiled_supported(a)))  // (the MFMA kernels bring a table in their own layout)
      hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n_tab + 255) / 256)), dim3(256), 0, stream, table, n_tab,
                         half, log2_theta);
    const int64_t n_q = (int64_t)a->L * a->B * a->N * a->H * half;
    hipLaunchKernelGGL(rope_q_kernel, dim3((unsigned)((n_q + 255) / 256)), dim3(256), 0, stream, p.q, q_rot, a->d_q_pos,
                       a->B, a->N, a->H, half, n_q, log2_theta);
    p.rope = table;
    p.q = q_rot;
  }

  // (the single-pass batch kernel does not look at the tile table)
  if (!(allow_mfma && tiled_supported(a) && seq_supported(a)))
    hipLaunchKernelGGL(tile_table_kernel, dim3(1), dim3(1024), 0, stream, p.B, p.cu, p.tile_cu);
  if (allow_mfma && tiled_supported(a)) {
    const sp_status st = tiled_score(a, p, ws, stream);
    clear_stream_status(a, stream);
    return st != SP_OK ? st : launch_status();
  }
  const dim3 grid1(p.max_tiles, p.H_kv, p.L);
  const int rows = p.L * p.B * p.N * p.H;
  if (p.d == 64) {
    hipLaunchKernelGGL(lse_partial_kernel<64>, grid1, dim3(64), 0, stream, p);
    hipLaunchKernelGGL(lse_combine_kernel, dim3(rows), dim3(64), 0, stream, p);
    hipLaunchKernelGGL(score_accum_kernel<64>, dim3(p.max_tiles), dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(lse_partial_kernel<128>, grid1, dim3(64), 0, stream, p);
    hipLaunchKernelGGL(lse_combine_kernel, dim3(rows), dim3(64), 0, stream, p);
    hipLaunchKernelGGL(score_accum_kernel<128>, dim3(p.max_tiles), dim3(256), 0, stream, p);
  }
  clear_stream_status(a, stream);
  return launch_status();
}

void fill_score_dev(const sp_score_args* a, ScoreDev* p) {
  p->B = a->B; p->N = a->N; p->L = a->L; p->H = a->H; p->H_kv = a->H_kv; p->G = a->H / a->H_kv; p->d = a->d;
  p->T = (int)a->T;
  p->max_tiles = 0;
  p->layer_reduce = a->layer_reduce;
  p->scale = a->scale;
  p->k_token_stride = a->k_token_stride;
  p->k_head_stride = a->k_head_stride;
  p->q = static_cast<const uint16_t*>(a->d_q);
  p->cu = a->d_cu_seqlens;
  p->n_valid = a->d_n_valid;
  p->tile_cu = nullptr; p->ws_lse = nullptr; p->part = nullptr;
  p->scores = a->d_scores;
  p->lse_out = a->d_lse;
  p->rope = nullptr;
  p->block_table = a->d_block_table;
  p->lg_page = 0;
  while (a->d_block_table && (1 << p->lg_page) < a->page_size) ++p->lg_page;
  p->blocks_per_seq = a->blocks_per_seq;
  p->k_page_stride = a->k_page_stride;
  p->k_fp8 = a->k_dtype == SP_K_FP8_E4M3;
  p->k_scale = a->d_k_scale;
  for (int l = 0; l < SP_MAX_LAYERS; ++l)
    p->k[l] = l < a->L ? static_cast<const uint16_t*>(a->k_layers[l]) : nullptr;
}

}  // namespace sp

extern "C" size_t sp_score_workspace_bytes(const sp_score_args* a) {
  if (!a || !sp::shape_ok(a)) return 0;
  // a shape that goes to the single-pass kernel never runs the tiled kernels on this workspace
  // (sp_score_general uses the plain kernels), so their kept-logits buffer is not asked for
  const bool single = sp::single_pass_wanted(a);
  const size_t general = sp::general_workspace_bytes(a, /*with_tiled=*/!single);
  const size_t stream = single ? std::max(sp::stream_workspace_bytes(a), sp::team_workspace_bytes(a)) : 0;
  // (sp_score_pool_select takes its logits' room from the same workspace)
  return std::max(std::max(general, stream), sp::fused_workspace_bytes(a));
}

static sp_status check_score_args(const sp_score_args* a) {
  if (!a) return SP_ENULL;
  if (!sp::shape_ok(a)) return SP_EINVAL;
  if (!a->d_q || !a->k_layers || !a->d_cu_seqlens || !a->d_scores) return SP_ENULL;
  for (int l = 0; l < a->L; ++l)
    if (!a->k_layers[l]) return SP_ENULL;
  if (!sp::finite_f32(a->rope_theta) || a->rope_theta < 0.f) return SP_EINVAL;
  if (a->rope_theta == 0.f && a->d_q_pos != nullptr) return SP_EINVAL;
  if (a->rope_theta > 0.f && a->d_q_pos == nullptr) return SP_ENULL;
  if (!sp::finite_f32(a->scale) || a->scale <= 0.f) return SP_EINVAL;
  if (a->flags & ~(uint32_t)(SP_SCORE_EXCLUSIVE_DEVICE | SP_SCORE_WORKSPACE_KEPT)) return SP_EINVAL;
  if (a->k_token_stride < 0 || a->k_head_stride < 0 || a->max_seqlen < 0) return SP_EINVAL;
  if (a->d_block_table) {
    if (a->page_size < 8 || (a->page_size & (a->page_size - 1)) != 0 || a->blocks_per_seq < 1) return SP_EINVAL;
    if (a->k_page_stride < 0) return SP_EINVAL;
    if (a->k_page_stride & 7) return SP_EALIGN;
  }
  if ((a->k_token_stride & 7) || (a->k_head_stride & 7) || !sp::aligned16(a->d_q)) return SP_EALIGN;
  if (a->k_dtype == SP_K_FP8_E4M3) {
    if (a->rope_theta > 0.f) return SP_EUNSUPPORTED;
    if ((a->k_token_stride & 15) || (a->k_head_stride & 15) || (a->d_block_table && (a->k_page_stride & 15))) return SP_EALIGN;
  } else if (a->d_k_scale) {
    return SP_EINVAL;
  }
  for (int l = 0; l < a->L; ++l)
    if (!sp::aligned16(a->k_layers[l])) return SP_EALIGN;
  if (!a->d_workspace || a->workspace_bytes < sp_score_workspace_bytes(a)) return SP_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(a->d_workspace) & 255u) return SP_EALIGN;
  return SP_OK;
}

extern "C" sp_status sp_score(const sp_score_args* a, void* hip_stream) {
  const sp_status st = check_score_args(a);
  if (st != SP_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (sp::single_pass_wanted(a)) return sp::team_supported(a) ? sp::team_score(a, stream) : sp::stream_score(a, stream);
  return sp::general_score(a, stream, /*allow_mfma=*/true);
}

extern "C" sp_status sp_score_check(const sp_score_args* a, void* hip_stream) {
  const sp_status st = check_score_args(a);
  if (st != SP_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (hipStreamSynchronize(stream) != hipSuccess) return SP_ELAUNCH;
  const size_t off = sp::single_pass_wanted(a) ? sp::single_pass_status_offset(a) : 0;
  if (off == 0) return SP_OK;
  uint32_t words[4] = {0, 0, 0, 0};  // (every single-pass workspace has 256 bytes at `off`)
  if (hipMemcpy(words, static_cast<const char*>(a->d_workspace) + off, sizeof(words), hipMemcpyDeviceToHost) !=
      hipSuccess)
    return SP_ELAUNCH;
  // the team kernel keeps one status word per epoch parity and has moved on to the next epoch
  const uint32_t word = sp::team_supported(a) ? words[(words[2] + 1u) & 1u] : words[0];
  return word == 0 ? SP_OK : SP_ETIMEOUT;
}

extern "C" sp_status sp_score_general(const sp_score_args* a, void* hip_stream) {
  const sp_status st = check_score_args(a);
  if (st != SP_OK) return st;
  return sp::general_score(a, static_cast<hipStream_t>(hip_stream), /*allow_mfma=*/false);
}
