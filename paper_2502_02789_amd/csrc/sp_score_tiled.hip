// Two-pass MFMA scorer for ragged batches (and every other shape the single-pass kernel does
// not take, as long as the query rows of one KV head fit a 32-column MFMA tile).
//
// Same quantity as the other scoring kernels: row softmax of the stored queries against the
// prompt keys (Sec. 3.2 equation of arXiv 2502.02789), max over heads, max/mean over layers,
// mean over queries (Sec. 3.2.2).  The K cache is read twice, as by the plain-FMA general
// kernels, whose workspace layout (64-key tiles numbered over the whole batch, per-tile
// (max, sum) partials, per-row log-sum-exps) is reused together with their tile-table and
// combine kernels:
//
//   pass 0  every wave owns one 64-key tile of one sequence and walks over (layer, KV head)
//           "slabs"; per slab it streams the KV head's 32 query rows and its two 32-key tiles
//           through a private two-slot LDS ring with direct global->LDS loads (XOR-swizzled so
//           that MFMA operand reads are conflict free), forms the 64 x 32 logits with
//           v_mfma_f32_32x32x16_bf16 and writes each row's (max, sum exp) over its keys;
//   combine the general kernels' combine step turns the partials into log-sum-exps;
//   pass 1  the same walk; the row's log-sum-exp arrives with the query tile, logits become
//           log2-probabilities, the max over the heads of a KV group is a quad DPP max, the
//           max over KV heads and layers (or the sum over layers of the per-layer max) stays
//           in registers: a wave owns its keys for all heads and layers of its layer group;
//   finish  the layer groups' results (the grid is cut along the layers too, to give the chip
//           several workgroups per CU to balance) are merged and averaged over the queries.
//
// No wave waits for another one: there is no cross-workgroup exchange in this path.
#include <mutex>

#include "sp_tile_walker.h"

namespace sp {

// (cos, sin) table for the MFMA kernels.  A lane of the key operand holds, for k-step t, the
// eight elements 16t + 8*half + i of row `col`; their rotation partners (Sec. 3.2 scores need the
// keys as the model sees them: rotated by their position) sit d/2 further on, i.e. in k-step
// t + KS/2 of the same lane.  So per 32-key tile and t < KS/2 a lane needs eight (cos, sin) pairs:
// four 16-byte loads, laid out here so that each of them is one dense 1 KiB wave-wide load:
//   entry [((tile32 * KS/2 + t) * 4 + j) * 64 + half * 32 + col] = (cos, sin) of frequencies
//   f = 16t + 8*half + 2j and f + 1 at position tile32 * 32 + col.
// Positions are counted inside a sequence, so only those below the longest sequence are filled in
// (the room is sized for one sequence of all T tokens).
__global__ __launch_bounds__(256) void rope_tile_table_kernel(float4* __restrict__ table, int64_t n, int ks_half,
                                                               int half_d, double log2_theta, int B,
                                                               const int32_t* __restrict__ cu) {
  __shared__ int longest;
  if (threadIdx.x == 0) longest = 0;
  __syncthreads();
  int mine = 0;
  for (int b = threadIdx.x; b < B; b += 256) mine = max(mine, cu[b + 1] - cu[b]);
  if (mine > 0) atomicMax(&longest, mine);
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n || ((i >> 8) / ks_half) * 32 >= longest) return;
  const int lane = (int)(i & 63), j = (int)((i >> 6) & 3);
  const int t = (int)((i >> 8) % ks_half);
  const int64_t tile32 = (i >> 8) / ks_half;
  const int f = 16 * t + 8 * (lane >> 5) + 2 * j;
  const double pos = (double)(tile32 * 32 + (lane & 31));
  const float2 a = rope_cos_sin(pos, f, half_d, log2_theta), b = rope_cos_sin(pos, f + 1, half_d, log2_theta);
  table[i] = make_float4(a.x, a.y, b.x, b.y);
}

// One slab's step along the stream: tiles in stream order are Q(s) K0(s) K1(s) Q(s+1) ...,
// tile number x of slab s sits in ring slot (3s + x) & 1.
struct SlabCursor {
  int l, g;
  __device__ __forceinline__ void advance(int H_kv, int l_last) {
    if (++g == H_kv) { g = 0; l = min(l + 1, l_last); }  // past the end: the last layer again (nobody consumes it)
  }
};

template <int D, int PASS, bool MEAN, bool ROPE, bool FP8>
__global__ __launch_bounds__(kTiledThreads) void tiled_score_kernel(const TiledDev p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  using TW = TileWalker<D, ROPE, FP8>;
  const int tile = blockIdx.x * kTiledWaves + (threadIdx.x >> 6);
  if (tile >= p.tile_cu[p.B]) return;  // (no workgroup barrier anywhere in this kernel)
  const int l0 = blockIdx.y * p.layers_per_group;
  const int l1 = min(p.L, l0 + p.layers_per_group);
  if (l0 >= l1) return;
  TW w(p, smem, __builtin_amdgcn_readfirstlane(tile));
  const int n_slabs = (l1 - l0) * p.H_kv;

  // PASS 0: row statistics; 1: probabilities; 2: row statistics, and the logits are kept for logit_score_kernel
  float smax[PASS == 1 ? 32 : 1], tot[(PASS == 1 && MEAN) ? 32 : 1];
#pragma unroll
  for (int i = 0; i < (PASS == 1 ? 32 : 1); ++i) smax[i] = -INFINITY;
#pragma unroll
  for (int i = 0; i < ((PASS == 1 && MEAN) ? 32 : 1); ++i) tot[i] = 0.f;

  // keep mode: up to kKeepHeld 16-byte units of logits wait here, entry held_first + k in held[k]
  constexpr int kKeepHeld = 8;
  u32x4 held[PASS == 2 ? kKeepHeld : 1];
  int held_n = 0, held_first = 0;
  auto flush_held = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < (PASS == 2 ? kKeepHeld : 1); ++k) {
      if (k < held_n) {
        const int e = held_first + k;  // entry number: slab * keep_units + unit
        const int sl = p.keep_units == 2 ? e >> 1 : e, unit = p.keep_units == 2 ? e & 1 : 0;
        w.store_logits(held[k], l0 + sl / p.H_kv, sl % p.H_kv, unit);
      }
    }
    held_first += held_n;
    held_n = 0;
  };
  SlabCursor cur{l0, 0}, nxt{l0, 0};
  int done = 0;  // pass 0: slabs whose statistics have been written out
  w.template issue_queries<PASS == 1>(l0, 0, 0, 0);
  w.issue_keys(l0, 0, 0, 1);
  w.issue_rope(0);
  nxt.advance(p.H_kv, l1 - 1);

  auto body = [&](auto par_tag) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_tag)::value;  // parity of the slab = ring slot of its query tile
    w.slab_scale(cur.l, cur.g);
    w.wait_tile(PAR);
    w.read_queries(PAR);
    float neg_lse2 = 0.f;
    if (PASS == 1) {
      int c = w.col;
      asm volatile("" : "+v"(c));
      neg_lse2 = -1.4426950408889634f * __uint_as_float(lds_peek(w.lse_lds + PAR * 256 + c * 4));
    }
    w.slot_free();
    w.issue_keys(cur.l, cur.g, 1, PAR);
    w.run_m = -INFINITY;
    w.run_s = 0.f;
    // key tile 0
    w.wait_tile(PAR ^ 1);
    w.mfma_tile(0, PAR ^ 1);
    w.slot_free();
    w.template issue_queries<PASS == 1>(nxt.l, nxt.g, PAR ^ 1, PAR ^ 1);
    if (PASS != 1) w.stats_tile(0);
    // key tile 1
    w.wait_tile(PAR);
    w.mfma_tile(1, PAR);
    w.slot_free();
    w.issue_keys(nxt.l, nxt.g, 0, PAR);
    if (PASS != 1) {
      w.stats_tile(1);
      if constexpr (PASS == 2) {
       for (int unit = 0; unit < p.keep_units; ++unit) {
        const u32x4 v = w.transposed_logits(unit);
        switch (held_n) {
          case 0: held[0] = v; break;
          case 1: held[1] = v; break;
          case 2: held[2] = v; break;
          case 3: held[3] = v; break;
          case 4: held[4] = v; break;
          case 5: held[5] = v; break;
          case 6: held[6] = v; break;
          default: held[7] = v; break;
        }
        held_n = __builtin_amdgcn_readfirstlane(held_n + 1);
        if (held_n == kKeepHeld) flush_held();
       }
      }
      w.keep_partial();
      if (w.partials_full(PASS == 2 ? kPartBufBytes - kKeepStageBytes : kPartBufBytes)) {
        done += w.part_n;
        w.flush_partials(done - w.part_n, l0, tile);
      }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = fmaf(w.acc[kb][i], w.c2, neg_lse2);
        if (p.lgG >= 1) {
#pragma unroll
          for (int i = 0; i < 16; ++i) x[i] = max_quad_xor1(x[i]);
        }
        if (p.lgG >= 2) {
#pragma unroll
          for (int i = 0; i < 16; ++i) x[i] = max_quad_xor2(x[i]);
        }
        if (p.lgG >= 3) {
#pragma unroll
          for (int i = 0; i < 16; ++i) x[i] = fmaxf(x[i], __shfl_xor(x[i], 4, kWave));
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) smax[kb * 16 + i] = fmaxf(smax[kb * 16 + i], x[i]);
      }
      if (MEAN && cur.g == p.H_kv - 1) {  // the layer is complete: its max probability joins the sum
#pragma unroll
        for (int i = 0; i < 32; ++i) {
          tot[i] += fast_exp2(smax[i]);
          smax[i] = -INFINITY;
        }
      }
    }
    cur = nxt;
    nxt.advance(p.H_kv, l1 - 1);
  };

  for (int s = 0; s < n_slabs; s += 2) {
    body(std::integral_constant<int, 0>{});
    if (s + 1 < n_slabs) body(std::integral_constant<int, 1>{});
  }
  if (PASS == 2 && held_n > 0) flush_held();
  if (PASS != 1 && w.part_n > 0) w.flush_partials(done, l0, tile);
  wait_vmcnt<0>();  // loads issued past the end land before the wave (and its LDS) goes away

  if (PASS == 1) {
    int c = w.col, h = w.half;
    asm volatile("" : "+v"(c), "+v"(h));
    if (c < p.Gp * p.N && (c & (p.Gp - 1)) == 0) {
      float* dst = p.group_scores + ((int64_t)blockIdx.y * p.N + (c >> p.lgG)) * p.T + w.tok0;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = kb * 32 + (i >> 2) * 8 + h * 4 + (i & 3);
          if (key < w.rows_in) dst[key] = MEAN ? tot[kb * 16 + i] : smax[kb * 16 + i];
        }
    }
  }
}

// keep mode, second pass: one thread per token walks over the kept logits of all layers and KV
// heads (16 bytes each, neighbouring tokens neighbouring in memory), turns them into
// log2-probabilities with the rows' log-sum-exps and aggregates as the other kernels do.
template <bool MEAN>
__global__ __launch_bounds__(256) void logit_score_kernel(const TiledDev p) {
  // four threads per token, each with every fourth layer: four times the loads in flight
  const int64_t tok = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 2;
  const int part = threadIdx.x & 3;
  if (tok >= p.T) return;  // (the four threads of a token leave together)
  const int b = upper_segment(p.cu, p.B, (int)tok);
  const int rows = p.Gp * p.N;
  float best[kKeepMaxRows], tot[kKeepMaxRows];  // per query (entries beyond N unused)
#pragma unroll
  for (int n = 0; n < kKeepMaxRows; ++n) { best[n] = -INFINITY; tot[n] = 0.f; }
  const float* lse_b = p.ws_lse + (int64_t)b * p.N * p.H;
  const bool one_query_four_heads = p.N == 1 && p.G == 4;  // the common shape: a KV head's four log-sum-exps are one 16-byte load
  for (int l = part; l < p.L; l += 4) {
    const float* lse_l = lse_b + (int64_t)l * p.B * p.N * p.H;
    const float* src = p.logits + ((int64_t)l * p.H_kv * p.keep_units * p.T + tok) * kKeepRows;
    if (one_query_four_heads) {
      float m = best[0];
#pragma unroll 8
      for (int g = 0; g < p.H_kv; ++g) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (int64_t)g * p.T * kKeepRows));
        const u32x4 e = *reinterpret_cast<const u32x4*>(lse_l + g * 4);
#pragma unroll
        for (int r = 0; r < 4; ++r) m = fmaxf(m, __uint_as_float(v[r]) - 1.4426950408889634f * __uint_as_float(e[r]));
      }
      best[0] = m;
      if (MEAN) { tot[0] += fast_exp2(best[0]); best[0] = -INFINITY; }
      continue;
    }
#pragma unroll 2
    for (int gu = 0; gu < p.H_kv * p.keep_units; ++gu) {
      const int g = p.keep_units == 2 ? gu >> 1 : gu, unit = p.keep_units == 2 ? gu & 1 : 0;
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (int64_t)gu * p.T * kKeepRows));
#pragma unroll
      for (int rr = 0; rr < kKeepRows; ++rr) {
        const int r = unit * kKeepRows + rr;
        if (r < rows) {
          const int n = r >> p.lgG, h = g * p.G + ((r & (p.Gp - 1)) < p.G ? (r & (p.Gp - 1)) : 0);
          const float x = __uint_as_float(v[rr]) - 1.4426950408889634f * lse_l[n * p.H + h];
#pragma unroll
          for (int q = 0; q < kKeepMaxRows; ++q)
            if (q == n) best[q] = fmaxf(best[q], x);
        }
      }
    }
    if (MEAN) {
#pragma unroll
      for (int n = 0; n < kKeepMaxRows; ++n) { tot[n] += fast_exp2(best[n]); best[n] = -INFINITY; }
    }
  }
#pragma unroll
  for (int n = 0; n < kKeepMaxRows; ++n) {  // fold the four threads of the token
    if (MEAN) {
      tot[n] += __shfl_xor(tot[n], 1, kWave);
      tot[n] += __shfl_xor(tot[n], 2, kWave);
    } else {
      best[n] = fmaxf(best[n], __shfl_xor(best[n], 1, kWave));
      best[n] = fmaxf(best[n], __shfl_xor(best[n], 2, kWave));
    }
  }
  if (part != 0) return;
  int nv = p.n_valid ? p.n_valid[b] : p.N;
  nv = max(1, min(nv, p.N));
  float sum = 0.f;
#pragma unroll
  for (int n = 0; n < kKeepMaxRows; ++n)
    if (n < nv) sum += MEAN ? tot[n] : fast_exp2(best[n]);
  p.scores[tok] = sum / (MEAN ? (float)nv * (float)p.L : (float)nv);
}

// merge the layer groups and average over the valid queries; one thread per token
__global__ __launch_bounds__(256) void tiled_finish_kernel(const TiledDev p) {
  const int64_t tok = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tok >= p.T) return;
  const int b = upper_segment(p.cu, p.B, (int)tok);
  int nv = p.n_valid ? p.n_valid[b] : p.N;
  nv = max(1, min(nv, p.N));
  float sum = 0.f;
  for (int n = 0; n < nv; ++n) {
    if (p.layer_reduce == SP_LAYER_MAX) {
      float m = -INFINITY;
      for (int g = 0; g < p.n_groups; ++g) m = fmaxf(m, p.group_scores[((int64_t)g * p.N + n) * p.T + tok]);
      sum += fast_exp2(m);
    } else {
      for (int g = 0; g < p.n_groups; ++g) sum += p.group_scores[((int64_t)g * p.N + n) * p.T + tok];
    }
  }
  const float denom = (p.layer_reduce == SP_LAYER_MAX) ? (float)nv : (float)nv * (float)p.L;
  p.scores[tok] = sum / denom;
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static int tiled_max_tiles(const sp_score_args* a) { return (int)(a->T / kWaveKeys) + a->B; }

static void tiled_grouping(const sp_score_args* a, int* layers_per_group, int* n_groups) {
  const int wgs = (tiled_max_tiles(a) + kTiledWaves - 1) / kTiledWaves;
  int groups = std::min(a->L, (kTiledTargetWGs + wgs - 1) / wgs);
  groups = std::max(groups, 1);
  *layers_per_group = (a->L + groups - 1) / groups;
  *n_groups = (a->L + *layers_per_group - 1) / *layers_per_group;
}

static int padded_group(const sp_score_args* a) {
  const int G = a->H / a->H_kv;
  return G <= 2 ? G : G <= 4 ? 4 : 8;
}

bool tiled_supported(const sp_score_args* a) {
  // (an 8-bit cache behind a block table: the 8 or 16 rows of one direct load must lie in one page)
  if (a->k_dtype == SP_K_FP8_E4M3 && a->d_block_table && a->page_size < (a->d == 64 ? 16 : 8)) return false;
  if (a->H / a->H_kv > 8) return false;
  if (padded_group(a) * a->N > 32) return false;
  if (a->T < 1) return false;
  return true;
}

// Keep mode: with few query rows per KV head the logits of a key (16 bytes per layer and KV
// head) are much smaller than the key itself (2*d bytes), so the second pass reads the logits
// the first pass wrote instead of reading the K cache again.
#ifndef SP_TILED_KEEP_MAX_BYTES
#define SP_TILED_KEEP_MAX_BYTES (16ull << 30)
#endif
static int keep_units(const sp_score_args* a) { return padded_group(a) * a->N <= kKeepRows ? 1 : 2; }
static size_t keep_bytes(const sp_score_args* a) {
  return sizeof(float) * kKeepRows * keep_units(a) * (size_t)a->L * a->H_kv * (size_t)a->T;
}
static bool keep_mode(const sp_score_args* a) {
  return padded_group(a) * a->N <= kKeepMaxRows && keep_bytes(a) <= SP_TILED_KEEP_MAX_BYTES;
}

static size_t tiled_main_workspace_bytes(const sp_score_args* a) {
  if (seq_supported(a)) return seq_workspace_bytes(a);
  if (keep_mode(a)) return align_up(keep_bytes(a), 256);
  int lpg, groups;
  tiled_grouping(a, &lpg, &groups);
  return align_up(sizeof(float) * (size_t)groups * a->N * (size_t)a->T, 256);
}
// 16-byte entries of the rotation table: positions 0 .. T-1 in whole 32-key tiles
static int64_t rope_tile_table_entries(const sp_score_args* a) { return (a->T + 31) / 32 * (a->d / 32) * 4 * 64; }

size_t tiled_extra_workspace_bytes(const sp_score_args* a) {
  if (!tiled_supported(a)) return 0;
  return tiled_main_workspace_bytes(a) +
         (a->rope_theta > 0.f ? align_up(sizeof(float4) * (size_t)rope_tile_table_entries(a), 256) : 0);
}

template <int D, int PASS, bool MEAN, bool ROPE, bool FP8>
static sp_status launch_tiled(const TiledDev& dev, hipStream_t stream) {
  auto kernel = tiled_score_kernel<D, PASS, MEAN, ROPE, FP8>;
  const size_t smem = TileWalker<D, ROPE, FP8>::smem_bytes();
  static std::mutex mu;  // once per kernel and device
  static bool prepared[kMaxDevices] = {};
  {
    std::lock_guard<std::mutex> lock(mu);
    const int slot = current_device();
    if (!prepared[slot]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)smem) != hipSuccess)
        return SP_ELAUNCH;
      prepared[slot] = true;
    }
  }
  const dim3 grid((dev.max_tiles + kTiledWaves - 1) / kTiledWaves, dev.n_groups);
  hipLaunchKernelGGL(kernel, grid, dim3(kTiledThreads), smem, stream, dev);
  return launch_status();
}

template <int D, bool ROPE, bool FP8>
static sp_status tiled_passes(const TiledDev& dev, const ScoreDev& gen, hipStream_t stream) {
  if (dev.logits) {
    const sp_status st = launch_tiled<D, 2, false, ROPE, FP8>(dev, stream);
    if (st != SP_OK) return st;
    launch_lse_combine(gen, stream);
    const dim3 grid((unsigned)((dev.T * 4 + 255) / 256));
    if (dev.layer_reduce == SP_LAYER_MEAN) hipLaunchKernelGGL(logit_score_kernel<true>, grid, dim3(256), 0, stream, dev);
    else hipLaunchKernelGGL(logit_score_kernel<false>, grid, dim3(256), 0, stream, dev);
    return launch_status();
  }
  sp_status st = launch_tiled<D, 0, false, ROPE, FP8>(dev, stream);
  if (st != SP_OK) return st;
  launch_lse_combine(gen, stream);
  st = dev.layer_reduce == SP_LAYER_MEAN ? launch_tiled<D, 1, true, ROPE, FP8>(dev, stream)
                                         : launch_tiled<D, 1, false, ROPE, FP8>(dev, stream);
  if (st != SP_OK) return st;
  hipLaunchKernelGGL(tiled_finish_kernel, dim3((unsigned)((dev.T + 255) / 256)), dim3(256), 0, stream, dev);
  return launch_status();
}

// `gen` carries the general kernels' workspace pointers (tile table, partials, log-sum-exps),
// already laid out and with the tile table kernel launched; `extra` is this path's own part.
sp_status tiled_score(const sp_score_args* a, const ScoreDev& gen, void* extra, hipStream_t stream) {
  TiledDev dev;
  dev.B = a->B; dev.N = a->N; dev.L = a->L; dev.H = a->H; dev.H_kv = a->H_kv; dev.G = a->H / a->H_kv;
  dev.lgG = dev.G == 1 ? 0 : dev.G == 2 ? 1 : dev.G <= 4 ? 2 : 3;
  dev.Gp = 1 << dev.lgG;
  tiled_grouping(a, &dev.layers_per_group, &dev.n_groups);
  dev.max_tiles = gen.max_tiles;
  dev.layer_reduce = a->layer_reduce;
  dev.scale = a->scale;
  dev.c = a->scale * 1.4426950408889634f;
  dev.ts = a->k_token_stride; dev.hs = a->k_head_stride; dev.T = a->T;
  dev.q = gen.q; dev.cu = gen.cu; dev.n_valid = gen.n_valid; dev.tile_cu = gen.tile_cu;
  dev.ws_lse = gen.ws_lse; dev.part = gen.part;
  dev.lse_out = a->d_lse;
  dev.k_scale = a->d_k_scale;
  dev.seq_limit = 0;
  dev.seq_order = nullptr;
  if (seq_supported(a)) {  // one pass over K, a workgroup per (sequence, layer group)
    seq_grouping(a, &dev.slabs_per_group, &dev.n_groups, &dev.groups_per_layer);
    if (dev.lgG < 2) { dev.lgG = 2; dev.Gp = 4; }  // (one or two heads per KV head: padded to four on this path)
    dev.layers_per_group = 0;
    dev.group_scores = static_cast<float*>(extra);
    dev.logits = nullptr;
    dev.keep_units = 0;
    dev.scores = a->d_scores;
    dev.block_table = gen.block_table; dev.lg_page = gen.lg_page; dev.blocks_per_seq = gen.blocks_per_seq;
    dev.page_stride = gen.k_page_stride;
    for (int l = 0; l < SP_MAX_LAYERS; ++l) dev.k[l] = gen.k[l];
    dev.rope_tiles = nullptr;
    dev.seq_limit = seq_max_keys(a);
    return seq_score(a, dev, stream);
  }
  const bool keep = keep_mode(a);
  dev.group_scores = keep ? nullptr : static_cast<float*>(extra);
  dev.logits = keep ? static_cast<float*>(extra) : nullptr;
  dev.keep_units = keep_units(a);
  dev.scores = a->d_scores;
  dev.block_table = gen.block_table; dev.lg_page = gen.lg_page; dev.blocks_per_seq = gen.blocks_per_seq;
  dev.page_stride = gen.k_page_stride;
  for (int l = 0; l < SP_MAX_LAYERS; ++l) dev.k[l] = gen.k[l];
  dev.rope_tiles = nullptr;
  if (a->rope_theta > 0.f) {  // the table follows this path's other workspace part
    float4* table = reinterpret_cast<float4*>(static_cast<char*>(extra) + tiled_main_workspace_bytes(a));
    const int64_t n = rope_tile_table_entries(a);
    hipLaunchKernelGGL(rope_tile_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, table, n,
                       a->d / 32, a->d / 2, std::log2((double)a->rope_theta), a->B, a->d_cu_seqlens);
    dev.rope_tiles = table;
    return a->d == 64 ? tiled_passes<64, true, false>(dev, gen, stream) : tiled_passes<128, true, false>(dev, gen, stream);
  }
  if (a->k_dtype == SP_K_FP8_E4M3)
    return a->d == 64 ? tiled_passes<64, false, true>(dev, gen, stream) : tiled_passes<128, false, true>(dev, gen, stream);
  return a->d == 64 ? tiled_passes<64, false, false>(dev, gen, stream) : tiled_passes<128, false, false>(dev, gen, stream);
}

}  // namespace sp
