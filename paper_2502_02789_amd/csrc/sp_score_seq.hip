// Single-pass MFMA scorer for batches of short prompts whose KV heads carry few query rows (the
// paper's variants without look-ahead, Sec. 4.3, served many prompts at a time).
//
// Same quantity as the other scoring kernels: row softmax of the stored queries against the
// prompt keys (Sec. 3.2 equation of arXiv 2502.02789), max over heads, max/mean over layers,
// mean over queries (Sec. 3.2.2).  The K cache is read ONCE and no logit ever leaves the chip:
//
//   * A workgroup owns one whole sequence for a group of layers and walks over the group's
//     (layer, KV head) slabs.  Inside a slab its eight waves take the sequence's 64-key tiles in
//     turn (wave w: tiles w, w + 8, ...), stream them through the per-wave two-slot LDS ring of
//     the tiled kernels and multiply them with the KV head's query rows on the matrix cores --
//     with the QUERY rows as the rows of the result, so that a lane ends up with all R <= 8 logits
//     of one key (one v_permlane32_swap per register joins the two 32-key halves of a tile).
//   * Those R logits per key stay in registers for the whole slab (R registers per tile), each
//     lane keeps a running (max, sum exp2) per row, and at the end of the slab the lanes' and the
//     eight waves' statistics are merged (shuffles, one small LDS table, ONE workgroup barrier):
//     every wave then knows the rows' log-sum-exps and turns its held logits into
//     log2-probabilities, folds the heads of a group and keeps the running maximum over KV heads
//     and layers (or the sum over layers of the per-layer maxima) per key in registers.
//   * The stream of tiles never stops at a slab's end: the loads of the next slab's first tiles
//     are in flight while the statistics are merged, and the barrier is a bare s_barrier (no
//     vector-memory wait in front of it).
//   * Each (sequence, layer group) writes its [N][M] partial result; the tiled kernels' finish
//     kernel merges the layer groups and averages over the valid queries.
//
// A sequence must fit the registers: 64 * 8 * kSeqMaxTiles<R> keys.  The host cannot see the
// sequence lengths (they live on the device), so this path is taken only on the caller's promise
// sp_score_args.max_seqlen; a sequence that breaks the promise gets NaN scores (finish kernel).
#include <mutex>

#include "sp_tile_walker.h"

namespace sp {

template <int R> struct SeqLimits { static constexpr int kMaxTiles = (R == 4) ? 16 : 8; };  // tiles per wave

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose counter is a constant in
// every copy of the body (register arrays indexed by it must never be indexed at run time)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

template <int D>
struct SeqAhead {  // the next item of a wave's stream: ph < 0 the slab's query tile, else 32-key half-tile ph of the wave
  int l, g, ph;
};

template <int D, int R, int LG, bool MEAN>
__global__ __launch_bounds__(kTiledThreads) void seq_score_kernel(const TiledDev p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  using TW = TileWalker<D, false>;
  constexpr int MAXT = SeqLimits<R>::kMaxTiles;
  constexpr int GP = 1 << LG;   // heads of a KV group, padded to a power of two
  constexpr int NQ = R >> LG;   // queries whose rows fit the R held rows
  const int b = blockIdx.x;
  const int seq0 = p.cu[b];
  const int M = p.cu[b + 1] - seq0;
  const int n_tiles = (M + kWaveKeys - 1) / kWaveKeys;
  const int l0 = blockIdx.y * p.layers_per_group;
  const int l1 = min(p.L, l0 + p.layers_per_group);
  if (l0 >= l1) return;
  if (M <= 0 || n_tiles > MAXT * kTiledWaves) {
    // no keys: the rows' log-sum-exps are 0 by convention; too many: the sequence is not scored
    // (NaN here, and the finish kernel writes NaN scores for it)
    if (p.lse_out)
      for (int i = threadIdx.x; i < (l1 - l0) * p.N * p.H; i += kTiledThreads)
        p.lse_out[(((int64_t)(l0 + i / (p.N * p.H)) * p.B + b) * p.N) * p.H + i % (p.N * p.H)] =
            M <= 0 ? 0.f : __uint_as_float(0x7FC00000u);
    return;
  }
  TW w(p, smem, typename TW::WholeSequence{}, b);
  const int nt = __builtin_amdgcn_readfirstlane((n_tiles - w.wave + kTiledWaves - 1) / kTiledWaves);  // this wave's tiles
  const int n_slabs = (l1 - l0) * p.H_kv;
  const uint32_t xchg = (uint32_t)reinterpret_cast<uintptr_t>(smem) + kTiledWaves * 2 * TW::TILE_B;  // [2][waves][R] (max, sum)

  float held[MAXT][R];
  float smax[MAXT][NQ], tot[MEAN ? MAXT : 1][NQ];
#pragma unroll
  for (int t = 0; t < MAXT; ++t)
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      smax[t][n] = -INFINITY;
      if (MEAN) tot[MEAN ? t : 0][n] = 0.f;
    }

  SeqAhead<D> ah{l0, 0, -1};
  auto issue_next = [&](int slot) __attribute__((always_inline)) {
    if (ah.ph < 0) {
      w.template issue_queries<false>(ah.l, ah.g, slot, 0);
    } else {
      const int key_first = ((w.wave + (ah.ph >> 1) * kTiledWaves) * 2 + (ah.ph & 1)) * 32;
      const int rows = min(32, M - key_first);
      w.issue_key_rows(ah.l, ah.g, rows > 0 ? key_first : 0, rows, slot);
    }
    if (++ah.ph == 2 * nt) {
      ah.ph = -1;
      if (++ah.g == p.H_kv) { ah.g = 0; ah.l = min(ah.l + 1, l1 - 1); }  // past the end: the last layer again (nobody consumes it)
    }
  };
  issue_next(0);
  issue_next(1);
  int pos = 0;  // items consumed so far; item number x sits in ring slot x & 1
  int l = l0, g = 0;

#pragma unroll 1
  for (int s = 0; s < n_slabs; ++s) {
    {
      const int slot = pos & 1;
      w.wait_tile(slot);
      w.read_queries(slot);
      w.slot_free();
      issue_next(slot);
      ++pos;
    }
    float rm[R], rs[R];  // this lane's running max and sum of exp2 per row, base-2 logits
#pragma unroll
    for (int r = 0; r < R; ++r) { rm[r] = -INFINITY; rs[r] = 0.f; }

    static_for<0, MAXT>([&](auto tc) __attribute__((always_inline)) {
      constexpr int t = decltype(tc)::value;
      if (t < nt) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const int slot = pos & 1;
          w.wait_tile(slot);
          w.template mfma_tile<true>(kb, slot);
          w.slot_free();
          issue_next(slot);
          ++pos;
        }
        // rows 0..3 of a key sit in registers 0..3 of the lower half-wave (rows 4..7 in the upper one); joining
        // the two 32-key halves gives lane x the rows of key x of the 64-key tile
        int left = M - (w.wave + t * kTiledWaves) * kWaveKeys - w.lane;  // > 0: the lane's key exists
        asm volatile("" : "+v"(left));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(w.acc[0][i]), __float_as_uint(w.acc[1][i]), false, false);
          held[t][i] = left > 0 ? __uint_as_float(sw[0]) * p.c : -INFINITY;
          if (R == 8) held[t][4 + i] = left > 0 ? __uint_as_float(sw[1]) * p.c : -INFINITY;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float m_new = fmaxf(rm[r], held[t][r]);
          const float ref = (m_new == -INFINITY) ? 0.f : m_new;
          rs[r] = rs[r] * fast_exp2(rm[r] - ref) + fast_exp2(held[t][r] - ref);
          rm[r] = m_new;
        }
      }
    });

    // the rows' statistics over the wave's keys, then over the workgroup's
    const int par = s & 1;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float mw = wave_max(rm[r]);
      const float ref = (mw == -INFINITY) ? 0.f : mw;
      const float sw = wave_sum(rs[r] * fast_exp2(rm[r] - ref));
      int ln = w.lane;
      asm volatile("" : "+v"(ln));
      if (ln == 0)
        lds_poke64<0>(xchg + ((par * kTiledWaves + w.wave) * R + r) * 8, ((uint64_t)__float_as_uint(sw) << 32) | __float_as_uint(mw));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    float lse2[R];
    {
      int ln = w.lane;
      asm volatile("" : "+v"(ln));
      const uint64_t v = lds_peek64(xchg + (par * kTiledWaves * R + (ln & (kTiledWaves * R - 1))) * 8);  // entry wave * R + row
      float m = __uint_as_float((uint32_t)v), z = __uint_as_float((uint32_t)(v >> 32));
#pragma unroll
      for (int off = R; off < kTiledWaves * R; off <<= 1) {
        const float pm = __shfl_xor(m, off, kWave), pz = __shfl_xor(z, off, kWave);
        const float mn = fmaxf(m, pm);
        const float ref = (mn == -INFINITY) ? 0.f : mn;
        z = z * fast_exp2(m - ref) + pz * fast_exp2(pm - ref);
        m = mn;
      }
      const float lse = m + __builtin_amdgcn_logf(z);  // base 2; lanes x and x + R, x + 2R, ... all hold row x & (R - 1)
#pragma unroll
      for (int r = 0; r < R; ++r) lse2[r] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(lse), r));
      if (p.lse_out && w.wave == 0) {
        const int n = ln >> LG, j = ln & (GP - 1);
        if (ln < R && n < p.N && j < p.G)
          p.lse_out[(((int64_t)l * p.B + b) * p.N + n) * p.H + g * p.G + j] = lse * 0.6931471805599453f;
        w.note_issued(1);
      }
    }

    // log2-probabilities; max over the heads of a group, over KV heads and layers
    static_for<0, MAXT>([&](auto tc) __attribute__((always_inline)) {
      constexpr int t = decltype(tc)::value;
      if (t < nt) {
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
          float v = held[t][n * GP] - lse2[n * GP];
#pragma unroll
          for (int j = 1; j < GP; ++j) v = fmaxf(v, held[t][n * GP + j] - lse2[n * GP + j]);
          smax[t][n] = fmaxf(smax[t][n], v);
        }
      }
    });
    if (MEAN && g == p.H_kv - 1) {  // the layer is complete: its max probability joins the sum
#pragma unroll
      for (int t = 0; t < MAXT; ++t)
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
          tot[MEAN ? t : 0][n] += fast_exp2(smax[t][n]);
          smax[t][n] = -INFINITY;
        }
    }
    if (++g == p.H_kv) { g = 0; ++l; }
  }
  wait_vmcnt<0>();  // loads issued past the end land before the wave (and its LDS) goes away

  static_for<0, MAXT>([&](auto tc) __attribute__((always_inline)) {
    constexpr int t = decltype(tc)::value;
    if (t < nt) {
      const int key = (w.wave + t * kTiledWaves) * kWaveKeys + w.lane;
      if (key < M) {
#pragma unroll
        for (int n = 0; n < NQ; ++n)
          if (n < p.N)
            p.group_scores[((int64_t)blockIdx.y * p.N + n) * p.T + seq0 + key] = MEAN ? tot[MEAN ? t : 0][n] : smax[t][n];
      }
    }
  });
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static int seq_padded_group(const sp_score_args* a) {
  const int G = a->H / a->H_kv;
  return G <= 2 ? G : G <= 4 ? 4 : 8;
}
static int seq_rows(const sp_score_args* a) {  // held rows per key: 4 or 8 (0: too many)
  const int rows = seq_padded_group(a) * a->N;
  return rows <= 4 ? 4 : rows <= 8 ? 8 : 0;
}
int seq_max_keys(const sp_score_args* a) {
  const int R = seq_rows(a);
  return R == 0 ? 0 : kWaveKeys * kTiledWaves * (R == 4 ? SeqLimits<4>::kMaxTiles : SeqLimits<8>::kMaxTiles);
}

// the cut along the layers: about kTiledTargetWGs workgroups
void seq_grouping(const sp_score_args* a, int* layers_per_group, int* n_groups) {
  int groups = std::min(a->L, (kTiledTargetWGs + a->B - 1) / a->B);
  groups = std::max(groups, 1);
  *layers_per_group = (a->L + groups - 1) / groups;
  *n_groups = (a->L + *layers_per_group - 1) / *layers_per_group;
}

bool seq_supported(const sp_score_args* a) {
  if (a->rope_theta > 0.f || a->max_seqlen <= 0) return false;
  const int R = seq_rows(a), Gp = seq_padded_group(a);
  if (R == 0 || a->max_seqlen > seq_max_keys(a)) return false;
  if (Gp < 4) return false;                                 // instantiated: groups of 3..8 heads
  if ((int64_t)a->B * a->L < 512) return false;             // too few (sequence, layer) units to fill the device
  return true;
}

size_t seq_workspace_bytes(const sp_score_args* a) {
  if (!seq_supported(a)) return 0;
  int lpg, groups;
  seq_grouping(a, &lpg, &groups);
  return align_up(sizeof(float) * (size_t)groups * a->N * (size_t)a->T, 256);
}

template <int D, int R, int LG, bool MEAN>
static sp_status launch_seq(const TiledDev& dev, hipStream_t stream) {
  auto kernel = seq_score_kernel<D, R, LG, MEAN>;
  const size_t smem = TileWalker<D, false>::smem_bytes();
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
  hipLaunchKernelGGL(kernel, dim3(dev.B, dev.n_groups), dim3(kTiledThreads), smem, stream, dev);
  return launch_status();
}

template <int D, bool MEAN>
static sp_status seq_by_rows(const TiledDev& dev, int R, hipStream_t stream) {
  if (dev.lgG == 2) return R == 4 ? launch_seq<D, 4, 2, MEAN>(dev, stream) : launch_seq<D, 8, 2, MEAN>(dev, stream);
  return launch_seq<D, 8, 3, MEAN>(dev, stream);
}

// `dev` as the tiled kernels fill it in, with group_scores, layers_per_group, n_groups and
// seq_limit set for this path; the caller runs the finish kernel afterwards
sp_status seq_score(const sp_score_args* a, const TiledDev& dev, hipStream_t stream) {
  const int R = seq_rows(a);
  const bool mean = a->layer_reduce == SP_LAYER_MEAN;
  if (a->d == 64) return mean ? seq_by_rows<64, true>(dev, R, stream) : seq_by_rows<64, false>(dev, R, stream);
  return mean ? seq_by_rows<128, true>(dev, R, stream) : seq_by_rows<128, false>(dev, R, stream);
}

}  // namespace sp
