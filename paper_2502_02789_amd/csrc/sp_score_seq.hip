// Single-pass MFMA scorer for batches of short prompts whose KV heads carry few query rows (the
// paper's variants without look-ahead, Sec. 4.3): many prompts at a time, or one prompt of a few thousand tokens.
//
// Same quantity as the other scoring kernels: row softmax of the stored queries against the
// prompt keys (Sec. 3.2 equation of arXiv 2502.02789), max over heads, max/mean over layers,
// mean over queries (Sec. 3.2.2).  The K cache is read ONCE and no logit ever leaves the chip:
//
//   * The work is cut into units (one whole sequence, one run of (layer, KV head) slabs), numbered with
//     the longest sequences first, and dealt out to one workgroup per compute unit in rounds whose
//     direction alternates: every workgroup gets nearly the same number of keys without any shared
//     counter, and nobody ever waits for another workgroup.
//   * A workgroup walks over the (layer, KV head) slabs of its unit.  Inside a slab its eight waves
//     take the sequence's 64-key tiles in turn (wave w: tiles w, w + 8, ...), stream them through
//     the per-wave two-slot LDS ring of the tiled kernels and multiply them with the KV head's
//     query rows on the matrix cores -- with the QUERY rows as the rows of the result, so that a
//     lane ends up with all R <= 8 logits of one key (one v_permlane32_swap per register joins
//     the two 32-key halves of a tile).
//   * Those R logits per key stay in registers for the whole slab (R registers per tile), each
//     lane keeps a running (max, sum exp2) per row, and at the end of the slab the lanes' and the
//     eight waves' statistics are merged (shuffles, one small LDS table, ONE workgroup barrier):
//     every wave then knows the rows' log-sum-exps and turns its held logits into
//     log2-probabilities, folds the heads of a group and keeps the running maximum over KV heads
//     and layers (or the sum over layers of the per-layer maxima) per key in registers.
//   * The stream of tiles never stops, neither at a slab's end nor between units: the loads run two
//     tiles ahead of the arithmetic straight into the next slab or unit, and the barrier is a bare
//     s_barrier (no vector-memory wait in front of it).
//   * Each unit writes its [N][M] partial result; seq_finish_kernel merges the units of a sequence and
//     averages over the valid queries.
//
// A sequence must fit the registers: 64 * 8 * SeqLimits<R>::kMaxTiles keys.  The host cannot see the
// sequence lengths of a batch (they live on the device), so for B > 1 this path is taken only on the caller's
// promise sp_score_args.max_seqlen; a sequence that breaks the promise gets NaN scores (seq_finish_kernel).
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

// One unit of work: sequence b for the slabs [s0, s1) of slab group grp (slab s = KV head s % H_kv of layer
// s / H_kv; with SP_LAYER_MEAN a group holds whole layers).  Units are numbered with the longest sequences
// first (all groups of a sequence next to each other).
struct SeqUnit {
  int k;  // position in this workgroup's list of units
  int b, grp, seq0, M, nt, s0, s1;
};

// Units are dealt out to the gridDim.x workgroups in rounds, the direction changing with every round
// (workgroup j: units j, 2W-1-j, 2W+j, ...): with the sizes in descending order every workgroup gets
// nearly the same number of keys, and no counter has to be shared.
template <int MAXT>
__device__ __forceinline__ bool seq_next_unit(const TiledDev& p, int wave, int k, SeqUnit* u) {
  const int W = gridDim.x, n_units = p.B * p.n_groups;
  for (;; ++k) {
    const int idx = k * W + ((k & 1) ? W - 1 - (int)blockIdx.x : (int)blockIdx.x);
    if (idx >= n_units) return false;
    const int grp = idx % p.n_groups;
    const int b = p.seq_order ? p.seq_order[idx / p.n_groups] : idx / p.n_groups;  // (no table: batch order)
    const int seq0 = p.cu[b];
    const int M = p.cu[b + 1] - seq0;
    const int n_tiles = (M + kWaveKeys - 1) / kWaveKeys;
    const int s0 = grp * p.slabs_per_group;
    const int s1 = min(p.L * p.H_kv, s0 + p.slabs_per_group);
    // (no keys, or more than the registers hold: nothing to do here, see seq_order_kernel and seq_finish_kernel)
    if (M <= 0 || n_tiles > MAXT * kTiledWaves || s0 >= s1) continue;
    u->k = k; u->b = b; u->grp = grp; u->seq0 = seq0; u->M = M; u->s0 = s0; u->s1 = s1;
    u->nt = __builtin_amdgcn_readfirstlane((n_tiles - wave + kTiledWaves - 1) / kTiledWaves);  // this wave's tiles
    return true;
  }
}

template <int D, int R, int LG, bool MEAN, bool FP8>
__global__ __launch_bounds__(kTiledThreads) void seq_score_kernel(const TiledDev p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  using TW = TileWalker<D, false, FP8>;
  constexpr int MAXT = SeqLimits<R>::kMaxTiles;
  constexpr int GP = 1 << LG;   // heads of a KV group, padded to a power of two
  constexpr int NQ = R >> LG;   // queries whose rows fit the R held rows
  TW w(p, smem, typename TW::WholeSequence{}, 0);
  SeqUnit cur;
  if (!seq_next_unit<MAXT>(p, w.wave, 0, &cur)) return;
  const uint32_t xchg = (uint32_t)reinterpret_cast<uintptr_t>(smem) + kTiledWaves * 2 * TW::TILE_B;  // [2][waves][R] (max, sum)

  // The stream of tiles runs two items ahead of the arithmetic and straight on into the workgroup's
  // next unit: `ah` is the unit, slab and item that is requested next.
  SeqUnit ahu = cur;
  bool ah_live = true;  // false: past the last unit (the last slab is requested again, nobody consumes it)
  int ah_s = cur.s0, ah_ph = -1;  // the slab; ph < 0: its query tile, else 32-key half-tile ph of this wave
  auto issue_next = [&](int slot) __attribute__((always_inline)) {
    w.b = ahu.b;
    w.seq0 = ahu.seq0;
    const int ah_l = ah_s / p.H_kv, ah_g = ah_s - ah_l * p.H_kv;
    if (ah_ph < 0) {
      w.template issue_queries<false>(ah_l, ah_g, slot, 0);
    } else {
      const int key_first = ((w.wave + (ah_ph >> 1) * kTiledWaves) * 2 + (ah_ph & 1)) * 32;
      const int rows = min(32, ahu.M - key_first);
      w.issue_key_rows(ah_l, ah_g, rows > 0 ? key_first : 0, rows, slot);
    }
    if (++ah_ph == 2 * ahu.nt) {
      ah_ph = -1;
      if (++ah_s == ahu.s1) {
        if (ah_live && seq_next_unit<MAXT>(p, w.wave, ahu.k + 1, &ahu)) {
          ah_s = ahu.s0;
        } else {
          ah_live = false;
          ah_s = ahu.s1 - 1;
        }
      }
    }
  };
  issue_next(0);
  issue_next(1);
  int pos = 0;    // items consumed so far; item number x sits in ring slot x & 1
  int slabs = 0;  // slabs finished so far (the exchange table has two halves used in turn)

  float held[MAXT][R];
  float smax[MAXT][NQ], tot[MEAN ? MAXT : 1][NQ];

#pragma unroll 1
  for (;;) {
  const int nt = cur.nt, M = cur.M, b = cur.b;
#pragma unroll
  for (int t = 0; t < MAXT; ++t)
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      smax[t][n] = -INFINITY;
      if (MEAN) tot[MEAN ? t : 0][n] = 0.f;
    }
#pragma unroll 1
  for (int s = cur.s0; s < cur.s1; ++s) {
    const int l = s / p.H_kv, g = s - l * p.H_kv;
    {
      const int slot = pos & 1;
      w.wait_tile(slot);
      w.read_queries(slot);
      w.slot_free();
      issue_next(slot);
      ++pos;
    }
    w.slab_scale(l, g);
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
          held[t][i] = left > 0 ? __uint_as_float(sw[0]) * w.c2 : -INFINITY;
          if (R == 8) held[t][4 + i] = left > 0 ? __uint_as_float(sw[1]) * w.c2 : -INFINITY;
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
    const int par = slabs & 1;
    ++slabs;
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
        if (ln < R && n < p.N && j < p.G)  // (never empty: lane 0 is always inside)
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
  }

  // the unit's result.  (These stores are left out of the count of vector-memory instructions in
  // flight -- a store whose lanes are all beyond the sequence may not be issued at all --, which only
  // makes the next tile waits stricter than they need be.)
  static_for<0, MAXT>([&](auto tc) __attribute__((always_inline)) {
    constexpr int t = decltype(tc)::value;
    if (t < nt) {
      const int key = (w.wave + t * kTiledWaves) * kWaveKeys + w.lane;
      if (key < M) {
#pragma unroll
        for (int n = 0; n < NQ; ++n)
          if (n < p.N)
            p.group_scores[((int64_t)cur.grp * p.N + n) * p.T + cur.seq0 + key] = MEAN ? tot[MEAN ? t : 0][n] : smax[t][n];
      }
    }
  });
  if (!seq_next_unit<MAXT>(p, w.wave, cur.k + 1, &cur)) break;
  }
  wait_vmcnt<0>();  // loads issued past the end land before the wave (and its LDS) goes away
}

// order[r] = the sequence with the r-th most keys (equal lengths: lower index first); one workgroup,
// every thread ranks its sequences by counting those ahead of them
// (and the log-sum-exp rows of the sequences the scoring kernel leaves out: 0 by convention where there are no
// keys, NaN where there are more than `limit`)
__global__ __launch_bounds__(1024) void seq_order_kernel(int B, const int32_t* __restrict__ cu, int32_t* __restrict__ order,
                                                         float* __restrict__ lse_out, int limit, int L, int rows) {
  constexpr int kChunk = 4096;
  __shared__ int32_t len[kChunk];
  for (int b0 = 0; b0 < B; b0 += 1024) {  // (all threads take part in every round: barriers inside)
    const int b = b0 + threadIdx.x;
    const int mine = b < B ? cu[b + 1] - cu[b] : 0;
    int rank = 0;
    for (int c0 = 0; c0 < B; c0 += kChunk) {
      const int n = min(kChunk, B - c0);
      __syncthreads();
      for (int i = threadIdx.x; i < n; i += 1024) len[i] = cu[c0 + i + 1] - cu[c0 + i];
      __syncthreads();
      for (int i = 0; i < n; ++i) rank += (len[i] > mine || (len[i] == mine && c0 + i < b)) ? 1 : 0;
    }
    if (b < B) order[rank] = b;
    if (b < B && lse_out && (mine <= 0 || mine > limit))
      for (int i = 0; i < L * rows; ++i)
        lse_out[((int64_t)(i / rows) * B + b) * rows + i % rows] = mine <= 0 ? 0.f : __uint_as_float(0x7FC00000u);
  }
}

// Merge of the units' partial results and the average over the valid queries (Sec. 3.2.2): a workgroup takes 64
// tokens, each of its 16 waves every sixteenth slab group (one 256-byte read per group and query), the waves'
// results meet in LDS.  Sequences the scoring kernel left out (longer than promised) get NaN.
constexpr int kSeqFinishParts = 16;
__global__ __launch_bounds__(64 * kSeqFinishParts) void seq_finish_kernel(const TiledDev p) {
  __shared__ float red[kSeqFinishParts][2][64];
  const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int64_t tok = (int64_t)blockIdx.x * 64 + lane;
  const bool inside = tok < p.T;
  const bool mean = p.layer_reduce != SP_LAYER_MAX;
  float v[2] = {mean ? 0.f : -INFINITY, mean ? 0.f : -INFINITY};  // (this path has at most two queries per sequence)
  if (inside && mean && p.groups_per_layer > 0) {
    // mean over layers from units smaller than a layer: the groups of a layer hold the log2 of its maxima over
    // their KV heads; the layer's maximum over all heads is their maximum, and the layers' maxima add up
    for (int l = part; l < p.L; l += kSeqFinishParts)
#pragma unroll
      for (int n = 0; n < 2; ++n)
        if (n < p.N) {
          float m = -INFINITY;
          for (int j = 0; j < p.groups_per_layer; ++j)
            m = fmaxf(m, p.group_scores[((int64_t)(l * p.groups_per_layer + j) * p.N + n) * p.T + tok]);
          v[n] += fast_exp2(m);
        }
  } else if (inside) {
    for (int g = part; g < p.n_groups; g += kSeqFinishParts)
#pragma unroll
      for (int n = 0; n < 2; ++n)
        if (n < p.N) {
          const float x = p.group_scores[((int64_t)g * p.N + n) * p.T + tok];
          v[n] = mean ? v[n] + x : fmaxf(v[n], x);
        }
  }
  red[part][0][lane] = v[0];
  red[part][1][lane] = v[1];
  __syncthreads();
  if (part != 0 || !inside) return;
  const int b = upper_segment(p.cu, p.B, (int)tok);
  if (p.cu[b + 1] - p.cu[b] > p.seq_limit) {
    p.scores[tok] = __uint_as_float(0x7FC00000u);
    return;
  }
  int nv = p.n_valid ? p.n_valid[b] : p.N;
  nv = max(1, min(nv, p.N));
  float sum = 0.f;
#pragma unroll
  for (int n = 0; n < 2; ++n)
    if (n < nv) {
      float x = red[0][n][lane];
      for (int q = 1; q < kSeqFinishParts; ++q) x = mean ? x + red[q][n][lane] : fmaxf(x, red[q][n][lane]);
      sum += mean ? x : fast_exp2(x);
    }
  p.scores[tok] = sum / (mean ? (float)nv * (float)p.L : (float)nv);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// heads per KV head as this path lays them out: padded to four or eight (columns of padding heads repeat head
// 0, which changes neither a maximum nor a row's own statistics; one or two heads per KV head are padded to four
// as well, so that the same kernel variants serve them)
static int seq_padded_group(const sp_score_args* a) {
  const int G = a->H / a->H_kv;
  return G <= 4 ? 4 : 8;
}
static int seq_rows(const sp_score_args* a) {  // held rows per key: 4 or 8 (0: too many)
  const int rows = seq_padded_group(a) * a->N;
  return rows <= 4 ? 4 : rows <= 8 ? 8 : 0;
}
int seq_max_keys(const sp_score_args* a) {
  const int R = seq_rows(a);
  return R == 0 ? 0 : kWaveKeys * kTiledWaves * (R == 4 ? SeqLimits<4>::kMaxTiles : SeqLimits<8>::kMaxTiles);
}

// The cut along the (layer, KV head) slabs into units.  With the maximum over layers a
// group may be any run of slabs (a maximum can be completed in any order); with the mean over layers a group
// holds whole layers (a layer's maximum over heads must be complete before it joins the sum).
void seq_grouping(const sp_score_args* a, int* slabs_per_group, int* n_groups, int* groups_per_layer) {
  *groups_per_layer = 0;
  if (a->layer_reduce == SP_LAYER_MEAN && (int64_t)a->B * a->L < 256) {
    // too few whole layers to fill the device: units of a part of a layer's KV heads (the scoring kernel then
    // hands on maxima, as for the maximum over layers, and the merge adds the layers up)
    int per = 1;
    for (int cand = a->H_kv; cand >= 1; --cand)
      if (a->H_kv % cand == 0 && (int64_t)a->B * a->L * (a->H_kv / cand) >= 256) { per = cand; break; }
    if (per < a->H_kv) {
      *slabs_per_group = per;
      *groups_per_layer = a->H_kv / per;
      *n_groups = a->L * *groups_per_layer;
      return;
    }
  }
  const int step = a->layer_reduce == SP_LAYER_MEAN ? a->H_kv : 1;
  const int slabs = a->L * a->H_kv;
  // Units per workgroup (of 256): a unit's end costs several microseconds (its results go out, the next unit's
  // table entries come in), so few large units are better as long as the workgroups' shares stay even, which
  // takes more units the more sequences of different lengths there are.  Measured best (32 layers, 8 KV
  // heads, prompts of 1K to 4K keys): 2 per workgroup for 16 prompts, 2 to 4 for 64, 8 for 256.
  const int per_wg = std::min(8, std::max(2, a->B / 32));
  const int target = 256 * per_wg;
  int groups = std::min(slabs / step, (target + a->B - 1) / a->B);
  groups = std::max(groups, 1);
  int per = (slabs + groups - 1) / groups;
  per = (per + step - 1) / step * step;
  *slabs_per_group = per;
  *n_groups = (slabs + per - 1) / per;
}
// the longest sequence the caller vouches for (one sequence: its length is the host's to see)
static int64_t seq_stated_max(const sp_score_args* a) { return a->B == 1 ? a->T : a->max_seqlen; }

bool seq_supported(const sp_score_args* a) {
  if (a->rope_theta > 0.f || seq_stated_max(a) <= 0) return false;
  if (a->k_dtype == SP_K_FP8_E4M3 && a->d_block_table && a->page_size < (a->d == 64 ? 16 : 8)) return false;
  const int R = seq_rows(a);
  if (R == 0 || seq_stated_max(a) > seq_max_keys(a)) return false;
  if (a->B > 8192) return false;                            // (the sequences are ranked by counting: quadratic in B)
  // too few units to fill the device?
  if ((int64_t)a->B * a->L * a->H_kv < 256) return false;
  return true;
}

static size_t seq_scores_bytes(const sp_score_args* a) {
  int lpg, groups, gpl;
  seq_grouping(a, &lpg, &groups, &gpl);
  return align_up(sizeof(float) * (size_t)groups * a->N * (size_t)a->T, 256);
}

size_t seq_workspace_bytes(const sp_score_args* a) {
  if (!seq_supported(a)) return 0;
  return seq_scores_bytes(a) + align_up(sizeof(int32_t) * (size_t)a->B, 256);  // partial results, then the sequence order
}

static int seq_cu_count() {  // compute units of the current device
  static std::mutex mu;
  static int cached[kMaxDevices] = {};
  std::lock_guard<std::mutex> lock(mu);
  const int slot = current_device();
  if (cached[slot] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, slot) != hipSuccess || n < 1) {
      (void)hipGetLastError();
      n = 256;
    }
    cached[slot] = n;
  }
  return cached[slot];
}

template <int D, int R, int LG, bool MEAN, bool FP8>
static sp_status launch_seq(const TiledDev& dev, hipStream_t stream) {
  auto kernel = seq_score_kernel<D, R, LG, MEAN, FP8>;
  const size_t smem = TileWalker<D, false, FP8>::smem_bytes();
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
  // one workgroup per compute unit walks over its share of the (sequence, layer group) units
  const int wgs = std::min(dev.B * dev.n_groups, seq_cu_count());
  hipLaunchKernelGGL(kernel, dim3(wgs), dim3(kTiledThreads), smem, stream, dev);
  return launch_status();
}

template <int D, bool MEAN, bool FP8>
static sp_status seq_by_rows(const TiledDev& dev, int R, hipStream_t stream) {
  if (dev.lgG == 2) return R == 4 ? launch_seq<D, 4, 2, MEAN, FP8>(dev, stream) : launch_seq<D, 8, 2, MEAN, FP8>(dev, stream);
  return launch_seq<D, 8, 3, MEAN, FP8>(dev, stream);
}
template <int D, bool FP8>
static sp_status seq_by_mode(const TiledDev& dev, int R, bool mean, hipStream_t stream) {
  return mean ? seq_by_rows<D, true, FP8>(dev, R, stream) : seq_by_rows<D, false, FP8>(dev, R, stream);
}

// `dev` as the tiled kernels fill it in, with group_scores, slabs_per_group, n_groups and
// seq_limit set for this path
sp_status seq_score(const sp_score_args* a, const TiledDev& dev_, hipStream_t stream) {
  TiledDev dev = dev_;
  dev.seq_order = nullptr;
  if (a->B > 1) {  // (one sequence: nothing to order, and the host has seen that its length fits)
    int32_t* order = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(dev.group_scores) + seq_scores_bytes(a));
    hipLaunchKernelGGL(seq_order_kernel, dim3(1), dim3(1024), 0, stream, a->B, a->d_cu_seqlens, order, a->d_lse,
                       seq_max_keys(a), a->L, a->N * a->H);
    dev.seq_order = order;
  }
  const int R = seq_rows(a);
  // (units smaller than a layer: the kernel variant that hands on maxima, whatever the layer reduction)
  const bool mean = a->layer_reduce == SP_LAYER_MEAN && dev.groups_per_layer == 0;
  const bool fp8 = a->k_dtype == SP_K_FP8_E4M3;
  const sp_status st = a->d == 64 ? (fp8 ? seq_by_mode<64, true>(dev, R, mean, stream) : seq_by_mode<64, false>(dev, R, mean, stream))
                                  : (fp8 ? seq_by_mode<128, true>(dev, R, mean, stream) : seq_by_mode<128, false>(dev, R, mean, stream));
  if (st != SP_OK) return st;
  hipLaunchKernelGGL(seq_finish_kernel, dim3((unsigned)((dev.T + 63) / 64)), dim3(64 * kSeqFinishParts), 0, stream, dev);
  return launch_status();
}

}  // namespace sp
