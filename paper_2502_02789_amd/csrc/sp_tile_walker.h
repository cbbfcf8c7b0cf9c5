// What the MFMA scoring kernels for batches share: the kernel-side argument block, and the per-wave
// walker that streams query and key tiles through a two-slot LDS ring with direct global->LDS loads,
// multiplies them on the matrix cores and keeps row statistics (Sec. 3.2 equation of arXiv 2502.02789).
#pragma once

#include "sp_score_internal.h"
#include "sp_lds.h"

namespace sp {

constexpr int kTiledWaves = 8;
constexpr int kTiledThreads = kTiledWaves * kWave;
constexpr int kWaveKeys = 64;        // keys per wave = the general kernels' tile size (shared tile table)
constexpr int kPartBufBytes = 3072;  // per wave: pass 0 collects the slabs' row statistics here before writing them out
constexpr int kKeepRows = 4;         // "keep" mode: logits are kept in units of four query rows (16 bytes per key) ...
constexpr int kKeepMaxRows = 8;      // ... one or two units per KV head
constexpr int kKeepStageBytes = kWaveKeys * kKeepRows * 4;  // taken from the end of the statistics buffer
#ifndef SP_TILED_TARGET_WGS
#define SP_TILED_TARGET_WGS 2048
#endif
constexpr int kTiledTargetWGs = SP_TILED_TARGET_WGS;  // cut the layers into groups until the grid has about this many workgroups

struct TiledDev {
  // G heads per KV head; their query rows are laid out with the group size padded to a power of
  // two, Gp = 1 << lgG (columns of padding heads repeat head 0 and are masked where it matters)
  int B, N, L, H, H_kv, G, Gp, lgG, layers_per_group, n_groups, max_tiles, layer_reduce;
  float scale;  // logits -> natural-log domain (what the partials and log-sum-exps are kept in)
  float c;      // scale * log2(e)
  int64_t ts, hs, T;
  const uint16_t* q;
  const int32_t* cu;
  const int32_t* n_valid;
  const int32_t* tile_cu;
  const float* ws_lse;   // [L][B][N][H]
  float2* part;          // [(l*N + n)*H + h][max_tiles]
  float* group_scores;   // [n_groups][N][T]: per layer group, log2 of the max probability (layer max) or the
                         // sum over its layers of the per-layer max probability (layer mean)
  float* logits;         // keep mode: [L][H_kv][keep_units][T][kKeepRows] base-2 logits (scale * log2(e) applied), else null
  int keep_units;        // 1 or 2: units of four query rows per KV head
  float* scores;
  float* lse_out;        // optional [L][B][N][H] natural-log row log-sum-exps (written by the single-pass batch kernel itself)
  const int32_t* seq_order;  // single-pass batch kernel: sequence numbers, longest first
  int slabs_per_group;   // single-pass batch kernel: (layer, KV head) slabs per unit (n_groups of them cover the L * H_kv slabs)
  int groups_per_layer;  // single-pass batch kernel, mean over layers with units smaller than a layer: slab groups per layer, else 0
  int seq_limit;         // single-pass batch kernel: sequences longer than this many keys are not scored (NaN), 0 = no limit
  const int32_t* block_table;  // paged cache: [B][blocks_per_seq] page numbers, else null
  int lg_page, blocks_per_seq;
  int64_t page_stride;
  // un-rotated cache: (cos, sin) of every position's rotation, in the order the waves consume it
  // (see rope_tile_table_kernel), else null
  const float4* rope_tiles;
  const float* k_scale;  // 8-bit cache (FP8 kernels): [L][H_kv] scales of the keys, or null (all 1)
  const uint16_t* k[SP_MAX_LAYERS];
};

// "at most n vector-memory instructions still in flight" for the kernels that also stream the
// rotation table (more instructions per tile than wait_vmcnt_upto distinguishes)
__device__ __forceinline__ void wait_vmcnt_upto_wide(int n) {
  if (n >= 40) wait_vmcnt<40>();
  else if (n >= 32) wait_vmcnt<32>();
  else if (n >= 28) wait_vmcnt<28>();
  else if (n >= 24) wait_vmcnt<24>();
  else if (n >= 20) wait_vmcnt<20>();
  else if (n >= 16) wait_vmcnt<16>();
  else wait_vmcnt_upto(n);
}

// FP8: the keys are OCP E4M3 bytes (one byte per element, a scale per layer and KV head); the query
// rows stay bf16.  A key row is then half as long; its 16-byte units hold 16 elements, i.e. TWO MFMA
// k-steps, so a lane reads whole units (upper half-wave: the odd ones), widens the bytes to bf16 in
// registers (exact) and the query operand is read in the matching order (k-step 2j + e of half-wave h
// multiplies elements 16 (2j + h) + 8e ... + 7: any order will do as long as both operands agree).
template <int D, bool ROPE, bool FP8 = false>
struct TileWalker {
  static_assert(!(ROPE && FP8), "8-bit caches are taken as already rotated");
  static constexpr int KS = D / 16;            // MFMA k-steps per tile
  static constexpr int ROW_B = D * 2;          // bytes of one query row (and of one bf16 key)
  static constexpr int TILE_B = 32 * ROW_B;    // 32 rows: a ring slot
  static constexpr int UNITS = ROW_B / 16;     // 16-byte units per row
  static constexpr int LOADS = TILE_B / 1024;  // wave-wide 16-byte loads per tile
  static constexpr int RPI = 64 / UNITS;       // rows covered by one such load
  static constexpr int ESZ = FP8 ? 1 : 2;      // bytes per key element
  static constexpr int KROW_B = D * ESZ;       // the same for a key tile
  static constexpr int KUNITS = KROW_B / 16;
  static constexpr int KLOADS = 32 * KROW_B / 1024;
  static constexpr int KRPI = 64 / KUNITS;

  const TiledDev& p;
  int wave, lane, half, col;
  int b, seq0, key0, rows_in;  // sequence, its first token, the tile's first key within it, valid keys of the tile (1..64)
  int64_t tok0;          // flat token index of the tile's first key
  int issued, seq_a, seq_b;  // vector-memory instructions issued so far; value right after the loads into slot 0 / 1
  uint32_t ring_lds, lse_lds, part_lds, rd0, u0;
  uint32_t krd0, qrd0;   // FP8: where this lane reads its key units / its query units from (ring slot 0)
  float c2, scale;        // logits -> base-2 / natural-log domain for the current slab (an 8-bit cache's key scale included)
  int part_n;            // slabs waiting in the statistics buffer
  uint32_t ld_off[4];
  bf16x8 qf[KS];
  f32x16 acc[2];
  float run_m, run_s;
  float4 cs[ROPE ? KS / 2 : 1][4];  // ROPE: the (cos, sin) pairs of the key tile that is rotated next

  // a wave that owns 64-key tile `tile` (numbered over the whole batch) ...
  __device__ __forceinline__ TileWalker(const TiledDev& p_, unsigned char* smem, int tile) : p(p_) {
    b = upper_segment(p.tile_cu, p.B, tile);
    seq0 = p.cu[b];
    key0 = (tile - p.tile_cu[b]) * kWaveKeys;
    rows_in = min(kWaveKeys, p.cu[b + 1] - seq0 - key0);
    tok0 = (int64_t)seq0 + key0;
    set_up(smem);
  }
  // ... or a wave that walks over several tiles of sequence b_ (the caller names the keys of every load)
  struct WholeSequence {};
  __device__ __forceinline__ TileWalker(const TiledDev& p_, unsigned char* smem, WholeSequence, int b_) : p(p_) {
    b = b_;
    seq0 = p.cu[b];
    key0 = 0;
    rows_in = 0;
    tok0 = seq0;
    set_up(smem);
  }
  __device__ __forceinline__ void set_up(unsigned char* smem) {
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    lane = threadIdx.x & 63;
    half = lane >> 5;
    col = lane & 31;
    issued = seq_a = seq_b = 0;
    const uint32_t smem_lds = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    ring_lds = smem_lds + wave * 2 * TILE_B;
    lse_lds = smem_lds + kTiledWaves * 2 * TILE_B + wave * 512;
    part_lds = smem_lds + kTiledWaves * (2 * TILE_B + 512) + wave * kPartBufBytes;
    part_n = 0;
    // LDS layout of a tile: row r at r*ROW_B; inside a row the 16-byte unit holding head-dim
    // elements [8u, 8u+8) sits at position u ^ key(r), key(r) = r & 15 (D=128) or (r >> 1) & 7
    // (D=64): the 16 lanes of an operand read hit 16 distinct bank groups, and a wave-wide
    // direct load still fills 1 KiB of consecutive LDS.
    const int key = (D == 128) ? (col & 15) : ((col >> 1) & 7);
    rd0 = ring_lds + col * ROW_B + ((half ^ (key & 1)) << 4) + ((key >> 1) << 5);
    const int i = lane / UNITS;
    const int key_i = (D == 128) ? i : (i >> 1);
    u0 = (lane % UNITS) ^ key_i;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      ld_off[jj] = (uint32_t)((int64_t)i * p.ts * 2) + (uint32_t)((u0 ^ ((4 * jj) & (UNITS - 1))) << 4);
    c2 = p.c;
    scale = p.scale;
    krd0 = qrd0 = 0;
    if constexpr (FP8) {
      // key tile: row r at r*KROW_B, unit u at position u ^ (r & (KUNITS - 1)); the lane of a wave-wide load
      // that fills row (lane / KUNITS) of its KRPI rows, position lane % KUNITS, fetches that unit
      const int ki = lane / KUNITS;
      u0 = (lane % KUNITS) ^ (ki & (KUNITS - 1));
      ld_off[0] = (uint32_t)((int64_t)ki * p.ts) + (u0 << 4);
      krd0 = ring_lds + col * KROW_B + ((half ^ (col & (KUNITS - 1))) << 4);
      qrd0 = ring_lds + col * ROW_B + (((2 * half) ^ key) << 4);
    }
  }
  // the scale of the keys of (layer l, KV head g) joins the logit scale (8-bit cache)
  __device__ __forceinline__ void slab_scale(int l, int g) {
    if constexpr (FP8) {
      if (p.k_scale) {
        const float ks = p.k_scale[l * p.H_kv + g];
        c2 = p.c * ks;
        scale = p.scale * ks;
      }
    }
  }

  static size_t smem_bytes() { return (size_t)kTiledWaves * (2 * TILE_B + 512 + kPartBufBytes); }

  __device__ __forceinline__ static __attribute__((address_space(3))) void* lds_ptr(uint32_t addr) {
    return reinterpret_cast<__attribute__((address_space(3))) void*>(addr);
  }
  __device__ __forceinline__ void note_issued(int k) { issued = __builtin_amdgcn_readfirstlane(issued + k); }
  __device__ __forceinline__ void mark_slot(int slot) { if (slot & 1) seq_b = issued; else seq_a = issued; }
  __device__ __forceinline__ void wait_tile(int slot) {
    const int newer = __builtin_amdgcn_readfirstlane(issued - ((slot & 1) ? seq_b : seq_a));
    if (ROPE) wait_vmcnt_upto_wide(newer); else wait_vmcnt_upto(newer);
  }
  // ROPE: request the (cos, sin) pairs for key tile kb of this wave (the same for every slab; a
  // tile wholly beyond the sequence takes tile 0's, its keys are masked anyway)
  __device__ __forceinline__ void issue_rope(int kb) {
    if constexpr (ROPE) {
      const int tile32 = (key0 >> 5) + (kb * 32 < rows_in ? kb : 0);
      const float4* src = p.rope_tiles + (int64_t)tile32 * (KS / 2) * 4 * 64 + lane;
#pragma unroll
      for (int t = 0; t < KS / 2; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) cs[t][j] = src[(t * 4 + j) * 64];
      note_issued(KS / 2 * 4);
    }
  }
  // ROPE: turn the key operand in registers (kf[t] and kf[t + KS/2] hold the two halves of the pairs)
  __device__ __forceinline__ void rotate_keys(bf16x8 (&kf)[KS]) {
    if constexpr (ROPE) {
#pragma unroll
      for (int t = 0; t < KS / 2; ++t) {
        u32x4 lo = __builtin_bit_cast(u32x4, kf[t]), hi = __builtin_bit_cast(u32x4, kf[t + KS / 2]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {  // word w: elements 2w (low half) and 2w + 1 (high half)
          const float4 c = cs[t][w];
          const float2 e = rope_turn_exact(__uint_as_float(lo[w] << 16), __uint_as_float(hi[w] << 16), make_float2(c.x, c.y));
          const float2 o = rope_turn_exact(__uint_as_float(lo[w] & 0xFFFF0000u), __uint_as_float(hi[w] & 0xFFFF0000u), make_float2(c.z, c.w));
          lo[w] = pack_bf16_pair(e.x, o.x);
          hi[w] = pack_bf16_pair(e.y, o.y);
        }
        kf[t] = __builtin_bit_cast(bf16x8, lo);
        kf[t + KS / 2] = __builtin_bit_cast(bf16x8, hi);
      }
    }
  }
  // the slot is about to be overwritten: every LDS read of its previous tile must have been performed
  __device__ __forceinline__ void slot_free() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

  // Key tile kb (0/1) of KV head g in layer l -> ring slot.  Always exactly LOADS wave-wide
  // loads; rows beyond the sequence re-read the tile's (or the wave's) first row and are masked later.
  __device__ __forceinline__ void issue_keys(int l, int g, int kb, int slot) {
    const int rows = min(32, rows_in - kb * 32);
    issue_key_rows(l, g, rows > 0 ? key0 + kb * 32 : key0, rows, slot);
  }
  // 32 keys of the walker's sequence starting at key `key_first` (a multiple of 32 inside the
  // sequence) of which the first `rows_` exist (<= 0: none, the load only keeps the stream in step)
  __device__ __forceinline__ void issue_key_rows(int l, int g, int key_first, int rows_, int slot) {
    const uint32_t dst = ring_lds + slot * TILE_B;
    int rows = rows_;
    asm volatile("" : "+s"(rows));
    if (p.block_table) {
      issue_keys_paged(l, g, key_first, rows, dst);
      note_issued(KLOADS);
      mark_slot(slot);
      return;
    }
    const int64_t tok = (int64_t)seq0 + key_first;
    const unsigned char* base = reinterpret_cast<const unsigned char*>(p.k[l]) + ESZ * ((int64_t)g * p.hs + tok * p.ts);
    if (rows == 32) {
#pragma unroll
      for (int j = 0; j < KLOADS; ++j) {
        uint32_t lane_off = ld_off[FP8 ? 0 : (j & 3)];
        asm volatile("" : "+v"(lane_off));
        __builtin_amdgcn_global_load_lds(base + (int64_t)(j * KRPI) * p.ts * ESZ + (size_t)lane_off, lds_ptr(dst + j * 1024),
                                         16, 0, kKeyLoadPolicy);
      }
    } else {
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int i = ln / KUNITS;
#pragma unroll
      for (int j = 0; j < KLOADS; ++j) {
        const int r = j * KRPI + i;
        const int64_t row_off = r < rows ? (int64_t)r * p.ts * ESZ : 0;
        const uint32_t unit = FP8 ? u0 : (u0 ^ ((4 * j) & (UNITS - 1)));
        __builtin_amdgcn_global_load_lds(base + row_off + (unit << 4), lds_ptr(dst + j * 1024), 16, 0, kKeyLoadPolicy);
      }
    }
    note_issued(KLOADS);
    mark_slot(slot);
  }

  // The same from a paged cache.  key_first: in-sequence index of the tile's row 0 (a multiple of
  // 32).  The KRPI (4 or 8; 8 or 16 with an 8-bit cache) rows of one load lie in one page: pages hold a power of
  // two >= 8 keys (>= 16 where a load has 16 rows; the host checks).
  // Loads whose rows are all beyond the sequence, and lanes beyond it, re-read a valid row.
  __device__ __forceinline__ void issue_keys_paged(int l, int g, int key_first, int rows, uint32_t dst) {
    const unsigned char* layer = reinterpret_cast<const unsigned char*>(p.k[l]) + ESZ * (int64_t)g * p.hs;
    const int32_t* table = p.block_table + (int64_t)b * p.blocks_per_seq;
    const int pmask = (1 << p.lg_page) - 1;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int i = ln / KUNITS;
    const unsigned char* base = layer;
#pragma unroll
    for (int j = 0; j < KLOADS; ++j) {
      const bool inside = j * KRPI < rows;
      const int kk = inside ? key_first + j * KRPI : key_first;
      if (j == 0 || !inside || ((j * KRPI) & pmask) == 0)  // first load, fallback row, or a new page begins
        base = layer + ESZ * ((int64_t)table[kk >> p.lg_page] * p.page_stride + (int64_t)(kk & pmask) * p.ts);
      else
        base += (int64_t)KRPI * p.ts * ESZ;
      const int64_t row_off = (j * KRPI + i < rows) ? (int64_t)i * p.ts * ESZ : 0;
      const uint32_t unit = FP8 ? u0 : (u0 ^ ((4 * j) & (UNITS - 1)));
      __builtin_amdgcn_global_load_lds(base + row_off + (unit << 4), lds_ptr(dst + j * 1024), 16, 0, kKeyLoadPolicy);
    }
  }

  // Query tile of (layer l, KV head g) of this wave's sequence: row r = n*G + j holds
  // Q[l, b, n, g*G + j, :] (rows beyond G*N repeat row 0; their columns are never used).  With
  // WITH_LSE the rows' log-sum-exps follow into lse zone `zone` and land with the tile.
  template <bool WITH_LSE>
  __device__ __forceinline__ void issue_queries(int l, int g, int slot, int zone) {
    int rows = p.Gp * p.N;
    asm volatile("" : "+s"(rows));
    const uint32_t dst = ring_lds + slot * TILE_B;
    const int64_t row0 = (((int64_t)l * p.B + b) * p.N) * p.H + g * p.G;
    const unsigned char* base = reinterpret_cast<const unsigned char*>(p.q) + 2 * row0 * D;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int i = ln / UNITS;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int r = j * RPI + i;
      const int key = (D == 128) ? (r & 15) : ((r >> 1) & 7);
      const int unit = (ln % UNITS) ^ key;
      const int rr = r < rows ? r : 0;
      const int jj = (rr & (p.Gp - 1)) < p.G ? (rr & (p.Gp - 1)) : 0;
      const uint32_t off = (uint32_t)((rr >> p.lgG) * p.H * ROW_B + jj * ROW_B + unit * 16);
      __builtin_amdgcn_global_load_lds(base + off, lds_ptr(dst + j * 1024), 16, 0, 0);
    }
    note_issued(LOADS);
    if (WITH_LSE) {
      const int cc = (ln & 31) < rows ? (ln & 31) : 0;
      const int cj = (cc & (p.Gp - 1)) < p.G ? (cc & (p.Gp - 1)) : 0;
      const float* src = p.ws_lse + row0 + (cc >> p.lgG) * p.H + cj;
      __builtin_amdgcn_global_load_lds(src, lds_ptr(lse_lds + zone * 256), 4, 0, 0);
      note_issued(1);
    }
    mark_slot(slot);
  }

  __device__ __forceinline__ bf16x8 read_unit(int t, int slot) const {
    uint32_t base = rd0;
    asm volatile("" : "+v"(base));
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
        lds_ptr((base ^ (uint32_t)(t << 5)) + slot * TILE_B));
  }
  __device__ __forceinline__ void read_queries(int slot) {
    if constexpr (FP8) {  // k-step 2j + e of this half-wave: query elements 16 (2j + h) + 8e ... = unit 4j + 2h + e
      uint32_t base = qrd0;
      asm volatile("" : "+v"(base));
#pragma unroll
      for (int t = 0; t < KS; ++t)
        qf[t] = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
            lds_ptr((base ^ (uint32_t)((4 * (t >> 1) + (t & 1)) << 4)) + slot * TILE_B));
      return;
    }
#pragma unroll
    for (int t = 0; t < KS; ++t) qf[t] = read_unit(t, slot);
  }
  // FP8: the key operand of all k-steps: unit 2j + h of the lane's key, its 16 bytes widened to bf16 (exact)
  __device__ __forceinline__ void read_keys_fp8(bf16x8 (&kf)[KS], int slot) {
    uint32_t base = krd0;
    asm volatile("" : "+v"(base));
#pragma unroll
    for (int j = 0; j < KS / 2; ++j) {
      const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(
          lds_ptr((base ^ (uint32_t)((2 * j) << 4)) + slot * TILE_B));
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        u32x4 o;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          o[2 * x] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v[2 * e + x], 1.0f, false));
          o[2 * x + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v[2 * e + x], 1.0f, true));
        }
        kf[2 * j + e] = __builtin_bit_cast(bf16x8, o);
      }
    }
  }
  // QROWS = false: register i of acc[kb] holds key (i / 4) * 8 + (i % 4) (+ 4 for the upper half-wave) of the
  // tile for query row `col`; QROWS = true: the operands change places, so that it holds that QUERY ROW for
  // key `col` of the tile (a lane then has all of a key's first rows, see sp_score_seq.hip)
  template <bool QROWS = false>
  __device__ __forceinline__ void mfma_tile(int kb, int slot) {
    f32x16 a = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8 kf[KS];
    if constexpr (FP8) {
      read_keys_fp8(kf, slot);
#pragma unroll
      for (int t = 0; t < KS; ++t)
        a = QROWS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[t], a, 0, 0, 0)
                  : __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], a, 0, 0, 0);
      acc[kb] = a;
      return;
    }
#pragma unroll
    for (int t = 0; t < KS; ++t) kf[t] = read_unit(t, slot);
    if constexpr (ROPE) {  // rotate, ask for the other tile's table (the registers are free now), multiply
      rotate_keys(kf);
      issue_rope(kb ^ 1);
#pragma unroll
      for (int t = 0; t < KS; ++t) a = QROWS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[t], a, 0, 0, 0)
                : __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], a, 0, 0, 0);
      acc[kb] = a;
      return;
    }
#pragma unroll
    for (int t = 0; t < KS; ++t) a = QROWS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[t], a, 0, 0, 0)
                : __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], a, 0, 0, 0);
    constexpr int kAhead = KS < 4 ? KS : 4;
    __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
    for (int t = 0; t < KS - kAhead; ++t) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
    acc[kb] = a;
  }

  // Register i of a 32x32 accumulator tile holds key (i / 4) * 8 + (i % 4) (+ 4 for the upper
  // half-wave) of the tile, for query column `col`.
  __device__ __forceinline__ void stats_tile(int kb) {
    f32x16& a = acc[kb];
    if ((kb + 1) * 32 > rows_in) {  // ragged tail: keys beyond the sequence do not count
      int left = rows_in - kb * 32 - half * 4;
      asm volatile("" : "+v"(left));
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if ((i >> 2) * 8 + (i & 3) >= left) a[i] = -INFINITY;
    }
    float tm = a[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tm = fmaxf(tm, a[i]);
    const float m_new = fmaxf(run_m, tm);
    const float ref = (m_new == -INFINITY) ? 0.f : m_new;
    const float off = -ref * c2;
    float s0 = run_s * fast_exp2(fmaf(run_m, c2, off)), s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
      s0 += fast_exp2(fmaf(a[i], c2, off));
      s1 += fast_exp2(fmaf(a[i + 1], c2, off));
      s2 += fast_exp2(fmaf(a[i + 2], c2, off));
      s3 += fast_exp2(fmaf(a[i + 3], c2, off));
    }
    run_m = m_new;
    run_s = (s0 + s1) + (s2 + s3);
  }

  // pass 0, end of a slab: the row's (max, sum exp) over this wave's keys, in the natural-log
  // domain, goes into the wave's LDS buffer.  (Vector-memory instructions of a wave complete in
  // order: a store per slab makes the next tile's wait sit out the store's round trip.)
  __device__ __forceinline__ void keep_partial() {
    const float pm = __shfl_xor(run_m, 32, kWave), ps = __shfl_xor(run_s, 32, kWave);
    const float mn = fmaxf(run_m, pm);
    const float ref = (mn == -INFINITY) ? 0.f : mn;
    const float z = run_s * fast_exp2((run_m - ref) * c2) + ps * fast_exp2((pm - ref) * c2);
    int c = col;
    asm volatile("" : "+v"(c));
    const int rows = p.Gp * p.N;
    if (half == 0 && c < rows)
      lds_poke64<0>(part_lds + (part_n * rows + c) * 8, ((uint64_t)__float_as_uint(z) << 32) | __float_as_uint(mn * scale));
    part_n = __builtin_amdgcn_readfirstlane(part_n + 1);
  }
  __device__ __forceinline__ bool partials_full(int buf_bytes) const { return (part_n + 1) * p.Gp * p.N * 8 > buf_bytes; }

  // keep mode, end of a slab: the wave's 64 x (G*N <= 4) logits, scaled to base 2, as 16 bytes
  // per key in the key's lane, after a turn through LDS (a lane holds one query row of 32 keys,
  // the store wants one key's rows per lane).  A slab's logits are one dense 1 KiB store; the
  // caller collects several slabs in registers and stores them together (a store per slab would
  // make the tile waits sit out a store round trip every slab).
  __device__ __forceinline__ u32x4 transposed_logits(int unit) {  // unit: query rows 4*unit .. 4*unit + 3
    const uint32_t stage = part_lds + kPartBufBytes - kKeepStageBytes;
    int c = col - unit * kKeepRows, h = half, ln = lane;
    asm volatile("" : "+v"(c), "+v"(h), "+v"(ln));
    if (c >= 0 && c < kKeepRows) {  // (columns beyond G*N repeat row 0: finite values nobody reads)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          lds_poke32(stage + ((kb * 32 + (i >> 2) * 8 + h * 4 + (i & 3)) * kKeepRows + c) * 4,
                     __float_as_uint(acc[kb][i] * c2));
    }
    return lds_peek128(stage + ln * 16);  // (LDS operations of a wave are performed in order)
  }
  __device__ __forceinline__ void store_logits(const u32x4& v, int l, int g, int unit) {
    int ln = lane;
    asm volatile("" : "+v"(ln));
    if (ln < rows_in)  // (never empty: a tile has at least one key)
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(
          p.logits + ((((int64_t)l * p.H_kv + g) * p.keep_units + unit) * p.T + tok0 + ln) * kKeepRows));
    note_issued(1);
  }
  // write the buffered statistics of slabs [first, first + part_n) of the layer group starting
  // at layer l0 out, 64 (slab, row) pairs per store instruction
  __device__ __forceinline__ void flush_partials(int first, int l0, int tile) {
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int rows = p.Gp * p.N, total = part_n * rows;
#pragma unroll 1
    for (int base = 0; base < total; base += kWave) {
      const int idx = base + ln;
      if (idx < total) {  // (never empty: lane 0 is always inside)
        const uint64_t v = lds_peek64(part_lds + idx * 8);
        const int j = idx / rows, c = idx - j * rows;
        const int s = first + j;
        const int l = l0 + s / p.H_kv, g = s % p.H_kv;
        // (a padding column repeats head 0 of its query: same statistics, written to the same place)
        const int n = c >> p.lgG, h = g * p.G + ((c & (p.Gp - 1)) < p.G ? (c & (p.Gp - 1)) : 0);
        p.part[((int64_t)(l * p.N + n) * p.H + h) * p.max_tiles + tile] =
            make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
      }
      note_issued(1);
    }
    part_n = 0;
  }
};

// single-pass kernel for batches of short prompts (sp_score_seq.hip)
bool seq_supported(const sp_score_args* a);
int seq_max_keys(const sp_score_args* a);
void seq_grouping(const sp_score_args* a, int* slabs_per_group, int* n_groups, int* groups_per_layer);
size_t seq_workspace_bytes(const sp_score_args* a);
sp_status seq_score(const sp_score_args* a, const TiledDev& dev, hipStream_t stream);

}  // namespace sp
