// The streaming core shared by the single-pass scoring kernels (sp_score_stream.hip: all
// workgroups exchange row statistics with each other; sp_score_team.hip: teams of workgroups each
// take a subset of the KV heads and exchange only inside the team).
//
// What lives here is everything a wave does on its own: it streams 32-row tiles (one tile of
// query rows, then TPW tiles of keys per slab) from global memory through a private two-slot LDS
// ring with direct global->LDS loads, multiplies them with v_mfma_f32_32x32x16_bf16 (keys as
// matrix rows, the 32 (query, head-in-group) rows of one KV head as columns), keeps the raw
// logits of the last NSETS slabs in registers, computes per-row (max, sum 2^(x-max)) of a slab
// over its own keys, and -- once a slab's row log-sum-exps are known -- turns the stored logits
// into log2-probabilities (Sec. 3.2 equation of arXiv 2502.02789) and maxes them over the heads
// of the KV group (DPP) and into a per-workgroup [query][key] running maximum in LDS
// (Sec. 3.2.2).  How the row statistics of all the workgroups that share a softmax row are
// brought together is the business of the two kernels.
#pragma once

#include <utility>

#include "sp_score_internal.h"
#include "sp_lds.h"

namespace sp {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * kWave;
constexpr int kMaxWG = 256;
constexpr uint32_t kEmpty32 = ~0u;        // a cross-workgroup word nobody has written yet
constexpr uint32_t kPending32 = ~0u - 1;  // in an LDS landing zone: the load has not arrived yet
constexpr int kDefaultSpinBudget = 1 << 16;  // polls per wave over the whole call before giving up (~0.1 s)

// Shape and addressing of one call, as the streaming core needs it.  S, slabs_per_layer, KPW
// and G are powers of two.
struct StreamShape {
  int M, L, N, H, G, lgG;
  int S, lgS;                    // KV heads a workgroup's waves work on side by side in one slab
  int slabs_per_layer, lgSPL;    // slabs per layer (of this workgroup's sequence of slabs)
  int layer_step;                // the workgroup's layers are layer_base, layer_base + layer_step, ...
  int n_slabs;
  int KPW, lgKPW;                // keys owned by a workgroup
  int own_step, tile_step;       // key tile x of owner o starts at key o * own_step + x * tile_step: (KPW, 32) gives
                                 // every workgroup one run of KPW keys, (32, owners * 32) deals the 32-key
                                 // tiles out to the workgroups in turn
  int spin_budget;               // polls a wave may spend waiting for other workgroups over the whole call
  float c;                       // scale * log2(e): logits are handled in the base-2 domain
  int64_t ts, hs;                // token / head stride of the K cache, elements
  const uint16_t* q;
  const int32_t* block_table;    // paged cache: page numbers of the (single) prompt, else null
  int lg_page;
  int64_t page_stride;
  const float* k_scale;          // 8-bit cache (FP8 kernels): [L][H_kv] scales of the keys, or null (all 1)
  int H_kv;
  const uint16_t* k[SP_MAX_LAYERS];
};

// start-of-call state of the exchange area: every word "empty", the status word clear
static __global__ __launch_bounds__(256) void fill_empty_kernel(uint4* __restrict__ dst, size_t n_vec, uint32_t* status) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
    dst[i] = make_uint4(kEmpty32, kEmpty32, kEmpty32, kEmpty32);
  if (blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;
}

// Register i of a 32x32 accumulator tile holds key (i / 4) * 8 + (i % 4) (+ 4 for the upper
// half-wave).  In the running-max array that key sits at cell (i / 4) * 8 + (i % 4) * 2 (+ 1 for
// the upper half-wave) of its tile, and query rows are kSmaxPad cells apart modulo 32: the 16
// lanes of one atomic (8 queries x 2 half-waves) then fall into 16 different LDS banks.
constexpr int kSmaxPad = 2;
__device__ __forceinline__ int smax_cell(int key) {  // key within the workgroup's slice -> cell in a row
  return (key & ~7) | ((key & 3) << 1) | ((key >> 2) & 1);
}
template <int... I>
__device__ __forceinline__ void lds_fmax_tile(uint32_t lds_addr, const float (&x)[16], std::integer_sequence<int, I...>) {
  (lds_fmax<((I >> 2) * 8 + (I & 3) * 2) * 4>(lds_addr, x[I]), ...);
}

// FP8: the keys are OCP E4M3 bytes (one byte per element, a scale per layer and KV head); the query
// rows stay bf16.  A key row is then half as long; its 16-byte units hold 16 elements, i.e. TWO MFMA
// k-steps, so a lane reads whole units (upper half-wave: the odd ones), widens the bytes to bf16 in
// registers (exact), and the query operand is read in the matching order (k-step 2j + e of half-wave h
// multiplies elements 16 (2j + h) + 8e ... + 7: any order will do as long as both operands agree).  The
// key scale is applied to the products' sums right after the matrix instructions.
// per-lane state only the 8-bit form has (an empty base otherwise, so the bf16 kernels carry nothing of it)
template <bool FP8> struct Fp8Lane {};
template <> struct Fp8Lane<true> {
  uint32_t krd0, qrd0;   // where this lane reads its key units / its query units from (ring slot 0)
  uint32_t kunit;        // the 16-byte unit of a key row this lane fetches in every load
  float ks;              // the key scale of the slab at hand
};

template <int D, int TPW, bool PAGED, bool FP8 = false>
struct StreamCore : Fp8Lane<FP8> {
  static_assert(!(PAGED && FP8), "8-bit caches behind a block table take the two-pass kernels");
  static constexpr int NSETS = 8 / TPW;        // slabs of logits alive in registers
  static constexpr int TPS = TPW + 1;          // stream tiles per slab: query tile + key tiles
  static constexpr int KS = D / 16;            // MFMA k-steps per tile
  static constexpr int ROW_B = D * 2;          // bytes of one row (one key / one query row)
  static constexpr int TILE_B = 32 * ROW_B;    // 32 rows
  static constexpr int UNITS = ROW_B / 16;     // 16-byte units per row
  static constexpr int LOADS = TILE_B / 1024;  // wave-wide 16-byte loads per tile
  static constexpr int RPI = 64 / UNITS;       // rows covered by one such load
  static constexpr int RING_BYTES = kWaves * 2 * TILE_B;
  static constexpr int ESZ = FP8 ? 1 : 2;      // bytes per key element
  static constexpr int KROW_B = D * ESZ;       // bytes of one key; units, loads and rows per load of a key tile
  static constexpr int KUNITS = KROW_B / 16;
  static constexpr int KLOADS = 32 * KROW_B / 1024;
  static constexpr int KRPI = 64 / KUNITS;

  const StreamShape& p;
  float* smax;           // [N][KPW + kSmaxPad] running max of log2-probabilities (cells: smax_cell)
  int wave, lane, half, col;
  int owner;             // which share of the prompt's key tiles this workgroup owns (see own_step, tile_step)
  int kvh_base;          // first KV head of this workgroup's sequence of slabs
  int layer_base;        // first layer of it
  int kvh_local, kbg;    // this wave's KV head inside a slab, and its group of key tiles
  int budget;            // polls left; a wait that finds it used up gives up and sets `expired`
  bool expired;
  int issued;            // vector-memory instructions issued so far by this wave (never over-counted)
  int seq0, seq1;        // value of `issued` right after the loads of the tile in ring slot 0 / 1
  uint32_t ring_lds;     // LDS byte address of this wave's two-slot ring
  uint32_t rd0;          // LDS byte address of this lane's operand unit for k-step 0 in slot 0
  uint32_t ld_off[4];    // per-lane global byte offset of key load j (depends on j & 3 only)
  bf16x8 qf[KS];
  f32x16 acc[NSETS][TPW];
  float run_m, run_s;    // running (max of raw logits, sum of 2^((x-max)*c)) of this lane's row

  // LDS layout of a tile: row r at r*ROW_B; inside a row the 16-byte unit holding head-dim
  // elements [8u, 8u+8) sits at position u ^ key(r), key(r) = r & 15 (D=128) or (r >> 1) & 7
  // (D=64).  With it the 16 lanes of an operand read hit 16 distinct bank groups, and a
  // wave-wide direct load still fills 1 KiB of consecutive LDS.
  // ring_base: LDS byte address of the workgroup's RING_BYTES of tile ring.
  __device__ __forceinline__ StreamCore(const StreamShape& p_, uint32_t ring_base, float* smax_, int owner_, int kvh_base_,
                                        int layer_base_ = 0)
      : p(p_), smax(smax_), owner(owner_), kvh_base(kvh_base_), layer_base(layer_base_) {
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    lane = threadIdx.x & 63;
    half = lane >> 5;
    col = lane & 31;
    kvh_local = wave & (p.S - 1);
    kbg = wave >> p.lgS;
    ring_lds = ring_base + wave * 2 * TILE_B;
    budget = p.spin_budget;
    expired = false;
    issued = 0;
    seq0 = seq1 = 0;
    // operand read: unit (2t + half) of row col lives at position (2t + half) ^ key(col)
    //             = 2 * (t ^ (key >> 1)) + (half ^ (key & 1)), so the address is rd0 ^ (t << 5)
    const int key = (D == 128) ? (col & 15) : ((col >> 1) & 7);
    rd0 = ring_lds + col * ROW_B + ((half ^ (key & 1)) << 4) + ((key >> 1) << 5);
    // loads: lane covers row j*RPI + i (i = lane / UNITS) and LDS position lane % UNITS, i.e.
    // data unit (lane % UNITS) ^ key(row); key(row) = key(i) ^ ((4j) & (UNITS-1)) (disjoint bits)
    const int i = lane / UNITS;
    const int key_i = (D == 128) ? i : (i >> 1);
    const int u0 = (lane % UNITS) ^ key_i;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      ld_off[jj] = (uint32_t)((int64_t)i * p.ts * 2) + (uint32_t)((u0 ^ ((4 * jj) & (UNITS - 1))) << 4);
    if constexpr (FP8) {
      this->ks = 1.f;
      // key tile: row r at r*KROW_B, unit u at position u ^ (r & (KUNITS - 1)); the lane of a wave-wide load
      // that fills row lane / KUNITS of its KRPI rows, position lane % KUNITS, fetches that unit
      const int ki = lane / KUNITS;
      this->kunit = (uint32_t)(((lane % KUNITS) ^ (ki & (KUNITS - 1))) << 4);
      ld_off[0] = (uint32_t)((int64_t)ki * p.ts) + this->kunit;
      this->krd0 = ring_lds + col * KROW_B + ((half ^ (col & (KUNITS - 1))) << 4);
      this->qrd0 = ring_lds + col * ROW_B + (((2 * half) ^ key) << 4);
    }
  }
  __device__ __forceinline__ uint32_t fallback_unit(uint32_t lo) const {
    if constexpr (FP8) return this->kunit; else return lo & (uint32_t)(ROW_B - 1);
  }
  // FP8: the scale of the keys of slab `slab` (this wave's KV head)
  __device__ __forceinline__ void slab_scale(int slab) {
    if constexpr (FP8) {
      if (p.k_scale) this->ks = p.k_scale[layer_of(slab) * p.H_kv + kvh_of(slab)];
    }
  }

  __device__ __forceinline__ static __attribute__((address_space(3))) void* lds_ptr(uint32_t addr) {
    return reinterpret_cast<__attribute__((address_space(3))) void*>(addr);
  }
  __device__ __forceinline__ static uint32_t lds_addr_of(const void* generic) {
    return (uint32_t)reinterpret_cast<uintptr_t>(generic);
  }

  // One more round of a bounded wait?  False (and the wave remembers it) once the budget is gone.
  __device__ __forceinline__ bool may_poll() {
    if (budget > 0) { --budget; return true; }
    expired = true;
    return false;
  }

  // first key (in the prompt) of this workgroup's key tile x; of this wave's tile kb
  __device__ __forceinline__ int tile_key(int x) const { return owner * p.own_step + x * p.tile_step; }
  __device__ __forceinline__ int wave_tile_key(int kb) const { return tile_key(kbg * TPW + kb); }
  // prompt key of the workgroup's local key number `local` (tile local / 32, position local % 32)
  __device__ __forceinline__ int key_of_local(int local) const { return tile_key(local >> 5) + (local & 31); }

  __device__ __forceinline__ int layer_of(int slab) const { return layer_base + (slab >> p.lgSPL) * p.layer_step; }
  __device__ __forceinline__ int kvh_of(int slab) const {
    return kvh_base + ((slab & (p.slabs_per_layer - 1)) << p.lgS) + kvh_local;
  }

  // Direct global->LDS load of one key tile into ring slot `slot`.  Always exactly LOADS
  // wave-wide loads (the vmcnt bookkeeping counts on it): rows beyond the prompt re-read row 0
  // of the last in-range tile and are masked later.
  __device__ __forceinline__ void issue_keys(int slab, int kb, int slot) {
    int key_start = wave_tile_key(kb);
    // keep the address arithmetic at its point of use: hoisted out of the slab loop it would
    // pin dozens of registers for the whole kernel
    asm volatile("" : "+s"(key_start));
    const uint32_t dst = ring_lds + slot * TILE_B;
    if constexpr (PAGED) {
      // Paged cache: the RPI (4 or 8) rows of one load lie in one page (pages hold a power of two
      // >= 8 keys, tiles start at multiples of 32); a scalar table lookup where a load enters a
      // new page.  Loads and lanes beyond the prompt re-read a valid row (masked later).
      int rows = min(32, p.M - key_start);
      asm volatile("" : "+s"(rows));
      const int first = rows > 0 ? key_start : 0;
      const unsigned char* layer = reinterpret_cast<const unsigned char*>(p.k[layer_of(slab)]) +
                                   2 * (int64_t)kvh_of(slab) * p.hs;
      const int pmask = (1 << p.lg_page) - 1;
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int i = ln / UNITS;
      const uint32_t row_part = (uint32_t)((int64_t)i * p.ts * 2);
      const unsigned char* base = layer;
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const bool inside = j * RPI < rows;
        const int kk = inside ? first + j * RPI : first;
        if (j == 0 || !inside || ((j * RPI) & pmask) == 0)
          base = layer + 2 * ((int64_t)p.block_table[kk >> p.lg_page] * p.page_stride + (int64_t)(kk & pmask) * p.ts);
        else
          base += (int64_t)RPI * p.ts * 2;
        uint32_t lane_off = ld_off[j & 3];
        asm volatile("" : "+v"(lane_off));
        if (j * RPI + i >= rows) lane_off -= row_part;  // this lane's row is beyond the prompt: the load's first row instead
        __builtin_amdgcn_global_load_lds(base + (size_t)lane_off, lds_ptr(dst + j * 1024), 16, 0, kKeyLoadPolicy);
      }
      return;
    }
    const int start_eff = min(key_start, (p.M - 1) & ~31);
    const unsigned char* base = reinterpret_cast<const unsigned char*>(p.k[layer_of(slab)]) +
                                ESZ * ((int64_t)kvh_of(slab) * p.hs + (int64_t)start_eff * p.ts);
    if (start_eff + 32 <= p.M) {  // whole tile inside the prompt
#pragma unroll
      for (int j = 0; j < KLOADS; ++j) {
        uint32_t lane_off = ld_off[FP8 ? 0 : (j & 3)];
        asm volatile("" : "+v"(lane_off));  // scalar row base + 32-bit lane offset; nothing 64-bit per lane to keep around
        const unsigned char* src = base + (int64_t)(j * KRPI) * p.ts * ESZ + (size_t)lane_off;
        __builtin_amdgcn_global_load_lds(src, lds_ptr(dst + j * 1024), 16, 0, kKeyLoadPolicy);
      }
    } else {
      const int rows_in = p.M - start_eff;  // 1..31
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int i = ln / KUNITS;
#pragma unroll
      for (int j = 0; j < KLOADS; ++j) {
        const bool in = j * KRPI + i < rows_in;
        const uint32_t lo = ld_off[FP8 ? 0 : (j & 3)];
        const int64_t row_off = in ? (int64_t)(j * KRPI) * p.ts * ESZ + (int64_t)lo
                                   : (int64_t)fallback_unit(lo);  // same unit of row 0
        __builtin_amdgcn_global_load_lds(base + row_off, lds_ptr(dst + j * 1024), 16, 0, kKeyLoadPolicy);
      }
    }
  }

  // Direct global->LDS load of the slab's query tile: row r = n*G + g holds Q[layer, n, kvh*G + g, :]
  // (rows beyond G*N repeat row 0; their columns of the logit tiles are never used).
  __device__ __forceinline__ void issue_queries(int slab, int slot) {
    int rows = p.G * p.N;
    asm volatile("" : "+s"(rows));
    const uint32_t dst = ring_lds + slot * TILE_B;
    const unsigned char* base = reinterpret_cast<const unsigned char*>(p.q) +
                                2 * (((int64_t)layer_of(slab) * p.N * p.H + kvh_of(slab) * p.G) * D);
    int ln = lane;
    asm volatile("" : "+v"(ln));  // per-load offsets are cheap to recompute and expensive to keep
    const int i = ln / UNITS;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int r = j * RPI + i;
      const int key = (D == 128) ? (r & 15) : ((r >> 1) & 7);
      const int unit = (ln % UNITS) ^ key;
      const int rr = r < rows ? r : 0;
      const uint32_t off = (uint32_t)((rr >> p.lgG) * p.H * ROW_B + (rr & (p.G - 1)) * ROW_B + unit * 16);
      __builtin_amdgcn_global_load_lds(base + off, lds_ptr(dst + j * 1024), 16, 0, 0);
    }
  }

  // issue stream tile number IDX counted from the start of slab `slab` (0 = its queries,
  // 1..TPW = its keys, TPW+1 = the next slab's queries, ...); past the end of the call the
  // last slab is read again (nobody consumes it)
  template <int IDX>
  __device__ __forceinline__ void issue_stream(int slab, int slot) {
    constexpr int ADV = IDX / TPS, I = IDX % TPS;
    // the slot is about to be overwritten: every LDS read of its previous tile must have been
    // performed (a freshly issued read could otherwise lose the race against an L2-hit load)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const int s = min(slab + ADV, p.n_slabs - 1);
    if (I == 0) issue_queries(s, slot); else issue_keys(s, I - 1, slot);
    note_issued(I == 0 ? LOADS : KLOADS);
    if (slot & 1) seq1 = issued; else seq0 = issued;
  }
  // the tile in ring slot `slot` has landed once at most the instructions issued after its
  // loads are still in flight (vector-memory instructions of a wave complete in order)
  __device__ __forceinline__ void wait_tile(int slot) {
    wait_vmcnt_upto(__builtin_amdgcn_readfirstlane(issued - ((slot & 1) ? seq1 : seq0)));
  }
  // the bookkeeping is wave-uniform; saying so keeps it in scalar registers
  __device__ __forceinline__ void note_issued(int k) { issued = __builtin_amdgcn_readfirstlane(issued + k); }

  __device__ __forceinline__ bf16x8 read_unit(int t, int slot) const {
    uint32_t base = rd0;
    asm volatile("" : "+v"(base));  // one XOR per read beats KS addresses held in registers all along
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
        lds_ptr((base ^ (uint32_t)(t << 5)) + slot * TILE_B));
  }

  __device__ __forceinline__ void read_queries(int slot) {
    if constexpr (FP8) {  // k-step 2j + e of this half-wave: query elements 16 (2j + h) + 8e ... = unit 4j + 2h + e
      uint32_t base = 0;
      if constexpr (FP8) base = this->qrd0;
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
    uint32_t base = 0;
    if constexpr (FP8) base = this->krd0;
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

  template <int SET>
  __device__ __forceinline__ void mfma_tile(int kb, int slot) {
    f32x16 a = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8 kf[KS];
    if constexpr (FP8) {
      read_keys_fp8(kf, slot);
#pragma unroll
      for (int t = 0; t < KS; ++t) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], a, 0, 0, 0);
      float k = 1.f;
      if constexpr (FP8) k = this->ks;
#pragma unroll
      for (int i = 0; i < 16; ++i) a[i] *= k;
      acc[SET][kb] = a;
      return;
    }
#pragma unroll
    for (int t = 0; t < KS; ++t) kf[t] = read_unit(t, slot);
#pragma unroll
    for (int t = 0; t < KS; ++t) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], a, 0, 0, 0);
    // operand reads run kAhead steps ahead of the matrix instructions that use them
    constexpr int kAhead = KS < 4 ? KS : 4;
    __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
    for (int t = 0; t < KS - kAhead; ++t) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
    acc[SET][kb] = a;
  }

  template <int SET>
  __device__ __forceinline__ void stats_tile(int kb) {
    f32x16& a = acc[SET][kb];
    const int inside = p.M - wave_tile_key(kb);  // keys of this tile that belong to the prompt (may be <= 0 or >= 32)
    if (inside < 32) {  // ragged tail: keys beyond the prompt do not count
      int left = inside - half * 4;  // keys of this half-wave's first register still inside
      asm volatile("" : "+v"(left));           // compare here, when needed: 16 hoisted lane masks would cost 32 SGPRs
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if ((i >> 2) * 8 + (i & 3) >= left) a[i] = -INFINITY;
    }
    float tm = a[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tm = fmaxf(tm, a[i]);
    const float m_new = fmaxf(run_m, tm);
    const float ref = (m_new == -INFINITY) ? 0.f : m_new;
    const float off = -ref * p.c;
    // four independent chains: the exponentials are long-latency and a single chain would
    // serialise on them
    float s0 = run_s * fast_exp2(fmaf(run_m, p.c, off)), s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
      s0 += fast_exp2(fmaf(a[i], p.c, off));
      s1 += fast_exp2(fmaf(a[i + 1], p.c, off));
      s2 += fast_exp2(fmaf(a[i + 2], p.c, off));
      s3 += fast_exp2(fmaf(a[i + 3], p.c, off));
    }
    run_m = m_new;
    run_s = (s0 + s1) + (s2 + s3);
  }

  // fold two (max, sum) pairs
  __device__ __forceinline__ void fold(float& m, float& s, float pm, float ps) const {
    const float mn = fmaxf(m, pm);
    const float ref = (mn == -INFINITY) ? 0.f : mn;
    s = s * fast_exp2((m - ref) * p.c) + ps * fast_exp2((pm - ref) * p.c);
    m = mn;
  }

  // Turn the stored logits of set SET into log2-probabilities and max them into smax: over the
  // heads of the KV group across lanes, over KV heads / layers in LDS.
  template <int SET>
  __device__ __forceinline__ void finish_set(float lse) {
    const float neg_lse = -lse;
    int c = col, h = half;
    asm volatile("" : "+v"(c), "+v"(h));  // recompute the few lane-dependent values here rather than keep them all along
    const bool writer = c < p.G * p.N && (c & (p.G - 1)) == 0;
    // LDS address of this lane's first key of tile 0 in its query's row of smax
    const uint32_t dst0 = lds_addr_of(smax + (c >> p.lgG) * (p.KPW + kSmaxPad) + kbg * TPW * 32 + h);
#pragma unroll
    for (int kb = 0; kb < TPW; ++kb) {
      float x[16];
      // step by step over all 16 registers: a DPP read right after the write of its source
      // register would cost wait states
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = fmaf(acc[SET][kb][i], p.c, neg_lse);
      if (p.lgG >= 1) {  // group size is uniform: these are scalar branches around one copy of the code
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
      const int inside = p.M - wave_tile_key(kb);
      if (inside < 32) {  // ragged tail: keys beyond the prompt never beat the -inf start value
        const int left = inside - h * 4;
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if ((i >> 2) * 8 + (i & 3) >= left) x[i] = -INFINITY;
      }
      if (writer) lds_fmax_tile(dst0 + kb * 128, x, std::make_integer_sequence<int, 16>{});
    }
  }
};

}  // namespace sp
