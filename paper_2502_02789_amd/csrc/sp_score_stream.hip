// Single-pass streaming scorer for one long prompt (B = 1, 8 KV heads).
//
// Computes the same quantity as the general kernels -- row softmax of the stored queries
// against the prompt keys (Sec. 3.2 equation of arXiv 2502.02789) followed by the max/mean
// aggregation of Sec. 3.2.2 -- but reads every K-cache byte from HBM exactly once.
//
// Why one pass is hard: the probability of key i in row (layer, head, query) needs that row's
// log-sum-exp over ALL keys, and the max over heads has to be taken on probabilities.  So the
// logits of a whole layer must stay somewhere until the row statistics are known.  Here they
// stay in registers:
//
//   * one persistent workgroup per CU owns a fixed slice of the prompt (KPW keys) for the
//     whole call; the work is cut into "slabs" = (layer, group of S KV heads), S chosen so
//     that a slab's logits (KPW keys x S heads x 32 query rows, fp32) fit in the accumulator
//     registers of the 8 waves, twice (two slabs are alive at any time);
//   * each wave streams the K rows of its own (KV head, key blocks) through a private
//     two-tile LDS ring with direct global->LDS loads, in an XOR-swizzled layout that makes
//     the MFMA operand reads conflict-free, and runs v_mfma_f32_32x32x16_bf16 with the keys
//     as matrix rows and the (query, head-in-group) pairs as columns;
//   * per slab every workgroup publishes, for each row, (max, sum 2^(x-max)) over its keys;
//     one designated workgroup per row folds the 256 partials into the row's log-sum-exp and
//     publishes it; these two hops overlap with the next slab's streaming (the exchange for
//     slab s-1 happens while slab s is being computed, which is why two logit sets are kept);
//   * with the row's log-sum-exp known, a slab's logits become log-probabilities; the max over
//     the heads of a KV group is a quad DPP max, the max over KV heads / layers an LDS float
//     atomic max per (query, key); the mean over layers (if asked) and queries is taken at the
//     layer end / kernel end.
//
// Cross-workgroup exchange uses 64-bit (max,sum) words and 32-bit log-sum-exp words that are
// "empty" (all ones) until written, written and polled with agent-scope atomics; the
// workspace is re-filled with the empty pattern by a small kernel at the start of each call.
// Every wait is bounded; the launch is cooperative so all workgroups are co-resident.
#include "sp_score_internal.h"

namespace sp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * kWave;
constexpr int kMaxWG = 256;
constexpr uint64_t kEmpty64 = ~0ull;
constexpr uint32_t kEmpty32 = ~0u;
constexpr int kSpinBudget = 1 << 22;  // polls per wave over the whole call before giving up

struct StreamDev {
  int M, L, N, H, G, S, slabs_per_layer, n_slabs, KPW, nwg, wpr, layer_reduce;
  float c;  // scale * log2(e): logits are handled in the base-2 domain
  int64_t ts, hs;
  const uint16_t* q;
  const int32_t* n_valid;
  uint64_t* partial;  // [rows][nwg][wpr]
  uint32_t* lse2;     // [rows]
  uint32_t* status;   // [0] != 0: a bounded wait ran out (results invalid)
  float* scores;
  float* lse_out;
  const uint16_t* k[SP_MAX_LAYERS];
};

__global__ __launch_bounds__(256) void fill_empty_kernel(uint4* __restrict__ dst, size_t n_vec, uint32_t* status) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
    dst[i] = make_uint4(kEmpty32, kEmpty32, kEmpty32, kEmpty32);
  if (blockIdx.x == 0 && threadIdx.x == 0) status[0] = 0;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

__device__ __forceinline__ uint64_t poll64(const uint64_t* p, int& budget) {
  uint64_t v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  while (v == kEmpty64 && budget > 0) {
    __builtin_amdgcn_s_sleep(2);
    --budget;
    v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return v;
}
__device__ __forceinline__ uint32_t poll32(const uint32_t* p, int& budget) {
  uint32_t v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  while (v == kEmpty32 && budget > 0) {
    __builtin_amdgcn_s_sleep(2);
    --budget;
    v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return v;
}

__device__ __forceinline__ float quad_xor1(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_xor2(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
}

template <int D, int TPW>
struct Streamer {
  static constexpr int KS = D / 16;          // MFMA k-steps per tile
  static constexpr int ROW_B = D * 2;        // bytes of one (token, KV head) row
  static constexpr int TILE_B = 32 * ROW_B;  // one 32-key tile of one KV head
  static constexpr int UNITS = ROW_B / 16;   // 16-byte units per row
  static constexpr int LOADS = TILE_B / 1024;  // wave-wide 16-byte loads per tile
  static constexpr int RPI = 64 / UNITS;     // rows covered by one such load

  const StreamDev& p;
  float* smax;           // [N][KPW] running max of log2-probabilities
  int wave, lane, half, col, wg;
  int kvh_local, kbg;
  int keys_wg;           // valid keys owned by this workgroup
  int n_tiles;           // tiles this wave streams over the whole call
  int budget;
  uint32_t ring_lds;     // LDS byte address of this wave's two-tile ring
  uint32_t rd0;          // LDS byte address of this lane's operand unit for k-step 0 in buffer 0
  uint32_t ld_off[4];    // per-lane global byte offset of load j (depends on j & 3 only)
  bf16x8 qf[KS];
  f32x16 acc[2][TPW];
  float run_m, run_s;    // running (max of raw logits, sum of 2^((x-max)*c)) of this lane's row

  // LDS layout of a tile: row r (one key) at r*ROW_B; inside a row the 16-byte unit holding
  // head-dim elements [8u, 8u+8) sits at position u ^ key(r), key(r) = r & 15 (D=128) or
  // (r >> 1) & 7 (D=64).  With it the 16 lanes of an operand read hit 16 distinct bank groups,
  // and a wave-wide direct load still fills 1 KiB of consecutive LDS.
  __device__ __forceinline__ Streamer(const StreamDev& p_, unsigned char* smem) : p(p_) {
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    lane = threadIdx.x & 63;
    half = lane >> 5;
    col = lane & 31;
    wg = blockIdx.x;
    kvh_local = wave % p.S;
    kbg = wave / p.S;
    ring_lds = (uint32_t)reinterpret_cast<uintptr_t>(smem) + wave * 2 * TILE_B;
    smax = reinterpret_cast<float*>(smem + kWaves * 2 * TILE_B);
    keys_wg = max(0, min(p.KPW, p.M - wg * p.KPW));
    n_tiles = p.n_slabs * TPW;
    budget = kSpinBudget;
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
  }

  __device__ __forceinline__ static __attribute__((address_space(3))) void* lds_ptr(uint32_t addr) {
    return reinterpret_cast<__attribute__((address_space(3))) void*>(addr);
  }

  // direct global->LDS load of tile f (flattened slab*TPW + kb) into ring buffer `buf`.
  // Always issues exactly LOADS wave-wide loads (the vmcnt bookkeeping counts on it): rows
  // beyond the prompt re-read row 0 of the last in-range tile and are masked later.
  __device__ __forceinline__ void issue_tile(int f, int buf) {
    const int slab = f / TPW, kb = f % TPW;
    const int l = slab / p.slabs_per_layer;
    const int kvh = (slab % p.slabs_per_layer) * p.S + kvh_local;
    int key_start = wg * p.KPW + (kbg * TPW + kb) * 32;
    // keep the address arithmetic below at its point of use: hoisted out of the slab loop it
    // would pin dozens of registers for the whole kernel
    asm volatile("" : "+s"(key_start));
    const uint32_t dst = ring_lds + buf * TILE_B;
    const int start_eff = min(key_start, (p.M - 1) & ~31);
    const unsigned char* base = reinterpret_cast<const unsigned char*>(p.k[l]) +
                                2 * ((int64_t)kvh * p.hs + (int64_t)start_eff * p.ts);
    if (start_eff + 32 <= p.M) {  // whole tile inside the prompt
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const unsigned char* src = base + (int64_t)(j * RPI) * p.ts * 2 + (size_t)ld_off[j & 3];
        __builtin_amdgcn_global_load_lds(src, lds_ptr(dst + j * 1024), 16, 0, 0);
      }
    } else {
      const int rows_in = p.M - start_eff;  // 1..31
      const int i = lane / UNITS;
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const bool in = j * RPI + i < rows_in;
        const int64_t row_off = in ? (int64_t)(j * RPI) * p.ts * 2 + (int64_t)ld_off[j & 3]
                                   : (int64_t)(ld_off[j & 3] & (uint32_t)(ROW_B - 1));  // same unit of row 0
        __builtin_amdgcn_global_load_lds(base + row_off, lds_ptr(dst + j * 1024), 16, 0, 0);
      }
    }
  }

  // query fragments of this wave's KV head for slab `slab` (B operand: column = query row)
  __device__ __forceinline__ void load_q(int slab) {
    const int l = slab / p.slabs_per_layer;
    const int kvh = (slab % p.slabs_per_layer) * p.S + kvh_local;
    const bool real = col < p.G * p.N;
    const int n = col / p.G, g = col % p.G;
    const uint16_t* row = p.q + (((int64_t)l * p.N + (real ? n : 0)) * p.H + kvh * p.G + (real ? g : 0)) * D +
                          half * 8;
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (real) v = *reinterpret_cast<const bf16x8*>(row + t * 16);
      qf[t] = v;
    }
  }

  template <int CUR>
  __device__ __forceinline__ void mfma_tile(int kb, int buf) {
    f32x16 a = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      const bf16x8 kfrag = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
          lds_ptr((rd0 ^ (uint32_t)(t << 5)) + buf * TILE_B));
      a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qf[t], a, 0, 0, 0);
    }
    acc[CUR][kb] = a;
  }

  // key (within the workgroup's slice) held by accumulator register i of tile kb in this lane
  __device__ __forceinline__ int key_of(int kb, int i) const {
    return (kbg * TPW + kb) * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
  }

  template <int CUR>
  __device__ __forceinline__ void stats_tile(int kb) {
    f32x16& a = acc[CUR][kb];
    const int first = (kbg * TPW + kb) * 32;
    if (first + 32 > keys_wg) {  // ragged tail: keys beyond the prompt do not count
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (key_of(kb, i) >= keys_wg) a[i] = -INFINITY;
    }
    float tm = a[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tm = fmaxf(tm, a[i]);
    const float m_new = fmaxf(run_m, tm);
    const float ref = (m_new == -INFINITY) ? 0.f : m_new;
    const float off = -ref * p.c;
    float s = run_s * fast_exp2(fmaf(run_m, p.c, off));
#pragma unroll
    for (int i = 0; i < 16; ++i) s += fast_exp2(fmaf(a[i], p.c, off));
    run_m = m_new;
    run_s = s;
  }

  __device__ __forceinline__ int row_base(int slab) const { return (slab * p.S + kvh_local) * 32; }

  // publish this wave's (max, sum) of every row of the slab over the keys it has seen
  __device__ __forceinline__ void publish(int slab) {
    const float m_o = __shfl_xor(run_m, 32, kWave);
    const float s_o = __shfl_xor(run_s, 32, kWave);
    const float mm = fmaxf(run_m, m_o);
    const float ref = (mm == -INFINITY) ? 0.f : mm;
    const float ss = run_s * fast_exp2((run_m - ref) * p.c) + s_o * fast_exp2((m_o - ref) * p.c);
    if (half == 0) {
      const uint64_t word = ((uint64_t)__float_as_uint(ss) << 32) | __float_as_uint(mm);
      uint64_t* dst = p.partial + ((int64_t)(row_base(slab) + col) * p.nwg + wg) * p.wpr + kbg;
      __hip_atomic_store(dst, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // fold all workgroups' partials of the rows this workgroup is responsible for (one wave)
  __device__ __forceinline__ void reduce_rows(int slab) {
    const int rows = p.S * 32;
    const int base = slab * rows;
    const int per_row = p.nwg * p.wpr;
    int first = base + ((wg - base) % p.nwg + p.nwg) % p.nwg;
    for (int row = first; row < base + rows; row += p.nwg) {
      const uint64_t* src = p.partial + (int64_t)row * per_row;
      float m = -INFINITY, s = 0.f;
      for (int e = lane; e < per_row; e += kWave) {
        const uint64_t w = poll64(src + e, budget);
        const float pm = __uint_as_float((uint32_t)w), ps = __uint_as_float((uint32_t)(w >> 32));
        const float mn = fmaxf(m, pm);
        const float ref = (mn == -INFINITY) ? 0.f : mn;
        s = s * fast_exp2((m - ref) * p.c) + ps * fast_exp2((pm - ref) * p.c);
        m = mn;
      }
      const float mw = wave_max(m);
      const float zw = wave_sum(s * fast_exp2((m - mw) * p.c));  // mw is finite: the prompt is not empty
      if (lane == 0) {
        const float lse2 = fmaf(mw, p.c, __builtin_amdgcn_logf(zw));  // v_log_f32 is log2
        __hip_atomic_store(p.lse2 + row, __float_as_uint(lse2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p.lse_out) {
          const int in_slab = row - base;
          const int qrow = in_slab & 31;
          if (qrow < p.G * p.N) {
            const int l = slab / p.slabs_per_layer;
            const int kvh = (slab % p.slabs_per_layer) * p.S + (in_slab >> 5);
            const int n = qrow / p.G, g = qrow % p.G;
            p.lse_out[((int64_t)l * p.N + n) * p.H + kvh * p.G + g] = lse2 * 0.6931471805599453f;
          }
        }
      }
    }
  }

  // turn the stored logits of slab `slab` (set PREV) into log2-probabilities and max them
  // into smax over the heads of the KV group (cross-lane) and over KV heads / layers (LDS)
  template <int PREV>
  __device__ __forceinline__ void finish_slab(int slab) {
    const uint32_t bits = poll32(p.lse2 + row_base(slab) + col, budget);
    const float neg_lse = -__uint_as_float(bits);
    const bool real = col < p.G * p.N;
    const int n = col / p.G, g = col % p.G;
    float* dst_row = smax + n * p.KPW;
#pragma unroll
    for (int kb = 0; kb < TPW; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float x = real ? fmaf(acc[PREV][kb][i], p.c, neg_lse) : -INFINITY;
        if (p.G >= 2) x = fmaxf(x, quad_xor1(x));
        if (p.G >= 4) x = fmaxf(x, quad_xor2(x));
        if (p.G >= 8) x = fmaxf(x, __shfl_xor(x, 4, kWave));
        const int key = key_of(kb, i);
        if (real && g == 0 && key < keys_wg)
          __hip_atomic_fetch_max(dst_row + key, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
  }
};

template <int D, int TPW>
__global__ __launch_bounds__(kThreads) void stream_score_kernel(const StreamDev p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  using St = Streamer<D, TPW>;
  St st(p, smem);
  const int cells = p.N * p.KPW;  // (query, key) cells of this workgroup
  float tot[8];                   // layer-mean mode: sum over layers, cell = threadIdx + 512*j
#pragma unroll
  for (int j = 0; j < 8; ++j) tot[j] = 0.f;
  for (int i = threadIdx.x; i < cells; i += kThreads) st.smax[i] = -INFINITY;
  __syncthreads();

  st.load_q(0);
  st.issue_tile(0, 0);
  if (st.n_tiles > 1) st.issue_tile(1, 1);

  auto body = [&](auto cur_tag, int slab) {
    constexpr int CUR = decltype(cur_tag)::value;
    st.run_m = -INFINITY;
    st.run_s = 0.f;
#pragma unroll
    for (int kb = 0; kb < TPW; ++kb) {
      const int f = slab * TPW + kb;
      if (f + 1 < st.n_tiles) wait_vmcnt<St::LOADS>(); else wait_vmcnt<0>();
      st.template mfma_tile<CUR>(kb, f & 1);
      if (kb == TPW - 1 && slab + 1 < p.n_slabs) st.load_q(slab + 1);  // next slab's queries, behind this slab's MFMAs
      if (f + 2 < st.n_tiles) st.issue_tile(f + 2, f & 1);
      if (kb == (TPW >= 2 ? TPW / 2 - 1 : 0) && slab >= 1 && st.wave == ((slab - 1) & 7)) st.reduce_rows(slab - 1);
      st.template stats_tile<CUR>(kb);
    }
    st.publish(slab);
    if (slab >= 1) {
      st.template finish_slab<1 - CUR>(slab - 1);
      if (p.layer_reduce == SP_LAYER_MEAN && slab % p.slabs_per_layer == 0) {  // slab-1 closed a layer
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int cell = threadIdx.x + kThreads * j;
          if (cell < cells) {
            const float v = st.smax[cell];
            tot[j] += fast_exp2(v);
            st.smax[cell] = -INFINITY;
          }
        }
        __syncthreads();
      }
    }
  };

  for (int slab = 0; slab < p.n_slabs; slab += 2) {
    body(std::integral_constant<int, 0>{}, slab);
    if (slab + 1 < p.n_slabs) body(std::integral_constant<int, 1>{}, slab + 1);
  }
  // last slab: the exchange cannot hide behind further streaming
  const int last = p.n_slabs - 1;
  if (st.wave == (last & 7)) st.reduce_rows(last);
  if (last & 1) st.template finish_slab<1>(last); else st.template finish_slab<0>(last);
  __syncthreads();

  int nv = p.n_valid ? p.n_valid[0] : p.N;
  nv = max(1, min(nv, p.N));
  if (p.layer_reduce == SP_LAYER_MEAN) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int cell = threadIdx.x + kThreads * j;
      if (cell < cells) st.smax[cell] = tot[j] + fast_exp2(st.smax[cell]);  // + the last layer
    }
    __syncthreads();
  }
  for (int key = threadIdx.x; key < st.keys_wg; key += kThreads) {
    float sum = 0.f;
    for (int n = 0; n < nv; ++n) {
      const float v = st.smax[n * p.KPW + key];
      sum += (p.layer_reduce == SP_LAYER_MEAN) ? v : fast_exp2(v);
    }
    const float denom = (p.layer_reduce == SP_LAYER_MEAN) ? (float)nv * (float)p.L : (float)nv;
    p.scores[(int64_t)blockIdx.x * p.KPW + key] = sum / denom;
  }
  if (st.budget <= 0 && st.lane == 0) atomicOr(p.status, 1u);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
struct StreamPlan {
  bool ok;
  int nwg, KPW, S, TPW, wpr, slabs_per_layer, n_slabs;
  size_t rows, partial_bytes, lse_bytes, smem_bytes;
};

static int device_cu_count() {
  static int cached = -1;
  if (cached >= 0) return cached;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return kMaxWG;  // no device visible (sizing queries on a CPU-only host): assume the full chip
  }
  cached = cus;
  return cached;
}

static StreamPlan make_plan(const sp_score_args* a, int nwg) {
  StreamPlan pl{};
  pl.ok = false;
  const int G = a->H / a->H_kv;
  if (a->B != 1 || a->H_kv != 8 || a->T < 1) return pl;
  if (G != 1 && G != 2 && G != 4 && G != 8) return pl;
  if (G * a->N > 32 || a->N > 8) return pl;
  nwg = std::min(nwg, kMaxWG);
  int kb = (int)((a->T + (int64_t)nwg * 32 - 1) / ((int64_t)nwg * 32));
  int kb2 = 1;
  while (kb2 < kb) kb2 <<= 1;
  if (kb2 > 16) return pl;  // beyond 16 key blocks per workgroup the slabs no longer fit
  pl.nwg = nwg;
  pl.KPW = kb2 * 32;
  if (kb2 <= 4) { pl.S = 8; pl.TPW = kb2; } else { pl.S = 32 / kb2; pl.TPW = 4; }
  pl.wpr = kWaves / pl.S;
  pl.slabs_per_layer = a->H_kv / pl.S;
  pl.n_slabs = a->L * pl.slabs_per_layer;
  pl.rows = (size_t)a->L * a->H_kv * 32;
  pl.partial_bytes = align_up(pl.rows * nwg * pl.wpr * sizeof(uint64_t), 256);
  pl.lse_bytes = align_up(pl.rows * sizeof(uint32_t), 256);
  pl.smem_bytes = (size_t)kWaves * 2 * 32 * a->d * 2 + (size_t)a->N * pl.KPW * sizeof(float);
  if (pl.smem_bytes > 160 * 1024) return pl;
  if ((size_t)a->N * pl.KPW > 8 * kThreads) return pl;
  pl.ok = true;
  return pl;
}

bool stream_supported(const sp_score_args* a) { return make_plan(a, device_cu_count()).ok; }

size_t stream_workspace_bytes(const sp_score_args* a) {
  const StreamPlan pl = make_plan(a, kMaxWG);  // sized for the full chip
  if (!pl.ok) return 0;
  return pl.partial_bytes + pl.lse_bytes + 256;
}

template <int D, int TPW>
static sp_status launch_stream(const StreamDev& dev, const StreamPlan& pl, hipStream_t stream) {
  auto kernel = stream_score_kernel<D, TPW>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)pl.smem_bytes) != hipSuccess)
    return SP_ELAUNCH;
  StreamDev copy = dev;
  void* args[] = {&copy};
  if (hipLaunchCooperativeKernel(reinterpret_cast<const void*>(kernel), dim3(pl.nwg), dim3(kThreads), args,
                                 (unsigned)pl.smem_bytes, stream) != hipSuccess)
    return SP_ELAUNCH;
  return SP_OK;
}

sp_status stream_score(const sp_score_args* a, hipStream_t stream) {
  const StreamPlan pl = make_plan(a, device_cu_count());
  if (!pl.ok) return SP_EUNSUPPORTED;
  StreamDev dev;
  dev.M = (int)a->T; dev.L = a->L; dev.N = a->N; dev.H = a->H; dev.G = a->H / a->H_kv; dev.S = pl.S;
  dev.slabs_per_layer = pl.slabs_per_layer; dev.n_slabs = pl.n_slabs; dev.KPW = pl.KPW; dev.nwg = pl.nwg;
  dev.wpr = pl.wpr; dev.layer_reduce = a->layer_reduce;
  dev.c = a->scale * 1.4426950408889634f;
  dev.ts = a->k_token_stride; dev.hs = a->k_head_stride;
  dev.q = static_cast<const uint16_t*>(a->d_q);
  dev.n_valid = a->d_n_valid;
  char* ws = static_cast<char*>(a->d_workspace);
  dev.partial = reinterpret_cast<uint64_t*>(ws);
  dev.lse2 = reinterpret_cast<uint32_t*>(ws + pl.partial_bytes);
  dev.status = reinterpret_cast<uint32_t*>(ws + pl.partial_bytes + pl.lse_bytes);
  dev.scores = a->d_scores; dev.lse_out = a->d_lse;
  for (int l = 0; l < SP_MAX_LAYERS; ++l)
    dev.k[l] = l < a->L ? static_cast<const uint16_t*>(a->k_layers[l]) : nullptr;

  const size_t n_vec = (pl.partial_bytes + pl.lse_bytes) / 16;
  const int fill_blocks = (int)std::min<size_t>((n_vec + 255) / 256, 2048);
  hipLaunchKernelGGL(fill_empty_kernel, dim3(fill_blocks), dim3(256), 0, stream, reinterpret_cast<uint4*>(ws),
                     n_vec, dev.status);
  if (hipGetLastError() != hipSuccess) return SP_ELAUNCH;
  if (a->d == 128) {
    switch (pl.TPW) {
      case 1: return launch_stream<128, 1>(dev, pl, stream);
      case 2: return launch_stream<128, 2>(dev, pl, stream);
      default: return launch_stream<128, 4>(dev, pl, stream);
    }
  }
  switch (pl.TPW) {
    case 1: return launch_stream<64, 1>(dev, pl, stream);
    case 2: return launch_stream<64, 2>(dev, pl, stream);
    default: return launch_stream<64, 4>(dev, pl, stream);
  }
}

}  // namespace sp
