// Single-pass streaming scorer for one long prompt (B = 1, 8 KV heads).
//
// Computes the same quantity as the general kernels -- row softmax of the stored queries
// against the prompt keys (Sec. 3.2 equation of arXiv 2502.02789) followed by the max/mean
// aggregation of Sec. 3.2.2 -- but reads every K-cache byte from HBM exactly once.
//
// Why one pass is hard: the probability of key i in row (layer, head, query) needs that row's
// log-sum-exp over ALL keys, and the max over heads has to be taken on probabilities.  So the
// logits must stay somewhere until the row statistics are known.  Here they stay in registers:
//
//   * one persistent workgroup per CU owns a fixed slice of the prompt (KPW keys) for the whole
//     call; the work is cut into "slabs" = (layer, group of S KV heads).  A slab's logits are
//     TPW accumulator tiles (32 keys x 32 query rows, fp32) per wave; the register file holds
//     NSETS = 8 / TPW slabs at once, so a slab's logits survive NSETS further slabs of
//     streaming -- the window in which the cross-workgroup exchange below has to finish;
//   * every wave streams its own sequence of 32-row tiles through a private two-slot LDS ring
//     with direct global->LDS loads: per slab one tile of query rows (its KV head's 32
//     (query, head-in-group) rows) followed by TPW tiles of keys.  Tiles are stored with an
//     XOR swizzle that makes the MFMA operand reads bank-conflict free; the MFMA is
//     v_mfma_f32_32x32x16_bf16 with keys as matrix rows and query rows as columns;
//   * exchange, publication: per slab every wave deposits, for each of its rows, (max, sum
//     2^(x-max)) over its keys in LDS.  The wave that deposits last only flags the slab; a wave
//     of the workgroup that has time (typically one waiting for a log-sum-exp) merges the
//     deposits into one base-2 log-sum-exp per row and stores them, 16 bytes per four rows
//     (every coherent access costs the chip's memory pipeline time in proportion to its size,
//     so a publication is as small as it can be);
//   * exchange, reduction: for every four rows one workgroup (round-robin) owns the reduction
//     as a duty kept in LDS.  A step of it -- sample all workgroups' words with four
//     direct-to-LDS loads, or look at the landed sample and, once no word is empty, fold it into
//     the four rows' log-sum-exps and store those -- is done by whichever wave comes by, at the
//     end of every slab and all the time while it waits for a log-sum-exp of its own;
//   * exchange, consumption: each wave fetches the 32 log-sum-exps of its rows with one more
//     direct-to-LDS load, issued one tile before they are needed;
//   * nothing of this is ever waited for through vmcnt: a sample's LDS landing zone is filled
//     with a "pending" pattern before the load is issued and simply looked at later, so the
//     stream of key tiles is never drained for the exchange (a drained wave publishes late, and
//     everybody waits for the last publication).  vmcnt waits are for key/query tiles only and
//     count exactly the instructions issued after the tile waited for;
//   * with the log-sum-exp known a slab's logits become log2-probabilities; the max over the
//     heads of a KV group is a quad DPP max, the max over KV heads / layers an LDS float
//     atomic max per (query, key); the layer mean (if asked) and the query mean are taken at
//     layer end / kernel end.
//
// Cross-workgroup words are "empty" (all ones) until written, and are written and read with
// agent-scope coherence; a small kernel refills the workspace with the empty pattern at the
// start of each call.  Every wait is bounded (a status word records an expired wait), and a
// wave that waits, or is about to park at a barrier or to exit, keeps serving its workgroup's
// duties, so waiting waves cannot starve each other.  The grid is one workgroup per CU, each
// needing more than half of a CU's LDS, so all of them are resident together on an otherwise
// idle device; that residency is what every wait relies on.
#include <atomic>
#include <mutex>

#include "sp_stream_core.h"

namespace sp {

constexpr int kCtlBytes = 128;         // arrival counters and the workgroup's duty words
constexpr int kStageBytes = kMaxWG * 16;  // landing zone of a reducer's sample: 4 rows x 4 bytes per workgroup
constexpr int kDepSlotBytes = 8 * 32 * 8;  // one slab's deposits: 8 waves x 32 rows x (max, sum)

struct StreamDev : StreamShape {
  int nwg, wpr, layer_reduce;
  const int32_t* n_valid;
  uint32_t* partial;  // [quad of rows][nwg][4]: each workgroup's log-sum-exp (base 2) of the quad's rows
  uint32_t* lse2;     // [rows]
  uint32_t* status;   // [0] != 0: a bounded wait ran out (results invalid)
  float* scores;
  float* lse_out;
};

__device__ __forceinline__ uint64_t pack_stat(float m, float s) {
  return ((uint64_t)__float_as_uint(s) << 32) | __float_as_uint(m);
}

template <int D, int TPW, bool PAGED = false, bool FP8 = false>
struct Streamer : StreamCore<D, TPW, PAGED, FP8> {
  using Core = StreamCore<D, TPW, PAGED, FP8>;
  using Core::NSETS; using Core::TILE_B; using Core::RING_BYTES;
  using Core::wave; using Core::lane; using Core::half; using Core::col; using Core::kvh_local;
  using Core::budget; using Core::issued; using Core::run_m; using Core::run_s;
  using Core::may_poll; using Core::note_issued; using Core::fold; using Core::lds_ptr; using Core::layer_of;
  // slab s: published by the last wave to finish it, reduced by its reducers as soon as every
  // workgroup's words are seen, its log-sum-exps requested at the end of slab s + NSETS - 1 and
  // used at the start of slab s + NSETS (just before its register set is reused)

  const StreamDev& p;
  int wg;
  int duty_k;            // reducer rotation: this workgroup reduces quad duty_k of the slab if duty_k < quads
  uint32_t dep_lds;      // LDS: [NSETS][8 waves][32 rows] (max, sum) deposits
  uint32_t cnt_lds;      // LDS control block: words 0..7 arrival counters per set; 8 reducer duty (quad or -1);
                         // 9 mask of sets waiting to be published; 10, 11 the two duties' locks; 12 reducer
                         // sample flag; 13 "a wait of some wave expired"; 16..23 slab number of the set
                         // waiting to be published
  uint32_t lse_lds;      // LDS: this wave's [2][32] fetched log-sum-exps
  uint32_t stage_lds;    // LDS: landing zone of a reducer sample (one per workgroup)

  static constexpr int kFixedBytes = RING_BYTES + NSETS * kDepSlotBytes + kCtlBytes + kWaves * 256 + kStageBytes;

  __device__ __forceinline__ Streamer(const StreamDev& p_, unsigned char* smem)
      : Core(p_, (uint32_t)reinterpret_cast<uintptr_t>(smem), reinterpret_cast<float*>(smem + kFixedBytes),
             (int)blockIdx.x, 0),
        p(p_) {
    wg = blockIdx.x;
    const uint32_t smem_lds = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    dep_lds = smem_lds + RING_BYTES;
    cnt_lds = dep_lds + NSETS * kDepSlotBytes;
    lse_lds = cnt_lds + kCtlBytes + wave * 256;
    stage_lds = cnt_lds + kCtlBytes + kWaves * 256;
    duty_k = wg;
  }

  __device__ __forceinline__ int row_base(int slab) const { return ((slab << p.lgS) + kvh_local) * 32; }

  // Hop 1, sending side.  Deposit this wave's (max, sum) of each of its 32 rows in LDS and count
  // the arrival; the wave that arrives last publishes the slab (LDS operations of a wave are
  // performed in order, so whoever sees the count complete also sees every deposit).
  template <int SET>
  __device__ __forceinline__ void deposit(int slab) {
    float m = run_m, s = run_s;
    fold(m, s, __shfl_xor(run_m, 32, kWave), __shfl_xor(run_s, 32, kWave));
    uint32_t dst = dep_lds + (wave * 32 + col) * 8;
    asm volatile("" : "+v"(dst));  // one address plus an immediate per set, not NSETS addresses kept alive
    if (half == 0) lds_poke64<SET * kDepSlotBytes>(dst, pack_stat(m, s));
    uint32_t old = 0;
    if (lane == 0) old = lds_add_rtn(cnt_lds + SET * 4, 1);
    old = __builtin_amdgcn_readfirstlane(old);
    const bool last = (old & 7) == 7;
    // the slab is complete: leave its publication to whoever has time (this wave is the one that
    // has none: it is the workgroup's last)
    if (last && lane == 0) {
      lds_poke32(cnt_lds + 64 + SET * 4, (uint32_t)slab);
      lds_or(cnt_lds + 36, 1u << SET);
    }
    advance_duty(slab, last);
  }

  // Merge the deposits of the waves that share rows into one base-2 log-sum-exp per row and
  // send the workgroup's S*32 rows out, four rows (16 bytes) per lane.  The words of one quad
  // from all workgroups are neighbours in memory: the reducer's sample is one dense 4 KiB read
  // (what is scattered is these writes, once; reads may have to be repeated).  Deposits are
  // indexed [kbg * S + kvh_local][query row].
  __device__ __forceinline__ void publish(int slab, uint32_t dep) {
    const int quads = p.S * 8;
    int ln = lane;
    asm volatile("" : "+v"(ln));  // address arithmetic of this rare path stays here instead of being hoisted
    if (ln < quads) {
      float m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY}, z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
      for (int g = 0; g < p.wpr; ++g) {
        const uint32_t a = dep + ((g * p.S + (ln >> 3)) * 32 + (ln & 7) * 4) * 8;
        const u32x4 w0 = lds_peek128(a), w1 = lds_peek128(a + 16);
        fold(m[0], z[0], __uint_as_float(w0.x), __uint_as_float(w0.y));
        fold(m[1], z[1], __uint_as_float(w0.z), __uint_as_float(w0.w));
        fold(m[2], z[2], __uint_as_float(w1.x), __uint_as_float(w1.y));
        fold(m[3], z[3], __uint_as_float(w1.z), __uint_as_float(w1.w));
      }
      // (-inf, 0) -- no key of the prompt in this workgroup -- gives -inf, which is a value, not "empty"
      u32x4 out;
#pragma unroll
      for (int r = 0; r < 4; ++r) out[r] = __float_as_uint(fmaf(m[r], p.c, __builtin_amdgcn_logf(z[r])));  // v_log_f32 is log2
      store128_agent(p.partial + (((int64_t)slab * quads + ln) * p.nwg + wg) * 4, out);
    }
    note_issued(1);
  }

  // Reducer rotation.  Quad number x (four rows; counted over the whole call) is reduced by
  // workgroup x % nwg.  Every wave keeps the rotation in step (called once per slab, in slab
  // order); the wave that has just published the slab posts the workgroup's duty for it, if it
  // has one, in LDS, where any wave of the workgroup can pick it up.
  __device__ __forceinline__ void advance_duty(int slab, bool post) {
    const int quads = p.S * 8;
    if (post && duty_k < quads) {
      while ((int)__builtin_amdgcn_readfirstlane(lds_peek(cnt_lds + 32)) >= 0 && may_poll()) {
        service_reduce();  // the previous duty is still open: cannot happen unless the exchange is badly late
        __builtin_amdgcn_s_sleep(4);
      }
      if (lane == 0) {
        lds_poke32(cnt_lds + 48, 0);                               // nothing sampled yet
        lds_poke32(cnt_lds + 32, (uint32_t)(slab * quads + duty_k));  // (LDS writes of a wave are performed in order)
      }
    }
    duty_k -= quads;
    if (duty_k < 0) duty_k += p.nwg;
  }
  // anything left that only this workgroup can do for the others?
  __device__ __forceinline__ bool duty_open() {
    const uint64_t v = lds_peek64(cnt_lds + 32);
    return (int)__builtin_amdgcn_readfirstlane((uint32_t)v) >= 0 || __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32)) != 0;
  }
  // Publish one complete slab, if one is waiting and nobody else is at it.  `not_set`: the set this
  // wave has just completed itself (it leaves that one to a wave with time on its hands), or -1.
  __device__ __forceinline__ void service_publish(uint32_t mask, int not_set) {
    if (not_set >= 0) mask &= ~(1u << not_set);
    if (mask == 0) return;
    uint32_t held = 1;
    if (lane == 0) held = lds_or_rtn(cnt_lds + 44, 1);
    if (__builtin_amdgcn_readfirstlane(held) != 0) return;
    uint32_t now = __builtin_amdgcn_readfirstlane(lds_peek(cnt_lds + 36));
    if (not_set >= 0) now &= ~(1u << not_set);
    if (now != 0) {
      const int set = __builtin_ctz(now);
      const int slab = (int)__builtin_amdgcn_readfirstlane(lds_peek(cnt_lds + 64 + set * 4));
      publish(slab, dep_lds + set * kDepSlotBytes);
      if (lane == 0) lds_and(cnt_lds + 36, ~(1u << set));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lane == 0) lds_poke32(cnt_lds + 44, 0);
  }

  // Hop 1, receiving side: one step of the workgroup's reducer duty, by whichever wave comes
  // by -- at the end of every slab, and all the time while it waits for a log-sum-exp, so the
  // waves that are ahead of the others do this work.  Never waits.  No sample out yet: send one
  // of the quad's nwg x 4 values on its way into the landing zone (marked "pending" first).
  // Sample out: look at the zone (LDS reads only); words still pending -> later; a value still
  // empty -> sample again; all there -> fold them into the four rows' log-sum-exps and publish.
  __device__ __forceinline__ void service_reduce(int not_set = -1) {
    const uint64_t duties = lds_peek64(cnt_lds + 32);
    const int quad = (int)__builtin_amdgcn_readfirstlane((uint32_t)duties);
    const uint32_t mask = __builtin_amdgcn_readfirstlane((uint32_t)(duties >> 32));
    if (mask != 0) service_publish(mask, not_set);
    if (quad < 0) return;
    // the duty is one wave's at a time: test-and-set (an add that is taken back when it finds the
    // lock held would make the lock look held to everybody else in the meantime, and with eight
    // waves asking in a tight loop nobody would ever get it)
    uint32_t held = 1;
    if (lane == 0) held = lds_or_rtn(cnt_lds + 40, 1);
    if (__builtin_amdgcn_readfirstlane(held) != 0) return;
    // (the duty may have been finished between the two looks above)
    const int quad2 = (int)__builtin_amdgcn_readfirstlane(lds_peek(cnt_lds + 32));
    if (quad2 == quad) reduce_step(quad);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lane == 0) lds_poke32(cnt_lds + 40, 0);
  }
  __device__ __forceinline__ void reduce_step(int quad) {
    int ln = lane;
    asm volatile("" : "+v"(ln));  // address arithmetic of this rare path stays here instead of being hoisted
    const bool sampled = __builtin_amdgcn_readfirstlane(lds_peek(cnt_lds + 48)) != 0;
    const int groups = (p.nwg + kWave - 1) / kWave;
    bool pending = false, empty = false;
    u32x4 w[kMaxWG / kWave];
    if (sampled) {
#pragma unroll
      for (int i = 0; i < kMaxWG / kWave; ++i) {
        if (i < groups) {
          w[i] = lds_peek128(stage_lds + (ln + i * kWave) * 16);
          pending |= w[i].x == kPending32 || w[i].y == kPending32 || w[i].z == kPending32 || w[i].w == kPending32;
          empty |= w[i].x == kEmpty32 || w[i].y == kEmpty32 || w[i].z == kEmpty32 || w[i].w == kEmpty32;
        } else {
          w[i] = u32x4{0xff800000u, 0xff800000u, 0xff800000u, 0xff800000u};  // -inf: contributes nothing
        }
      }
      if (__any(pending)) return;
    }
    if (!sampled || __any(empty)) {
      const uint32_t* src = p.partial + (int64_t)quad * p.nwg * 4;
      const u32x4 fill = {kPending32, kPending32, kPending32, kPending32};
#pragma unroll 1  // rare path: keep its register appetite small
      for (int i = 0; i < groups; ++i) lds_poke128(stage_lds + (ln + i * kWave) * 16, fill);
      if (ln == 0) lds_poke32(cnt_lds + 48, 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the pattern is in place before any answer can land
#pragma unroll
      for (int i = 0; i < kMaxWG / kWave; ++i) {
        if (i < groups) {
          const int e = min(ln + i * kWave, p.nwg - 1);  // lanes past the end repeat the last workgroup
          __builtin_amdgcn_global_load_lds(src + (int64_t)e * 4, lds_ptr(stage_lds + i * 1024), 16, 0, /*sc1*/ 16);
        }
      }
      note_issued(groups);
      return;
    }
    const int slab = quad >> (p.lgS + 3);
    const int q4 = (quad - (slab << (p.lgS + 3))) * 4;  // first of the four rows, within the slab
    float lse4[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float v[kMaxWG / kWave];
#pragma unroll
      for (int i = 0; i < kMaxWG / kWave; ++i)  // lanes past the last workgroup hold a repeat: count it as nothing
        v[i] = ln + i * kWave < p.nwg ? __uint_as_float(w[i][r]) : -INFINITY;
      float m = v[0];
#pragma unroll
      for (int i = 1; i < kMaxWG / kWave; ++i) m = fmaxf(m, v[i]);
      m = wave_max(m);  // finite: the prompt is not empty
      float z = 0.f;
#pragma unroll
      for (int i = 0; i < kMaxWG / kWave; ++i) z += fast_exp2(v[i] - m);
      lse4[r] = m + __builtin_amdgcn_logf(wave_sum(z));
    }
    if (ln == 0) {
      const u32x4 out = {__float_as_uint(lse4[0]), __float_as_uint(lse4[1]), __float_as_uint(lse4[2]), __float_as_uint(lse4[3])};
      store128_agent(p.lse2 + (int64_t)quad * 4, out);
      if (p.lse_out) {
        const int kvh = ((slab & (p.slabs_per_layer - 1)) << p.lgS) + (q4 >> 5);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int qrow = (q4 & 31) + r;
          if (qrow < p.G * p.N)
            p.lse_out[((int64_t)layer_of(slab) * p.N + (qrow >> p.lgG)) * p.H + kvh * p.G + (qrow & (p.G - 1))] =
                lse4[r] * 0.6931471805599453f;
        }
      }
      lds_poke32(cnt_lds + 32, ~0u);  // duty done
    }
    note_issued(1);  // (the optional log-sum-exp output is not counted: counting less only waits more)
  }

  // Hop 2.  Request the log-sum-exps of this wave's 32 rows of the slab with one direct-to-LDS
  // load (agent-coherent) into a landing zone marked "pending".  One request per slab: every
  // coherent access costs the whole chip a little, repeats did not pay.
  __device__ __forceinline__ void request_lse(int slab) {
    int c = col;
    asm volatile("" : "+v"(c));
    if (half == 0) {
      lds_poke32(lse_lds + (slab & 1) * 128 + c * 4, kPending32);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_global_load_lds(p.lse2 + row_base(slab) + c, lds_ptr(lse_lds + (slab & 1) * 128), 4, 0, /*sc1*/ 16);
    }
    note_issued(1);
  }
  // Take this lane's log-sum-exp.  Normally it is there; if the exchange is late, ask again
  // whenever an answer came back empty, and keep this wave's own reducer duty going meanwhile
  // (another wave may be waiting for exactly that).
  __device__ __forceinline__ float take_lse(int slab) {
    int c = col;
    asm volatile("" : "+v"(c));
    const uint32_t addr = lse_lds + (slab & 1) * 128 + c * 4;
    uint32_t bits = lds_peek(addr);
    while (__any(bits == kPending32 || bits == kEmpty32) && may_poll()) {
      if (!__any(bits == kPending32)) request_lse(slab);
      service_reduce();
      __builtin_amdgcn_s_sleep(4);
      bits = lds_peek(addr);
    }
    return __uint_as_float(bits);
  }
};

template <int D, int TPW, bool MEAN, bool PAGED, bool FP8>
__global__ __launch_bounds__(kThreads) void stream_score_kernel(const StreamDev p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  using St = Streamer<D, TPW, PAGED, FP8>;
  constexpr int NSETS = St::NSETS, TPS = St::TPS;
  St st(p, smem);
  const int cells = p.N * p.KPW;  // (query, key) cells of this workgroup
  auto cell_at = [&](int c) __attribute__((always_inline)) { return st.smax + c + kSmaxPad * (c >> p.lgKPW); };  // skips the row padding
  float tot[MEAN ? 8 : 1];        // layer-mean mode: sum over layers, cell = threadIdx + 512*j
#pragma unroll
  for (int j = 0; j < (MEAN ? 8 : 1); ++j) tot[j] = 0.f;
  for (int i = threadIdx.x; i < cells; i += kThreads) *cell_at(i) = -INFINITY;
  if (threadIdx.x < 16)  // arrival counters, duty lock and flag: 0; the duty itself: none
    *reinterpret_cast<uint32_t*>(smem + St::RING_BYTES + NSETS * kDepSlotBytes + threadIdx.x * 4) = threadIdx.x == 8 ? ~0u : 0u;
  __syncthreads();

  // layer-mean mode: slab `done` was just finished by this wave; if it closes a layer (other
  // than the last), fold the layer's maxima into the running sums.  Needs every wave's
  // contribution, hence the workgroup barriers; the condition is the same in every wave.
  auto close_layer = [&](int done) __attribute__((always_inline)) {
    if (MEAN && ((done + 1) & (p.slabs_per_layer - 1)) == 0 && done + 1 < p.n_slabs) {
      // a wave parked at a barrier serves nobody: finish the reducer duty first (it only needs
      // publications of slabs every wave of the grid has already left behind)
      while (st.duty_open() && st.may_poll()) {
        st.service_reduce();
        __builtin_amdgcn_s_sleep(4);
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's LDS atomics have been performed
      __syncthreads();
      int t = threadIdx.x;
      asm volatile("" : "+v"(t));  // the cells' addresses are formed here, once per layer, not kept in registers all along
                                   // (kept, they spill, and a reload from scratch drains the tile prefetch)
#pragma unroll
      for (int j = 0; j < (MEAN ? 8 : 1); ++j) {
        const int cell = t + kThreads * j;
        if (cell < cells) {
          const uint32_t addr = St::lds_addr_of(cell_at(cell));
          tot[j] += fast_exp2(__uint_as_float(lds_peek(addr)));
          lds_poke32(addr, 0xff800000u);  // -inf
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __syncthreads();
    }
  };

  st.template issue_stream<0>(0, 0);
  st.template issue_stream<1>(0, 1);

  // One slab.  Stream tile x of the slab sits in ring slot (SET*TPS + x) & 1 (NSETS is even, so
  // the slab's parity is SET's).
  auto body = [&](auto set_tag, int slab) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value;
    constexpr int SLOT0 = (SET * TPS) & 1;
    // The two waves that share a SIMD take turns at being the one the instruction arbiter
    // prefers; left alone it favours the older wave throughout, and the slab is only published
    // when the slowest wave is done with it.
    if ((slab ^ (st.wave >> 2)) & 1) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(0);
    st.slab_scale(slab);
    st.wait_tile(SLOT0);
    st.read_queries(SLOT0);
    st.template issue_stream<2>(slab, SLOT0);
    if (slab >= NSETS) {  // set SET still holds slab - NSETS, whose log-sum-exps were requested a tile ago
      st.template finish_set<SET>(st.take_lse(slab - NSETS));
      close_layer(slab - NSETS);
    }
    st.run_m = -INFINITY;
    st.run_s = 0.f;
#pragma unroll
    for (int kb = 0; kb < TPW; ++kb) {
      const int slot = (SLOT0 + 1 + kb) & 1;
      st.wait_tile(slot);
      st.template mfma_tile<SET>(kb, slot);
      if (kb == TPW - 1 && slab + 1 >= NSETS) st.request_lse(slab + 1 - NSETS);
      switch (kb) {  // a compile-time constant after unrolling
        case 0: st.template issue_stream<3>(slab, slot); break;
        case 1: st.template issue_stream<4>(slab, slot); break;
        case 2: st.template issue_stream<5>(slab, slot); break;
        default: st.template issue_stream<6>(slab, slot); break;
      }
      st.template stats_tile<SET>(kb);
    }
    st.template deposit<SET>(slab);
    // a step of the workgroup's duties, here, where the fewest registers are live
    st.service_reduce(SET);
  };

  for (int s0 = 0; s0 < p.n_slabs; s0 += NSETS) {
    body(std::integral_constant<int, 0>{}, s0);
    if (s0 + 1 < p.n_slabs) body(std::integral_constant<int, 1>{}, s0 + 1);
    if (NSETS > 2) {
      if (s0 + 2 < p.n_slabs) body(std::integral_constant<int, 2 % NSETS>{}, s0 + 2);
      if (s0 + 3 < p.n_slabs) body(std::integral_constant<int, 3 % NSETS>{}, s0 + 3);
    }
    if (NSETS > 4) {
      if (s0 + 4 < p.n_slabs) body(std::integral_constant<int, 4 % NSETS>{}, s0 + 4);
      if (s0 + 5 < p.n_slabs) body(std::integral_constant<int, 5 % NSETS>{}, s0 + 5);
      if (s0 + 6 < p.n_slabs) body(std::integral_constant<int, 6 % NSETS>{}, s0 + 6);
      if (s0 + 7 < p.n_slabs) body(std::integral_constant<int, 7 % NSETS>{}, s0 + 7);
    }
  }

  // drain: the exchange of the last slabs cannot hide behind further streaming
  wait_vmcnt<0>();
  for (int s = max(0, p.n_slabs - NSETS); s < p.n_slabs; ++s) {
    st.request_lse(s);
    const float lse = st.take_lse(s);
    switch (s % NSETS) {
      case 0: st.template finish_set<0>(lse); break;
      case 1: st.template finish_set<1 % NSETS>(lse); break;
      case 2: st.template finish_set<2 % NSETS>(lse); break;
      case 3: st.template finish_set<3 % NSETS>(lse); break;
      case 4: st.template finish_set<4 % NSETS>(lse); break;
      case 5: st.template finish_set<5 % NSETS>(lse); break;
      case 6: st.template finish_set<6 % NSETS>(lse); break;
      default: st.template finish_set<7 % NSETS>(lse); break;
    }
    close_layer(s);
  }
  while (st.duty_open() && st.may_poll()) {  // nobody gets its log-sum-exps before this duty is done
    st.service_reduce();
    __builtin_amdgcn_s_sleep(4);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's LDS atomics have been performed
  // A wait of any wave of this workgroup gave up: its tokens' scores may rest on statistics that
  // never arrived.  They are written as NaN so that no consumer can take them for scores.  (The
  // waves tell each other through a word of the control block: a library workgroup reduction
  // would bring static LDS of its own, which the LDS budget of this kernel has no room for.)
  if (st.expired && st.lane == 0) lds_or(st.cnt_lds + 52, 1u);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();
  const bool gave_up = __builtin_amdgcn_readfirstlane(lds_peek(st.cnt_lds + 52)) != 0;

  int nv = p.n_valid ? p.n_valid[0] : p.N;
  nv = max(1, min(nv, p.N));
  if (MEAN) {
#pragma unroll
    for (int j = 0; j < (MEAN ? 8 : 1); ++j) {
      const int cell = threadIdx.x + kThreads * j;
      if (cell < cells) *cell_at(cell) = tot[j] + fast_exp2(*cell_at(cell));  // + the last layer
    }
    __syncthreads();
  }
  for (int key = threadIdx.x; key < p.KPW; key += kThreads) {
    const int token = st.key_of_local(key);
    if (token >= p.M) continue;
    float sum = 0.f;
    for (int n = 0; n < nv; ++n) {
      const float v = st.smax[n * (p.KPW + kSmaxPad) + smax_cell(key)];
      sum += MEAN ? v : fast_exp2(v);
    }
    const float denom = MEAN ? (float)nv * (float)p.L : (float)nv;
    p.scores[token] = gave_up ? __uint_as_float(0x7fc00000u) : sum / denom;
  }
  if (gave_up && threadIdx.x == 0) atomicOr(p.status, 1u);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
struct StreamPlan {
  bool ok;
  int nwg, KPW, S, TPW, wpr, slabs_per_layer, n_slabs;
  size_t rows, partial_bytes, lse_bytes, smem_bytes;
};

// compute units of the current device; cached per device (0 = not asked yet)
static int device_cu_count() {
  static std::atomic<int> cached[kMaxDevices];
  const int slot = current_device();
  const int have = cached[slot].load(std::memory_order_relaxed);
  if (have > 0) return have;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return kMaxWG;  // no device visible (sizing queries on a CPU-only host): assume the full chip
  }
  cached[slot].store(cus, std::memory_order_relaxed);
  return cus;
}

static std::atomic<int> g_spin_budget{kDefaultSpinBudget};

#ifndef SP_STREAM_TPW_PREF
#define SP_STREAM_TPW_PREF 2  // preferred key tiles per wave per slab (smaller = longer exchange window)
#endif

static StreamPlan make_plan(const sp_score_args* a, int nwg) {
  StreamPlan pl{};
  pl.ok = false;
  const int G = a->H / a->H_kv;
  if (a->B != 1 || a->H_kv != 8 || a->T < 1) return pl;
  if (a->rope_theta != 0.f) return pl;  // un-rotated caches take the general kernels
  if (a->k_dtype == SP_K_FP8_E4M3 && (a->d != 128 || a->d_block_table)) return pl;  // 8-bit caches: head dim 128, contiguous
  if (G != 1 && G != 2 && G != 4 && G != 8) return pl;
  if (G * a->N > 32 || a->N > 8) return pl;
  nwg = std::min(nwg, kMaxWG);
  const int kb = (int)((a->T + (int64_t)nwg * 32 - 1) / ((int64_t)nwg * 32));
  int kb2 = 1;
  while (kb2 < kb) kb2 <<= 1;
  if (kb2 > 16) return pl;  // beyond 16 key blocks per workgroup the slabs no longer fit
  // S * kb2 = 8 * TPW with S in {1,2,4,8} and TPW in {1,2}: start from the preferred TPW and
  // move it into range
  int tpw = SP_STREAM_TPW_PREF;
  while (tpw < 2 && 8 * tpw < kb2) tpw <<= 1;
  while (tpw > 1 && 8 * tpw / kb2 > 8) tpw >>= 1;
  const int S = 8 * tpw / kb2;
  if (S < 1 || S > 8 || S * kb2 != 8 * tpw) return pl;
  pl.nwg = nwg;
  pl.KPW = kb2 * 32;
  pl.TPW = tpw;
  pl.S = S;
  pl.wpr = kWaves / pl.S;
  pl.slabs_per_layer = a->H_kv / pl.S;
  pl.n_slabs = a->L * pl.slabs_per_layer;
  pl.rows = (size_t)a->L * a->H_kv * 32;
  if (pl.S * 8 > nwg) return pl;  // reducer rotation: at most one quad of rows per workgroup and slab
  pl.partial_bytes = align_up(pl.rows * nwg * sizeof(uint32_t), 256);
  pl.lse_bytes = align_up(pl.rows * sizeof(uint32_t), 256);
  pl.smem_bytes = (size_t)kWaves * 2 * 32 * a->d * 2 + (size_t)(8 / tpw) * kDepSlotBytes + kCtlBytes + kWaves * 256 +
                  kStageBytes + (size_t)a->N * (pl.KPW + kSmaxPad) * sizeof(float);
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

// byte offset of the status word inside the workspace, or 0 if the shape does not use this kernel
size_t stream_status_offset(const sp_score_args* a) {
  const StreamPlan pl = make_plan(a, device_cu_count());
  return pl.ok ? pl.partial_bytes + pl.lse_bytes : 0;
}

template <int D, int TPW, bool MEAN, bool PAGED = false, bool FP8 = false>
static sp_status launch_stream(const StreamDev& dev, const StreamPlan& pl, hipStream_t stream) {
  auto kernel = stream_score_kernel<D, TPW, MEAN, PAGED, FP8>;
  // once per kernel and device, under a lock: allow the large dynamic LDS size and make sure a
  // workgroup fits on a compute unit (the grid is one workgroup per unit; the plan has already
  // bounded the LDS size by what a unit has)
  static std::mutex mu;
  static bool prepared[kMaxDevices] = {};
  {
    std::lock_guard<std::mutex> lock(mu);
    const int slot = current_device();
    if (!prepared[slot]) {
      hipFuncAttributes fa;
      if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kernel)) != hipSuccess) return SP_ELAUNCH;
      const int max_dynamic = 160 * 1024 - (int)fa.sharedSizeBytes;  // a unit's LDS less the kernel's static part
      if ((int)pl.smem_bytes > max_dynamic) return SP_ELAUNCH;
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              max_dynamic) != hipSuccess)
        return SP_ELAUNCH;
      int per_cu = 0;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kernel), kThreads,
                                                       pl.smem_bytes) != hipSuccess || per_cu < 1)
        return SP_ELAUNCH;
      prepared[slot] = true;
    }
  }
  hipLaunchKernelGGL(kernel, dim3(pl.nwg), dim3(kThreads), pl.smem_bytes, stream, dev);
  return launch_status();
}

sp_status stream_score(const sp_score_args* a, hipStream_t stream) {
  const StreamPlan pl = make_plan(a, device_cu_count());
  if (!pl.ok) return SP_EUNSUPPORTED;
  StreamDev dev;
  dev.M = (int)a->T; dev.L = a->L; dev.N = a->N; dev.H = a->H; dev.G = a->H / a->H_kv; dev.S = pl.S;
  dev.lgG = dev.G == 1 ? 0 : dev.G == 2 ? 1 : dev.G == 4 ? 2 : 3;
  dev.lgS = pl.S == 1 ? 0 : pl.S == 2 ? 1 : pl.S == 4 ? 2 : 3;
  dev.lgSPL = pl.slabs_per_layer == 1 ? 0 : pl.slabs_per_layer == 2 ? 1 : pl.slabs_per_layer == 4 ? 2 : 3;
  dev.slabs_per_layer = pl.slabs_per_layer; dev.n_slabs = pl.n_slabs; dev.KPW = pl.KPW; dev.nwg = pl.nwg;
  dev.layer_step = 1;
  dev.lgKPW = 0;
  while ((1 << dev.lgKPW) < pl.KPW) ++dev.lgKPW;
  dev.own_step = pl.KPW; dev.tile_step = 32;  // every workgroup one run of KPW keys (and all KV heads of them)
  dev.wpr = pl.wpr; dev.layer_reduce = a->layer_reduce;
  dev.spin_budget = g_spin_budget.load(std::memory_order_relaxed);
  dev.c = a->scale * 1.4426950408889634f;
  dev.ts = a->k_token_stride; dev.hs = a->k_head_stride;
  dev.q = static_cast<const uint16_t*>(a->d_q);
  dev.n_valid = a->d_n_valid;
  char* ws = static_cast<char*>(a->d_workspace);
  dev.partial = reinterpret_cast<uint32_t*>(ws);
  dev.lse2 = reinterpret_cast<uint32_t*>(ws + pl.partial_bytes);
  dev.status = reinterpret_cast<uint32_t*>(ws + pl.partial_bytes + pl.lse_bytes);
  dev.scores = a->d_scores; dev.lse_out = a->d_lse;
  dev.block_table = a->d_block_table;
  dev.lg_page = 0;
  while (a->d_block_table && (1 << dev.lg_page) < a->page_size) ++dev.lg_page;
  dev.page_stride = a->k_page_stride;
  dev.k_scale = a->d_k_scale;
  dev.H_kv = a->H_kv;
  for (int l = 0; l < SP_MAX_LAYERS; ++l)
    dev.k[l] = l < a->L ? static_cast<const uint16_t*>(a->k_layers[l]) : nullptr;

  const size_t n_vec = (pl.partial_bytes + pl.lse_bytes) / 16;
  const int fill_blocks = (int)std::min<size_t>((n_vec + 255) / 256, 2048);
  hipLaunchKernelGGL(fill_empty_kernel, dim3(fill_blocks), dim3(256), 0, stream, reinterpret_cast<uint4*>(ws),
                     n_vec, dev.status);
  if (hipGetLastError() != hipSuccess) return SP_ELAUNCH;
  const bool mean = a->layer_reduce == SP_LAYER_MEAN;
  if (a->k_dtype == SP_K_FP8_E4M3) {  // (head dim 128, contiguous: make_plan takes nothing else)
    if (pl.TPW == 1) return mean ? launch_stream<128, 1, true, false, true>(dev, pl, stream) : launch_stream<128, 1, false, false, true>(dev, pl, stream);
    return mean ? launch_stream<128, 2, true, false, true>(dev, pl, stream) : launch_stream<128, 2, false, false, true>(dev, pl, stream);
  }
  if (a->d_block_table) {
    if (a->d == 128) {
      if (pl.TPW == 1) return mean ? launch_stream<128, 1, true, true>(dev, pl, stream) : launch_stream<128, 1, false, true>(dev, pl, stream);
      return mean ? launch_stream<128, 2, true, true>(dev, pl, stream) : launch_stream<128, 2, false, true>(dev, pl, stream);
    }
    if (pl.TPW == 1) return mean ? launch_stream<64, 1, true, true>(dev, pl, stream) : launch_stream<64, 1, false, true>(dev, pl, stream);
    return mean ? launch_stream<64, 2, true, true>(dev, pl, stream) : launch_stream<64, 2, false, true>(dev, pl, stream);
  }
  if (a->d == 128) {
    if (pl.TPW == 1) return mean ? launch_stream<128, 1, true>(dev, pl, stream) : launch_stream<128, 1, false>(dev, pl, stream);
    return mean ? launch_stream<128, 2, true>(dev, pl, stream) : launch_stream<128, 2, false>(dev, pl, stream);
  }
  if (pl.TPW == 1) return mean ? launch_stream<64, 1, true>(dev, pl, stream) : launch_stream<64, 1, false>(dev, pl, stream);
  return mean ? launch_stream<64, 2, true>(dev, pl, stream) : launch_stream<64, 2, false>(dev, pl, stream);
}

}  // namespace sp

extern "C" int32_t sp_set_wait_budget(int32_t polls) {
  if (polls < 0) return sp::g_spin_budget.load(std::memory_order_relaxed);
  return sp::g_spin_budget.exchange(polls, std::memory_order_relaxed);
}
