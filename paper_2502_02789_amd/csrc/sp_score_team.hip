// Single-pass scorer for one prompt of up to 32K keys: teams of workgroups, one team per group
// of KV heads (SP_LAYER_MAX, Sec. 3.2.2 of arXiv 2502.02789 as printed: maximum over heads and
// layers, mean over queries) or per group of layers (SP_LAYER_MEAN: maximum over heads, mean over
// layers and queries).
//
// Same arithmetic and the same per-wave streaming as sp_score_stream.hip (see sp_stream_core.h):
// every K-cache byte is read from HBM once, the raw logits of the last NSETS slabs wait in
// registers for their rows' log-sum-exps.  What differs is who shares a softmax row.  There, every
// workgroup owns 1/256 of the keys for ALL KV heads, so each row's statistics come from 256
// workgroups and travel in two hops.  Here the grid is cut into TC teams; team t owns the KV heads
// [t * H_kv/TC, (t+1) * H_kv/TC) and walks over (layer, own KV head) slabs; inside a team the
// prompt's 32-key tiles are dealt out to the workgroups in turn (KPW keys each) and all eight
// waves of a workgroup work on the SAME KV head, TPW tiles each.  A softmax row therefore has only
// P = 256 / TC partners (64 for a 32K prompt), and because the maximum over heads and layers
// commutes with everything, teams never talk to each other until the very end.  (With the mean
// over layers team t owns the layers t, t + TC, ... and all their KV heads instead: a layer's
// maximum over heads is then complete inside a workgroup, which adds the layer's maxima to a
// running sum at each end of a layer, and the teams' sums add up at the very end.)
//
//   * per slab a workgroup publishes ONE 128-byte line: the base-2 log-sum-exp of its keys for
//     the slab's 32 rows, written by the wave that completes the slab (the waves' own values are
//     merged through LDS);
//   * the lines of a slab's P partners are contiguous, so what a workgroup needs to turn its own
//     stored logits into probabilities is one dense P * 128-byte read.  Every workgroup does that
//     read for itself (one hop; nobody reduces on behalf of others): a wave that passes by at the
//     end of a slab sends the read on its way into an LDS landing zone marked "pending"; a later
//     passer-by looks at the zone, re-requests the lines that were still empty, or folds the P
//     values per row into the row's log-sum-exp and leaves the 32 results in LDS for all waves;
//   * no wave ever waits through vmcnt for any of this; a wave waits (bounded, by polling LDS) only
//     if the log-sum-exps of slab s - NSETS are not there when it is about to reuse the registers;
//   * at the end each workgroup writes its [query][key] maxima of log2-probabilities to a per-team
//     array and counts itself in; of the TC workgroups that own the same keys the one that arrives
//     last takes the maximum over teams, exponentiates and averages over the valid queries.
//
// Publications per workgroup and slab: one full line instead of 32 scattered 16-byte stores;
// coherent reads: P lines once (plus re-reads of late lines) instead of a two-hop chain.  Words
// are "empty" (all ones) until written, written and read with agent-scope coherence.  The
// exchange lines exist twice: a call works in one copy and, line by line as it publishes, puts
// "empty" back into the other, so the next call finds its copy clean (the epoch word in the
// workspace says which is which; counters and status words are handed on the same way).  A small
// kernel sets all of that up in front of a call that cannot rely on the previous one
// (no SP_SCORE_WORKSPACE_KEPT).  As in the other single-pass
// kernel all workgroups must be resident together (the caller's SP_SCORE_EXCLUSIVE_DEVICE
// promise), every wait is bounded, and an expired wait turns the call's scores into NaN.
#include <atomic>
#include <mutex>

#include "sp_stream_core.h"

namespace sp {

constexpr int kTeamCtlBytes = 128;
constexpr int kTeamMaxPartners = 64;                       // landing zone: one line per partner
constexpr int kTeamLandBytes = kTeamMaxPartners * 128;
constexpr int kTeamDepBytes = 8 * 32 * 4;                  // one slab's deposits: 32 rows x 8 waves

struct TeamDev : StreamShape {
  int TC, lgTC;       // teams; team = workgroup % TC, index in team = workgroup / TC
  int by_layers;      // 0: a team owns KV heads (SP_LAYER_MAX); 1: it owns every TC-th layer (SP_LAYER_MEAN)
  int P;              // workgroups per team (a multiple of 32, at most kTeamMaxPartners)
  int M_pad;          // P * KPW
  uint32_t* partial;  // two copies of [team][slab][partner][32]: base-2 log-sum-exp of the partner's
                      // keys, per row.  A call works in copy (epoch & 1) and leaves the other one
                      // "empty" for the call after it.
  size_t partial_words;  // 32-bit words of one copy
  float* part;        // [team][N][M_pad]: the team's max over its heads and all layers of log2 p
  uint32_t* arrived;  // [P]: how many of the TC workgroups that own key slice j are done (+ 65536 per
                      // workgroup one of whose waits expired); zero at the start of the call
  uint32_t* status;   // [epoch & 1] != 0: a bounded wait of this call ran out (results invalid); [2]: epoch,
                      // the number of calls this workspace has served since it was last filled; [3]: key
                      // slices finished (zero at the start of the call)
  const int32_t* n_valid;
  float* scores;
  float* lse_out;
};

template <int D, int TPW, bool PAGED, bool FP8>
struct Teamer : StreamCore<D, TPW, PAGED, FP8> {
  using Core = StreamCore<D, TPW, PAGED, FP8>;
  using Core::NSETS; using Core::RING_BYTES;
  using Core::wave; using Core::lane; using Core::half; using Core::col;
  using Core::issued; using Core::run_m; using Core::run_s;
  using Core::may_poll; using Core::note_issued; using Core::fold; using Core::lds_ptr; using Core::layer_of;
  using Core::kvh_of;

  const TeamDev& p;
  int team, pidx;
  uint32_t epoch;          // of this call
  uint32_t* partial_cur;   // the exchange lines of this call
  uint32_t* partial_nxt;   // ... and of the next one
  uint32_t dep_lds;   // LDS: [NSETS][32 rows][8 waves] each wave's base-2 log-sum-exp of the row over its keys
  uint32_t ctl_lds;   // LDS control block: words 0..7 arrival counters per set; 8 last slab whose row
                      // log-sum-exps are in LDS (-1: none); 9 last slab this workgroup has published
                      // (-1: none); 10 the sampler's lock; 11 "a sample of slab [8]+1 has been requested";
                      // 12 "a wait of some wave expired"; 13 arrival count of this key slice (kernel end)
  uint32_t lse_lds;   // LDS: [NSETS][32] finished row log-sum-exps (slot = slab % NSETS)
  uint32_t land_lds;  // LDS: landing zone of a sample, [P][32]

  static constexpr int kFixedBytes = RING_BYTES + NSETS * kTeamDepBytes + kTeamCtlBytes + NSETS * 128 + kTeamLandBytes;
  static size_t smem_bytes(int n_queries, int kpw) {
    return (size_t)kFixedBytes + (size_t)n_queries * (kpw + kSmaxPad) * sizeof(float);
  }

  __device__ __forceinline__ Teamer(const TeamDev& p_, unsigned char* smem)
      : Core(p_, (uint32_t)reinterpret_cast<uintptr_t>(smem), reinterpret_cast<float*>(smem + kFixedBytes),
             (int)(blockIdx.x >> p_.lgTC), p_.by_layers ? 0 : (int)(blockIdx.x & (p_.TC - 1)) * p_.slabs_per_layer,
             p_.by_layers ? (int)(blockIdx.x & (p_.TC - 1)) : 0),
        p(p_) {
    team = blockIdx.x & (p.TC - 1);
    pidx = blockIdx.x >> p.lgTC;
    epoch = __builtin_amdgcn_readfirstlane(p.status[2]);  // (changed only after every workgroup is past this point)
    partial_cur = p.partial + (size_t)(epoch & 1u) * p.partial_words;
    partial_nxt = p.partial + (size_t)(~epoch & 1u) * p.partial_words;
    const uint32_t smem_lds = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    dep_lds = smem_lds + RING_BYTES;
    ctl_lds = dep_lds + NSETS * kTeamDepBytes;
    lse_lds = ctl_lds + kTeamCtlBytes;
    land_lds = lse_lds + NSETS * 128;
  }

  // log2(2^a + 2^b + ...) of eight values, -inf if all are
  __device__ __forceinline__ static float lse2_of8(const u32x4& a, const u32x4& b) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = __uint_as_float(a[i]); v[4 + i] = __uint_as_float(b[i]); }
    float m = v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) m = fmaxf(m, v[i]);
    const float ref = (m == -INFINITY) ? 0.f : m;
    float z = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) z += fast_exp2(v[i] - ref);
    return (m == -INFINITY) ? -INFINITY : m + __builtin_amdgcn_logf(z);  // v_log_f32 is log2
  }

  // This wave is done with the slab's keys: leave the base-2 log-sum-exp of each of its 32 rows
  // over its own keys in LDS and count the arrival; the wave that arrives last merges the eight
  // waves' values and publishes the workgroup's line (LDS operations of a wave are performed in
  // order, so whoever sees the count complete also sees every deposit).
  template <int SET>
  __device__ __forceinline__ void deposit(int slab) {
    float m = run_m, s = run_s;
    fold(m, s, __shfl_xor(run_m, 32, kWave), __shfl_xor(run_s, 32, kWave));
    const float v = (m == -INFINITY) ? -INFINITY : fmaf(m, p.c, __builtin_amdgcn_logf(s));
    uint32_t dst = dep_lds + col * 32 + wave * 4;
    asm volatile("" : "+v"(dst));  // one address plus an immediate per set, not NSETS addresses kept alive
    if (half == 0) lds_poke32_at<SET * kTeamDepBytes>(dst, __float_as_uint(v));
    uint32_t old = 0;
    if (lane == 0) old = lds_add_rtn(ctl_lds + SET * 4, 1);
    old = __builtin_amdgcn_readfirstlane(old);
    if ((old & 7) == 7) publish(slab, dep_lds + SET * kTeamDepBytes);
  }

  __device__ __forceinline__ void publish(int slab, uint32_t dep) {
    int ln = lane;
    asm volatile("" : "+v"(ln));  // address arithmetic of this once-per-slab path stays here instead of being hoisted
    if (ln < 32) {
      const u32x4 a = lds_peek128(dep + ln * 32), b = lds_peek128(dep + ln * 32 + 16);
      const float out = lse2_of8(a, b);  // (-inf -- no key of the prompt in this workgroup -- is a value, not "empty")
      const int64_t at = ((int64_t)(team * p.n_slabs + slab) * p.P + pidx) * 32 + ln;
      store32_agent(partial_cur + at, __float_as_uint(out));
      // the same line of the other copy: "empty" again for the call after this one (nobody reads
      // that copy during this call, and the end of the kernel makes the store visible)
      asm volatile("global_store_dword %0, %1, off" : : "v"(partial_nxt + at), "v"(kEmpty32) : "memory");
    }
    note_issued(2);
    if (ln == 0) lds_poke32(ctl_lds + 36, (uint32_t)slab);
  }

  // By whichever wave comes by: bring the row log-sum-exps of the next slab that lacks them a step
  // forward (never beyond slab `limit`, and never before this workgroup itself has published
  // that slab: its partners are then about as far).  A landed sample is folded and the next
  // slab's sample is sent on its way in the same visit: the waves of a workgroup pass by in a
  // cluster, once per slab, and those that find the lock taken do nothing.  Never waits.
  __device__ __forceinline__ void service(int limit) {
    const uint64_t st = lds_peek64(ctl_lds + 32);
    const int r0 = (int)__builtin_amdgcn_readfirstlane((uint32_t)st) + 1;
    const int pub = (int)__builtin_amdgcn_readfirstlane((uint32_t)(st >> 32));
    if (r0 > limit || r0 > pub) return;
    // one wave at a time: test-and-set
    uint32_t held = 1;
    if (lane == 0) held = lds_or_rtn(ctl_lds + 40, 1);
    if (__builtin_amdgcn_readfirstlane(held) != 0) return;
#pragma unroll 1
    for (int visit = 0; visit < 2; ++visit) {
      // (another wave may have finished slab r0 between the two looks)
      const int r = (int)__builtin_amdgcn_readfirstlane(lds_peek(ctl_lds + 32)) + 1;
      if (r > limit || r > pub) break;
      if (!sample_step(r)) break;  // not folded yet: nothing more to do now
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lane == 0) lds_poke32(ctl_lds + 40, 0);
  }

  // No sample of slab r out yet: mark the landing zone "pending" and request the P partner lines
  // (P / 8 wave-wide 16-byte direct-to-LDS loads).  Sample out: look at the zone (LDS reads only);
  // words still pending -> come back later; pieces still empty -> request those pieces again;
  // everything there -> fold the P values of each row and leave the 32 log-sum-exps in LDS
  // (returns true: slab r is done).
  __device__ __forceinline__ bool sample_step(int r) {
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const bool sampled = __builtin_amdgcn_readfirstlane(lds_peek(ctl_lds + 44)) != 0;
    const int groups = p.P >> 3;
    const unsigned char* src = reinterpret_cast<const unsigned char*>(partial_cur + (int64_t)(team * p.n_slabs + r) * p.P * 32) + ln * 16;
    const u32x4 fill = {kPending32, kPending32, kPending32, kPending32};
    if (!sampled) {
#pragma unroll 1  // rare path: keep its register appetite small
      for (int i = 0; i < groups; ++i) lds_poke128(land_lds + i * 1024 + ln * 16, fill);
      if (ln == 0) lds_poke32(ctl_lds + 44, 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the pattern is in place before any answer can land
#pragma unroll
      for (int i = 0; i < kTeamMaxPartners / 8; ++i)
        if (i < groups) __builtin_amdgcn_global_load_lds(src + i * 1024, lds_ptr(land_lds + i * 1024), 16, 0, /*sc1*/ 16);
      note_issued(groups);
      return false;
    }
    // Look at the zone.  Lane ln holds, of load i, the 16 bytes of partner i * 8 + ln / 8 that carry
    // rows 4 * (ln % 8) .. + 3: what it needs to check, and exactly one partner's share of a row
    // quad's fold.  Pass 1: pending / empty words and the rows' maxima; pass 2: the sums.
    bool pending = false;
    uint32_t miss = 0;  // bit i: this lane's 16 bytes of load i hold an empty word
    const uint32_t zone = land_lds + ln * 16;
    float m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int i0 = 0; i0 < kTeamMaxPartners / 8; i0 += 4) {
      if (i0 < groups) {  // (groups is a multiple of four)
        const u32x4x4 w = lds_peek128x4<1024>(zone + i0 * 1024);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const u32x4 x = w.v[j];
          pending |= x.x == kPending32 || x.y == kPending32 || x.z == kPending32 || x.w == kPending32;
          if (x.x == kEmpty32 || x.y == kEmpty32 || x.z == kEmpty32 || x.w == kEmpty32) miss |= 1u << (i0 + j);
#pragma unroll
          for (int c = 0; c < 4; ++c) m[c] = fmaxf(m[c], __uint_as_float(x[c]));  // (the NaN patterns never win a max)
        }
      }
    }
    if (__any(pending)) return false;
    if (__any(miss != 0)) {
#pragma unroll
      for (int i = 0; i < kTeamMaxPartners / 8; ++i)
        if (i < groups && ((miss >> i) & 1)) lds_poke128(land_lds + i * 1024 + ln * 16, fill);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < kTeamMaxPartners / 8; ++i) {
        if (i < groups && __any((miss >> i) & 1)) {  // wave-uniform: the instruction is issued, for the lanes that miss
          if ((miss >> i) & 1)
            __builtin_amdgcn_global_load_lds(src + i * 1024, lds_ptr(land_lds + i * 1024), 16, 0, /*sc1*/ 16);
          note_issued(1);
        }
      }
      return false;
    }
    // all P lines are here: finish the maxima across the eight lanes that share a row quad
    // (lanes ln, ln ^ 8, ln ^ 16, ln ^ 32), then the sums the same way
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      m[c] = fmaxf(m[c], __shfl_xor(m[c], 8, kWave));
      m[c] = fmaxf(m[c], __shfl_xor(m[c], 16, kWave));
      m[c] = fmaxf(m[c], __shfl_xor(m[c], 32, kWave));  // finite: the prompt is not empty
    }
    float z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i0 = 0; i0 < kTeamMaxPartners / 8; i0 += 4) {
      if (i0 < groups) {
        const u32x4x4 w = lds_peek128x4<1024>(zone + i0 * 1024);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int c = 0; c < 4; ++c) z[c] += fast_exp2(__uint_as_float(w.v[j][c]) - m[c]);
      }
    }
    u32x4 out;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      z[c] += __shfl_xor(z[c], 8, kWave);
      z[c] += __shfl_xor(z[c], 16, kWave);
      z[c] += __shfl_xor(z[c], 32, kWave);
      out[c] = __float_as_uint(m[c] + __builtin_amdgcn_logf(z[c]));
    }
    if (ln < 8) lds_poke128(lse_lds + (r & (NSETS - 1)) * 128 + ln * 16, out);  // rows 4 * ln .. + 3
    if (ln == 0) {
      lds_poke32(ctl_lds + 44, 0);            // no sample out for the next slab
      lds_poke32(ctl_lds + 32, (uint32_t)r);  // after the values: LDS writes of a wave are performed in order
    }
    if (p.lse_out && pidx == 0 && ln < 8) {  // (not counted in `issued`: counting less only waits more)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int row = ln * 4 + c;
        if (row < p.G * p.N)
          p.lse_out[((int64_t)layer_of(r) * p.N + (row >> p.lgG)) * p.H + kvh_of(r) * p.G + (row & (p.G - 1))] =
              __uint_as_float(out[c]) * 0.6931471805599453f;
      }
    }
    return true;
  }

  // 1 KiB (16 bytes per lane, src = this lane's address) straight into LDS, agent scope.  (The
  // builtin has to sit in a device function: in the body of a kernel template it keeps the host
  // pass from emitting the kernel's launch stub.)
  __device__ __forceinline__ void load_kib_agent(const void* src, uint32_t lds) {
    __builtin_amdgcn_global_load_lds(src, lds_ptr(lds), 16, 0, /*sc1*/ 16);
  }

  // This lane's row log-sum-exp of `slab`.  Normally it is there; if not, keep the sampling going
  // until it is (bounded).
  __device__ __forceinline__ float take_lse(int slab) {
    if ((int)__builtin_amdgcn_readfirstlane(lds_peek(ctl_lds + 32)) < slab) {
      // A waiting wave must cost the working ones as little as possible: lowest issue priority (it
      // shares its SIMD with a wave that streams) and long naps between looks.  Measured on the
      // 32K-token workload (whole call, steady state): naps of 8 x 64 cycles 409 us, 20: 400, 40: 397,
      // 80: 394, 127: 394.
      __builtin_amdgcn_s_setprio(0);
      while ((int)__builtin_amdgcn_readfirstlane(lds_peek(ctl_lds + 32)) < slab && may_poll()) {
        service(slab);
        __builtin_amdgcn_s_sleep(80);
      }
      if (((slab + NSETS) ^ (wave >> 2)) & 1) __builtin_amdgcn_s_setprio(2);  // back to the priority of the slab in progress
    }
    int c = col;
    asm volatile("" : "+v"(c));
    return __uint_as_float(lds_peek(lse_lds + (slab & (NSETS - 1)) * 128 + c * 4));
  }
};

template <int D, int TPW, bool PAGED, bool MEAN, bool FP8>
__global__ __launch_bounds__(kThreads) void team_score_kernel(const TeamDev p) {
  extern __shared__ __align__(1024) unsigned char smem[];
  using Tm = Teamer<D, TPW, PAGED, FP8>;
  constexpr int NSETS = Tm::NSETS, TPS = Tm::TPS;
  Tm tm(p, smem);
  const int cells = p.N * p.KPW;  // (query, key) cells of this workgroup
  auto cell_at = [&](int c) __attribute__((always_inline)) { return tm.smax + c + kSmaxPad * (c >> p.lgKPW); };  // skips the row padding
  // SP_LAYER_MEAN: the team owns whole layers, so a layer's maximum over heads is complete inside
  // the workgroup; the sum over the team's layers of these maxima (as probabilities) is kept here,
  // cell = threadIdx + 512 * j.  Slab `done` was just finished by this wave: if it closes a layer,
  // the layer's maxima join the sums and the cells start over; after the last slab the sums go
  // back into the cells.  (The cells of a wave's keys are touched by no other wave, so this could
  // be done wave by wave without the barriers; measured, that is 8 us slower per call on the
  // 32K-token shape, 416 against 408 us.)
  float tot[MEAN ? 8 : 1];
#pragma unroll
  for (int j = 0; j < (MEAN ? 8 : 1); ++j) tot[j] = 0.f;
  auto close_layer = [&](int done) __attribute__((always_inline)) {
    if (MEAN && ((done + 1) & (p.slabs_per_layer - 1)) == 0) {
      const bool last = done + 1 == p.n_slabs;
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's LDS atomics have been performed
      __syncthreads();
      int t = threadIdx.x;
      asm volatile("" : "+v"(t));  // the cells' addresses are formed here, once per layer, not kept in registers all along
#pragma unroll
      for (int j = 0; j < (MEAN ? 8 : 1); ++j) {
        const int cell = t + kThreads * j;
        if (cell < cells) {
          const uint32_t addr = Tm::lds_addr_of(cell_at(cell));
          tot[j] += fast_exp2(__uint_as_float(lds_peek(addr)));
          lds_poke32(addr, last ? __float_as_uint(tot[j]) : 0xff800000u);  // the sum at the end, else -inf
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __syncthreads();
    }
  };
  for (int i = threadIdx.x; i < cells; i += kThreads) *cell_at(i) = -INFINITY;
  if (threadIdx.x < 16)  // arrival counters, lock and flag: 0; "last slab done / published": none
    *reinterpret_cast<uint32_t*>(smem + Tm::RING_BYTES + NSETS * kTeamDepBytes + threadIdx.x * 4) =
        (threadIdx.x == 8 || threadIdx.x == 9) ? ~0u : 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0) p.status[~tm.epoch & 1u] = 0;  // the next call's status word
  __syncthreads();

  tm.template issue_stream<0>(0, 0);
  tm.template issue_stream<1>(0, 1);
  // When a slab's query rows move from their ring slot into registers (the slot then takes the stream tile
  // two further on): at the slab's start, or, EARLY_Q, already behind the last product of the slab before,
  // so that the next key tile is requested before that slab's statistics, publication and sampling rather
  // than after them.  Measured on the 32K-token prompt: mean over layers 394 -> 381 us (its layer ends hold
  // the waves up, a deeper stream bridges that), maximum over layers 358 / 359 us, 16K keys 201 / 204 us.
  constexpr bool EARLY_Q = MEAN;
  if (EARLY_Q) {
    tm.wait_tile(0);
    tm.read_queries(0);
    tm.template issue_stream<2>(0, 0);
  }

  // One slab.  Stream tile x of the slab sits in ring slot (SET*TPS + x) & 1 (NSETS is even, so
  // the slab's parity is SET's).
  auto body = [&](auto set_tag, int slab) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value;
    constexpr int SLOT0 = (SET * TPS) & 1;
    constexpr int NEXT_SLOT0 = ((SET + 1) * TPS) & 1;  // where the next slab's query tile lands
    // The two waves that share a SIMD take turns at being the one the instruction arbiter
    // prefers; left alone it favours the older wave throughout, and the slab is only published
    // when the slowest wave is done with it.
    if ((slab ^ (tm.wave >> 2)) & 1) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(0);
    tm.slab_scale(slab);
    if (!EARLY_Q) {
      tm.wait_tile(SLOT0);
      tm.read_queries(SLOT0);
      tm.template issue_stream<2>(slab, SLOT0);
    }
    if (slab >= NSETS) {  // set SET still holds slab - NSETS
      tm.template finish_set<SET>(tm.take_lse(slab - NSETS));
      close_layer(slab - NSETS);
    }
    tm.run_m = -INFINITY;
    tm.run_s = 0.f;
#pragma unroll
    for (int kb = 0; kb < TPW; ++kb) {
      const int slot = (SLOT0 + 1 + kb) & 1;
      tm.wait_tile(slot);
      tm.template mfma_tile<SET>(kb, slot);
      switch (kb) {  // a compile-time constant after unrolling
        case 0: tm.template issue_stream<3>(slab, slot); break;
        case 1: tm.template issue_stream<4>(slab, slot); break;
        case 2: tm.template issue_stream<5>(slab, slot); break;
        default: tm.template issue_stream<6>(slab, slot); break;
      }
      if (EARLY_Q && kb == TPW - 1) {  // the slab's last product is under way and the query registers are free
        tm.wait_tile(NEXT_SLOT0);
        tm.read_queries(NEXT_SLOT0);
        tm.template issue_stream<TPS + 2>(slab, NEXT_SLOT0);
      }
      tm.template stats_tile<SET>(kb);
      // between the key tiles too: with one visit per slab a sampler that has fallen behind
      // (a sample that had to be repeated) could never catch up again
      if (kb + 1 < TPW) tm.service(slab - 2);
    }
    tm.template deposit<SET>(slab);
    // A step towards the log-sum-exps of an earlier slab, here, where the fewest registers are
    // live.  Two slabs behind: a sample that comes back with lines still empty has to be repeated
    // and costs more than it gains (whole call with the limit at slab: 430 us, slab - 1: 397 us,
    // slab - 2: 389 us; three behind is too late: 418 us).
    tm.service(slab - 2);
  };

  for (int s0 = 0; s0 < p.n_slabs; s0 += NSETS) {
    body(std::integral_constant<int, 0>{}, s0);
    if (s0 + 1 < p.n_slabs) body(std::integral_constant<int, 1>{}, s0 + 1);
    if (s0 + 2 < p.n_slabs) body(std::integral_constant<int, 2>{}, s0 + 2);
    if (s0 + 3 < p.n_slabs) body(std::integral_constant<int, 3>{}, s0 + 3);
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
    const float lse = tm.take_lse(s);
    switch (s % NSETS) {
      case 0: tm.template finish_set<0>(lse); break;
      case 1: tm.template finish_set<1>(lse); break;
      case 2: tm.template finish_set<2>(lse); break;
      case 3: tm.template finish_set<3>(lse); break;
      case 4: tm.template finish_set<4 % NSETS>(lse); break;
      case 5: tm.template finish_set<5 % NSETS>(lse); break;
      case 6: tm.template finish_set<6 % NSETS>(lse); break;
      default: tm.template finish_set<7 % NSETS>(lse); break;
    }
    close_layer(s);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's LDS atomics have been performed
  if (tm.expired && tm.lane == 0) {  // a wait of this wave gave up
    atomicOr(p.status + (tm.epoch & 1u), 1u);
    lds_or(tm.ctl_lds + 48, 1u);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();  // every wave's maxima (and give-up marks) are in LDS

  // The team's maxima for this workgroup's keys go out as [team][query][key].  The TC workgroups
  // that own the same key slice (one per team) count their arrivals; the one that arrives last
  // takes the maximum over the teams -- now the maximum over all heads and layers --,
  // exponentiates and averages over the valid queries (Sec. 3.2.2).  The workgroups sit on
  // different dies: the values are stored with agent scope and are complete before the count,
  // and the last one fetches them with agent-scope loads (straight into the idle tile ring,
  // all at once).
  for (int i = threadIdx.x; i < p.N * p.KPW; i += kThreads) {
    const int n = i >> p.lgKPW, key = i & (p.KPW - 1);  // (keys beyond the prompt carry -inf: never read back)
    store32_agent(p.part + ((int64_t)tm.team * p.N + n) * p.M_pad + (int64_t)tm.pidx * p.KPW + key,
                  __float_as_uint(tm.smax[n * (p.KPW + kSmaxPad) + smax_cell(key)]));
  }
  wait_vmcnt<0>();
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t mine = 1u + (__builtin_amdgcn_readfirstlane(lds_peek(tm.ctl_lds + 48)) != 0 ? 65536u : 0u);
    const uint32_t before = atomicAdd(p.arrived + tm.pidx, mine);
    lds_poke32(tm.ctl_lds + 52, before + mine);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();
  const uint32_t count = __builtin_amdgcn_readfirstlane(lds_peek(tm.ctl_lds + 52));
  if ((int)(count & 65535u) != p.TC) return;  // somebody else will be last
  if (threadIdx.x == 0) {  // leave the workspace as the next call expects it; the last slice of all turns the epoch
    p.arrived[tm.pidx] = 0;
    if (atomicAdd(p.status + 3, 1u) == (uint32_t)p.P - 1u) {
      p.status[3] = 0;
      p.status[2] = tm.epoch + 1u;
    }
  }
  const bool void_result = (count >> 16) != 0;  // a wait expired in one of the TC workgroups: no score of this slice can be trusted
  int nv = p.n_valid ? p.n_valid[0] : p.N;
  nv = max(1, min(nv, p.N));
  // queries in groups whose TC x group x KPW values fit the ring; 1 KiB (256 keys of one team and
  // query) per wave-wide load
  const int per_query = p.TC * p.KPW * 4;                 // bytes
  const int group = min(nv, Tm::RING_BYTES / per_query);  // >= 1: at most 16 KiB per query
  const int chunks_per_row = p.KPW >> 8;                  // KPW is 256 or 512
  float sum[2] = {0.f, 0.f};                              // this thread's keys: threadIdx.x (+ 512)
  const uint32_t ring = (uint32_t)reinterpret_cast<uintptr_t>(smem);
  for (int n0 = 0; n0 < nv; n0 += group) {
    const int gq = min(group, nv - n0);
    const int rows = p.TC * gq;                           // (team, query) rows of KPW values each
    for (int c = tm.wave; c < rows * chunks_per_row; c += kWaves) {
      const int row = c / chunks_per_row, piece = c - row * chunks_per_row;
      const int t = row / gq, n = n0 + row - t * gq;
      const float* src = p.part + ((int64_t)t * p.N + n) * p.M_pad + (int64_t)tm.pidx * p.KPW + piece * 256 + tm.lane * 4;
      tm.load_kib_agent(src, ring + (uint32_t)c * 1024);
    }
    wait_vmcnt<0>();
    __syncthreads();
    for (int j = 0; j < 2; ++j) {
      const int key = threadIdx.x + j * kThreads;
      if (key < p.KPW && tm.key_of_local(key) < p.M) {
        for (int q = 0; q < gq; ++q) {
          if (MEAN) {  // the teams' sums over their layers add up to the sum over all layers
            for (int t = 0; t < p.TC; ++t) sum[j] += __uint_as_float(lds_peek(ring + ((t * gq + q) * p.KPW + key) * 4));
          } else {
            float m = -INFINITY;
            for (int t = 0; t < p.TC; ++t) m = fmaxf(m, __uint_as_float(lds_peek(ring + ((t * gq + q) * p.KPW + key) * 4)));
            sum[j] += fast_exp2(m);
          }
        }
      }
    }
    __syncthreads();
  }
  for (int j = 0; j < 2; ++j) {
    const int key = threadIdx.x + j * kThreads;
    if (key < p.KPW && tm.key_of_local(key) < p.M)
      p.scores[tm.key_of_local(key)] = void_result ? __uint_as_float(0x7fc00000u) : sum[j] / (MEAN ? (float)nv * (float)p.L : (float)nv);
  }
}

// start-of-call state of the exchange area: every line "empty", arrival counts and status word clear
__global__ __launch_bounds__(256) void team_fill_kernel(uint4* __restrict__ dst, size_t n_vec, uint32_t* __restrict__ arrived,
                                                        int n_arrived, uint32_t* __restrict__ status) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
    dst[i] = make_uint4(kEmpty32, kEmpty32, kEmpty32, kEmpty32);
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < n_arrived; i += 256) arrived[i] = 0;
    if (threadIdx.x < 4) status[threadIdx.x] = 0;  // both status words, the epoch, the slice count
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
struct TeamPlan {
  bool ok;
  int TC, P, TPW, KPW, kpt, n_slabs, M_pad;
  size_t partial_bytes, part_bytes, smem_bytes;
};

static int team_device_cu_count() {
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

static TeamPlan make_team_plan(const sp_score_args* a, int cus) {
  TeamPlan pl{};
  pl.ok = false;
  const int G = a->H / a->H_kv;
  if (a->B != 1 || a->T < 1) return pl;
  const bool by_layers = a->layer_reduce == SP_LAYER_MEAN;  // teams own layers instead of KV heads
  // Where both single-pass kernels fit, this one is taken where it was measured to be the faster
  // (16 layers, 8 look-ahead rows; team / all-workgroup kernel, us): head dim 128: 8K keys 90 / 83,
  // 12K 109 / 113, 16K 126 / 135, 32K 218 / 230; head dim 64: 8K 75 / 64, 16K 86 / 84, 32K 163 / 158.
  if (a->d != 128 || a->T <= 8192) return pl;
  if (a->rope_theta != 0.f) return pl;  // un-rotated caches take the general kernels
  if (a->k_dtype == SP_K_FP8_E4M3 && a->d_block_table) return pl;  // 8-bit caches: contiguous only here
  if (G != 1 && G != 2 && G != 4 && G != 8) return pl;
  if (G * a->N > 32) return pl;
  cus = std::min(cus, kMaxWG);
  // the most teams (fewest partners per softmax row) and the fewest key tiles per wave and slab
  // that still cover the prompt
  for (int tc = 8; tc >= 4; tc >>= 1) {
    if (by_layers ? a->L % tc != 0 : a->H_kv % tc != 0) continue;
    const int kpt = by_layers ? a->H_kv : a->H_kv / tc;  // slabs per layer of a team
    if (kpt & (kpt - 1)) continue;  // a power of two
    const int partners = std::min(kTeamMaxPartners, cus / tc) / 32 * 32;  // the sampler reads lines in batches of 32
    if (partners < 32) continue;
    for (int tpw = 1; tpw <= 2; ++tpw) {
      const int kpw = kWaves * tpw * 32;
      if ((int64_t)partners * kpw < a->T) continue;
      const size_t smem = (size_t)kWaves * 2 * 32 * a->d * 2 + (size_t)(8 / tpw) * (kTeamDepBytes + 128) + kTeamCtlBytes +
                          kTeamLandBytes + (size_t)a->N * (kpw + kSmaxPad) * sizeof(float);
      if (smem > 160 * 1024) continue;
      pl.ok = true;
      pl.TC = tc; pl.P = partners; pl.TPW = tpw; pl.KPW = kpw; pl.kpt = kpt;
      pl.n_slabs = (by_layers ? a->L / tc : a->L) * kpt;
      pl.M_pad = partners * kpw;
      pl.partial_bytes = align_up((size_t)tc * pl.n_slabs * partners * 128, 256);
      pl.part_bytes = align_up((size_t)tc * a->N * pl.M_pad * sizeof(float), 256);
      pl.smem_bytes = smem;
      return pl;
    }
  }
  return pl;
}

bool team_supported(const sp_score_args* a) { return make_team_plan(a, team_device_cu_count()).ok; }

size_t team_workspace_bytes(const sp_score_args* a) {
  const TeamPlan pl = make_team_plan(a, kMaxWG);  // sized for the full chip
  if (!pl.ok) return 0;
  return 2 * pl.partial_bytes + pl.part_bytes + 256 + 256;  // + status words and epoch + arrival counts
}

// byte offset of the status word inside the workspace, or 0 if the shape does not use this kernel
size_t team_status_offset(const sp_score_args* a) {
  const TeamPlan pl = make_team_plan(a, team_device_cu_count());
  return pl.ok ? 2 * pl.partial_bytes + pl.part_bytes : 0;
}

// Every variant the dispatch below names, instantiated explicitly: left to implicit instantiation, the
// host side of half of them (the launch stubs) was not emitted.
template __global__ void team_score_kernel<128, 1, false, false, false>(const TeamDev);
template __global__ void team_score_kernel<128, 1, false, true, false>(const TeamDev);
template __global__ void team_score_kernel<128, 1, true, false, false>(const TeamDev);
template __global__ void team_score_kernel<128, 1, true, true, false>(const TeamDev);
template __global__ void team_score_kernel<128, 2, false, false, false>(const TeamDev);
template __global__ void team_score_kernel<128, 2, false, true, false>(const TeamDev);
template __global__ void team_score_kernel<128, 2, true, false, false>(const TeamDev);
template __global__ void team_score_kernel<128, 2, true, true, false>(const TeamDev);
template __global__ void team_score_kernel<128, 1, false, false, true>(const TeamDev);  // 8-bit caches (contiguous only)
template __global__ void team_score_kernel<128, 1, false, true, true>(const TeamDev);
template __global__ void team_score_kernel<128, 2, false, false, true>(const TeamDev);
template __global__ void team_score_kernel<128, 2, false, true, true>(const TeamDev);

template <int D, int TPW, bool PAGED, bool MEAN, bool FP8 = false>
static sp_status launch_team(const TeamDev& dev, const TeamPlan& pl, hipStream_t stream) {
  auto kernel = team_score_kernel<D, TPW, PAGED, MEAN, FP8>;
  // once per kernel and device, under a lock: allow the large dynamic LDS size and make sure the
  // whole grid can be resident at once
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
  hipLaunchKernelGGL(kernel, dim3(pl.TC * pl.P), dim3(kThreads), pl.smem_bytes, stream, dev);
  return launch_status();
}

sp_status team_score(const sp_score_args* a, hipStream_t stream) {
  const TeamPlan pl = make_team_plan(a, team_device_cu_count());
  if (!pl.ok) return SP_EUNSUPPORTED;
  TeamDev dev;
  dev.M = (int)a->T; dev.L = a->L; dev.N = a->N; dev.H = a->H; dev.G = a->H / a->H_kv;
  dev.lgG = dev.G == 1 ? 0 : dev.G == 2 ? 1 : dev.G == 4 ? 2 : 3;
  dev.S = 1; dev.lgS = 0;
  dev.by_layers = a->layer_reduce == SP_LAYER_MEAN ? 1 : 0;
  dev.layer_step = dev.by_layers ? pl.TC : 1;
  dev.slabs_per_layer = pl.kpt;
  dev.lgSPL = 0;
  while ((1 << dev.lgSPL) < pl.kpt) ++dev.lgSPL;
  dev.n_slabs = pl.n_slabs;
  dev.KPW = pl.KPW;
  dev.lgKPW = 0;
  while ((1 << dev.lgKPW) < pl.KPW) ++dev.lgKPW;
  // The 32-key tiles are dealt out to the team's workgroups in turn (tile x of workgroup j is tile
  // x * P + j of the prompt): what the grid reads at any moment is then spread evenly over the
  // layer.  A read-only copy of this kernel's access pattern ran at 6.36 TB/s this way against
  // 6.15 TB/s with one run of KPW keys per workgroup; the kernel itself, which is not bound by that
  // alone, came out the same either way.
  dev.own_step = 32; dev.tile_step = pl.P * 32;
  dev.spin_budget = sp_set_wait_budget(-1);
  dev.c = a->scale * 1.4426950408889634f;
  dev.ts = a->k_token_stride; dev.hs = a->k_head_stride;
  dev.q = static_cast<const uint16_t*>(a->d_q);
  dev.block_table = a->d_block_table;
  dev.lg_page = 0;
  while (a->d_block_table && (1 << dev.lg_page) < a->page_size) ++dev.lg_page;
  dev.page_stride = a->k_page_stride;
  dev.k_scale = a->d_k_scale;
  dev.H_kv = a->H_kv;
  for (int l = 0; l < SP_MAX_LAYERS; ++l)
    dev.k[l] = l < a->L ? static_cast<const uint16_t*>(a->k_layers[l]) : nullptr;
  dev.TC = pl.TC;
  dev.lgTC = pl.TC == 8 ? 3 : 2;
  dev.P = pl.P;
  dev.M_pad = pl.M_pad;
  char* ws = static_cast<char*>(a->d_workspace);
  dev.partial = reinterpret_cast<uint32_t*>(ws);
  dev.partial_words = pl.partial_bytes / 4;
  dev.part = reinterpret_cast<float*>(ws + 2 * pl.partial_bytes);
  dev.status = reinterpret_cast<uint32_t*>(ws + 2 * pl.partial_bytes + pl.part_bytes);
  dev.arrived = reinterpret_cast<uint32_t*>(ws + 2 * pl.partial_bytes + pl.part_bytes + 256);  // kTeamMaxPartners words
  dev.n_valid = a->d_n_valid;
  dev.scores = a->d_scores;
  dev.lse_out = a->d_lse;

  if (!(a->flags & SP_SCORE_WORKSPACE_KEPT)) {
    // epoch 0: the first copy of the exchange lines "empty", counts and status clear.  (A call
    // leaves all of that behind in the state the next call needs, one epoch on.)
    const size_t n_vec = pl.partial_bytes / 16;
    const int fill_blocks = (int)std::min<size_t>((n_vec + 255) / 256, 1024);
    hipLaunchKernelGGL(team_fill_kernel, dim3(fill_blocks), dim3(256), 0, stream, reinterpret_cast<uint4*>(ws), n_vec,
                       dev.arrived, dev.P, dev.status);
    if (hipGetLastError() != hipSuccess) return SP_ELAUNCH;
  }
  sp_status st;
  // (head dim 128 only: make_team_plan takes nothing else)
  const bool paged = a->d_block_table != nullptr, mean = dev.by_layers != 0;
  if (a->k_dtype == SP_K_FP8_E4M3) {
    if (pl.TPW == 1) st = mean ? launch_team<128, 1, false, true, true>(dev, pl, stream) : launch_team<128, 1, false, false, true>(dev, pl, stream);
    else st = mean ? launch_team<128, 2, false, true, true>(dev, pl, stream) : launch_team<128, 2, false, false, true>(dev, pl, stream);
  } else if (pl.TPW == 1) {
    st = paged ? (mean ? launch_team<128, 1, true, true>(dev, pl, stream) : launch_team<128, 1, true, false>(dev, pl, stream))
               : (mean ? launch_team<128, 1, false, true>(dev, pl, stream) : launch_team<128, 1, false, false>(dev, pl, stream));
  } else {
    st = paged ? (mean ? launch_team<128, 2, true, true>(dev, pl, stream) : launch_team<128, 2, true, false>(dev, pl, stream))
               : (mean ? launch_team<128, 2, false, true>(dev, pl, stream) : launch_team<128, 2, false, false>(dev, pl, stream));
  }
  return st;
}

}  // namespace sp
