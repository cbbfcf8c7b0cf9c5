// Internal helpers shared by the HIP translation units of libspecprefill (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "specprefill.h"

namespace sp {

constexpr int kWave = 64;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// finite (neither NaN nor infinite), decided on the bit pattern so that no floating-point
// compile option can fold the test away
inline bool finite_f32(float x) {
  uint32_t u;
  memcpy(&u, &x, sizeof(u));
  return (u & 0x7f800000u) != 0x7f800000u;
}
inline bool finite_f64(double x) {
  uint64_t u;
  memcpy(&u, &x, sizeof(u));
  return (u & 0x7ff0000000000000ull) != 0x7ff0000000000000ull;
}

// Index of the current device, clamped into [0, kMaxDevices) (per-device set-up is cached by it).
constexpr int kMaxDevices = 64;
inline int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = 0; }
  return dev < 0 ? 0 : (dev >= kMaxDevices ? kMaxDevices - 1 : dev);
}

inline sp_status launch_status() { return hipGetLastError() == hipSuccess ? SP_OK : SP_ELAUNCH; }

// bf16 bit pattern -> fp32 (exact)
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Largest b in [0, B) with table[b] <= x, for a non-decreasing table[0..B] with table[0] <= x < table[B].
__device__ __forceinline__ int upper_segment(const int32_t* __restrict__ table, int B, int x) {
  int lo = 0, hi = B;  // invariant: table[lo] <= x < table[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (table[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

// Exclusive prefix over per-sequence counts f(b), b in [0,B), by one workgroup; writes out[0..B].
// Call with all threads of a 1024-thread block.
template <typename F>
__device__ void block_prefix_table(int B, F count_of, int32_t* __restrict__ out) {
  __shared__ int32_t part[1024];
  const int t = threadIdx.x;
  const int per = (B + 1023) / 1024;
  const int b0 = min(B, t * per), b1 = min(B, b0 + per);
  int32_t sum = 0;
  for (int b = b0; b < b1; ++b) sum += count_of(b);
  part[t] = sum;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    int32_t v = (t >= off) ? part[t - off] : 0;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  int32_t run = part[t] - sum;  // exclusive
  for (int b = b0; b < b1; ++b) { out[b] = run; run += count_of(b); }
  if (t == 1023) out[B] = part[1023];
  __syncthreads();
}

}  // namespace sp
