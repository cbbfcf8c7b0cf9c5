// Low-level pieces shared by the MFMA scoring kernels: waits on the vector-memory counter,
// LDS accesses the compiler does not track, agent-coherent stores, quad maxima.
#pragma once

#include "sp_common.h"

namespace sp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Cache-policy bits of the direct global->LDS loads that stream key tiles: 2 = "nt" (non-temporal: the line
// is used once).  Every key byte is read once per pass, so nothing is lost by not keeping it; measured on a
// read-only stream of the 32K-token cache in the scorer's tile order: 7.2 TB/s with the bit, 6.4 TB/s without
// (plain register loads: 7.1 / 6.35).  Query tiles, which every workgroup re-reads from L2, keep policy 0.
#ifndef SP_KEY_LOAD_POLICY
#define SP_KEY_LOAD_POLICY 2
#endif
constexpr int kKeyLoadPolicy = SP_KEY_LOAD_POLICY;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// "at most n vector-memory instructions of this wave still in flight", n known only at run time.
// Rounded down to a value there is an instruction for (stricter than asked is always correct).
__device__ __forceinline__ void wait_vmcnt_upto(int n) {
  if (n >= 12) {
    if (n >= 16) wait_vmcnt<16>();
    else if (n >= 14) { if (n >= 15) wait_vmcnt<15>(); else wait_vmcnt<14>(); }
    else { if (n >= 13) wait_vmcnt<13>(); else wait_vmcnt<12>(); }
  } else if (n >= 8) {
    if (n >= 10) { if (n >= 11) wait_vmcnt<11>(); else wait_vmcnt<10>(); }
    else { if (n >= 9) wait_vmcnt<9>(); else wait_vmcnt<8>(); }
  } else if (n >= 4) {
    wait_vmcnt<4>();
  } else {
    wait_vmcnt<0>();
  }
}

// LDS accesses the compiler does not see as such.  The words touched this way (deposits, counters,
// fetched log-sum-exps, the running maxima) are never the target of a direct-to-LDS TILE load, so
// there is no reason to wait for the tile loads in flight before touching them -- which an
// ordinary LDS access would be made to do.  LDS operations of one wave are performed in order.
__device__ __forceinline__ uint32_t lds_peek(uint32_t lds_addr) {
  uint32_t v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_addr) : "memory");
  return v;
}
__device__ __forceinline__ u32x4 lds_peek128(uint32_t lds_addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_addr) : "memory");
  return v;
}
__device__ __forceinline__ void lds_poke32(uint32_t lds_addr, uint32_t v) {
  asm volatile("ds_write_b32 %0, %1" : : "v"(lds_addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_poke128(uint32_t lds_addr, u32x4 v) {
  asm volatile("ds_write_b128 %0, %1" : : "v"(lds_addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_add(uint32_t lds_addr, uint32_t v) {
  asm volatile("ds_add_u32 %0, %1" : : "v"(lds_addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_or(uint32_t lds_addr, uint32_t v) {
  asm volatile("ds_or_b32 %0, %1" : : "v"(lds_addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_and(uint32_t lds_addr, uint32_t v) {
  asm volatile("ds_and_b32 %0, %1" : : "v"(lds_addr), "v"(v) : "memory");
}
__device__ __forceinline__ uint64_t lds_peek64(uint32_t lds_addr) {
  uint64_t v;
  asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_addr) : "memory");
  return v;
}
__device__ __forceinline__ uint32_t lds_or_rtn(uint32_t lds_addr, uint32_t v) {
  uint32_t old;
  asm volatile("ds_or_rtn_b32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(old) : "v"(lds_addr), "v"(v) : "memory");
  return old;
}
__device__ __forceinline__ uint32_t lds_add_rtn(uint32_t lds_addr, uint32_t v) {
  uint32_t old;
  asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(old) : "v"(lds_addr), "v"(v) : "memory");
  return old;
}
// 16-byte store with agent-scope coherence (written through to where every XCD can see it)
__device__ __forceinline__ void store128_agent(void* dst, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(v) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_poke64(uint32_t lds_addr, uint64_t v) {
  asm volatile("ds_write_b64 %0, %1 offset:%2" : : "v"(lds_addr), "v"(v), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_poke32_at(uint32_t lds_addr, uint32_t v) {
  asm volatile("ds_write_b32 %0, %1 offset:%2" : : "v"(lds_addr), "v"(v), "n"(OFF) : "memory");
}
// four words STRIDE bytes apart, one wait for all of them
template <int STRIDE>
__device__ __forceinline__ u32x4 lds_peek4(uint32_t lds_addr) {
  uint32_t a, b, c, d;
  asm volatile(
      "ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:%5\n\tds_read_b32 %2, %4 offset:%6\n\t"
      "ds_read_b32 %3, %4 offset:%7\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d)
      : "v"(lds_addr), "n"(STRIDE), "n"(2 * STRIDE), "n"(3 * STRIDE)
      : "memory");
  return u32x4{a, b, c, d};
}
// four 16-byte reads STRIDE bytes apart, one wait for all of them
struct u32x4x4 { u32x4 v[4]; };
template <int STRIDE>
__device__ __forceinline__ u32x4x4 lds_peek128x4(uint32_t lds_addr) {
  u32x4x4 r;
  asm volatile(
      "ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:%5\n\tds_read_b128 %2, %4 offset:%6\n\t"
      "ds_read_b128 %3, %4 offset:%7\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(r.v[0]), "=&v"(r.v[1]), "=&v"(r.v[2]), "=&v"(r.v[3])
      : "v"(lds_addr), "n"(STRIDE), "n"(2 * STRIDE), "n"(3 * STRIDE)
      : "memory");
  return r;
}
// 4-byte store with agent-scope coherence
__device__ __forceinline__ void store32_agent(void* dst, uint32_t v) {
  asm volatile("global_store_dword %0, %1, off sc1" : : "v"(dst), "v"(v) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_fmax(uint32_t lds_addr, float v) {
  asm volatile("ds_max_f32 %0, %1 offset:%2" : : "v"(lds_addr), "v"(v), "n"(OFF) : "memory");
}
// max with the value of lane ^ 1 / lane ^ 2 (inside the quad); folds into v_max_f32_dpp
__device__ __forceinline__ float max_quad_xor1(float v) {
  return fmaxf(v, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true)));
}
__device__ __forceinline__ float max_quad_xor2(float v) {
  return fmaxf(v, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true)));
}

}  // namespace sp
