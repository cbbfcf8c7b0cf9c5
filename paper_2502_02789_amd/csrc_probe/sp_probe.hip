// Read-only probes for the benchmark: what plain streaming of the K cache achieves on this device
// (see sp_probe.h).  No part of the scoring path uses anything in this file.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sp_probe.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct Layers {
  const unsigned char* p[SP_PROBE_MAX_LAYERS];
};

__global__ __launch_bounds__(256) void read_kernel(const Layers layers, int L, size_t vecs_per_layer, unsigned* sink) {
  u32x4 acc = {0, 0, 0, 0};
  const size_t stride = (size_t)gridDim.x * 256;
  for (int l = 0; l < L; ++l) {
    const u32x4* src = reinterpret_cast<const u32x4*>(layers.p[l]);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < vecs_per_layer; i += stride)
      acc ^= __builtin_nontemporal_load(src + i);
  }
  const unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (r == 0x9e3779b9u) sink[threadIdx.x & 63] = r;  // (practically never: keeps the loads alive)
}

__device__ __forceinline__ __attribute__((address_space(3))) void* lds_ptr(uint32_t a) {
  return reinterpret_cast<__attribute__((address_space(3))) void*>(a);
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

constexpr int kTile = 32 * 256;  // 32 keys x 128 bf16

// 256 workgroups x 8 waves; workgroup = (team = wg % 4, j = wg / 4); team t walks (layer, KV head
// 2t + s) slabs; the prompt's 32-key tiles are dealt out to the 64 workgroups of a team in turn: wave
// w of workgroup j reads tiles (2w + kb) * 64 + j, kb = 0, 1, of the slab, 8 KiB each, as 8 wave-wide
// loads of 4 keys x 256 bytes.
// POLICY: cache-policy bits of the loads (0 = default, 2 = non-temporal, what the scorer's key loads use).
template <int POLICY>
__device__ __forceinline__ void tiled_body(const Layers& layers, int L, int64_t ts_bytes, int64_t hs_bytes, unsigned* sink,
                                           unsigned char* smem) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int team = blockIdx.x & 3, j = blockIdx.x >> 2;
  const uint32_t ring = (uint32_t)reinterpret_cast<uintptr_t>(smem) + wave * 2 * kTile;
  const int n_tiles = L * 2 * 2;  // layers x KV heads of the team x tiles per slab
  const int64_t lane_off = (int64_t)(lane >> 4) * ts_bytes + (lane & 15) * 16;
  auto issue = [&](int f, int slot) {
    const int slab = f >> 1, kb = f & 1;
    const int layer = slab >> 1, kvh = team * 2 + (slab & 1);
    const unsigned char* src = layers.p[layer] + kvh * hs_bytes + (int64_t)(((wave * 2 + kb) * 64 + j) * 32) * ts_bytes + lane_off;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      __builtin_amdgcn_global_load_lds(src + (int64_t)(4 * i) * ts_bytes, lds_ptr(ring + slot * kTile + i * 1024), 16, 0, POLICY);
  };
  u32x4 acc = {0, 0, 0, 0};
  issue(0, 0);
  issue(1, 1);
  for (int f = 0; f < n_tiles; ++f) {
    const int slot = f & 1;
    if (f + 1 < n_tiles) wait_vmcnt<8>(); else wait_vmcnt<0>();
    acc ^= *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(lds_ptr(ring + slot * kTile + lane * 16));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the slot has been read before it is refilled
    if (f + 2 < n_tiles) issue(f + 2, slot);
  }
  const unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (r == 0x9e3779b9u) sink[lane] = r;
}

extern __shared__ __align__(1024) unsigned char tile_ring[];
__global__ __launch_bounds__(512) void tiled_kernel(const Layers layers, int L, int64_t ts_bytes, int64_t hs_bytes,
                                                    unsigned* sink) {
  tiled_body<2>(layers, L, ts_bytes, hs_bytes, sink, tile_ring);
}
__global__ __launch_bounds__(512) void tiled_default_policy_kernel(const Layers layers, int L, int64_t ts_bytes,
                                                                   int64_t hs_bytes, unsigned* sink) {
  tiled_body<0>(layers, L, ts_bytes, hs_bytes, sink, tile_ring);
}

}  // namespace

extern "C" int sp_probe_read(const void* const* h_layers, int32_t L, size_t bytes_per_layer, int32_t blocks, void* d_sink,
                             void* hip_stream) {
  if (!h_layers || !d_sink || L < 1 || L > SP_PROBE_MAX_LAYERS || blocks < 1 || (bytes_per_layer & 15)) return -1;
  Layers ls{};
  for (int l = 0; l < L; ++l) {
    if (!h_layers[l]) return -1;
    ls.p[l] = static_cast<const unsigned char*>(h_layers[l]);
  }
  hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), ls, L,
                     bytes_per_layer / 16, static_cast<unsigned*>(d_sink));
  return hipGetLastError() == hipSuccess ? 0 : -6;
}

typedef void (*tiled_kernel_t)(const Layers, int, int64_t, int64_t, unsigned*);

static int launch_tiled(tiled_kernel_t kernel, bool* prepared, const void* const* h_layers, int32_t L, int32_t T, int32_t H_kv,
                        int32_t d, int64_t k_token_stride, int64_t k_head_stride, void* d_sink, void* hip_stream) {
  if (!h_layers || !d_sink || L < 1 || L > SP_PROBE_MAX_LAYERS) return -1;
  if (T != 32768 || H_kv != 8 || d != 128 || k_token_stride < 128 || k_head_stride < 128) return -1;
  Layers ls{};
  for (int l = 0; l < L; ++l) {
    if (!h_layers[l]) return -1;
    ls.p[l] = static_cast<const unsigned char*>(h_layers[l]);
  }
  const int smem = 8 * 2 * kTile;
  if (!*prepared) {  // (benchmark helper: single-threaded use)
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
        hipSuccess)
      return -6;
    *prepared = true;
  }
  hipLaunchKernelGGL(kernel, dim3(256), dim3(512), smem, static_cast<hipStream_t>(hip_stream), ls, L, k_token_stride * 2,
                     k_head_stride * 2, static_cast<unsigned*>(d_sink));
  return hipGetLastError() == hipSuccess ? 0 : -6;
}

extern "C" int sp_probe_tiled(const void* const* h_layers, int32_t L, int32_t T, int32_t H_kv, int32_t d,
                              int64_t k_token_stride, int64_t k_head_stride, void* d_sink, void* hip_stream) {
  static bool prepared = false;
  return launch_tiled(tiled_kernel, &prepared, h_layers, L, T, H_kv, d, k_token_stride, k_head_stride, d_sink, hip_stream);
}

extern "C" int sp_probe_tiled_default_policy(const void* const* h_layers, int32_t L, int32_t T, int32_t H_kv, int32_t d,
                                             int64_t k_token_stride, int64_t k_head_stride, void* d_sink, void* hip_stream) {
  static bool prepared = false;
  return launch_tiled(tiled_default_policy_kernel, &prepared, h_layers, L, T, H_kv, d, k_token_stride, k_head_stride, d_sink,
                      hip_stream);
}
