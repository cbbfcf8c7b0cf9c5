// sp_gather: restore the original position ids of the kept tokens (Sec. 3.2.4 and
// Algorithm 1, restore_pos_ids, of arXiv 2502.02789) and gather what the base model's
// prefill consumes: token ids and embedding rows.  Pure integer work and byte copies.
#include "sp_common.h"

namespace sp {

struct GatherDev {
  int B;
  int D;
  int64_t capacity;
  const int32_t* cu;
  const int32_t* cu_keep;
  const int32_t* kept_idx;
  const int32_t* token_ids;
  const u32x4* embed;
  int32_t* kept_ids;
  int32_t* kept_pos;
  int32_t* decode_pos;
  u32x4* out_embed;
};

__global__ __launch_bounds__(256) void gather_meta_kernel(const GatherDev p) {
  const int64_t n_keep = min((int64_t)p.cu_keep[p.B], p.capacity);
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x; s < max(n_keep, (int64_t)p.B); s += stride) {
    if (s < p.B) p.decode_pos[s] = p.cu[s + 1] - p.cu[s];
    if (s < n_keep) {
      const int b = upper_segment(p.cu_keep, p.B, (int)s);
      const int idx = p.kept_idx[s];
      p.kept_pos[s] = idx - p.cu[b];
      if (p.token_ids) p.kept_ids[s] = p.token_ids[idx];
    }
  }
}

// one workgroup per kept row, 16 bytes per lane per step; the row's position and token id and the
// sequences' decode positions are written here too (one launch instead of two)
__global__ __launch_bounds__(256) void gather_rows_kernel(const GatherDev p) {
  const int64_t n_keep = min((int64_t)p.cu_keep[p.B], p.capacity);
  const int vec_per_row = p.D / 8;
  for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < p.B; b += (int64_t)gridDim.x * 256)
    p.decode_pos[b] = p.cu[b + 1] - p.cu[b];
  for (int64_t s = blockIdx.x; s < n_keep; s += gridDim.x) {
    const int idx = p.kept_idx[s];
    const int64_t id = p.token_ids[idx];
    if (threadIdx.x == 0) {
      p.kept_pos[s] = idx - p.cu[upper_segment(p.cu_keep, p.B, (int)s)];
      p.kept_ids[s] = (int32_t)id;
    }
    const u32x4* src = p.embed + id * vec_per_row;
    u32x4* dst = p.out_embed + s * vec_per_row;
    for (int v = threadIdx.x; v < vec_per_row; v += 256) dst[v] = __builtin_nontemporal_load(src + v);
  }
}

}  // namespace sp

extern "C" sp_status sp_gather(const sp_gather_args* a, void* hip_stream) {
  using namespace sp;
  if (!a) return SP_ENULL;
  if (a->B < 1 || a->kept_capacity < 0) return SP_EINVAL;
  if (!a->d_cu_seqlens || !a->d_cu_keep || !a->d_kept_idx || !a->d_kept_pos || !a->d_decode_pos) return SP_ENULL;
  if (a->d_token_ids && !a->d_kept_ids) return SP_ENULL;
  const bool rows = a->d_out_embed != nullptr;
  if (rows) {
    if (!a->d_embed || !a->d_token_ids) return SP_ENULL;
    if (a->V < 1 || a->D < 8 || (a->D & 7)) return SP_EINVAL;
    if (!aligned16(a->d_embed) || !aligned16(a->d_out_embed)) return SP_EALIGN;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  GatherDev p;
  p.B = a->B; p.D = a->D; p.capacity = a->kept_capacity;
  p.cu = a->d_cu_seqlens; p.cu_keep = a->d_cu_keep; p.kept_idx = a->d_kept_idx;
  p.token_ids = a->d_token_ids;
  p.embed = static_cast<const u32x4*>(a->d_embed);
  p.kept_ids = a->d_kept_ids; p.kept_pos = a->d_kept_pos; p.decode_pos = a->d_decode_pos;
  p.out_embed = static_cast<u32x4*>(a->d_out_embed);
  const int64_t work = std::max<int64_t>(a->kept_capacity, a->B);
  const int meta_blocks = (int)std::min<int64_t>((work + 255) / 256, 4096);
  if (rows && a->kept_capacity > 0) {
    const int row_blocks = (int)std::min<int64_t>(a->kept_capacity, 16384);
    hipLaunchKernelGGL(gather_rows_kernel, dim3(row_blocks), dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(gather_meta_kernel, dim3(std::max(meta_blocks, 1)), dim3(256), 0, stream, p);
  }
  return launch_status();
}

extern "C" const char* sp_strerror(sp_status status) {
  switch (status) {
    case SP_OK: return "ok";
    case SP_EINVAL: return "a size, rate or enum is out of range";
    case SP_ENULL: return "a required pointer is NULL";
    case SP_EALIGN: return "a pointer or stride is not 16-byte aligned (workspace: 256)";
    case SP_EWORKSPACE: return "workspace missing or too small";
    case SP_EUNSUPPORTED: return "request not supported by this build";
    case SP_ELAUNCH: return "the HIP runtime refused a kernel launch";
    case SP_ETIMEOUT: return "a bounded device-side wait expired; results are invalid";
  }
  return "unknown status";
}

extern "C" int32_t sp_version(void) { return 200; }
