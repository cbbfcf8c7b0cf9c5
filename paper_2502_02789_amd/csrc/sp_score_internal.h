// Declarations shared by the two scoring translation units.
#pragma once

#include "sp_common.h"

namespace sp {

// Kernel-side view of sp_score_args (passed by value).
struct ScoreDev {
  int B, N, L, H, H_kv, G, d;
  int T;
  int max_tiles;
  int layer_reduce;
  float scale;
  int64_t k_token_stride, k_head_stride;
  const uint16_t* q;
  const int32_t* cu;
  const int32_t* n_valid;
  int32_t* tile_cu;
  float* ws_lse;
  float2* part;
  float* scores;
  float* lse_out;
  const float2* rope;  // [position][d/2] (cos, sin) if keys are stored un-rotated, else null
  const int32_t* block_table;  // paged cache: [B][blocks_per_seq] page numbers, else null
  int lg_page, blocks_per_seq;
  int64_t k_page_stride;
  const float* k_scale;  // 8-bit cache: [L][H_kv] scales (null: all 1); the layers then hold bytes
  int k_fp8;
  const uint16_t* k[SP_MAX_LAYERS];
};

void fill_score_dev(const sp_score_args* a, ScoreDev* p);

// Rotary position encoding of an un-rotated cache (rope_theta > 0): the pair (t, t + d/2) of a row
// at position pos turns by pos * theta^(-2t/d).  The angle is formed in fp64, its cosine and sine
// are rounded to fp32, the two products and their sum or difference are separate fp32
// operations, and the result is rounded to bf16 (nearest even) as a cache would hold it -- every
// kernel that rotates goes through these two functions, so all of them produce the same bits.
__device__ __forceinline__ float2 rope_cos_sin(double pos, int t, int half, double log2_theta) {
  const double inv_freq = exp2(-((double)t / (double)half) * log2_theta);
  double sn, cs;
  sincos(pos * inv_freq, &sn, &cs);
  return make_float2((float)cs, (float)sn);
}
// lo, hi: the pair's values (exact bf16 values held as fp32); returns the rotated pair before rounding
__device__ __forceinline__ float2 rope_turn_exact(float lo, float hi, float2 cs) {
#pragma clang fp contract(off)
  const float a = lo * cs.x, b = hi * cs.y, c = hi * cs.x, d = lo * cs.y;
  return make_float2(a - b, c + d);
}
// ... and rounded to bf16 (nearest even), as fp32 values
__device__ __forceinline__ float2 rope_turn(float lo, float hi, float2 cs) {
  const float2 r = rope_turn_exact(lo, hi, cs);
  const uint32_t ul = __float_as_uint(r.x), uh = __float_as_uint(r.y);
  return make_float2(__uint_as_float((ul + 0x7FFFu + ((ul >> 16) & 1u)) & 0xFFFF0000u),
                     __uint_as_float((uh + 0x7FFFu + ((uh >> 16) & 1u)) & 0xFFFF0000u));
}
// two fp32 values -> two bf16 (nearest even) in one word, `even` in the low half: one instruction on gfx950
__device__ __forceinline__ uint32_t pack_bf16_pair(float even, float odd) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {even, odd};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// general two-pass kernels (sp_score.hip)
size_t general_workspace_bytes(const sp_score_args* a, bool with_tiled);
bool single_pass_wanted(const sp_score_args* a);
// allow_mfma: hand the two passes to the tiled MFMA kernels when the shape fits them
sp_status general_score(const sp_score_args* a, hipStream_t stream, bool allow_mfma);
void launch_lse_combine(const ScoreDev& p, hipStream_t stream);

// two-pass MFMA kernels for ragged batches (sp_score_tiled.hip); they share the general kernels'
// tile table, partials and log-sum-exps (`gen`), `extra` is their own workspace part
bool tiled_supported(const sp_score_args* a);
size_t tiled_extra_workspace_bytes(const sp_score_args* a);
sp_status tiled_score(const sp_score_args* a, const ScoreDev& gen, void* extra, hipStream_t stream);

// single-pass kernel for batches of short prompts with few query rows per KV head (sp_score_seq.hip)
bool seq_supported(const sp_score_args* a);

// single-pass streaming kernel (sp_score_stream.hip)
bool stream_supported(const sp_score_args* a);
size_t stream_workspace_bytes(const sp_score_args* a);
sp_status stream_score(const sp_score_args* a, hipStream_t stream);
size_t stream_status_offset(const sp_score_args* a);

// single-pass kernel with per-KV-head teams of workgroups (sp_score_team.hip): one prompt of up
// to 32K keys, SP_LAYER_MAX
bool team_supported(const sp_score_args* a);
size_t team_workspace_bytes(const sp_score_args* a);
sp_status team_score(const sp_score_args* a, hipStream_t stream);
size_t team_status_offset(const sp_score_args* a);

// single-launch scoring + selection of one short prompt (sp_fused.hip); 0 if the shape is not covered
size_t fused_workspace_bytes(const sp_score_args* a);

}  // namespace sp
