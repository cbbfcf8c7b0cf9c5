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
  const uint16_t* k[SP_MAX_LAYERS];
};

void fill_score_dev(const sp_score_args* a, ScoreDev* p);

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
