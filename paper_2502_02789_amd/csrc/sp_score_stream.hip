// Single-pass streaming scorer (placeholder until the MFMA kernel lands): reports that no
// shape is supported, so the dispatcher always takes the general kernels.
#include "sp_score_internal.h"

namespace sp {
bool stream_supported(const sp_score_args*) { return false; }
size_t stream_workspace_bytes(const sp_score_args*) { return 0; }
sp_status stream_score(const sp_score_args*, hipStream_t) { return SP_EUNSUPPORTED; }
}  // namespace sp
