"""MI355X-native SpecPrefill token-importance path: C-ABI HIP library + thin binding."""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    SP_LAYER_MAX, SP_LAYER_MEAN, SpError, load_library,
    sp_gather, sp_keep_upper_bound, sp_pool_select, sp_pool_select_workspace_bytes,
    sp_score, sp_score_check, sp_score_general, sp_score_workspace_bytes, sp_version,
)
