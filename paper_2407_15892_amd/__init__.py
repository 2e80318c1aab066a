"""Mini-sequence LM-head + cross-entropy and mini-sequence MLP for MI355X (gfx950): ctypes bindings of the HIP libraries."""
from .binding import (  # noqa: F401
    MstError,
    load_library,
    mst_lmhead_ce_bwd,
    mst_lmhead_ce_fwd,
    mst_mfma_probe,
    mst_profile_collect,
    mst_profile_enable,
    mst_shift_labels,
    mst_strerror,
    mst_suggest_m,
    mst_version,
    mst_workspace_bytes,
)
from .mlp_binding import (  # noqa: F401
    load_mlp_library,
    mst_mlp_bwd,
    mst_mlp_fwd,
    mst_mlp_profile_collect,
    mst_mlp_profile_enable,
    mst_mlp_suggest_m,
    mst_mlp_version,
    mst_mlp_workspace_bytes,
)
