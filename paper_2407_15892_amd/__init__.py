"""Mini-sequence LM-head + cross-entropy for MI355X (gfx950): ctypes binding of the HIP library."""
from .binding import (  # noqa: F401
    MstError,
    load_library,
    mst_lmhead_ce_bwd,
    mst_lmhead_ce_fwd,
    mst_profile_collect,
    mst_profile_enable,
    mst_strerror,
    mst_suggest_m,
    mst_version,
    mst_workspace_bytes,
)
