"""SageBwd hot path for MI355X (gfx950): fused INT8 attention forward and
backward behind a C-ABI library, with a thin ctypes binding."""
from .binding import (  # noqa: F401
    SageParams,
    lib_path,
    load_library,
    workspace_bytes,
    sagebwd_quantize,
    sagebwd_fwd,
    sagebwd_bwd,
    sagebwd_strerror,
)
