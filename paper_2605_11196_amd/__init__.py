"""MI355X-native Variational Linear Attention forward (thin binding over libvla.so)."""
from .binding import (  # noqa: F401
    VLA_BF16,
    VLA_F32,
    MODE_AUTO,
    MODE_CHUNKED,
    MODE_SCAN,
    MODE_TIME_PARALLEL,
    MODE_TWO_PHASE,
    VlaError,
    lib_path,
    load_library,
    resolve_mode,
    status_string,
    version,
    vla_forward,
    vla_forward_raw,
    vla_forward_workspace_bytes,
)
