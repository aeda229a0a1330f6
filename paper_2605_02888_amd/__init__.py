"""MI355X-native verify-and-select stage of SpecKV: thin Python binding over libspeckv.so.

Importing this package does not load the HIP library; the first call that needs it does, and
fails loudly if it has not been built (``python -m paper_2605_02888_amd.build``).
"""
from .binding import (  # noqa: F401
    SpecKV,
    SpecKVError,
    Batch,
    load_library,
    workspace_bytes,
    STATUS_NAMES,
    DTYPES,
    FEATURES,
    FLAG_NONFINITE,
    FLAG_BAD_TOKEN,
    FLAG_FALLBACK,
    FLAG_BAD_GAMMA,
    STATIC_WS_BYTES,
)
