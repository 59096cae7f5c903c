"""MI355X-native selective-recompute path of InfoFlow KV (HIP kernels behind a
C ABI, see include/ifkv.h).  The shared library is loaded on first use."""
from .binding import (  # noqa: F401
    IFKV_FLAG_FORCE_GENERIC,
    IFKV_FLAG_VALIDATE,
    IfkvError,
    Layer,
    LIB_PATH,
    load_library,
)
