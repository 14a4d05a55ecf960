"""MI355X-native TOVA bounded-KV-cache decode step (arXiv 2401.06104).

The package is a thin ctypes binding over libtova.so, the C-ABI library declared in
include/tova.h; every step of the path runs in its HIP kernels.  PyTorch is used for
device memory and streams only.
"""
from .binding import (  # noqa: F401
    TovaConfig, TovaLayout, TovaCache, TovaError, load_library, library_path,
    tova_cache_bytes, tova_cache_layout, tova_strerror,
    TOVA_F32, TOVA_BF16, TOVA_POLICY_TOVA, TOVA_POLICY_WINDOW, TOVA_POLICY_H2O, TOVA_OK, TOVA_EINVAL, TOVA_ENOSUP, TOVA_EHIP, TOVA_ENOMEM, TOVA_ETOOBIG,
)
