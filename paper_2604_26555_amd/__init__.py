"""MI355X-native batch-SOM epoch (BMU search, per-BMU accumulation, neighbourhood update, host streaming).

The compute lives in ``libsom.so`` (hand-written HIP for gfx950, C ABI declared in ``include/som.h``);
``Som`` is the thin ctypes binding.  ``topology`` builds neighbourhood-distance matrices on the host.
"""
from .som import (  # noqa: F401
    Som, SomError, SomStats, EpochStats, load_library, LIB_PATH, EXPORTS, SOM_KERNEL_GAUSSIAN,
    SOM_OK, SOM_EINVAL, SOM_ENOMEM, SOM_EHIP, SOM_EIO, SOM_ESTATE,
)
from . import topology  # noqa: F401
