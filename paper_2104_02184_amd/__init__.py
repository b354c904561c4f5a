"""MI355X-native stochastic pulsed update of an analog crossbar tile.

Thin Python front-end of ``libaht.so`` (C ABI in ``include/aht.h``).  All
computation runs in the library's HIP kernels; PyTorch only provides device
memory and the stream.  There is no CPU fallback: if the library cannot be
loaded every call raises.
"""
from .workloads import WORKLOADS, HEADLINE, SMALL, Workload  # noqa: F401
from .binding import (  # noqa: F401
    AhtError, DeviceParams, IOParams, Tile, UnitCell, pulsed_update_many, load_library, library_path, debug_philox, debug_gauss,
    CONSTANT_STEP, LINEAR_STEP, SOFT_BOUNDS, PLANE_NAMES,
)

__all__ = ["AhtError", "DeviceParams", "IOParams", "Tile", "UnitCell", "pulsed_update_many", "load_library", "library_path", "debug_philox",
           "debug_gauss", "CONSTANT_STEP", "LINEAR_STEP", "SOFT_BOUNDS", "PLANE_NAMES",
           "WORKLOADS", "HEADLINE", "SMALL", "Workload"]
