"""libdsk for MI355X: whole-image forward / backward propagation of patch CNNs
with d-regularly sparse kernels (arXiv 1412.4526), hand-written HIP for gfx950.

Importing this package loads paper_1412_4526_amd/libdsk.so and fails if it has
not been built; there is no CPU or framework fallback.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
from .binding import DskError, lib, LIB_PATH, SYMBOLS, status_string, torch_dtype  # noqa: F401
from .net import WholeImageNet  # noqa: F401
from .fastscan import FastScanNet  # noqa: F401
from .video import WholeVideoNet  # noqa: F401
