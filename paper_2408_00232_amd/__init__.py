"""MI355X-native per-partition GCN layer step of cache-based distributed full-batch
training: HIP kernels behind a C ABI (libcdf.so) and a thin binding over it."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
from .layer import DeviceCsr, LayerBuffers, TfLayerBuffers  # noqa: F401
