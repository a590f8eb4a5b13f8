"""Condensed constant fan-in sparse linear layer (SRigL inference hot path) for AMD MI355X.

The product is libsrigl.so, a C-ABI library of hand-written gfx950 kernels declared in
include/srigl.h; `binding` is its ctypes front end and `layer` a small convenience
holder of the device buffers.  Importing the package loads the library and fails if it
has not been built.
"""
from . import binding  # noqa: F401  (loads libsrigl.so, raises if it is missing)
from .binding import (BF16, F32, FWD_AUTO, FWD_GENERIC, FWD_KLANE, FWD_ROWLANE, SriglError,  # noqa: F401
                      srigl_check_fanin, srigl_condense, srigl_condensed_linear_fwd, srigl_seg_stride,
                      srigl_workspace_bytes)
from .layer import CondensedLinear, CondensedMLP, condense_layer, fold_mlp  # noqa: F401
