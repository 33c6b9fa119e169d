"""MI355X-native Recurrent Residual Module: thin Python binding over the C-ABI HIP library.

The binding only marshals arguments (device pointers, shapes, the current HIP stream); every
step of the per-layer delta update runs in the library's gfx950 kernels.  There is no CPU or
PyTorch fallback: if the built library is missing, importing :mod:`.binding` symbols that need
it raises.
"""
from .binding import (  # noqa: F401
    BF16, BIN, CONV, FC, I8, Layer, RRMError, Shape, StackEntry, Stats, lib, lib_path, probe_copy, probe_mfma, relu_requant_pool_i8, stack_step,
)
