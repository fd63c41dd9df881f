"""MI355X-native DropIT hot path: min-k compress + weight gradient from the sparse cache.

The compute lives in ``libdropit.so`` (hand-written gfx950 HIP behind a C ABI,
declared in ``include/dropit.h``).  This package is only the ctypes binding:
argument marshalling from torch tensors (device memory + streams) to raw
pointers.  There is no CPU fallback: without the built library, or without a
GPU, the calls raise.
"""
from . import nn  # noqa: F401  (autograd wrappers: nn.Linear, nn.Conv2d, nn.apply_dropit)
from .binding import (  # noqa: F401
    DropitError,
    compress,
    compress_random,
    compress_random_workspace_bytes,
    compress_mask,
    compress_rows,
    compress_static,
    compress_workspace_bytes,
    keep_count,
    lib,
    lib_path,
    set_fc_recover,
    set_select_mode,
    trace_events,
    weight_grad,
    weight_grad_mask,
    weight_grad_rows,
    weight_grad_workspace_bytes,
    weight_grad_path,
)
