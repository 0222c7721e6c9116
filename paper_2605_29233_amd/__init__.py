"""BlockBatch branch-batched denoising path for MI355X: thin ctypes binding over libblockbatch.so.

The binding only marshals arguments; every step of the path runs in the library's HIP kernels.
PyTorch is used for the device workspace allocation and the stream handle.
"""
from .binding import (BlockBatch, Limits, BranchState, RequestStats, StepView, BBError, lib_path, load_library,
                      BB_INIT, BB_PERIODIC)  # noqa: F401
