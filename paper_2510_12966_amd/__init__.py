"""MI355X-native Pyramid Speculative Decoding: thin Python binding over libpsd.so.

Everything on the decoding path runs inside the HIP library; this package only marshals
arguments (ctypes) and offers the seeded synthetic-input generator under ``synth``.
"""
from .binding import (PsdError, Context, ModelDesc, Adapt, accept, accept_assisted, row_stats, accept_batch, accept_batch_noalloc, accept_noalloc_capacity, accept_noalloc_init, accept_workspace_bytes, set_accept_path, get_accept_path, get_accept_expiries, sample, sample_device, philox_block, lib, DeviceBuffer, dev_sync,
                      lib_path, F32, BF16, FLAG_GRAPH, FLAG_ASSISTED, FLAG_ROW_STATS, FLAG_GREEDY, MAX_WIDTH)

__all__ = ["PsdError", "Context", "ModelDesc", "Adapt", "accept", "accept_assisted", "row_stats", "accept_batch", "accept_batch_noalloc", "accept_noalloc_capacity", "accept_noalloc_init", "accept_workspace_bytes", "set_accept_path", "get_accept_path", "get_accept_expiries", "sample", "sample_device", "philox_block", "lib", "DeviceBuffer", "dev_sync",
           "lib_path", "F32", "BF16", "FLAG_GRAPH", "FLAG_ASSISTED", "FLAG_ROW_STATS", "FLAG_GREEDY", "MAX_WIDTH"]
