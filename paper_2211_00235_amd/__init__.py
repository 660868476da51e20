"""Parallel Evoformer block for AMD MI355X: thin Python binding over the C ABI.

All compute runs in the HIP library `libpe_mi355x.so` (built in-tree by
`paper_2211_00235_amd.build.build()`); this package only marshals arguments.
There is no CPU fallback: importing works without a GPU (shape queries are
host-only), compute calls need the built library and a device.
"""
from .binding import (PEDims, Handle, lib, param_count, param_table, ctx_table, ctx_bytes,
                      workspace_bytes, stack_workspace_bytes, check_dims, dims_error, block_fwd, block_bwd,
                      stack_fwd_bwd, strerror, PE_F32, PE_BF16, PEError, block_fwd_static,
                      static_scratch_bytes)

__all__ = ["PEDims", "Handle", "lib", "param_count", "param_table", "ctx_table", "ctx_bytes",
           "workspace_bytes", "stack_workspace_bytes", "check_dims", "dims_error", "block_fwd", "block_bwd",
           "stack_fwd_bwd", "strerror", "PE_F32", "PE_BF16", "PEError", "block_fwd_static",
           "static_scratch_bytes"]
