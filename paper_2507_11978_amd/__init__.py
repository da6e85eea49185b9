"""MI355X-native arrange-and-apply tiled contraction: thin Python binding over libnt.so.

Every step of the hot path runs in the HIP library; this package only marshals arguments
(torch tensors -> device pointers, sizes, strides, current stream).  There is no CPU or
PyTorch fallback: a missing library or device is an error.
"""
from .binding import (  # noqa: F401
    NtError, TileCfg, arrange_levels, arrange_tile, arrange_gemm, arrange_bmm, arrange_conv2d,
    program_order, tile_supported, gemm, gemm_noalloc, mfma_probe, addmm, bmm, matmul_views, last_kernel_path, last_k_split, PATH_GENERIC, PATH_STAGED, PATH_DIRECT, PATH_CONV, PATH_CONV_DIRECT, PATH_CONV_UNFOLD, PATH_CONV_TAP, add, silu, softmax, rms_norm, sdpa, conv2d_implicit, trace_tile, trace_loader_slice, version, lib_path, load, prepare,
    OP_TILE, OP_EXPAND, OP_SQUEEZE, OP_PERMUTE, OP_FLATTEN, OP_RAVEL, OP_DESCEND, OP_ASCEND,
)
