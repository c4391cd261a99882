"""MI355X-native per-partition einsum of GSPMD: thin Python binding over libgspmd.so.

Every step of the path runs in the HIP/C++ library; this package only marshals
arguments (see include/gspmd.h for the contract).  There is no CPU fallback: a
missing library raises.
"""
from .binding import (  # noqa: F401
    AXIS_BATCH, AXIS_CONTRACTING, AXIS_CONTRACTING_SCATTER, AXIS_LHS_FREE, AXIS_RHS_FREE, AXIS_UNUSED,
    EPILOGUE_NONE, EPILOGUE_RELU, KERNEL_MFMA, KERNEL_MFMA_STAGED, KERNEL_SCALAR,
    BF16, F32, LAYOUT_LHS_K_MAJOR, LAYOUT_RHS_K_CONTIGUOUS, DotDims, GspmdError, Mesh, Sharding, ShardBuf,
    classify_dot, compatible_operand_shardings, dot_workspace_bytes, resharded_dot, resharded_dot_workspace_bytes, grouped_dot, grouped_dot_noalloc, NOALLOC_MAX_WORKSPACE_BYTES, library_path, load_library,
    infer_out_sharding, local_dot, plan_dot, reduce_partials, reshard, reshard_workspace_bytes, shard_assemble, shard_bounds, shard_extract,
    status_string, EXPORTED_SYMBOLS, set_tile_timeline, TILE_TIMELINE_WORDS,
)
