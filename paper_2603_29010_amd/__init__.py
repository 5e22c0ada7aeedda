"""MI355X (gfx950) fused-epilogue GEMM / conv library: Python binding of the C ABI in include/ucl.h.

The compute lives in ``libucl.so`` (hand-written HIP kernels).  This package only marshals
arguments; importing it never compiles anything and never falls back to another implementation:
if the library has not been built, the first call raises.
"""
from .binding import (UclError, Epilogue, Tuning, ucl_gemm, ucl_gemm_static_workspace, ucl_batched_gemm, ucl_grouped_gemm,  # noqa: F401
                      ucl_conv2d_fprop, ucl_conv2d_dgrad, ucl_conv2d_wgrad, ucl_transpose, ucl_sol_bound, ucl_select_tuning, ucl_workspace_size,
                      ucl_workspace_init, ucl_tile_map, ucl_num_variants,
                      ucl_variant, ucl_last_error, ucl_version, library_path, DTYPES, EPI_OPS)
