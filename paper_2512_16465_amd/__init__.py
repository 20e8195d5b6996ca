"""libgemm for MI355X: a C-ABI GEMM library (HIP, gfx950) and its thin ctypes binding.

Importing the package does not load the shared library; the first call does, and fails loudly
if it has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTED_SYMBOLS, GemmError, gemm_create, gemm_destroy, gemm_epilogue_t,
                      gemm_get_last_plan, gemm_plan_query, gemm_plan_t, gemm_run, gemm_run_batched, gemm_run_noalloc, gemm_roofline_class, gemm_set_plan,
                      gemm_status_string, gemm_reserve_workspace, gemm_workspace_size,
                      gemm_variant_name, load_library, make_epilogue)
