"""MI355X-native 4x1 structured-sparse INT8 SpMM (hot path of arxiv 2306.16601).

The product is the C-ABI library built from csrc/ (declared in include/spmm.h);
this package is its thin ctypes binding.  Importing it does not load the
library; the first call does, and fails loudly if it was not built.
"""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, LIB_PATH, SpmmError, lib, make_epilogue, spmm_destroy, spmm_info,
                      spmm_kernel_name, spmm_kernel_variant, spmm_layout_dims, spmm_layout_export, spmm_make_gelu_lut,
                      spmm_pack, spmm_pack_ex, spmm_pack_host, spmm_plan, spmm_row_order, spmm_run, spmm_run_bound, spmm_run_status, spmm_run_tiled, spmm_run_tiled_bound, tile_major, from_tile_major, spmm_set_tuning,
                      spmm_status_string, spmm_unpack)
