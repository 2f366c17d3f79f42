"""Operator-split linear layer of OSDP (arXiv 2209.13258, Section 3.3) for AMD MI355X.

The product is ``libosdp.so`` (hand-written HIP for gfx950 behind a C ABI, see
``include/osdp.h``); this package is its thin ctypes binding.  Importing it
fails when the library has not been built: there is no fallback path.
"""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, KERNEL_NAMES, OsdpError, Plan, lib, osdp_cost_model, osdp_granularity_candidates,
                      osdp_plan_search,
                      osdp_granularity_measure, osdp_granularity_select, osdp_profile_begin, osdp_profile_end,
                      osdp_row_slice_range, osdp_slice_range, osdp_split_linear_bwd, osdp_split_linear_bwd_mixed,
                      osdp_split_linear_fwd, osdp_split_linear_fwd_mixed,
                      osdp_split_linear_gather_row_slice, osdp_split_linear_gather_slice,
                      osdp_split_linear_workspace_bytes, osdp_version)
