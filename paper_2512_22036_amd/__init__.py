"""MI355X-native MoE token shuffle with the layout transformation fused into the data movement.

The work is done by hand-written HIP kernels in libfusco.so behind the C boundary declared in
include/fusco.h; this package is a thin ctypes binding with the same names.  PyTorch supplies
device memory and streams only.  There is no CPU or PyTorch fallback: without the built library
every call raises.
"""
from .binding import (BF16, F32, DISPATCH_EXPERT, DISPATCH_WIRE, DISPATCH_TWO_HOP, DISPATCH_STREAMING, FuscoError, Layout, library_path,
                      load_library, fusco_version, fusco_plan, fusco_plan_static, fusco_dispatch, fusco_dispatch_in_transfer_order, fusco_combine, fusco_plan_dispatch,
                      fusco_probe_copy, fusco_probe_rows, fusco_probe_pieces, fusco_probe_consume_slices, fusco_probe_time_next_call, fusco_probe_source_chunk_bytes, fusco_probe_dispatch_kernel, fusco_probe_dispatch_occupancy, fusco_probe_dispatch_pull, fusco_probe_dispatch_walk,
                      fusco_combine_two_hop, fusco_balance_groups, fusco_cross_node_load, fusco_segments_scan,
                      fusco_segments_copy, fusco_disaggregated_plan, fusco_disaggregated_dispatch,
                      fusco_disaggregated_combine)

__all__ = ["BF16", "F32", "DISPATCH_EXPERT", "DISPATCH_WIRE", "DISPATCH_TWO_HOP", "DISPATCH_STREAMING", "FuscoError", "Layout",
           "library_path", "load_library", "fusco_version", "fusco_plan", "fusco_plan_static", "fusco_dispatch", "fusco_dispatch_in_transfer_order", "fusco_combine", "fusco_plan_dispatch",
           "fusco_probe_copy", "fusco_probe_rows", "fusco_probe_pieces", "fusco_probe_consume_slices", "fusco_probe_time_next_call", "fusco_probe_source_chunk_bytes", "fusco_probe_dispatch_kernel", "fusco_probe_dispatch_occupancy", "fusco_probe_dispatch_pull", "fusco_probe_dispatch_walk", "fusco_combine_two_hop", "fusco_balance_groups", "fusco_cross_node_load",
           "fusco_segments_scan", "fusco_segments_copy", "fusco_disaggregated_plan", "fusco_disaggregated_dispatch",
           "fusco_disaggregated_combine"]
