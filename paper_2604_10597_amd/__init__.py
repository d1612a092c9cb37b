"""COREY hot path on AMD MI355X: entropy histogram, chunk rule and the Mamba-1 selective-scan forward.

The work is done by hand-written HIP kernels in ``libcorey.so`` (sources under ``csrc/``, C ABI in
``include/corey.h``); ``binding`` marshals torch GPU tensors into it.  Importing the package does not
load the library; the first call does, and raises if it has not been built.
"""
from .binding import (CoreyError, Policy, causal_conv1d_silu_fwd, selective_state_update, corey_entropy_hist, corey_entropy_hist_static, corey_entropy_hist_onesweep, corey_entropy_hist_from_table, corey_pattern_table_workspace, corey_entropy_hist_workspace, corey_select_chunk,
                      corey_select_chunk_device, corey_route_device, corey_route_device_deferred, corey_ema_update, corey_version, policy_default, selective_scan_fwd,
                      selective_scan_fwd_workspace, selective_scan_fwd_plan, selective_scan_fwd_plan_steps, selective_scan_fwd_plan_split)

__all__ = ["CoreyError", "Policy", "causal_conv1d_silu_fwd", "selective_state_update", "corey_entropy_hist", "corey_entropy_hist_static", "corey_entropy_hist_onesweep", "corey_entropy_hist_from_table", "corey_pattern_table_workspace", "corey_entropy_hist_workspace", "corey_select_chunk",
           "corey_select_chunk_device", "corey_route_device", "corey_route_device_deferred", "corey_ema_update", "corey_version", "policy_default", "selective_scan_fwd", "selective_scan_fwd_workspace", "selective_scan_fwd_plan", "selective_scan_fwd_plan_steps", "selective_scan_fwd_plan_split"]
