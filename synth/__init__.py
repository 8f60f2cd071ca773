"""Seeded synthetic inputs for the HALoS server-side update path.

This package only *produces inputs*: tensor-list layouts, initial models,
worker pseudo-gradients and event schedules.  It contains none of the
method's arithmetic (no momentum step, no accumulation, no merge) and is
the one module that both the CPU oracle's tests and the HIP path's tests
are allowed to share.
"""
from .layouts import Layout, gpt_layout, flat_layout
from .configs import Workload, WORKLOADS, get_workload, delta_scales
from .tensors import normal_at, normal_flat, to_bf16_bits
from .schedule import Trace, make_trace, EV_ARRIVE_DELTA, EV_ARRIVE_GLOBAL, EV_LPS_STEP, EV_GPS_MERGE, EV_PULL

__all__ = [
    "Layout", "gpt_layout", "flat_layout", "Workload", "WORKLOADS", "get_workload", "delta_scales",
    "normal_at", "normal_flat", "to_bf16_bits", "Trace", "make_trace",
    "EV_ARRIVE_DELTA", "EV_ARRIVE_GLOBAL", "EV_LPS_STEP", "EV_GPS_MERGE", "EV_PULL",
]
