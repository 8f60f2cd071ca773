"""Seeded synthetic inputs for the HALoS server-side update path.

This package only *produces inputs*: tensor-list layouts, initial models,
worker pseudo-gradients and event schedules.  It contains none of the
method's arithmetic (no momentum step, no accumulation, no merge) and is
the one module that both the CPU oracle's tests and the HIP path's tests
are allowed to share.
"""
from .layouts import Layout, gpt_layout, flat_layout
from .configs import Workload, WORKLOADS, get_workload, delta_scales, staleness_weight
from .tensors import normal_at, normal_flat, to_bf16_bits, to_f16
from .schedule import Trace, EV_ARRIVE_DELTA, EV_ARRIVE_GLOBAL, EV_LPS_STEP, EV_GPS_MERGE, EV_PULL
from .schedule import make_trace as make_seeded_trace
from .paper_cluster import PaperClusterSpec, make_paper_trace


def make_trace(w: Workload, seed=None, with_pulls: bool = True) -> Trace:
    """The event schedule of a workload: the seeded simulator, or the paper's cluster model if the workload asks for it."""
    if w.schedule == "paper":
        spec = PaperClusterSpec(model=w.paper_model, n_params=w.layout.total, K=w.k_range[0], pool_slots=w.pool_slots,
                                seed=w.seed if seed is None else seed)
        return make_paper_trace(spec, w.n_updates, with_pulls)
    return make_seeded_trace(w, seed, with_pulls)


__all__ = [
    "Layout", "gpt_layout", "flat_layout", "Workload", "WORKLOADS", "get_workload", "delta_scales",
    "normal_at", "normal_flat", "to_bf16_bits", "to_f16", "staleness_weight", "Trace", "make_trace", "make_seeded_trace", "make_paper_trace",
    "PaperClusterSpec",
    "EV_ARRIVE_DELTA", "EV_ARRIVE_GLOBAL", "EV_LPS_STEP", "EV_GPS_MERGE", "EV_PULL",
]
