"""The five benchmark workloads (shapes, cluster sizes, event counts, seeds).

Hyper-parameter values are the best-performing ones the paper reports
(App. D, hyper-parameter table; Fig. 5): beta_l 0.9, beta_g 0.5, alpha 0.25,
local rate 0.2, global rate 0.15.  The accumulation count K is the paper's
ablation base (4, Table 2) for the Tiny case, its consistent-grouping value
(8, Sec. 5.3) for the fixed-K cases, and a seeded draw in [2, 8] where the
workload asks for seeded thresholds.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

from .layouts import Layout, flat_layout, gpt_layout


@dataclass(frozen=True)
class Workload:
    name: str
    description: str
    layout: Layout
    n_lps: int
    workers_per_lps: int
    n_updates: int                 # number of worker-delta arrivals in the trace
    delta_dtype: str               # "f32", "bf16" or "f16"
    delta_sigma: float = 1e-3      # base standard deviation of a worker delta
    scale_by_fan_in: bool = True   # multiply sigma by 1/sqrt(fan_in) per tensor
    init_sigma: float = 0.02
    hetero_rates: bool = False     # per-worker arrival rate ~ U[0.25, 1]
    k_range: Tuple[int, int] = (8, 8)   # accumulation threshold K drawn in [lo, hi] after each merge
    max_link_delay: int = 4        # LPS->GPS and GPS->LPS delays, in mean LPS inter-arrival times
    staleness_bound: int = 64      # asserted upper bound on worker staleness
    eta_l: float = 0.2
    beta_l: float = 0.9
    eta_g: float = 0.15
    beta_g: float = 0.5
    alpha: float = 0.25
    cg_l: float | None = None      # coefficient on the delta in the LPS rule; None = the paper's 1 - beta_l
    cg_g: float | None = None      # same for the GPS rule
    d_l: int = 1                   # momentum update delay of the LPS rule (delayed Nesterov momentum); 1 = plain rule
    d_g: int = 1                   # same for the GPS rule
    staleness_exponent: float = 0.0    # a > 0: every arriving delta carries the weight (1 + staleness)^-a (a caller-side
                                       # staleness scaling; 0 = HALoS itself, every weight 1)
    seed: int = 0
    pool_slots: int = 8            # number of distinct resident delta buffers
    schedule: str = "seeded"       # "seeded": synth.schedule; "paper": the paper's own cluster model (synth.paper_cluster)
    paper_model: str = ""          # key of the profiled-step-time table when schedule == "paper"

    def scaled(self, layout: Layout, n_updates: int | None = None, name: str | None = None) -> "Workload":
        """Same cluster / schedule recipe on another (usually smaller) layout."""
        return replace(self, layout=layout,
                       n_updates=self.n_updates if n_updates is None else n_updates,
                       name=self.name if name is None else name)


def delta_scales(w: Workload):
    """Per-tensor fp32 factor handed to the delta generator: sigma, divided by sqrt(fan_in) if the workload says so."""
    import numpy as np
    from .tensors import scale_f32
    out = np.empty(w.layout.n_tensors, dtype=np.float32)
    for i, fan in enumerate(w.layout.fan_in):
        sigma = w.delta_sigma / (float(fan) ** 0.5 if w.scale_by_fan_in else 1.0)
        out[i] = scale_f32(sigma)
    return out


def staleness_weight(w: Workload, staleness: int):
    """The fp32 weight a caller applying polynomial staleness scaling would hand over with a delta (an INPUT of the
    update path, like the delta itself; 1 when the workload uses none)."""
    import numpy as np
    if w.staleness_exponent <= 0.0:
        return np.float32(1.0)
    return np.float32((1.0 + float(staleness)) ** (-float(w.staleness_exponent)))


def _mk() -> Dict[str, Workload]:
    w = {}
    w["tiny"] = Workload(
        name="tiny",
        description="flat fp32 vector of 1,048,576 elements; 2 LPS x 2 workers; 32 updates",
        layout=flat_layout(1 << 20), n_lps=2, workers_per_lps=2, n_updates=32,
        delta_dtype="f32", scale_by_fan_in=False, k_range=(4, 4), max_link_delay=3,
        staleness_bound=3, seed=1001)
    w["70m"] = Workload(
        name="70m",
        description="70M-param GPT tensor list (d512, L6); 4 LPS x 4 workers; 256 updates; fp32 deltas",
        layout=gpt_layout(512, 6), n_lps=4, workers_per_lps=4, n_updates=256,
        delta_dtype="f32", k_range=(8, 8), max_link_delay=4, seed=1002)
    w["160m"] = Workload(
        name="160m",
        description="160M-param GPT tensor list (d768, L12); 4 LPS x 8 workers, rates U[0.25,1]; 512 updates; bf16 deltas",
        layout=gpt_layout(768, 12), n_lps=4, workers_per_lps=8, n_updates=512,
        delta_dtype="bf16", hetero_rates=True, k_range=(8, 8), max_link_delay=4, seed=1003)
    w["410m"] = Workload(
        name="410m",
        description="410M-param GPT tensor list (d1024, L24); 4 LPS x 4 workers; 512 updates; fp32 deltas; K seeded in [2,8]; link delay up to 16",
        layout=gpt_layout(1024, 24), n_lps=4, workers_per_lps=4, n_updates=512,
        delta_dtype="f32", k_range=(2, 8), max_link_delay=16, seed=1004)
    w["1b"] = Workload(
        name="1b",
        description="1B-param GPT tensor list (d2048, L16, ff8192); 8 LPS x 4 workers; 256 updates; bf16 deltas",
        layout=gpt_layout(2048, 16, d_ff=8192), n_lps=8, workers_per_lps=4, n_updates=256,
        delta_dtype="bf16", k_range=(8, 8), max_link_delay=4, seed=1005)
    # The paper's evaluation cluster (App. A): 4 regions x 4 workers, one LPS per region, K = 32, fp32 messages,
    # arrival order from its bandwidth, worker-speed and profiled-step-time tables.
    for key, lay in (("70m", gpt_layout(512, 6)), ("160m", gpt_layout(768, 12)), ("410m", gpt_layout(1024, 24))):
        w["paper-" + key] = Workload(
            name="paper-" + key,
            description=f"Pythia-{key.upper()}-shaped tensor list on the paper's 4-region x 4-worker cluster "
                        f"(its bandwidth / speed / step-time tables), K=32, 512 updates, fp32 deltas",
            layout=lay, n_lps=4, workers_per_lps=4, n_updates=512, delta_dtype="f32", k_range=(32, 32),
            staleness_bound=64, seed=2000 + len(w), schedule="paper", paper_model=key)
    # The optimizer setting of the paper's runs (App. D, hyper-parameter table): delayed Nesterov momentum with
    # d_l = 16, d_g = 2; the table lists the rates divided by the delays (0.2 and 0.15), so eta = rate x delay.
    for key in ("1b", "410m", "paper-410m"):
        base = w[key]
        w[key + "-dn"] = replace(base, name=key + "-dn", d_l=16, d_g=2, eta_l=0.2 * 16, eta_g=0.15 * 2,
                                 description=base.description + "; delayed Nesterov momentum d_l=16, d_g=2")
    return w


WORKLOADS: Dict[str, Workload] = _mk()


def get_workload(name: str) -> Workload:
    return WORKLOADS[name.lower()]
