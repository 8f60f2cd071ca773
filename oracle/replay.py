"""Replay a synthetic event trace through the CPU oracle (test infrastructure only)."""
from __future__ import annotations

from typing import Callable, List, Tuple

import numpy as np

from . import HalosOracle

# event kinds of the trace records (integers fixed by the trace format)
_ARRIVE_DELTA, _LPS_STEP, _GPS_MERGE, _ARRIVE_GLOBAL, _PULL = 0, 1, 2, 3, 4


def replay(oracle: HalosOracle, events: np.ndarray, delta_of_slot: Callable[[int], np.ndarray],
           on_pull: Callable[[int, int, np.ndarray], None] | None = None,
           weight_of: Callable[[int], float] | None = None) -> List[Tuple[int, int, int, int, int, int]]:
    """Feed every record to the oracle in order.

    delta_of_slot(slot) returns the pseudo-gradient held in that pool slot
    (float32 values or raw bf16 bit patterns), restricted to whatever index
    subset the oracle was created on.  weight_of(staleness), if given, is the caller's scalar on a delta that arrives
    with that staleness.  Returns the step log: one tuple
    (record index, kind, t, t_last, sent, accumulated) per LPS step.
    """
    log = []
    for i, ev in enumerate(events):
        kind, l = int(ev["kind"]), int(ev["lps"])
        if kind == _ARRIVE_DELTA:
            weight = 1.0 if weight_of is None else weight_of(int(ev["staleness"]))
            oracle.arrive_delta(l, int(ev["worker"]), delta_of_slot(int(ev["slot"])), weight)
        elif kind == _LPS_STEP:
            oracle.set_K(l, int(ev["k_cur"]))
            info = oracle.lps_step(l)
            log.append((i, info.kind, info.t, info.t_last, info.sent, info.accumulated))
        elif kind == _GPS_MERGE:
            oracle.gps_receive(l)
        elif kind == _ARRIVE_GLOBAL:
            oracle.arrive_global(l)
        elif kind == _PULL:
            if on_pull is not None:
                on_pull(l, int(ev["worker"]), oracle.get(0, l))
        else:
            raise ValueError(f"unknown event kind {kind}")
    return log
