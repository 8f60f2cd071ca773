"""Event schedule from the paper's own cluster model (App. A, "Details on Experimental Setup").

The paper's simulator takes (i) a resource specification -- bandwidths between four regions, the placement of
the GPS, one LPS per region, four workers per region with relative speeds --, (ii) the model size and (iii) a
profiled time of one training step on the fastest worker, computes the duration of every computation and
communication event, and emits the order in which model updates reach each LPS and the GPS.  This module does
the same for the HALoS method with the three tables the paper prints, so that the arrival pattern (who is
fast, which region waits longest for the global model, how many updates land while an accumulated update is in
flight) is the paper's rather than a uniform draw.  Like synth.schedule it decides when messages arrive; it
performs none of the update arithmetic.

Durations (App. A):
    point-to-point   T = alpha + C / B            (alpha: propagation delay, B: bandwidth, C: message size)
    ring all-reduce  T = 2 (N-1) C / (N B)        (B: slowest link of the best ring; used by the synchronous baseline)
    computation      T = H * T_profiled * S_fastest / S

Readings where the paper gives no number: alpha = 0 (no propagation delay is printed); messages are fp32
(4 bytes per parameter); a parameter server's own update takes no simulated time; a worker that has delivered
its delta pulls the new local model over the same intra-region link before it starts computing again.
"""
from __future__ import annotations

import heapq
import itertools
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .schedule import (EV_ARRIVE_DELTA, EV_ARRIVE_GLOBAL, EV_GPS_MERGE, EV_LPS_STEP, EV_PULL, STEP_MERGE, STEP_UPDATE,
                       TRACE_DTYPE, SplitMix64, Trace)

# Table "Inter- and intra-region communication bandwidths (Gbps)"
BANDWIDTH_GBPS = np.array([
    [100.0, 0.537, 0.935, 0.202],
    [0.537, 100.0, 0.386, 0.117],
    [0.935, 0.386, 100.0, 0.127],
    [0.202, 0.117, 0.127, 100.0],
])

# Table "Relative speeds of the 16 workers" (rows: regions R-1..R-4)
WORKER_SPEEDS = np.array([
    [10.0, 9.1, 3.8, 2.6],
    [9.4, 8.0, 6.3, 5.8],
    [9.9, 5.7, 2.1, 1.5],
    [9.1, 8.7, 5.8, 1.2],
])

# Table "Profiled computation times of different models" (ms per training step on the fastest worker)
PROFILED_STEP_MS = {"70m": 238.4, "160m": 623.0, "410m": 1589.7}

GPS_REGION = 0          # "By default, we place the GPS in the first region (R-1)"


def t_p2p(message_bytes: float, bandwidth_gbps: float, alpha_s: float = 0.0) -> float:
    """Seconds for a point-to-point transfer: alpha + C / B."""
    return alpha_s + message_bytes * 8.0 / (bandwidth_gbps * 1e9)


def t_allreduce(n: int, message_bytes: float, slowest_gbps: float) -> float:
    """Seconds for a ring all-reduce among n participants: 2 (n-1) C / (n B)."""
    return 2.0 * (n - 1) * message_bytes * 8.0 / (n * slowest_gbps * 1e9)


def best_ring_bandwidth(regions: Sequence[int], bw: np.ndarray = BANDWIDTH_GBPS) -> Tuple[float, Tuple[int, ...]]:
    """The ring over the given regions whose slowest link is fastest (exhaustive search, as App. A describes)."""
    regions = list(regions)
    if len(regions) == 1:
        return float(bw[regions[0], regions[0]]), tuple(regions)
    best, best_ring = -1.0, None
    first = regions[0]
    for perm in itertools.permutations(regions[1:]):
        ring = (first,) + perm
        slow = min(bw[ring[i], ring[(i + 1) % len(ring)]] for i in range(len(ring)))
        if slow > best:
            best, best_ring = slow, ring
    return float(best), best_ring


def t_compute(h: int, profiled_ms: float, speed: float, fastest: float) -> float:
    """Seconds for h local steps on a worker of the given relative speed."""
    return h * profiled_ms * 1e-3 * fastest / speed


@dataclass(frozen=True)
class PaperClusterSpec:
    model: str                      # key of PROFILED_STEP_MS
    n_params: int
    K: int = 32                     # best value of the sensitivity study
    H: int = 8                      # local steps per round (hyper-parameter table)
    dynamic_local_updates: bool = True   # H scaled with worker speed, as HALoS is run in the paper
    bytes_per_param: float = 4.0
    alpha_s: float = 0.0
    pool_slots: int = 8
    seed: int = 2025


def make_paper_trace(spec: PaperClusterSpec, n_updates: int, with_pulls: bool = True) -> Trace:
    """Simulate HALoS on the paper's 4-region x 4-worker cluster until n_updates worker deltas have been applied."""
    L, W = WORKER_SPEEDS.shape
    rng = SplitMix64(spec.seed)                      # only picks delta-pool slots
    C = spec.n_params * spec.bytes_per_param
    fastest = float(WORKER_SPEEDS.max())
    prof = PROFILED_STEP_MS[spec.model]
    US = 1e6                                          # integer microseconds

    def us(seconds: float) -> int:
        return int(round(seconds * US))

    intra = us(t_p2p(C, 100.0, spec.alpha_s))
    to_gps = [us(t_p2p(C, BANDWIDTH_GBPS[l, GPS_REGION], spec.alpha_s)) for l in range(L)]
    rounds = np.zeros((L, W), dtype=np.int64)
    for l in range(L):
        for k in range(W):
            s = float(WORKER_SPEEDS[l, k])
            h = max(1, int(round(spec.H * s / fastest))) if spec.dynamic_local_updates else spec.H
            rounds[l, k] = us(t_compute(h, prof, s, fastest))

    t = [0] * L
    t_last = [0] * L
    outstanding = [False] * L
    t_pull = [[0] * W for _ in range(L)]
    fifo: List[List[tuple]] = [[] for _ in range(L)]
    heap: list = []
    seq = 0

    def post(time, what, l, k=0):
        nonlocal seq
        heapq.heappush(heap, (int(time), l, k, seq, what))
        seq += 1

    for l in range(L):
        for k in range(W):
            post(rounds[l, k] + intra, "delta", l, k)        # compute, then ship the delta to the LPS

    out = []

    def emit(kind, time, l, worker=-1, slot=-1, stale=0, exp_kind=0, exp_send=0, exp_acc=0):
        out.append((kind, l, worker, slot, stale, spec.K, exp_kind, t[l], t_last[l], exp_send, exp_acc, time))

    applied = 0
    while heap and applied < n_updates:
        now, l, k, _, what = heapq.heappop(heap)
        if what == "delta":
            stale = t[l] + sum(1 for it in fifo[l] if it[0] == "delta") - t_pull[l][k]
            emit(EV_ARRIVE_DELTA, now, l, worker=k, slot=rng.below(spec.pool_slots), stale=stale)
            fifo[l].append(("delta", k))
            post(now, "service", l)
        elif what == "global":
            emit(EV_ARRIVE_GLOBAL, now, l)
            fifo[l].append(("global",))
            post(now, "service", l)
        elif what == "gps":
            emit(EV_GPS_MERGE, now, l)
            post(now + to_gps[l], "global", l)               # the updated global model travels back
        elif what == "service":
            if not fifo[l]:
                continue
            item = fifo[l].pop(0)
            if item[0] == "delta":
                k = item[1]
                t[l] += 1
                acc = 0 if outstanding[l] else 1
                send = 0
                if not outstanding[l] and t[l] - t_last[l] >= spec.K:
                    outstanding[l] = True
                    send = 1
                    post(now + to_gps[l], "gps", l)          # the accumulated update travels to the GPS
                emit(EV_LPS_STEP, now, l, worker=k, exp_kind=STEP_UPDATE, exp_send=send, exp_acc=acc)
                applied += 1
                t_pull[l][k] = t[l]
                if with_pulls:
                    emit(EV_PULL, now, l, worker=k)
                post(now + intra + rounds[l, k] + intra, "delta", l, k)   # pull, compute, ship
            else:
                t_last[l] = t[l]
                outstanding[l] = False
                emit(EV_LPS_STEP, now, l, exp_kind=STEP_MERGE)
    events = np.array(out, dtype=TRACE_DTYPE)
    return Trace(f"paper-{spec.model}", L, W, [spec.K] * L, events, rounds)
