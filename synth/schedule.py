"""Seeded event schedule: the order in which messages reach the servers.

The paper evaluates by generating a trace of model-update events with a
discrete-event simulator and replaying it in strictly enforced order
(App. A).  This module is a small integer-clock simulator in the same
spirit: workers finish local training at their own rates, their deltas
queue at the local server, accumulated updates travel to the global server
and the global model travels back with seeded link delays.  It decides
*when things arrive*; it performs none of the update arithmetic.

A trace is a structured array, one record per call a driver makes:

  ARRIVE_DELTA   worker `worker` of server `lps` delivers a delta (pool slot `slot`)
  LPS_STEP       server `lps` handles the head of its queue
  GPS_MERGE      the accumulated update of `lps` reaches the global server
  ARRIVE_GLOBAL  the global model sent back to `lps` reaches it
  PULL           worker `worker` of `lps` fetches the local model

The exp_* fields record what the simulator's own bookkeeping expects the
step to report (what was popped, the counters t and t_last, whether the
accumulation threshold fired), so every implementation that replays the
trace can be checked against it record by record.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass
from typing import List

import numpy as np

from .configs import Workload

EV_ARRIVE_DELTA = 0
EV_LPS_STEP = 1
EV_GPS_MERGE = 2
EV_ARRIVE_GLOBAL = 3
EV_PULL = 4

STEP_NONE = 0
STEP_UPDATE = 1
STEP_MERGE = 2

TRACE_DTYPE = np.dtype([
    ("kind", "<i4"), ("lps", "<i4"), ("worker", "<i4"), ("slot", "<i4"),
    ("staleness", "<i4"), ("k_cur", "<i4"),
    ("exp_kind", "<i4"), ("exp_t", "<i8"), ("exp_t_last", "<i8"), ("exp_send", "<i4"),
    ("exp_accumulate", "<i4"), ("time", "<i8"),
])

_TICKS = 1 << 20


class SplitMix64:
    """Steele/Lea/Flood SplitMix64: a 64-bit counter stepped by the golden-ratio
    increment and finalised with two xor-shift-multiply rounds."""

    def __init__(self, seed: int):
        self.s = seed & 0xFFFFFFFFFFFFFFFF

    def next(self) -> int:
        self.s = (self.s + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        return z ^ (z >> 31)

    def below(self, n: int) -> int:
        """Uniform integer in [0, n) (n small; modulo bias < 2**-40 is irrelevant here)."""
        return self.next() % n if n > 0 else 0

    def between(self, lo: int, hi: int) -> int:
        return lo + self.below(hi - lo + 1)


@dataclass
class Trace:
    workload: str
    n_lps: int
    workers_per_lps: int
    k_initial: List[int]            # K in force at each LPS before its first merge
    events: np.ndarray              # TRACE_DTYPE records in replay order
    worker_period: np.ndarray       # ticks per worker round, shape (n_lps, workers)

    def to_bytes(self) -> bytes:
        return self.events.tobytes()

    def count(self, kind: int) -> int:
        return int((self.events["kind"] == kind).sum())

    @property
    def n_update_steps(self) -> int:
        e = self.events
        return int(((e["kind"] == EV_LPS_STEP) & (e["exp_kind"] == STEP_UPDATE)).sum())

    @property
    def n_merge_steps(self) -> int:
        e = self.events
        return int(((e["kind"] == EV_LPS_STEP) & (e["exp_kind"] == STEP_MERGE)).sum())


def make_trace(w: Workload, seed: int | None = None, with_pulls: bool = True) -> Trace:
    """Simulate until `w.n_updates` worker deltas have been applied."""
    rng = SplitMix64(w.seed if seed is None else seed)
    L, W = w.n_lps, w.workers_per_lps

    period = np.zeros((L, W), dtype=np.int64)
    for l in range(L):
        for k in range(W):
            if w.hetero_rates:
                rate_q = 256 + rng.below(769)          # rate = rate_q / 1024 in [0.25, 1.0]
                period[l, k] = (_TICKS * 1024 + rate_q // 2) // rate_q
            else:
                period[l, k] = _TICKS
    mean_gap = np.maximum(1, (period.mean(axis=1) / W).astype(np.int64))   # mean delta inter-arrival per LPS

    # bookkeeping that mirrors the protocol counters (no parameter arithmetic)
    t = [0] * L
    t_last = [0] * L
    k_cur = [rng.between(*w.k_range) for _ in range(L)]
    k_initial = list(k_cur)
    outstanding = [False] * L
    t_pull = [[0] * W for _ in range(L)]
    fifo: List[List[tuple]] = [[] for _ in range(L)]
    busy_until = [0] * L
    service_pending = [False] * L

    heap: list = []
    seq = 0

    def post(time, what, l, k=0):
        nonlocal seq
        heapq.heappush(heap, (int(time), l, k, seq, what))
        seq += 1

    for l in range(L):
        for k in range(W):
            post(period[l, k] + rng.below(int(period[l, k] // 8) + 1), "done", l, k)

    out = []

    def emit(kind, time, l, worker=-1, slot=-1, stale=0, exp_kind=0, exp_send=0, exp_acc=0):
        out.append((kind, l, worker, slot, stale, k_cur[l], exp_kind, t[l], t_last[l], exp_send, exp_acc, time))

    def kick(l, now):
        if not service_pending[l] and fifo[l]:
            service_pending[l] = True
            post(max(now, busy_until[l]), "service", l)

    applied = 0
    max_stale = 0
    while heap and applied < w.n_updates:
        now, l, k, _, what = heapq.heappop(heap)
        if what == "done":
            ahead = sum(1 for it in fifo[l] if it[0] == "delta")
            stale = t[l] + ahead - t_pull[l][k]
            max_stale = max(max_stale, stale)
            slot = rng.below(w.pool_slots)
            emit(EV_ARRIVE_DELTA, now, l, worker=k, slot=slot, stale=stale)
            fifo[l].append(("delta", k))
            kick(l, now)
        elif what == "service":
            service_pending[l] = False
            item = fifo[l].pop(0)
            if item[0] == "delta":
                k = item[1]
                t[l] += 1
                acc = 0 if outstanding[l] else 1
                send = 0
                if not outstanding[l] and t[l] - t_last[l] >= k_cur[l]:
                    outstanding[l] = True
                    send = 1
                    post(now + rng.between(0, w.max_link_delay) * int(mean_gap[l]) + rng.below(int(mean_gap[l]) // 4 + 1),
                         "gps", l)
                emit(EV_LPS_STEP, now, l, worker=k, exp_kind=STEP_UPDATE, exp_send=send, exp_acc=acc)
                applied += 1
                t_pull[l][k] = t[l]
                if with_pulls:
                    emit(EV_PULL, now, l, worker=k)
                post(now + period[l, k] + rng.below(int(period[l, k] // 8) + 1), "done", l, k)
            else:
                t_last[l] = t[l]
                outstanding[l] = False
                emit(EV_LPS_STEP, now, l, exp_kind=STEP_MERGE)
                k_cur[l] = rng.between(*w.k_range)
            busy_until[l] = now + rng.below(int(mean_gap[l]) + 1)
            kick(l, now)
        elif what == "gps":
            emit(EV_GPS_MERGE, now, l)
            post(now + rng.between(0, w.max_link_delay) * int(mean_gap[l]) + rng.below(int(mean_gap[l]) // 4 + 1),
                 "global", l)
        elif what == "global":
            emit(EV_ARRIVE_GLOBAL, now, l)
            fifo[l].append(("global",))
            kick(l, now)

    if max_stale > w.staleness_bound:
        raise AssertionError(f"worker staleness {max_stale} exceeds bound {w.staleness_bound}")
    events = np.array(out, dtype=TRACE_DTYPE)
    return Trace(w.name, L, W, k_initial, events, period)
