"""Replay harness: holds a whole simulated cluster (GPS, every LPS, a pool of worker deltas) in one
GPU's memory and drives the C ABI from an event trace.

PyTorch is used for device memory, streams and events only; every update, merge and copy goes
through libhalos.  Nothing here imports the CPU oracle.
"""
from __future__ import annotations

import ctypes
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import synth
from synth.tensors import scale_f32

from . import binding as B

_ARRIVE_DELTA, _LPS_STEP, _GPS_MERGE, _ARRIVE_GLOBAL, _PULL = (
    synth.EV_ARRIVE_DELTA, synth.EV_LPS_STEP, synth.EV_GPS_MERGE, synth.EV_ARRIVE_GLOBAL, synth.EV_PULL)


def alloc_tensor_list(numel: Sequence[int], dtype: torch.dtype, device, arena: bool = False) -> List[torch.Tensor]:
    """One tensor per layout entry: separate allocations, or views into one arena at 256-byte aligned offsets."""
    if not arena:
        return [torch.empty(int(n), dtype=dtype, device=device) for n in numel]
    esize = torch.empty(0, dtype=dtype).element_size()
    align = 256 // esize
    offs, total = [], 0
    for n in numel:
        offs.append(total)
        total += (int(n) + align - 1) // align * align
    buf = torch.empty(max(total, 1), dtype=dtype, device=device)
    return [buf[o:o + int(n)] for o, n in zip(offs, numel)]


def fill_initial_model(w: synth.Workload, tensors: List[torch.Tensor]) -> None:
    off = w.layout.offsets
    for i, t in enumerate(tensors):
        if t.numel():
            synth.normal_flat(w.seed, 0, int(off[i]), t.numel(), scale_f32(w.init_sigma), out=t)


def fill_delta_slot(w: synth.Workload, slot: int, tensors: List[torch.Tensor]) -> None:
    off, sc = w.layout.offsets, synth.delta_scales(w)
    for i, t in enumerate(tensors):
        if t.numel():
            synth.normal_flat(w.seed, 1 + slot, int(off[i]), t.numel(), sc[i], out=t)


def gather_flat(tensors: List[torch.Tensor], offsets: np.ndarray, flat_idx: torch.Tensor) -> torch.Tensor:
    """Values at packed flat indices (sorted or not) of a tensor list, as one 1-D tensor in index order."""
    dev = tensors[0].device
    idx = flat_idx.to(dev)
    off_t = torch.as_tensor(offsets, device=dev)
    tid = torch.searchsorted(off_t, idx, right=True) - 1
    out = torch.empty(idx.numel(), dtype=tensors[0].dtype, device=dev)
    for i in torch.unique(tid).tolist():
        sel = (tid == i).nonzero(as_tuple=True)[0]
        out[sel] = tensors[i][idx[sel] - int(offsets[i])]
    return out


class Cluster:
    """GPS + n_lps LPSs + delta pool for one workload, resident on `device`."""

    def __init__(self, w: synth.Workload, device="cuda:0", arena: bool = False, hp: Optional[B.HParams] = None,
                 k_initial: Optional[Sequence[int]] = None, pull_buffers: bool = True):
        self.w = w
        self.device = torch.device(device)
        lay = w.layout
        self.numel = [int(x) for x in lay.numel]
        self.offsets = lay.offsets
        self.n = lay.total
        f32 = torch.float32
        mk = lambda dt=f32: alloc_tensor_list(self.numel, dt, self.device, arena)
        self.Theta, self.M = mk(), mk()
        fill_initial_model(w, self.Theta)
        self.hp = hp if hp is not None else B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0])
        self.gps = B.halos_gps_create(self.numel, self.hp, self.Theta, self.M)
        self.theta, self.m, self.acc, self.lps = [], [], [], []
        for l in range(w.n_lps):
            th, m, acc = mk(), mk(), mk()
            self.theta.append(th); self.m.append(m); self.acc.append(acc)
            h = B.halos_lps_create(self.gps, l, w.workers_per_lps, th, m, acc)
            if k_initial is not None:
                B.halos_lps_set_threshold(h, int(k_initial[l]))
            self.lps.append(h)
        self.delta_dtype = B.BF16 if w.delta_dtype == "bf16" else B.F32
        ddt = torch.bfloat16 if w.delta_dtype == "bf16" else f32
        self.pool = []
        for s in range(w.pool_slots):
            ts = mk(ddt)
            fill_delta_slot(w, s, ts)
            self.pool.append(ts)
        self.pull_dst = [mk() for _ in range(w.n_lps)] if pull_buffers else None
        # pointer arrays marshalled once: the replay loop then costs a few ctypes calls per event
        self._pool_ptrs = [B._ptrs(ts) for ts in self.pool]
        self._pull_ptrs = [B._ptrs(ts) for ts in self.pull_dst] if pull_buffers else None
        self._lib = B.load_library()
        torch.cuda.synchronize(self.device)

    def close(self):
        for h in self.lps:
            B.halos_lps_destroy(h)
        self.lps = []
        B.halos_gps_destroy(self.gps)
        self.gps = None

    # ------------------------------------------------------------------ replay
    def replay(self, events: np.ndarray, timed: bool = False):
        """Issue every record through the C ABI, in order, on the current stream.

        Returns (step_log, timings): step_log has one tuple (record index, kind, t, t_last, delta_ready,
        accumulated) per LPS step; timings (only if timed) maps a kernel label to a list of
        (start_event, end_event) pairs recorded around each launch on the launch stream.
        """
        lib, chk = self._lib, B._check
        stream = torch.cuda.current_stream(self.device)
        sp = stream.cuda_stream or None
        log = []
        timings: Dict[str, list] = {"lps_update_acc": [], "lps_update_noacc": [], "gps_update": [], "lps_merge": [],
                                    "pull": []}
        info = B.StepInfo()
        k_now = [None] * len(self.lps)

        def bracket(label, call):
            if not timed:
                return call()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            rc = call()
            b.record(stream)
            timings[label].append((a, b))
            return rc

        for i in range(len(events)):
            ev = events[i]
            kind, l = int(ev["kind"]), int(ev["lps"])
            h = self.lps[l]
            if kind == _ARRIVE_DELTA:
                chk(lib.halos_lps_push_update(h, int(ev["worker"]), self._pool_ptrs[int(ev["slot"])],
                                              self.delta_dtype, int(ev["staleness"])))
            elif kind == _LPS_STEP:
                k = int(ev["k_cur"])
                if k_now[l] != k:
                    chk(lib.halos_lps_set_threshold(h, k))
                    k_now[l] = k
                if int(ev["exp_kind"]) == 2:
                    label = "lps_merge"
                else:
                    label = "lps_update_acc" if int(ev["exp_accumulate"]) else "lps_update_noacc"
                chk(bracket(label, lambda: lib.halos_lps_step(h, sp, ctypes.byref(info))))
                log.append((i, info.kind, info.t, info.t_last, info.delta_ready, info.accumulated))
            elif kind == _GPS_MERGE:
                chk(bracket("gps_update", lambda: lib.halos_gps_merge(self.gps, h, sp)))
            elif kind == _ARRIVE_GLOBAL:
                chk(lib.halos_lps_push_global(h))
            elif kind == _PULL:
                if self._pull_ptrs is not None:
                    chk(bracket("pull", lambda: lib.halos_pull_model(h, 0, self._pull_ptrs[l], sp)))
            else:
                raise ValueError(f"unknown event kind {kind}")
        return log, (timings if timed else None)

    # ------------------------------------------------------------------ inspection
    def state_lists(self) -> Dict[str, List[torch.Tensor]]:
        out = {"Theta": self.Theta, "M": self.M}
        for l in range(len(self.theta)):
            out[f"theta{l}"] = self.theta[l]
            out[f"m{l}"] = self.m[l]
            out[f"aux{l}"] = self.acc[l]
        return out

    def gather(self, name: str, flat_idx: torch.Tensor) -> np.ndarray:
        return gather_flat(self.state_lists()[name], self.offsets, flat_idx).cpu().numpy()

    def flat(self, name: str) -> np.ndarray:
        return torch.cat([t.reshape(-1) for t in self.state_lists()[name]]).cpu().numpy()
