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


class _DeviceBytes:
    """Lets torch view memory that the library's arena owns (the CUDA array interface: address, length, bytes)."""

    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (int(nbytes),), "typestr": "|u1", "data": (int(ptr), False), "version": 2}


class RegionArena:
    """Device memory sorted by HBM region: the library's arena (halos_arena_*, include/halos.h), with the pointers it
    hands out wrapped as torch tensors.  need[c] is the number of bytes wanted in placement class c.  The search, the
    classification of slabs and the bookkeeping are the library's; nothing is measured or decided here."""

    def __init__(self, device, need: Sequence[int], max_bytes: Optional[int] = None, verbose: bool = False):
        self.device = torch.device(device)
        self.n_classes = len(need)
        with torch.cuda.device(self.device):
            torch.cuda.empty_cache()              # let the library see the memory torch's allocator is only caching
            self._h = B.halos_arena_create(need, max_bytes or 0)
        info = B.halos_arena_info(self._h, self.n_classes)
        self.n_regions = info["n_regions"]
        self.region_of_class = info["region_of_class"]
        self.info = info
        if verbose:
            import sys
            print(f"[arena] walked {info['walked_bytes'] >> 30} GiB, regions found: {self.n_regions}, same-region reference "
                  f"{info['same_region_gbps']:.0f} GB/s; slabs kept per class: {info['slabs_of_class']} in regions "
                  f"{self.region_of_class}", file=sys.stderr, flush=True)

    def alloc(self, cls: int, numel: int, dtype: torch.dtype) -> torch.Tensor:
        esize = torch.empty(0, dtype=dtype).element_size()
        nbytes = int(numel) * esize
        if nbytes == 0:
            return torch.empty(0, dtype=dtype, device=self.device)
        ptr = B.halos_arena_alloc(self._h, cls, nbytes)
        t = torch.as_tensor(_DeviceBytes(ptr, nbytes), device=self.device).view(dtype)
        assert t.data_ptr() == ptr
        return t

    def alloc_list(self, cls: int, numel: Sequence[int], dtype: torch.dtype) -> List[torch.Tensor]:
        return [self.alloc(cls, n, dtype) for n in numel]

    def close(self):
        """Frees the arena's memory: every tensor it handed out is dead after this."""
        if getattr(self, "_h", None):
            B.halos_arena_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


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
                 k_initial: Optional[Sequence[int]] = None, pull_buffers: bool = True, placement: str = "plain",
                 verbose: bool = False):
        """placement "plain": every tensor is its own torch allocation (or one arena per list if arena=True).
        placement "regions": momenta and third buffers / local models and deltas / worker model buffers are placed in
        three different HBM regions through a RegionArena (see the comment below for the measured reason)."""
        self.w = w
        self.device = torch.device(device)
        lay = w.layout
        self.numel = [int(x) for x in lay.numel]
        self.offsets = lay.offsets
        self.n = lay.total
        f32 = torch.float32
        self.region_arena = None
        self.hp = hp if hp is not None else B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0],
                                                                 cg_l=w.cg_l, cg_g=w.cg_g)
        self.snapshot = bool(self.hp.flags & B.FLAG_SNAPSHOT)
        self.defer_clear = bool(self.hp.flags & B.FLAG_DEFER_CLEAR)
        self.momentum_bf16 = bool(self.hp.flags & B.FLAG_BF16_MOMENTUM)
        mdt = torch.bfloat16 if self.momentum_bf16 else f32        # element type of the momentum arrays
        if placement == "regions":
            ddt_size = 4 if w.delta_dtype == "f32" else 2
            S = sum((n * 4 + 255) // 256 * 256 for n in self.numel)
            L = w.n_lps
            pool_bytes = w.pool_slots * S * ddt_size // 4
            # Measured on MI355X (all 243 assignments of m, theta, third buffer, delta, worker model to three regions,
            # bench.py --placement-search): everything in one region 5.4 TB/s, an even spread 6.2-6.4,
            # best (6.5) with the worker's model copy in a region of its own, momentum and third buffer in a second,
            # model and delta in the third.  That pattern also spreads the three written arrays of an update that leaves
            # the third buffer alone over three regions (6.3 instead of 6.0 TB/s for those).
            #   class 0: momenta m_l and third buffers acc_l (delayed momentum: the gradient buffer b_l takes m_l's
            #            place here, being what all but one update of a cycle read and write, and m_l moves to class 2)
            #   class 1: local models theta_l, the delta pool, and the GPS's momentum M (and gradient buffer)
            #   class 2: worker model buffers (pull destinations) and the GPS's model Theta
            # so that the GPS update (reads G = acc_l, M, Theta; writes M, Theta, acc_l) touches all three as well.
            cls_of = {"m": 2 if w.d_l > 1 else 0, "b": 0, "acc": 0, "theta": 1, "pool": 1, "M": 1, "B": 1,
                      "wm": 2, "Theta": 2}
            Sm = sum((n * 2 + 255) // 256 * 256 for n in self.numel) if self.momentum_bf16 else S
            size_of = {"Theta": S, "M": Sm, "B": S if w.d_g > 1 else 0, "theta": L * S, "m": L * Sm,
                       "b": L * S if w.d_l > 1 else 0, "acc": L * S, "pool": pool_bytes, "wm": L * S if pull_buffers else 0}
            need = [0, 0, 0]
            for role, c in cls_of.items():
                need[c] += size_of[role]
            self.region_arena = RegionArena(self.device, need, verbose=verbose)
            ra = self.region_arena
            mk = lambda dt=f32, role="theta": ra.alloc_list(cls_of[role], self.numel, dt)
        else:
            mk = lambda dt=f32, role="theta": alloc_tensor_list(self.numel, dt, self.device, arena)
        self.Theta = mk(role="Theta")
        self.M = None if self.hp.flags & B.FLAG_GPS_NO_MOMENTUM else mk(mdt, role="M")      # a momentum-free GPS has no M at all
        fill_initial_model(w, self.Theta)
        self.gps = B.halos_gps_create(self.numel, self.hp, self.Theta, self.M)
        self.gps_buffer = None
        if w.d_g > 1:
            self.gps_buffer = mk(role="B")
            B.halos_gps_set_momentum_delay(self.gps, w.d_g, self.gps_buffer)
        self.theta, self.m, self.acc, self.buffer, self.lps = [], [], [], [], []
        for l in range(w.n_lps):
            th, m, acc = mk(role="theta"), mk(mdt, role="m"), mk(role="acc")
            self.theta.append(th); self.m.append(m); self.acc.append(acc)
            h = B.halos_lps_create(self.gps, l, w.workers_per_lps, th, m, acc)
            if w.d_l > 1:
                self.buffer.append(mk(role="b"))
                B.halos_lps_set_momentum_delay(h, w.d_l, self.buffer[l])
            if k_initial is not None:
                B.halos_lps_set_threshold(h, int(k_initial[l]))
            self.lps.append(h)
        self.delta_dtype = {"f32": B.F32, "bf16": B.BF16, "f16": B.F16}[w.delta_dtype]
        ddt = {"f32": f32, "bf16": torch.bfloat16, "f16": torch.float16}[w.delta_dtype]
        self.pool = []
        for s in range(w.pool_slots):
            ts = mk(ddt, role="pool")
            fill_delta_slot(w, s, ts)
            self.pool.append(ts)
        self.pull_dst = [mk(role="wm") for _ in range(w.n_lps)] if pull_buffers else None
        # pointer arrays marshalled once: the replay loop then costs a few ctypes calls per event
        self._pool_ptrs = [B._ptrs(ts) for ts in self.pool]
        self._pull_ptrs = [B._ptrs(ts) for ts in self.pull_dst] if pull_buffers else None
        self._lib = B.load_library()
        if pull_buffers:       # every worker of an LPS hands its model back into that LPS's pull buffer
            for l, h in enumerate(self.lps):
                for k in range(w.workers_per_lps):
                    B.halos_lps_set_worker_model(h, k, self._pull_ptrs[l])
        torch.cuda.synchronize(self.device)

    def close(self):
        for h in self.lps:
            B.halos_lps_destroy(h)
        self.lps = []
        B.halos_gps_destroy(self.gps)
        self.gps = None
        if self.region_arena is not None:      # the state tensors are views into the arena's memory: drop them with it
            torch.cuda.synchronize(self.device)
            self.Theta = self.M = self.gps_buffer = self.pull_dst = None
            self.theta, self.m, self.acc, self.buffer, self.pool = [], [], [], [], []
            self.region_arena.close()
            self.region_arena = None

    # ------------------------------------------------------------------ replay
    def replay(self, events: np.ndarray, timed: bool = False, fuse_pull: bool = False, batch: int = 0):
        """Issue every record through the C ABI, in order, on the current stream.

        fuse_pull: an update step that is directly followed by the pull of the same worker is issued as one
        halos_lps_step_pull call (same results, one pass less).
        batch (2..4, needs fuse_pull): update steps of one server that follow each other directly in the trace (each with
        its pull; events of other servers in between do not touch this server's state) are issued as one
        halos_lps_step_batch call (same results; the server's state is read and written once for all of them).  A merge
        step whose server does nothing else until its next update step is held back and opens that update's pass (the
        returned model waits in the queue meanwhile; same results, the merge's own pass is saved).

        Returns (step_log, timings): step_log has one tuple (record index, kind, t, t_last, delta_ready,
        accumulated) per LPS step; timings (only if timed) maps a kernel label to a list of
        (start_event, end_event) pairs recorded around each launch on the launch stream.
        """
        lib, chk = self._lib, B._check
        stream = torch.cuda.current_stream(self.device)
        sp = stream.cuda_stream or None
        log = []
        from collections import defaultdict
        timings: Dict[str, list] = defaultdict(list)
        fuse_pull = fuse_pull and self._pull_ptrs is not None
        weighted = self.w.staleness_exponent > 0.0
        skip = -1
        consumed = set()
        # (with the norm monitors on, the library's batch call takes one item at a time: issue the steps as such)
        batch = batch if (fuse_pull and batch >= 2 and not (self.hp.flags & B.FLAG_NORMS)) else 0
        delayed = self.w.d_l > 1          # under a momentum delay only a merge and the one update behind it share a pass
        infos = (B.StepInfo * 4)()
        n_done = ctypes.c_int32()
        info = B.StepInfo()
        k_now = [None] * len(self.lps)
        # under deferred clearing: has this server merged and not accumulated since? (labels only; the library keeps its own state)
        restart = [False] * len(self.lps)
        if self.defer_clear:
            for j, hh in enumerate(self.lps):
                cnt = B.halos_lps_get_counters(hh)
                restart[j] = cnt["phase"] == B.PHASE_ACCUMULATING and cnt["t"] == cnt["t_last"] and cnt["t"] > 0
        held_merge = [None] * len(self.lps)      # record index of a merge step that waits to open the server's next pass
        seen_l = [B.halos_lps_get_momentum_delay(h)["seen"] for h in self.lps]
        seen_g = B.halos_gps_get_momentum_delay(self.gps)["seen"]

        def bracket(label, call):
            if not timed:
                return call()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            rc = call()
            b.record(stream)
            timings[label].append((a, b))
            return rc

        n_ev = len(events)

        def following_steps(i, l, limit):
            """Record indices of the update steps of server l that follow step i directly: l's own events after i must read
            pull, step, pull, step, ... (each pull for the worker of the step before it)."""
            group, want_pull, worker = [i], True, int(events[i]["worker"])
            pulls = []
            j = i + 1
            while j < n_ev and len(group) <= limit:
                e2 = events[j]
                if int(e2["lps"]) != l:
                    j += 1
                    continue
                k2 = int(e2["kind"])
                if want_pull:
                    if k2 != _PULL or int(e2["worker"]) != worker:
                        return None if not pulls else (group[:len(pulls)], pulls)
                    pulls.append(j)
                    want_pull = False
                    if len(group) == limit:
                        break
                else:
                    if k2 != _LPS_STEP or int(e2["exp_kind"]) != 1 or int(e2["k_cur"]) != int(events[i]["k_cur"]):
                        break
                    group.append(j)
                    worker = int(e2["worker"])
                    want_pull = True
                j += 1
            return (group[:len(pulls)], pulls) if pulls else None

        def merge_can_wait(i, l):
            """Is the server's next event after merge step i (arrivals of deltas aside) an update step?"""
            for j in range(i + 1, n_ev):
                e2 = events[j]
                if int(e2["lps"]) != l or int(e2["kind"]) == _ARRIVE_DELTA:
                    continue
                return int(e2["kind"]) == _LPS_STEP and int(e2["exp_kind"]) == 1
            return False

        for i in range(n_ev):
            if i == skip or i in consumed:
                continue
            ev = events[i]
            kind, l = int(ev["kind"]), int(ev["lps"])
            h = self.lps[l]
            if kind == _ARRIVE_DELTA:
                if weighted:
                    chk(lib.halos_lps_push_update_weighted(h, int(ev["worker"]), self._pool_ptrs[int(ev["slot"])], self.delta_dtype,
                                                           int(ev["staleness"]), synth.staleness_weight(self.w, int(ev["staleness"]))))
                else:
                    chk(lib.halos_lps_push_update(h, int(ev["worker"]), self._pool_ptrs[int(ev["slot"])],
                                                  self.delta_dtype, int(ev["staleness"])))
            elif kind == _LPS_STEP:
                k = int(ev["k_cur"])
                if k_now[l] != k:
                    chk(lib.halos_lps_set_threshold(h, k))
                    k_now[l] = k
                fused = False
                merge_label = "lps_merge_leave" if self.defer_clear else "lps_merge"
                lead, grp = 0, None
                if int(ev["exp_kind"]) == 2:
                    if batch and merge_can_wait(i, l):
                        held_merge[l] = i
                        continue
                    label = merge_label
                    restart[l] = self.defer_clear
                else:
                    lead = 1 if held_merge[l] is not None else 0
                    grp = following_steps(i, l, 1 if delayed else batch - lead) if batch and (lead or not delayed) else None
                    if lead and grp is None:        # this update shares no pass: the merge that waited goes first, on its own
                        chk(bracket(merge_label, lambda: lib.halos_lps_step(h, sp, ctypes.byref(info))))
                        log.append((held_merge[l], info.kind, info.t, info.t_last, info.delta_ready, info.accumulated))
                        held_merge[l], restart[l], lead = None, self.defer_clear, 0
                    if self.snapshot:      # third buffer untouched except by the update that completes the accumulation
                        label = "lps_update_freeze" if int(ev["exp_send"]) else "lps_update_noacc"
                    else:
                        label = "lps_update_acc" if int(ev["exp_accumulate"]) else "lps_update_noacc"
                        if restart[l] and int(ev["exp_accumulate"]):
                            label, restart[l] = "lps_update_restart", False      # stores 0 + step: the third buffer is not read
                    if self.w.d_l > 1:      # delayed momentum: an update that refreshes the momentum moves more bytes
                        seen = seen_l[l]
                        label += "_refresh" if seen + 1 == self.w.d_l else ("_first" if seen == 0 else "")
                        seen_l[l] = (seen + 1) % self.w.d_l
                    if fuse_pull and i + 1 < n_ev:
                        nx = events[i + 1]
                        fused = (int(nx["kind"]) == _PULL and int(nx["lps"]) == l and int(nx["worker"]) == int(ev["worker"]))
                    if grp is not None and len(grp[0]) >= 2 - lead:
                        steps, pulls = grp
                        # does the pass touch the third buffer? (snapshot form: only the update that completes the accumulation does)
                        any_acc = any(int(events[j]["exp_send" if self.snapshot else "exp_accumulate"]) for j in steps)
                        third = "merge" if lead else ("acc" if any_acc else "noacc")
                        cyc = "_refresh" if label.endswith("_refresh") else ("_first" if label.endswith("_first") else "")
                        blabel = f"lps_update_batch{len(steps)}_{third}{cyc}_pull"
                        chk(bracket(blabel, lambda: lib.halos_lps_step_batch(h, lead + len(steps), 1, sp, infos, ctypes.byref(n_done))))
                        assert n_done.value == lead + len(steps), (n_done.value, lead, len(steps))
                        if lead:
                            inf = infos[0]
                            log.append((held_merge[l], inf.kind, inf.t, inf.t_last, inf.delta_ready, inf.accumulated))
                            held_merge[l], restart[l] = None, False
                        for j, inf in zip(steps, list(infos)[lead:]):
                            log.append((j, inf.kind, inf.t, inf.t_last, inf.delta_ready, inf.accumulated))
                            if restart[l] and inf.accumulated:
                                restart[l] = False
                        consumed.update(steps[1:])
                        consumed.update(pulls)
                        continue
                if fused:
                    skip = i + 1
                    chk(bracket(label + "_pull", lambda: lib.halos_lps_step_pull(h, sp, ctypes.byref(info))))
                else:
                    chk(bracket(label, lambda: lib.halos_lps_step(h, sp, ctypes.byref(info))))
                log.append((i, info.kind, info.t, info.t_last, info.delta_ready, info.accumulated))
            elif kind == _GPS_MERGE:
                glabel = "gps_update_nomom" if self.M is None else "gps_update"
                if self.w.d_g > 1:
                    glabel += "_refresh" if seen_g + 1 == self.w.d_g else ("_first" if seen_g == 0 else "")
                    seen_g = (seen_g + 1) % self.w.d_g
                chk(bracket(glabel, lambda: lib.halos_gps_merge(self.gps, h, sp)))
            elif kind == _ARRIVE_GLOBAL:
                chk(lib.halos_lps_push_global(h))
            elif kind == _PULL:
                if self._pull_ptrs is not None:
                    chk(bracket("pull", lambda: lib.halos_pull_model(h, 0, self._pull_ptrs[l], sp)))
            else:
                raise ValueError(f"unknown event kind {kind}")
        log.sort(key=lambda rec: rec[0])          # batched steps were logged ahead of other servers' steps
        return log, (dict(timings) if timed else None)

    # ------------------------------------------------------------------ inspection
    def state_lists(self) -> Dict[str, List[torch.Tensor]]:
        out = {"Theta": self.Theta}
        if self.M is not None:
            out["M"] = self.M
        for l in range(len(self.theta)):
            out[f"theta{l}"] = self.theta[l]
            out[f"m{l}"] = self.m[l]
            out[f"aux{l}"] = self.acc[l]
            if self.buffer:
                out[f"buffer{l}"] = self.buffer[l]
        if self.gps_buffer is not None:
            out["B"] = self.gps_buffer
        return out

    def gather(self, name: str, flat_idx: torch.Tensor) -> np.ndarray:
        return gather_flat(self.state_lists()[name], self.offsets, flat_idx).float().cpu().numpy()     # bfloat16 -> float is exact

    def flat(self, name: str) -> np.ndarray:
        return torch.cat([t.reshape(-1) for t in self.state_lists()[name]]).float().cpu().numpy()
