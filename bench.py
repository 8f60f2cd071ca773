#!/usr/bin/env python3
"""Benchmark of the HALoS server-side update path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1b] [--also tiny,70m,...]

A "step" is one pass of the whole hot path over one batch of synthetic input: the replay of one
workload-sized slice of a seeded event trace (every worker-delta update, every accumulated-update
hand-over, GPS update, global-model merge and worker pull it contains), through the C ABI, with all
state resident in HBM.  One JSON line is printed.

  value        parameters updated per second = N x (LPS updates + GPS updates + merges) / elapsed,
               elapsed including the pull copies that belong to the same events
  roofline     the dominant kernel (the LPS update) against the 8 TB/s HBM peak, from HIP events
               recorded around every launch of the timed region on the launch stream
  cpu_baseline the CPU oracle, as it stands, timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# Algorithmic bytes per parameter per launch (fp32 state; delta fp32 or bf16).
def bytes_per_param(label: str, delta_dtype: str, delayed: bool, momentum_bytes: int = 4) -> int:
    """Algorithmic bytes per parameter of one launch, from the kernel label the harness gave it.

    Every array the event needs is read once and written once (fp32 = 4 bytes, a bf16 delta 2):
      lps_update_*  read g, theta; write theta (+4 with "_pull": the worker's model buffer).  "acc": the accumulated
                    update is read and written (+8); "noacc": it is in flight and untouched; "freeze": snapshot form,
                    read the snapshot and write theta_{t_last} - theta_t (+8).
                    Plain rule: momentum read and written (+8) -> 28/26 for "acc", 20/18 for "noacc".
                    Delayed momentum: "_first" writes the gradient buffer (+4), an inner update reads and writes it
                    (+8), "_refresh" reads it and reads and writes the momentum (+12).
      gps_update*   read G, Theta; write Theta and the returned model (16), plus the momentum (+8) or, delayed, the
                    same buffer / momentum terms as above.
      lps_merge     read theta and the returned model, write theta and the cleared third buffer (16);
                    "lps_merge_leave" does not clear (12), and the "restart" update after it writes the third buffer
                    without reading it (4 less than "acc").
      gps_update_nomom  no momentum array at all: read G, Theta; write Theta and the returned model (16).
      lps_update_batchK_*  K queued deltas in one pass: K deltas read, K worker models written, momentum, model and
                    (if any of them accumulates) the third buffer read and written once.  "_merge_": the pass opens with
                    the merge of the returned global model (read from the third buffer, which then restarts: +8, and
                    no separate 16-byte merge pass).
      pull          read and write a model (8).
    momentum_bytes = 2 (HALOS_FLAG_BF16_MOMENTUM): the momentum's read and write cost 4 instead of 8.
    """
    if label == "lps_merge":
        return 16
    if label == "lps_merge_leave":
        return 12
    if label == "gps_update_nomom":
        return 16
    if label == "pull":
        return 8
    parts = label.split("_")
    if label.startswith("lps_update_batch"):
        k = int(parts[2][len("batch"):])
        g = 4 if delta_dtype == "f32" else 2
        rule = (4 if "first" in parts else (12 if "refresh" in parts else 8)) if delayed else 2 * momentum_bytes
        return k * g + 8 + rule + (0 if "noacc" in parts else 8) + 4 * k
    if delayed:
        rule = 4 if "first" in parts else (12 if "refresh" in parts else 8)
    else:
        rule = 2 * momentum_bytes
    if label.startswith("gps_update"):
        return 16 + rule
    assert label.startswith("lps_update"), label
    g = 4 if delta_dtype == "f32" else 2
    third = 0 if "noacc" in parts else (4 if "restart" in parts else 8)
    return g + 8 + third + rule + (4 if "pull" in parts else 0)


# HBM traffic per parameter per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), valid
# only for the kernel source it was measured on: {sha256 of kernels.hip: {kernel label: bytes/param}}.
MEASURED_TRAFFIC: dict = {
    # profiles/lps_update_1b_hbm_traffic.md, profiles/lps_update_delayed_1b_dn.md, profiles/lps_update_1b_bf16_momentum.md
    "71e43cab53cd9043d20d729908c04d42e74f8a0f58ccdc5014d471e14fa755b4": {
        "1b:lps_update_acc_pull": 30.033,
        "1b:lps_update_noacc_pull": 22.031,
        "1b:lps_update_batch1_merge_pull": 30.031,
        "1b-dn:lps_update_acc_first_pull": 26.039,
        "1b-dn:lps_update_acc_pull": 30.032,
        "1b-dn:lps_update_acc_refresh_pull": 34.031,
        "1b-dn:lps_update_noacc_first_pull": 18.031,
        "1b-dn:lps_update_noacc_pull": 22.035,
        "1b-dn:lps_update_noacc_refresh_pull": 26.031,
        "1b+bf16m:lps_update_acc_pull": 26.031,
        "1b+bf16m:lps_update_noacc_pull": 18.031,
    },
}


def kernels_digest() -> str:
    with open(os.path.join(ROOT, "paper_2506_04531_amd", "csrc", "kernels.hip"), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def split_steps(events, n_updates_per_step: int, n_steps: int):
    """Cut a long trace into consecutive slices that each contain n_updates_per_step worker updates."""
    import numpy as np
    import synth
    is_upd = (events["kind"] == synth.EV_LPS_STEP) & (events["exp_kind"] == 1)
    cum = np.cumsum(is_upd)
    cuts = [0]
    for s in range(1, n_steps + 1):
        # slice s ends right after the pull that follows its last update (or after the update itself)
        pos = int(np.searchsorted(cum, s * n_updates_per_step, side="left")) + 1
        while pos < len(events) and events[pos]["kind"] == synth.EV_PULL and cum[pos] == s * n_updates_per_step:
            pos += 1
        cuts.append(min(pos, len(events)))
    return [events[cuts[i]:cuts[i + 1]] for i in range(n_steps)]


def run_workload(name: str, steps: int, warmup: int, verbose: bool, placement: str = "regions", fuse_pull: bool = True,
                 snapshot: bool = False, defer_clear: bool = False, gps_no_momentum: bool = False, batch: int = 0,
                 bf16_momentum: bool = False):
    import numpy as np
    import torch
    import synth
    from paper_2506_04531_amd.harness import Cluster

    w = synth.get_workload(name)
    long_w = w.scaled(w.layout, n_updates=w.n_updates * (steps + warmup))
    trace = synth.make_trace(long_w)
    slices = split_steps(trace.events, w.n_updates, steps + warmup)
    N = w.layout.total
    t0 = time.time()
    hp = None
    if bf16_momentum and (w.d_l > 1 or w.d_g > 1):
        raise SystemExit(f"bench.py: workload {name} uses a momentum delay; 16-bit momentum is not built for the delayed rule")
    if snapshot or defer_clear or gps_no_momentum or bf16_momentum:
        from paper_2506_04531_amd import binding as B
        flags = (B.FLAG_SNAPSHOT if snapshot else 0) | (B.FLAG_DEFER_CLEAR if defer_clear else 0) | \
                (B.FLAG_GPS_NO_MOMENTUM if gps_no_momentum else 0) | (B.FLAG_BF16_MOMENTUM if bf16_momentum else 0)
        hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, 0.0 if gps_no_momentum else w.beta_g, w.alpha, w.k_range[0],
                             cg_l=w.cg_l, cg_g=w.cg_g, flags=flags)
    c = Cluster(w, "cuda:0", k_initial=trace.k_initial, placement=placement, verbose=verbose, hp=hp)
    n_regions = c.region_arena.n_regions if c.region_arena is not None else 0
    if verbose:
        free_b, total_b = torch.cuda.mem_get_info()
        print(f"[bench] {name}: N={N} tensors={w.layout.n_tensors} state resident after {time.time() - t0:.1f}s, "
              f"{(total_b - free_b) / 2**30:.1f} GiB of device memory in use", file=sys.stderr, flush=True)
    try:
        for s in range(warmup):
            c.replay(slices[s], fuse_pull=fuse_pull, batch=batch)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        timings = {}
        for s in range(warmup, warmup + steps):
            log, tm = c.replay(slices[s], timed=True, fuse_pull=fuse_pull, batch=batch)
            for k, v in tm.items():
                timings.setdefault(k, []).extend(v)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
    finally:
        c.close()
        del c
        torch.cuda.empty_cache()

    kernels = {}
    for label, pairs in timings.items():
        if not pairs:
            continue
        ms = np.array([a.elapsed_time(b) for a, b in pairs], dtype=np.float64)
        bpp = bytes_per_param(label, w.delta_dtype, (w.d_g if label.startswith("gps") else w.d_l) > 1, 2 if bf16_momentum else 4)
        kernels[label] = {
            "launches": int(ms.size),
            "avg_ms": float(ms.mean()),
            "p10_ms": float(np.percentile(ms, 10)),
            "p50_ms": float(np.median(ms)),
            "p90_ms": float(np.percentile(ms, 90)),
            "bytes_per_param": bpp,
            "achieved_GBps": float(N * bpp / (ms.mean() * 1e-3) / 1e9),
            "params_per_s": float(N / (ms.mean() * 1e-3)),
            "total_ms": float(ms.sum()),
        }
    upd_labels = [k for k in kernels if k.startswith("lps_update")]
    per_launch = lambda k: int(k.split("_")[2][len("batch"):]) if k.startswith("lps_update_batch") else 1
    n_upd = sum(kernels[k]["launches"] * per_launch(k) for k in upd_labels)
    n_pull_events = kernels.get("pull", {}).get("launches", 0) + sum(
        kernels[k]["launches"] * per_launch(k) for k in upd_labels if k.endswith("_pull"))
    n_gps = sum(v["launches"] for k, v in kernels.items() if k.startswith("gps_update"))
    n_mrg = sum(v["launches"] for k, v in kernels.items() if k.startswith("lps_merge") or "_merge_" in k)   # own pass, or opening a batch
    updates = n_upd + n_gps + n_mrg
    value = N * updates / elapsed
    # dominant kernel: the LPS update variant that takes the most time
    dom = max(upd_labels, key=lambda k: kernels[k]["total_ms"])
    stored = MEASURED_TRAFFIC.get(kernels_digest())
    traffic = (stored or {}).get(f"{name}{'+bf16m' if bf16_momentum else ''}:{dom}")
    if traffic is not None:
        traffic_source = ("stored: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under profiles/, valid for the "
                          "kernel source with this sha256 only")
    elif stored is None:
        traffic_source = "none: the kernel source has changed since the counters under profiles/ were taken"
    else:
        traffic_source = "none: the counter runs under profiles/ cover the 1b workload (fp32 and bfloat16 momentum) and 1b-dn only"
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": kernels[dom]["achieved_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": kernels[dom]["achieved_GBps"] / HBM_PEAK_GBS,
        "traffic": (traffic * N) if traffic is not None else None, "traffic_source": traffic_source,
        "algorithmic_bytes_per_launch": N * kernels[dom]["bytes_per_param"],
        "avg_launch_ms": kernels[dom]["avg_ms"],
    }
    total_bytes = sum(v["launches"] * v["bytes_per_param"] * N for v in kernels.values())
    return {
        "workload": name, "description": w.description, "params": N, "tensors": w.layout.n_tensors,
        "delta_dtype": w.delta_dtype, "n_lps": w.n_lps, "workers_per_lps": w.workers_per_lps,
        "steps": steps, "warmup": warmup, "elapsed_s": elapsed, "ms_per_step": elapsed / steps * 1e3,
        "events_per_step": {"lps_update": n_upd / steps, "gps_update": n_gps / steps, "lps_merge": n_mrg / steps,
                            "pull": n_pull_events / steps},
        "params_updated_per_s": value,
        "whole_path_GBps": total_bytes / elapsed / 1e9,
        "whole_path_frac_of_peak": total_bytes / elapsed / 1e9 / HBM_PEAK_GBS,
        "kernels": kernels, "roofline": roofline, "placement": placement, "hbm_regions_found": n_regions,
        "fuse_pull": fuse_pull, "delta_form": "snapshot" if snapshot else "accumulator",
        "defer_clear": defer_clear, "gps_no_momentum": gps_no_momentum, "batch": batch,
        "momentum_dtype": "bf16" if bf16_momentum else "f32",
        "momentum_delay": {"d_l": w.d_l, "d_g": w.d_g},
    }


def end_model_ab(name: str, reps: int = 20, verbose: bool = True):
    """The update pass fed an fp32 delta against the same pass fed the worker's end model (halos_lps_push_end_model:
    the subtraction of Alg. 1's worker block done by the server), on the workload's tensor list with the same placement:
    one LPS, one worker, always accumulating, pull fused.  HIP events around every launch on the launch stream."""
    import numpy as np
    import torch
    import synth
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import RegionArena, fill_delta_slot, fill_initial_model

    w = synth.get_workload(name)
    numel = [int(x) for x in w.layout.numel]
    N = w.layout.total
    S = sum((n * 4 + 255) // 256 * 256 for n in numel)
    dev = torch.device("cuda:0")
    ra = RegionArena(dev, [2 * S, 3 * S, 2 * S], verbose=verbose)      # the placement classes of harness.Cluster
    f32 = torch.float32
    m, acc = ra.alloc_list(0, numel, f32), ra.alloc_list(0, numel, f32)
    th, inp, M = (ra.alloc_list(1, numel, f32) for _ in range(3))
    wm, Theta = ra.alloc_list(2, numel, f32), ra.alloc_list(2, numel, f32)
    fill_initial_model(w, Theta)
    fill_delta_slot(w, 0, inp)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, 1 << 30)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
    out = {}
    try:
        B.halos_lps_set_worker_model(lps, 0, wm)
        B.halos_pull_model(lps, False, wm)
        stream = torch.cuda.current_stream(dev)
        for mode, bpp in (("fp32_delta", 32), ("end_model", 36)):
            push = (lambda: B.halos_lps_push_update(lps, 0, inp, B.F32)) if mode == "fp32_delta" else \
                   (lambda: B.halos_lps_push_end_model(lps, 0, inp))
            pairs = []
            for i in range(reps + 2):
                push()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                B.halos_lps_step_pull(lps)
                b.record(stream)
                if i >= 2:
                    pairs.append((a, b))
            torch.cuda.synchronize()
            ms = np.array([a.elapsed_time(b) for a, b in pairs])
            out[mode] = {"launches": int(ms.size), "avg_ms": float(ms.mean()), "bytes_per_param": bpp,
                         "achieved_GBps": float(N * bpp / (ms.mean() * 1e-3) / 1e9),
                         "frac_of_peak": float(N * bpp / (ms.mean() * 1e-3) / 1e9 / HBM_PEAK_GBS)}
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
        torch.cuda.synchronize()
        del Theta, M, th, m, inp, acc, wm
        ra.close()
        torch.cuda.empty_cache()
    out["workload"] = name
    out["note"] = ("end_model: the server reads the worker's start and end models (8 B) instead of an fp32 delta (4 B) "
                   "and the worker skips its own 12 B/parameter subtraction pass")
    return out


def graph_ab(reps: int = 300):
    """Launch-bound case: one accumulation cycle of the Tiny workload's shape (one LPS, two workers, K = 4: four
    updates with the model handed back, the GPS update, the merge -- six kernels of 7-10 us) issued call by call
    against the same cycle captured once into a HIP graph and replayed.  Same results (tests/test_gpu_graph.py);
    the difference is launch overhead."""
    import torch
    import synth
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import alloc_tensor_list, fill_delta_slot, fill_initial_model

    w = synth.get_workload("tiny")
    numel = [int(x) for x in w.layout.numel]
    N, K, n_workers = w.layout.total, 4, 2
    dev = torch.device("cuda:0")
    mk = lambda: alloc_tensor_list(numel, torch.float32, dev)
    Theta, M, th, m, acc, g = mk(), mk(), mk(), mk(), mk(), mk()
    wm = [mk() for _ in range(n_workers)]
    fill_initial_model(w, Theta)
    fill_delta_slot(w, 0, g)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, K)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, n_workers, th, m, acc)
    try:
        for k in range(n_workers):
            B.halos_lps_set_worker_model(lps, k, wm[k])

        def cycle():
            for k in range(K):
                B.halos_lps_push_update(lps, k % n_workers, g, B.F32)
                B.halos_lps_step_pull(lps)
            B.halos_gps_merge(gps, lps)
            B.halos_lps_push_global(lps)
            B.halos_lps_step(lps)

        for _ in range(3):
            cycle()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            cycle()
        torch.cuda.synchronize()
        eager = (time.perf_counter() - t0) / reps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            cycle()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        replay = (time.perf_counter() - t0) / reps
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
    bytes_per_cycle = N * (K * 32 + 24 + 16)
    return {"cycle": f"{K} updates with fused pull + GPS update + merge on the tiny layout ({N} parameters, fp32 deltas)",
            "eager_us_per_cycle": eager * 1e6, "graph_us_per_cycle": replay * 1e6,
            "eager_GBps": bytes_per_cycle / eager / 1e9, "graph_GBps": bytes_per_cycle / replay / 1e9,
            "eager_params_per_s": N * (K + 2) / eager, "graph_params_per_s": N * (K + 2) / replay}


def cpu_baseline(name: str, budget_elements: int = 1 << 22):
    """Time the CPU oracle, as it stands, on a bounded sample: every event of one workload-sized trace, on
    `budget_elements` evenly spaced parameters of the workload, single thread.  `value` is the canonical figure (fp64,
    literal form: whole replay, wall clock around the replay loop, the Python-side hand-over of deltas included);
    `per_event` is the time inside the oracle's own C++ handlers per event type (its stopwatch), in fp64 and in the fp32
    same-order form, so that each GPU kernel has the oracle's figure for the same event beside it."""
    import numpy as np
    import torch
    import synth
    from oracle import FORM_ACCUMULATOR, FORM_LITERAL, HalosOracle
    from oracle.replay import replay
    from synth.tensors import scale_f32

    w = synth.get_workload(name)
    trace = synth.make_trace(w)
    N = w.layout.total
    n_s = min(N, budget_elements)
    idx = (np.arange(n_s, dtype=np.int64) * (N // n_s))
    tidx = torch.from_numpy(idx)
    theta0 = synth.normal_at(w.seed, 0, tidx, scale_f32(w.init_sigma)).numpy()
    scale = torch.from_numpy(synth.delta_scales(w)[w.layout.tensor_of(idx)])
    pool = {}
    for s in range(w.pool_slots):
        g = synth.normal_at(w.seed, 1 + s, tidx, scale)
        pool[s] = (synth.to_bf16_bits(g).numpy() if w.delta_dtype == "bf16" else
                   synth.to_f16(g).numpy() if w.delta_dtype == "f16" else g.numpy())
    ev = trace.events
    ev = ev[ev["kind"] != synth.EV_PULL]          # the oracle's pull is a host copy for tests, not timed work
    g_bytes = 4 if w.delta_dtype == "f32" else 2
    # algorithmic bytes per parameter of the same events in fp32 state (what the GPU kernels are charged); fp64 state doubles the state part
    alg = {"lps_update": g_bytes + 24, "gps_update": 24, "lps_merge": 16}
    out, per_event = None, {}
    for precision, form, tag in ((64, FORM_LITERAL, "f64"), (32, FORM_ACCUMULATOR, "f32")):
        o = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha,
                        K=trace.k_initial, precision=precision, form=form)
        if w.d_l > 1:
            for l in range(w.n_lps):
                o.set_delay(l, w.d_l)
        if w.d_g > 1:
            o.set_delay(-1, w.d_g)
        t0 = time.perf_counter()
        log = replay(o, ev, lambda s: pool[s])
        dt = time.perf_counter() - t0
        updates = len(log) + trace.count(synth.EV_GPS_MERGE)
        for kind, (sec, calls) in o.stopwatch().items():
            if calls:
                per_event.setdefault(kind, {})[tag] = {
                    "events": calls, "params_per_s": n_s * calls / sec,
                    "GBps_fp32_algorithmic": n_s * calls * alg[kind] / sec / 1e9}
        if precision == 64:
            out = {"value": n_s * updates / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
                   "sample": f"{n_s} evenly spaced parameters of the {name} workload, all {updates} update/merge events of one "
                             f"trace (fp64, literal form, single thread, {dt:.1f} s wall clock including the hand-over of every "
                             f"delta); host has {os.cpu_count()} logical cores"}
        o.close()
    out["per_event"] = per_event
    out["per_event_note"] = ("time inside the oracle's own loops per event type (stopwatch in the C++ handlers, no Python), fp64 literal "
                             "form and fp32 same-order form; GB/s counts the fp32 algorithmic bytes of the event, as for the GPU kernels")
    return out


def ceilings_mode(gib: float, reps: int, quick: bool = False):
    """`bench.py --ceilings`: what this device's memory system delivers to plain streaming kernels, by HBM region.

    Places buffers in each HBM region the library's arena finds, then times halos_probe_streams (read some buffers,
    write others, no arithmetic, the access pattern of the update kernels) for pure reads, pure writes, copies and the
    stream mix of the update pass with fused pull (4 read, 4 written) under several placements; then the same mix for
    other tile sizes (128-bit accesses per thread and stream before anything is consumed: 1 .. 16, tiles of 4 .. 64 KiB),
    other grid sizes, and with the streams' start addresses staggered inside ONE region.  Prints tables (plain text)."""
    import torch
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import RegionArena

    nbytes = int(gib * (1 << 30)) // (1 << 16) * (1 << 16)
    n = nbytes // 4
    dev = torch.device("cuda:0")
    per_region = 8
    pad = 64 << 20                                             # room to shift a buffer's start by up to 64 MiB
    assert nbytes + pad <= (1 << 31), "a buffer and its padding must fit one 2 GiB slab"
    slabs_per_buffer = 1 if 2 * (nbytes + pad) > (1 << 31) else 0.5
    need = int(per_region * slabs_per_buffer * (1 << 31))
    arena = RegionArena(dev, [need, need, need], verbose=True)
    if arena.n_regions < 3:
        print(f"only {arena.n_regions} region(s) found: placements below collapse onto fewer regions")
    X, Y, Z = ([arena.alloc(r, n + pad // 4, torch.float32).zero_() for _ in range(per_region)] for r in range(3))
    torch.cuda.synchronize()

    def run(reads, writes, unroll=0, shift=None):
        """shift: per-stream start offsets in bytes (reads first, then writes)."""
        bufs = list(reads) + list(writes)
        ptrs = [b.data_ptr() + (shift[i] if shift else 0) for i, b in enumerate(bufs)]
        return B.halos_probe_streams(ptrs[:len(reads)], ptrs[len(reads):], nbytes, reps, unroll)

    if quick:       # three patterns only, one kernel each: for counter runs (rocprofv3 --pmc), where every dispatch is listed
        for name, rd, wr in (("4 reads, one region", X[:4], []), ("4 writes over three regions", [], [X[4], Y[4], Z[4], X[5]]),
                             ("4 reads + 4 writes, the benchmark's placement", [X[0], X[1], X[2], Y[0]], [X[4], X[5], Y[4], Z[4]])):
            v = run(rd, wr)
            print(f"{name:60s} {v:8.0f} GB/s {v / HBM_PEAK_GBS:7.1%}")
        del X, Y, Z
        arena.close()
        return

    def table(title, rows):
        print(f"\n{title}")
        print(f"{'pattern':104s} {'GB/s':>8s} {'of 8 TB/s':>10s}")
        for name, v in rows:
            print(f"{name:104s} {v:8.0f} {v / HBM_PEAK_GBS:10.1%}")

    rows = [("1 read", run([X[0]], [])), ("2 reads, one region", run([X[0], X[1]], [])),
            ("4 reads, one region", run(X[:4], [])), ("4 reads over three regions", run([X[0], Y[0], Z[0], X[1]], [])),
            ("1 write", run([], [X[4]])), ("2 writes, one region", run([], [X[4], X[5]])),
            ("4 writes, one region", run([], X[4:8])), ("4 writes over three regions", run([], [X[4], Y[4], Z[4], X[5]])),
            ("copy (1 read, 1 write), one region", run([X[0]], [X[4]])), ("copy, two regions", run([X[0]], [Y[4]]))]
    r4, w4 = max(rows[2][1], rows[3][1]), max(rows[6][1], rows[7][1])
    mixes = [
        ("4 reads + 4 writes, all in one region", X[:4], X[4:8]),
        ("4 reads + 4 writes, spread evenly (reads X Y Z X, writes X Y Z Y)", [X[0], Y[0], Z[0], X[1]], [X[4], Y[4], Z[4], Y[5]]),
        ("4 reads + 4 writes, as the benchmark places the update pass (reads X X X Y, writes X X Y Z)",
         [X[0], X[1], X[2], Y[0]], [X[4], X[5], Y[4], Z[4]]),
        ("4 reads + 4 writes, no region both read and written (reads X X X X, writes Y Z Y Z)", X[:4], [Y[4], Z[4], Y[5], Z[5]]),
    ]
    for name, rd, wr in mixes:
        rows.append((name, run(rd, wr)))
    table(f"buffers of {nbytes / (1 << 30):.2f} GiB, {reps} timed sweeps each, 16 KiB tiles, default grid", rows)
    pred = 30.0 / (14.0 / r4 + 16.0 / w4)
    print(f"best 4-stream read rate {r4:.0f} GB/s, best 4-stream write rate {w4:.0f} GB/s; a pass that reads 14 and writes "
          f"16 bytes per parameter at those rates, if reads and writes did not disturb each other: {pred:.0f} GB/s = "
          f"{pred / HBM_PEAK_GBS:.1%} of 8 TB/s")

    # tile size x grid size, for the benchmark's placement of the 4 + 4 mix and for 3 + 3 (GPS update: reads X Y Z, writes X Y Z)
    bench_mix = ([X[0], X[1], X[2], Y[0]], [X[4], X[5], Y[4], Z[4]])
    gps_mix = ([X[0], Y[0], Z[0]], [X[4], Y[4], Z[4]])
    for title, (rd, wr) in (("4 reads + 4 writes in the benchmark's placement", bench_mix), ("3 reads + 3 writes, one per region", gps_mix)):
        print(f"\n{title}: GB/s by tile size (rows: 128-bit accesses per thread and stream) and workgroups per compute unit (columns)")
        bpcs = (1, 2, 4, 8, 16, 32)
        print("unroll  tile " + "".join(f"{b:>8d}" for b in bpcs))
        for unroll in (1, 2, 4, 8, 16):
            vals = []
            for bpc in bpcs:
                B.halos_set_launch_config(bpc, -1)
                vals.append(run(rd, wr, unroll))
            print(f"{unroll:6d} {unroll * 4:3d}KiB " + "".join(f"{v:8.0f}" for v in vals))
        B.halos_set_launch_config(1, -1)

    # staggered starts inside ONE region: does shifting the streams against each other do what separate regions do?
    rows = []
    for label, step in (("no shift", 0), ("256 B", 256), ("4 KiB", 4 << 10), ("68 KiB", 68 << 10), ("1 MiB + 4 KiB", (1 << 20) + (4 << 10)),
                        ("5 MiB + 20 KiB", (5 << 20) + (20 << 10)), ("7 MiB", 7 << 20)):
        shift = [k * step for k in range(8)]
        rows.append((f"4 reads + 4 writes in one region, stream k shifted by k x {label}", run(X[:4], X[4:8], 0, shift)))
    for label, step in (("no shift", 0), ("68 KiB", 68 << 10), ("5 MiB + 20 KiB", (5 << 20) + (20 << 10))):
        shift = [k * step for k in range(8)]
        rows.append((f"benchmark placement, stream k shifted by k x {label}", run(bench_mix[0], bench_mix[1], 0, shift)))
    table("start addresses staggered", rows)
    del X, Y, Z
    arena.close()


def placement_search_mode(elements: int, dtype_name: str):
    """`bench.py --placement-search`: time the library's fused update pass (halos_lps_step_pull: read delta, m, theta,
    third buffer; write m, theta, third buffer, worker model) for every assignment of those five arrays to the HBM regions
    the arena finds, and print the assignments grouped by pattern (regions renamed X, Y, Z in order of first use, arrays
    in the order m, theta, third, delta, worker model).  This is how the benchmark's placement classes were chosen."""
    import itertools
    from collections import defaultdict
    import torch
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import RegionArena

    n = elements
    dev = torch.device("cuda:0")
    dtype = B.BF16 if dtype_name == "bf16" else B.F32
    ddt = torch.bfloat16 if dtype_name == "bf16" else torch.float32
    need = 7 * n * 4 + (1 << 30)
    arena = RegionArena(dev, [need, need, need], verbose=True)
    if arena.n_regions < 3:
        print(f"only {arena.n_regions} region(s) found: nothing to compare")
        return
    pool = []
    for r in range(3):
        pool.append({"delta": [arena.alloc(r, n, ddt).zero_()], "m": [arena.alloc(r, n, torch.float32)],
                     "theta": [arena.alloc(r, n, torch.float32)], "third": [arena.alloc(r, n, torch.float32)],
                     "model": [arena.alloc(r, n, torch.float32)]})
    gps_bufs = {"Theta": [arena.alloc(0, n, torch.float32).zero_()], "M": [arena.alloc(0, n, torch.float32)]}
    bpp = (4 if dtype == B.F32 else 2) + 28
    roles = ("m", "theta", "third", "delta", "model")
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 1 << 30)
    groups = defaultdict(list)
    for assign in itertools.product(range(3), repeat=5):
        bufs = dict(gps_bufs)
        for role, r in zip(roles, assign):
            bufs[role] = pool[r][role]
        gps = B.halos_gps_create([n], hp, bufs["Theta"], bufs["M"])
        lps = B.halos_lps_create(gps, 0, 1, bufs["theta"], bufs["m"], bufs["third"])
        try:
            B.halos_lps_set_worker_model(lps, 0, bufs["model"])
            B.halos_lps_push_update(lps, 0, bufs["delta"], dtype)
            B.halos_lps_step_pull(lps)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(3):
                B.halos_lps_push_update(lps, 0, bufs["delta"], dtype)
                B.halos_lps_step_pull(lps)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / 3
        finally:
            B.halos_lps_destroy(lps)
            B.halos_gps_destroy(gps)
        rename, pat = {}, []
        for r in assign:
            if r not in rename:
                rename[r] = "XYZ"[len(rename)]
            pat.append(rename[r])
        groups["".join(pat)].append(n * bpp / ms / 1e6)
    print(f"update pass with fused pull, {n} elements per array, {dtype_name} delta, {bpp} B/parameter")
    print("pattern (m theta third delta model)   mean GB/s    min     max   assignments")
    for pat, v in sorted(groups.items(), key=lambda kv: -sum(kv[1]) / len(kv[1])):
        print(f"  {pat}                              {sum(v) / len(v):8.1f} {min(v):7.1f} {max(v):7.1f}   {len(v)}")
    del pool, gps_bufs
    arena.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="1b", help="headline workload: tiny, 70m, 160m, 410m, 1b; paper-70m/160m/410m (the paper's cluster model); "
                         "1b-dn, 410m-dn, paper-410m-dn (the same with delayed Nesterov momentum, d_l=16, d_g=2)")
    ap.add_argument("--also", default="tiny,70m,160m,410m,1b-dn",
                    help="comma-separated further workloads reported under 'workloads' ('' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--nontemporal", type=int, default=-1)
    ap.add_argument("--placement", default="regions", choices=["regions", "plain"],
                    help="regions: state arrays sorted into three HBM regions (harness.Cluster); plain: torch allocations")
    ap.add_argument("--no-fuse-pull", action="store_true",
                    help="issue every worker pull as its own copy instead of fusing it into the update pass")
    ap.add_argument("--snapshot", action="store_true",
                    help="form the accumulated update by subtracting the snapshot theta_{t_last} (the Delta of Alg. 1's LPS block as "
                         "written) instead of keeping a running sum: fewer bytes per update, larger rounding error")
    ap.add_argument("--defer-clear", action="store_true",
                    help="merges leave the third buffer (12 B/parameter instead of 16); the next update restarts it")
    ap.add_argument("--gps-no-momentum", action="store_true",
                    help="the global server keeps no momentum (beta_g = 0, Sec. 5.4): 16 B/parameter per GPS update instead of 24")
    ap.add_argument("--bf16-momentum", action="store_true",
                    help="both tiers keep their momentum in bfloat16, rounded at every update (HALOS_FLAG_BF16_MOMENTUM: 4 B/parameter "
                         "less per update, results differ by the rounding); workloads with a momentum delay are left out")
    ap.add_argument("--batch", type=int, default=4,
                    help="2..4: update steps of one server that follow each other directly go through one pass "
                         "(halos_lps_step_batch; same results bit for bit); 0 = every step its own pass")
    ap.add_argument("--no-plain-placement", action="store_true",
                    help="skip the second run of the headline workload with ordinary allocations instead of the region-sorted arena")
    ap.add_argument("--no-variants-ab", action="store_true",
                    help="skip the runs of the headline workload with one option changed at a time")
    ap.add_argument("--no-end-model-ab", action="store_true",
                    help="skip the A/B of the update pass fed a delta vs fed the worker's end model")
    ap.add_argument("--no-graph-ab", action="store_true",
                    help="skip the call-by-call vs HIP-graph comparison on the launch-bound tiny shape")
    ap.add_argument("--quiet", action="store_true")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark: print what the memory system delivers to plain streaming kernels "
                         "(reads, writes, the update pass's mix; by region, tile size, grid size and start offsets)")
    ap.add_argument("--ceilings-gib", type=float, default=1.0, help="buffer size for --ceilings")
    ap.add_argument("--ceilings-reps", type=int, default=5)
    ap.add_argument("--ceilings-quick", action="store_true", help="with --ceilings: only pure reads, pure writes and the update pass's mix")
    ap.add_argument("--placement-search", action="store_true",
                    help="instead of the benchmark: time the fused update pass for every assignment of its arrays to the HBM regions")
    ap.add_argument("--search-elements", type=int, default=1 << 29)
    ap.add_argument("--search-dtype", default="f32", choices=["f32", "bf16"])
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU: every server copy lives in one device's memory and links are a "
              "seeded schedule; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    import paper_2506_04531_amd as halos
    halos.load_library()
    if args.blocks_per_cu or args.nontemporal >= 0:
        halos.halos_set_launch_config(args.blocks_per_cu, args.nontemporal)
    if args.ceilings:
        return ceilings_mode(args.ceilings_gib, args.ceilings_reps, args.ceilings_quick)
    if args.placement_search:
        return placement_search_mode(args.search_elements, args.search_dtype)

    variant = dict(snapshot=args.snapshot, defer_clear=args.defer_clear, gps_no_momentum=args.gps_no_momentum, batch=args.batch,
                   bf16_momentum=args.bf16_momentum)
    head = run_workload(args.workload, args.steps, args.warmup, not args.quiet, args.placement, not args.no_fuse_pull, **variant)
    others = []
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        if args.bf16_momentum and name.endswith("-dn"):
            continue
        others.append(run_workload(name, args.steps, args.warmup, not args.quiet, args.placement, not args.no_fuse_pull, **variant))
    plain = None
    if args.placement == "regions" and not args.no_plain_placement:      # what a caller with ordinary allocations gets
        r = run_workload(args.workload, args.steps, args.warmup, not args.quiet, "plain", not args.no_fuse_pull, **variant)
        plain = {"placement": "plain", "value": r["params_updated_per_s"], "ms_per_step": r["ms_per_step"],
                 "whole_path_GBps": r["whole_path_GBps"], "roofline": r["roofline"],
                 "note": "same workload, every tensor an ordinary allocation of the framework's caching allocator"}
    vab = None
    if not args.no_variants_ab:         # the same workload with one option changed at a time (one warm-up + one timed step each)
        vab = {}
        for tag, kw in (("single_steps", dict(variant, batch=0)), ("defer_clear", dict(variant, defer_clear=True)),
                        ("gps_no_momentum", dict(variant, gps_no_momentum=True)), ("snapshot_form", dict(variant, snapshot=True)),
                        ("bf16_momentum", dict(variant, bf16_momentum=True))):
            if tag == "bf16_momentum" and args.workload.endswith("-dn"):
                continue
            r = run_workload(args.workload, 1, 1, False, args.placement, not args.no_fuse_pull, **kw)
            vab[tag] = {"value": r["params_updated_per_s"], "ms_per_step": r["ms_per_step"], "whole_path_GBps": r["whole_path_GBps"],
                        "kernels": {k: {"launches": v["launches"], "avg_ms": v["avg_ms"], "bytes_per_param": v["bytes_per_param"],
                                        "achieved_GBps": v["achieved_GBps"]} for k, v in r["kernels"].items()}}
        vab["note"] = ("single_steps: every update its own pass (no halos_lps_step_batch); defer_clear: merges leave the third buffer "
                       "(HALOS_FLAG_DEFER_CLEAR, same results); gps_no_momentum: beta_g = 0 without a momentum array (Sec. 5.4; "
                       "another optimizer setting); snapshot_form: Delta by subtraction (HALOS_FLAG_SNAPSHOT; rounds differently); "
                       "bf16_momentum: both tiers' momentum in bfloat16 (HALOS_FLAG_BF16_MOMENTUM; an option of this library that "
                       "changes results by the rounding)")
    ab = None if args.no_end_model_ab else end_model_ab(args.workload, verbose=not args.quiet)
    gab = None if args.no_graph_ab else graph_ab()
    cpu = None if args.no_cpu_baseline else cpu_baseline(args.workload)

    def brief(r):
        return {k: r[k] for k in ("workload", "params", "delta_dtype", "momentum_delay", "ms_per_step", "params_updated_per_s",
                                  "whole_path_GBps", "whole_path_frac_of_peak", "kernels", "roofline")}

    line = {
        "metric": "params_updated_per_sec", "value": head["params_updated_per_s"], "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {head['description']}", "params": head["params"],
                   "tensors": head["tensors"], "n_lps": head["n_lps"], "workers_per_lps": head["workers_per_lps"],
                   "delta_dtype": head["delta_dtype"], "events_per_step": head["events_per_step"],
                   "placement": head["placement"], "hbm_regions_found": head["hbm_regions_found"],
                   "fuse_pull": head["fuse_pull"], "delta_form": head["delta_form"],
                   "defer_clear": head["defer_clear"], "gps_no_momentum": head["gps_no_momentum"], "batch": head["batch"],
                   "momentum_dtype": head["momentum_dtype"], "momentum_delay": head["momentum_delay"]},
        "roofline": head["roofline"],
        "plain_placement": plain,
        "cpu_baseline": cpu,
        "whole_path_GBps": head["whole_path_GBps"],
        "kernels": head["kernels"],
        "workloads": [brief(r) for r in others],
        "variants_ab": vab,
        "end_model_ab": ab,
        "tiny_graph_ab": gab,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
