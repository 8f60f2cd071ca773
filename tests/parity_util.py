"""Shared helpers of the GPU parity tests: run the CPU oracle on (a sample of) a workload and
compare a GPU cluster's state with it."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

import oracle as O
import synth
from oracle import HalosOracle
from oracle.replay import replay as oracle_replay
from synth.tensors import scale_f32

# fp32 state vs the fp64 reference: tolerance of the benchmark definition (max relative error per
# element after the full event sequence).  "Relative" is taken against the element's error scale as
# the oracle tracks it: the largest magnitude among the values the element has held and the operands
# that were combined to make them (delta, momentum term, the two terms of a step, the merged global
# model).  fp32 rounding errors are proportional to those operand magnitudes -- a step whose two terms
# nearly cancel is tiny, its rounding error is not -- so this is the scale on which 2^-24-sized errors
# accumulate.  The scale is never smaller than the element's final magnitude.
REL_TOL = 1e-5


def sample_indices(lay: synth.Layout, n_random: int, seed: int = 0, tile: int = 4096, edge: int = 6) -> np.ndarray:
    """Random packed flat indices plus the places where indexing mistakes show: the first and last
    `edge` elements of every tensor, and of the first, second and last tile of every tensor."""
    rng = np.random.default_rng(seed)
    total = lay.total
    picks = [rng.integers(0, total, size=min(n_random, total), dtype=np.int64)]
    off, numel = lay.offsets, lay.numel
    for i in range(lay.n_tensors):
        n = int(numel[i])
        if n == 0:
            continue
        marks = {0, n}
        for b in (tile, 2 * tile, (n // tile) * tile, ((n - 1) // tile) * tile):
            if 0 < b < n:
                marks.add(b)
        loc = []
        for b in marks:
            loc.extend(range(max(0, b - edge), min(n, b + edge)))
        picks.append(off[i] + np.array(sorted(set(loc)), dtype=np.int64))
    return np.unique(np.concatenate(picks))


def oracle_run(w: synth.Workload, trace: synth.Trace, idx: Optional[np.ndarray], precision: int, form: int,
               momentum_bf16: bool = False):
    """Replay `trace` through the oracle on the packed flat indices `idx` (None = every element)."""
    lay = w.layout
    if idx is None:
        idx = np.arange(lay.total, dtype=np.int64)
    tidx = torch.from_numpy(idx)
    theta0 = synth.normal_at(w.seed, 0, tidx, scale_f32(w.init_sigma)).numpy()
    scale = torch.from_numpy(synth.delta_scales(w)[lay.tensor_of(idx)])
    cache: Dict[int, np.ndarray] = {}

    def delta(slot: int) -> np.ndarray:
        if slot not in cache:
            g = synth.normal_at(w.seed, 1 + slot, tidx, scale)
            cache[slot] = (synth.to_bf16_bits(g).numpy() if w.delta_dtype == "bf16" else
                           synth.to_f16(g).numpy() if w.delta_dtype == "f16" else g.numpy())
        return cache[slot]

    o = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g,
                    alpha=w.alpha, K=trace.k_initial, cg_l=w.cg_l, cg_g=w.cg_g, precision=precision, form=form,
                    momentum_bf16=momentum_bf16)
    if w.d_l > 1:
        for l in range(w.n_lps):
            o.set_delay(l, w.d_l)
    if w.d_g > 1:
        o.set_delay(-1, w.d_g)
    log = oracle_replay(o, trace.events, delta, weight_of=lambda st: synth.staleness_weight(w, st))
    return o, log


def snapshot_form_view(o: HalosOracle, l: int, with_scale: bool = True):
    """What the third buffer of an implementation that keeps the SNAPSHOT theta_{t_last} (instead of a running sum)
    holds, assembled from the oracle's raw state by protocol phase: the snapshot while accumulating, the frozen G
    once sent, the returned model afterwards.  Its error scale while it is G: G was formed by subtracting two
    model-sized numbers, so rounding errors of the model's size flowed into it."""
    phase = o.counters(l)["phase"]
    if phase == 0:
        return o.get(O.SNAP, l), (o.get(O.THETA + O.SCALE, l) if with_scale else None)
    if phase == 1:
        sc = np.maximum(o.get(O.AUX + O.SCALE, l), o.get(O.THETA + O.SCALE, l)) if with_scale else None
        return o.get(O.FROZEN, l), sc
    return o.get(O.INBOX, l), (o.get(O.AUX + O.SCALE, l) if with_scale else None)


def oracle_state(o: HalosOracle, n_lps: int, with_scale: bool = True, snapshot_form: bool = False):
    """Every state array of the oracle (value, error scale).  snapshot_form: the third buffers as an implementation
    that keeps theta_{t_last} holds them (only meaningful for an oracle created with FORM_LITERAL)."""
    names = {"Theta": (O.GPS_THETA, 0), "M": (O.GPS_MOM, 0)}
    for l in range(n_lps):
        names[f"theta{l}"] = (O.THETA, l)
        names[f"m{l}"] = (O.MOM, l)
        if not snapshot_form:
            names[f"aux{l}"] = (O.AUX, l)
    # gradient buffers of the delayed momentum: defined only while a cycle is open (after a refresh an
    # implementation may leave anything there until the next update overwrites it)
    for l in range(n_lps):
        if o.delay_seen(l) > 0:
            names[f"buffer{l}"] = (O.BUFFER, l)
    if o.delay_seen(-1) > 0:
        names["B"] = (O.GPS_BUFFER, 0)
    out = {}
    for k, (what, l) in names.items():
        out[k] = (o.get(what, l), o.get(what + O.SCALE, l) if with_scale else None)
    if snapshot_form:
        for l in range(n_lps):
            out[f"aux{l}"] = snapshot_form_view(o, l, with_scale)
    return out


def literal_metrics(values: Dict[str, np.ndarray], ref: Dict[str, tuple], floor_rms: float = 1e-3):
    """The tolerance read literally, for the record: per array, the largest |x - ref| / max(|ref|, floor_rms * rms(ref))
    and the largest |x - ref|.  Returns {array: (relative, absolute)} plus the overall worst under "*"."""
    out = {}
    worst_rel = worst_abs = 0.0
    for k, (x_ref, _scale) in ref.items():
        x = values[k].astype(np.float64)
        if not x.size:
            continue
        rms = float(np.sqrt(np.mean(x_ref * x_ref)))
        diff = np.abs(x - x_ref)
        rel = float((diff / np.maximum(np.abs(x_ref), max(floor_rms * rms, 1e-300))).max())
        out[k] = (rel, float(diff.max()))
        worst_rel, worst_abs = max(worst_rel, rel), max(worst_abs, float(diff.max()))
    out["*"] = (worst_rel, worst_abs)
    return out


def literal_where_not_tiny(values: Dict[str, np.ndarray], ref: Dict[str, tuple], floor_rms: float = 0.1) -> float:
    """Largest |x - ref| / |ref| over the elements whose reference magnitude is at least floor_rms of their array's
    rms -- the tolerance read literally, on every element that is not close to zero."""
    worst = 0.0
    for k, (x_ref, _scale) in ref.items():
        if not x_ref.size:
            continue
        rms = float(np.sqrt(np.mean(x_ref * x_ref)))
        sel = np.abs(x_ref) >= floor_rms * rms
        if rms > 0 and sel.any():
            x = values[k].astype(np.float64)
            worst = max(worst, float((np.abs(x[sel] - x_ref[sel]) / np.abs(x_ref[sel])).max()))
    return worst


def report_literal(tag: str, gpu_values: Dict[str, np.ndarray], o32: HalosOracle, ref64: Dict[str, tuple], n_lps: int) -> float:
    """Print, for the record, the tolerance read literally (error relative to the reference VALUE, floored at 1e-3 of
    the array's rms, and the plain absolute error) for the GPU state and for the fp32 oracle, both against fp64.
    Returns the GPU's literal relative error over the elements that are not close to zero (>= 10 % of the array's rms),
    which callers hold to the same 1e-5."""
    g = literal_metrics(gpu_values, ref64)["*"]
    o = literal_metrics({k: v[0].astype(np.float32) for k, v in oracle_state(o32, n_lps, with_scale=False).items()
                         if k in ref64}, ref64)["*"]
    big = literal_where_not_tiny(gpu_values, ref64)
    print(f"[parity] {tag}: literal metric |x-ref|/max(|ref|, 1e-3 rms): GPU vs fp64 {g[0]:.3g} (max abs {g[1]:.3g}); "
          f"fp32 oracle vs fp64 {o[0]:.3g} (max abs {o[1]:.3g}); GPU vs fp64 over elements >= 10% of rms: {big:.3g}", flush=True)
    return big


def compare_state(gpu_values: Dict[str, np.ndarray], ref: Dict[str, tuple], bitwise: bool):
    """Returns (worst relative error, number of differing elements, name of the worst array).

    bitwise=True  compares with an fp32 oracle that performs the same operations in the same order:
                  relative error against |ref| itself, and the count of elements whose bits differ.
    bitwise=False compares with the fp64 reference using the path-scale metric described above.
    """
    worst, worst_name, n_diff = 0.0, "", 0
    for k, (x_ref, scale) in ref.items():
        x = gpu_values[k].astype(np.float64)
        assert x.shape == x_ref.shape, k
        assert np.all(np.isfinite(x)), k
        if bitwise:
            r32 = x_ref.astype(np.float32)
            n_diff += int((gpu_values[k].view(np.uint32) != r32.view(np.uint32)).sum())
            denom = np.maximum(np.abs(x_ref), 1e-30)
        else:
            denom = np.maximum(np.maximum(np.abs(x_ref), scale), 1e-30)
            n_diff += int((x != x_ref).sum())
        err = float((np.abs(x - x_ref) / denom).max()) if x.size else 0.0
        if err > worst:
            worst, worst_name = err, k
    return worst, n_diff, worst_name


def check_step_logs(trace: synth.Trace, gpu_log, oracle_log):
    """Event ordering and protocol decisions must agree exactly: GPU library, oracle, and the schedule
    generator's own bookkeeping."""
    assert gpu_log == oracle_log
    ev = trace.events
    steps = ev[ev["kind"] == synth.EV_LPS_STEP]
    assert len(steps) == len(gpu_log)
    for rec, (i, kind, t, t_last, ready, acc) in zip(steps, gpu_log):
        assert (kind, t, t_last, ready, acc) == (int(rec["exp_kind"]), int(rec["exp_t"]), int(rec["exp_t_last"]),
                                                 int(rec["exp_send"]), int(rec["exp_accumulate"]))
