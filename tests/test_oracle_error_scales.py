"""Pins for the oracle's error-scale bookkeeping -- the denominator of the fp64 parity tolerance.

The GPU state is compared with the fp64 oracle relative to a per-element error scale that the oracle carries next
to every value (tests/parity_util.py).  A scale that is too generous would silently loosen that comparison, so the
scales themselves are pinned here, on the CPU, against values worked out by hand from the stated rules
(tests/golden/*.json) and against bounds that hold for any trace.  Nothing here re-types the oracle's loop.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle as O
from oracle import HalosOracle, FORM_LITERAL, FORM_ACCUMULATOR
from parity_util import snapshot_form_view

HERE = os.path.dirname(os.path.abspath(__file__))
F32 = np.float32
BOTH_FORMS = [FORM_LITERAL, FORM_ACCUMULATOR]
SCALE_IDS = {"theta": O.THETA + O.SCALE, "m": O.MOM + O.SCALE, "aux": O.AUX + O.SCALE,
             "Theta": O.GPS_THETA + O.SCALE, "M": O.GPS_MOM + O.SCALE}
RAW_IDS = {"snap": O.SNAP, "frozen": O.FROZEN, "inbox": O.INBOX}


def _eq(got, want, what):
    assert np.array_equal(got, np.asarray(want, dtype=np.float64)), (what, got, want)


@pytest.mark.parametrize("precision", [32, 64])
@pytest.mark.parametrize("form", BOTH_FORMS)
def test_worked_example_scales_and_raw_state(precision, form):
    """The worked example of Alg. 1, with the error scales and the raw snapshot / frozen update / returned model
    after selected steps, all derived by hand."""
    with open(os.path.join(HERE, "golden", "alg1_worked_example.json")) as f:
        ex = json.load(f)
    o = HalosOracle(np.array(ex["theta0"], dtype=F32), ex["n_lps"], eta_l=ex["eta_l"], beta_l=ex["beta_l"],
                    cg_l=ex["cg_l"], eta_g=ex["eta_g"], beta_g=ex["beta_g"], cg_g=ex["cg_g"], alpha=ex["alpha"],
                    K=ex["K"], precision=precision, form=form)
    checked = 0
    for i, step in enumerate(ex["script"]):
        l = step["lps"]
        if step["op"] == "delta":
            o.arrive_delta(l, step["worker"], np.array(step["g"], dtype=F32))
        elif step["op"] == "step":
            o.lps_step(l)
        elif step["op"] == "gps":
            o.gps_receive(l)
        elif step["op"] == "global":
            o.arrive_global(l)
        for name, want in step.get("expect_state", {}).items():
            if name == "scales":
                for arr, sc in want.items():
                    _eq(o.get(SCALE_IDS[arr], l), sc, (i, "scale", arr))
                    checked += 1
            elif name == "snap" and form == FORM_ACCUMULATOR:
                continue        # the running-sum form keeps no meaningful snapshot between sends
            else:
                _eq(o.get(RAW_IDS[name], l), want, (i, name))
                checked += 1
    assert checked >= 30
    fin = ex["final"]["scales"]
    for l in range(ex["n_lps"]):
        for arr in ("theta", "m", "aux"):
            _eq(o.get(SCALE_IDS[arr], l), fin[arr][l], ("final", arr, l))
    _eq(o.get(SCALE_IDS["Theta"]), fin["Theta"], "final Theta")
    _eq(o.get(SCALE_IDS["M"]), fin["M"], "final M")


def test_snapshot_form_view_follows_the_phases():
    """What an implementation that keeps theta_{t_last} in its third buffer must hold, by phase, on the worked example:
    the snapshot while accumulating, the frozen update once sent, the returned model afterwards -- and the scale it
    is judged on (the model's while it is a difference of two models)."""
    with open(os.path.join(HERE, "golden", "alg1_worked_example.json")) as f:
        ex = json.load(f)
    o = HalosOracle(np.array(ex["theta0"], dtype=F32), ex["n_lps"], eta_l=ex["eta_l"], beta_l=ex["beta_l"],
                    cg_l=ex["cg_l"], eta_g=ex["eta_g"], beta_g=ex["beta_g"], cg_g=ex["cg_g"], alpha=ex["alpha"],
                    K=ex["K"], precision=64, form=FORM_LITERAL)
    # hand-derived: (script index, lps) -> (value, scale) of the snapshot-form third buffer right after that entry
    want = {
        (1, 0): ([8, -4, 0, 16], [8, 6, 3, 16]),            # accumulating: theta_0, judged on scale(theta)
        (3, 0): ([3, 2, 1, 8], [8, 6, 3, 16]),              # sent: G, judged on max(scale(G), scale(theta))
        (8, 0): ([5, -6, -1, 8], [8, 6, 3, 16]),            # returning: Theta_1 with scale(Theta)
        (13, 0): ([4.5, -6.5, -1.5, 7.5], [8, 7, 3, 16]),   # merged: the post-merge model is the new snapshot
        (10, 1): ([4, 6, 4, 6], [8, 10, 4, 16]),
        (20, 1): ([2.5, -11, -4.5, 6], [8, 12, 5, 16]),
    }
    seen = 0
    for i, step in enumerate(ex["script"]):
        l = step["lps"]
        if step["op"] == "delta":
            o.arrive_delta(l, step["worker"], np.array(step["g"], dtype=F32))
        elif step["op"] == "step":
            o.lps_step(l)
        elif step["op"] == "gps":
            o.gps_receive(l)
        else:
            o.arrive_global(l)
        if (i, l) in want:
            val, sc = snapshot_form_view(o, l)
            _eq(val, want[(i, l)][0], (i, l, "value"))
            _eq(sc, want[(i, l)][1], (i, l, "scale"))
            seen += 1
    assert seen == len(want)


@pytest.mark.parametrize("precision", [32, 64])
@pytest.mark.parametrize("form", BOTH_FORMS)
def test_scale_rules_with_momentum_rate_and_coefficient(precision, form):
    """beta, eta, cg away from 0 and 1: values cancel, scales do not shrink; G's scale travels to the GPS and back."""
    with open(os.path.join(HERE, "golden", "scale_rules_example.json")) as f:
        ex = json.load(f)["plain"]
    o = HalosOracle(np.array(ex["theta0"], dtype=F32), 1, eta_l=ex["eta_l"], beta_l=ex["beta_l"], cg_l=ex["cg_l"],
                    eta_g=ex["eta_g"], beta_g=ex["beta_g"], cg_g=ex["cg_g"], alpha=ex["alpha"], K=ex["K"],
                    precision=precision, form=form)
    for k, st in enumerate(ex["steps"]):
        o.arrive_delta(0, 0, np.array(st["g"], dtype=F32))
        info = o.lps_step(0)
        assert info.sent == (1 if k == len(ex["steps"]) - 1 else 0)
        _eq(o.get(O.THETA), st["theta"], (k, "theta")); _eq(o.get(O.MOM), st["m"], (k, "m"))
        _eq(o.get(O.AUX), st["acc"], (k, "acc"))
        _eq(o.get(SCALE_IDS["theta"]), st["sc_theta"], (k, "sc_theta"))
        _eq(o.get(SCALE_IDS["m"]), st["sc_m"], (k, "sc_m"))
        _eq(o.get(SCALE_IDS["aux"]), st["sc_aux"], (k, "sc_aux"))
    o.gps_receive(0)
    g = ex["after_gps"]
    _eq(o.get(O.GPS_THETA), g["Theta"], "Theta"); _eq(o.get(O.GPS_MOM), g["M"], "M"); _eq(o.get(O.AUX), g["inbox"], "inbox")
    _eq(o.get(SCALE_IDS["Theta"]), g["sc_Theta"], "sc_Theta"); _eq(o.get(SCALE_IDS["M"]), g["sc_M"], "sc_M")
    _eq(o.get(SCALE_IDS["aux"]), g["sc_aux"], "sc_aux after gps")
    o.arrive_global(0); o.lps_step(0)
    m = ex["after_merge"]
    _eq(o.get(O.THETA), m["theta"], "merged theta")
    _eq(o.get(SCALE_IDS["theta"]), m["sc_theta"], "sc_theta after merge")
    _eq(o.get(SCALE_IDS["aux"]), m["sc_aux"], "sc_aux after merge")


@pytest.mark.parametrize("precision", [32, 64])
def test_scale_rules_of_the_delayed_rule(precision):
    """Delayed momentum: the buffer's scale adds magnitudes, the momentum's scale rises to their mean at the refresh,
    and a refresh step that cancels to zero still carries the scale of its terms."""
    with open(os.path.join(HERE, "golden", "scale_rules_example.json")) as f:
        ex = json.load(f)["delayed"]
    o = HalosOracle(np.array(ex["theta0"], dtype=F32), 1, eta_l=ex["eta_l"], beta_l=ex["beta_l"], cg_l=ex["cg_l"],
                    eta_g=1.0, beta_g=0.0, alpha=0.0, K=1 << 30, precision=precision, form=FORM_ACCUMULATOR)
    o.set_delay(0, ex["d"])
    for k, st in enumerate(ex["steps"]):
        o.arrive_delta(0, 0, np.array(st["g"], dtype=F32))
        o.lps_step(0)
        _eq(o.get(O.THETA), st["theta"], (k, "theta")); _eq(o.get(O.MOM), st["m"], (k, "m"))
        _eq(o.get(SCALE_IDS["theta"]), st["sc_theta"], (k, "sc_theta"))
        _eq(o.get(SCALE_IDS["m"]), st["sc_m"], (k, "sc_m"))
        _eq(o.get(O.BUFFER + O.SCALE), st["sc_buffer"], (k, "sc_buffer"))
        if "buffer" in st:
            _eq(o.get(O.BUFFER), st["buffer"], (k, "buffer"))


def _seeded_run(d_l=1, d_g=1, n=2048, seed=17):
    """A seeded trace replayed event by event; after every event the magnitudes of everything the oracle holds are
    folded into one elementwise running maximum (`seen`), and every delta applied into it as well."""
    import synth
    from dataclasses import replace
    w = replace(synth.get_workload("410m").scaled(synth.flat_layout(n), n_updates=80), d_l=d_l, d_g=d_g)
    tr = synth.make_trace(w, seed=seed)
    idx = torch.arange(n, dtype=torch.int64)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
    pool = {s: synth.normal_at(w.seed, 1 + s, idx, synth.tensors.scale_f32(w.delta_sigma)).numpy() for s in range(w.pool_slots)}
    o = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha,
                    K=tr.k_initial, precision=64, form=FORM_ACCUMULATOR)
    if d_l > 1:
        for l in range(w.n_lps):
            o.set_delay(l, d_l)
    if d_g > 1:
        o.set_delay(-1, d_g)
    seen = np.abs(theta0.astype(np.float64))
    arrays = [(O.GPS_THETA, 0), (O.GPS_MOM, 0)] + [(what, l) for l in range(w.n_lps) for what in (O.THETA, O.MOM, O.AUX)]

    def check_lower_bounds(tag):
        for what, l in arrays:
            v, sc = np.abs(o.get(what, l)), o.get(what + O.SCALE, l)
            assert np.all(sc >= v), (tag, what, l)

    last_scales = {a: o.get(a[0] + O.SCALE, a[1]) for a in arrays}
    for i, ev in enumerate(tr.events):
        kind, l = int(ev["kind"]), int(ev["lps"])
        if kind == synth.EV_ARRIVE_DELTA:
            g = pool[int(ev["slot"])]
            o.arrive_delta(l, int(ev["worker"]), g)
            seen = np.maximum(seen, np.abs(g.astype(np.float64)))
        elif kind == synth.EV_LPS_STEP:
            o.set_K(l, int(ev["k_cur"]))
            o.lps_step(l)
        elif kind == synth.EV_GPS_MERGE:
            o.gps_receive(l)
        elif kind == synth.EV_ARRIVE_GLOBAL:
            o.arrive_global(l)
        for what, ll in arrays:
            seen = np.maximum(seen, np.abs(o.get(what, ll)))
        check_lower_bounds(i)
        for a in arrays:                      # scales never shrink, except the accumulated update's at its restart
            sc = o.get(a[0] + O.SCALE, a[1])
            if a[0] != O.AUX:
                assert np.all(sc >= last_scales[a]), (i, a)
            last_scales[a] = sc
    return w, o, seen, arrays


@pytest.mark.parametrize("d_l,d_g", [(1, 1), (4, 2)])
def test_scales_are_bounded_on_both_sides_on_a_seeded_trace(d_l, d_g):
    """For every element and array: |x| <= scale at every event (checked inside the run), scales other than the
    accumulated update's never shrink, and at the end scale <= C * (largest magnitude that element has ever shown in
    any array or delta), with C = the product of the two rules' gains  max(1, |eta| (|cg| + |beta|) [d for the
    buffer's summed magnitudes]).  An over-generous scale breaks the upper bound on the many elements whose values stay small."""
    w, o, seen, arrays = _seeded_run(d_l, d_g)
    f = lambda eta, beta, d: max(1.0, abs(eta) * ((1.0 - beta) + beta)) * (d if d > 1 else 1)
    C = f(w.eta_l, w.beta_l, d_l) * f(w.eta_g, w.beta_g, d_g)
    for what, l in arrays:
        sc = o.get(what + O.SCALE, l)
        assert np.all(sc <= C * seen * (1 + 1e-12)), (what, l, float((sc / np.maximum(seen, 1e-300)).max()), C)
    # and the scales are of the order of the values themselves, not orders of magnitude above them
    for what, l in arrays:
        v, sc = np.abs(o.get(what, l)), o.get(what + O.SCALE, l)
        if np.any(v > 0):
            assert np.median(sc) <= 20 * np.median(v[v > 0]), (what, l)
