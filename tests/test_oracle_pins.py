"""Pins for the CPU oracle: closed forms, library special cases, invariants and a
hand-derived worked example.  None of these re-type the oracle's own loop; each
compares it with something fixed by the paper or by mathematics."""
import json
import os

import numpy as np
import pytest
import scipy.signal
import torch

import oracle as O
from oracle import HalosOracle, FORM_LITERAL, FORM_ACCUMULATOR

HERE = os.path.dirname(os.path.abspath(__file__))
BOTH_FORMS = [FORM_LITERAL, FORM_ACCUMULATOR]
F32 = np.float32


def single(theta0, **kw):
    base = dict(eta_l=1.0, beta_l=0.0, eta_g=1.0, beta_g=0.0, alpha=0.0, K=1 << 30)
    base.update(kw)
    return HalosOracle(np.asarray(theta0, dtype=F32), 1, **base)


def apply(o, l, w, g):
    o.arrive_delta(l, w, np.asarray(g, dtype=F32))
    return o.lps_step(l)


# ---------------------------------------------------------------- local SGD special case
@pytest.mark.parametrize("precision", [32, 64])
def test_zero_momentum_unit_rate_adopts_worker_end_model(precision):
    """One LPS, one worker, beta_l = 0, eta_l = 1: after the update the server model is the
    worker's end model (Alg. 1: the worker's delta and the LPS's ModelUpdate, App. E) -- plain local SGD."""
    rng = np.random.default_rng(0)
    start = (rng.integers(-2000, 2000, 257) / 64.0).astype(F32)        # dyadic: every op exact
    end = (rng.integers(-2000, 2000, 257) / 64.0).astype(F32)
    o = single(start, precision=precision)
    apply(o, 0, 0, start - end)                                         # pseudo-gradient = start - end
    assert np.array_equal(o.get(O.THETA), end.astype(np.float64))
    # non-dyadic data: equal up to the rounding of g = start - end in fp32
    start = rng.normal(0, 0.02, 1000).astype(F32)
    end = (start + rng.normal(0, 1e-3, 1000)).astype(F32)
    o = single(start, precision=64)
    apply(o, 0, 0, start - end)
    assert np.max(np.abs(o.get(O.THETA) - end)) <= np.spacing(F32(0.1))


# ---------------------------------------------------------------- K identical deltas
@pytest.mark.parametrize("form", BOTH_FORMS)
@pytest.mark.parametrize("precision", [32, 64])
def test_k_identical_deltas_accumulate_to_k_eta_g(form, precision):
    K, eta = 6, 0.25
    g = (np.arange(-8, 9) / 128.0).astype(F32)
    theta0 = (np.arange(17) / 4.0).astype(F32)
    o = single(theta0, eta_l=eta, K=K, form=form, precision=precision)
    for k in range(K):
        info = apply(o, 0, k % 3, g)
        assert info.kind == 1 and info.t == k + 1 and info.sent == (1 if k == K - 1 else 0)
    assert np.array_equal(o.get(O.AUX), K * eta * g.astype(np.float64))          # G = -Delta = K eta g
    assert np.array_equal(o.get(O.THETA), theta0 - K * eta * g.astype(np.float64))
    assert o.counters(0)["phase"] == 1                                           # Delta frozen, in flight


# ---------------------------------------------------------------- geometric momentum series
def test_constant_delta_gives_geometric_momentum_series_exactly_in_fp32():
    """beta = 0.5, eta = 0.25, g = k * 2^-10: every fp32 operation is exact for n <= 12, so the
    closed forms  m_n = g (1 - beta^n)/(1 - beta)  and
    theta_n = theta_0 - eta g [ n cg + beta/(1-beta) ( n - beta (1-beta^n)/(1-beta) ) ]  hold bit for bit."""
    beta, eta = 0.5, 0.25
    g = (np.arange(-5, 6) / 1024.0).astype(F32)
    theta0 = np.linspace(-1, 1, 11).astype(F32)
    for precision in (32, 64):
        o = single(theta0, eta_l=eta, beta_l=beta, precision=precision, form=FORM_ACCUMULATOR)
        for n in range(1, 13):
            apply(o, 0, 0, g)
            gd = g.astype(np.float64)
            m_closed = gd * (1 - beta ** n) / (1 - beta)
            th_closed = theta0 - eta * gd * (n * (1 - beta) + beta / (1 - beta) * (n - beta * (1 - beta ** n) / (1 - beta)))
            assert np.array_equal(o.get(O.MOM), m_closed), n
            assert np.array_equal(o.get(O.THETA), th_closed), n
            assert np.array_equal(o.get(O.AUX), theta0 - th_closed), n


@pytest.mark.parametrize("beta,eta", [(0.9, 0.2), (0.5, 0.15), (0.0, 1.0), (0.99, 0.01)])
def test_momentum_recursion_matches_iir_filter(beta, eta):
    """For ANY delta sequence, m is g filtered by 1/(1 - beta z^-1) and theta is theta_0 minus the running
    sum of eta[(1-beta) g + beta m]  (App. E, LPS rule).  scipy.signal.lfilter is the library reference."""
    rng = np.random.default_rng(3)
    T, n = 50, 33
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    bf, ef = float(F32(beta)), float(F32(eta))                # the oracle receives fp32 hyper-parameters
    cg = float(F32(1) - F32(beta))
    m_ref = scipy.signal.lfilter([1.0], [1.0, -bf], G.astype(np.float64), axis=0)
    theta_ref = theta0 - np.cumsum(ef * (cg * G.astype(np.float64) + bf * m_ref), axis=0)
    o = single(theta0, eta_l=eta, beta_l=beta)
    for k in range(T):
        apply(o, 0, 0, G[k])
        np.testing.assert_allclose(o.get(O.MOM), m_ref[k], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.THETA), theta_ref[k], rtol=1e-12, atol=1e-18)


def test_gps_rule_matches_iir_filter():
    """1 LPS, K = 1, beta_l = 0, eta_l = 1, alpha = 0: every Delta equals one worker delta, so the GPS
    model is a single momentum chain with (eta_g, beta_g) over the same sequence (App. E, GPS rule)."""
    rng = np.random.default_rng(4)
    T, n = 30, 19
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    beta_g, eta_g = 0.5, 0.15
    bf, ef, cg = float(F32(beta_g)), float(F32(eta_g)), float(F32(1) - F32(beta_g))
    M_ref = scipy.signal.lfilter([1.0], [1.0, -bf], G.astype(np.float64), axis=0)
    Theta_ref = theta0 - np.cumsum(ef * (cg * G.astype(np.float64) + bf * M_ref), axis=0)
    o = single(theta0, eta_g=eta_g, beta_g=beta_g, K=1, alpha=0.0, form=FORM_ACCUMULATOR)
    for k in range(T):
        assert apply(o, 0, 0, G[k]).sent == 1
        o.gps_receive(0)
        np.testing.assert_allclose(o.get(O.GPS_MOM), M_ref[k], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.GPS_THETA), Theta_ref[k], rtol=1e-12, atol=1e-18)
        np.testing.assert_array_equal(o.get(O.AUX), o.get(O.GPS_THETA))      # the model sent back is this Theta_i
        o.arrive_global(0)
        assert o.lps_step(0).kind == 2
    assert o.counters(0)["gps_updates"] == T


# ---------------------------------------------------------------- library special case / paper identity
def test_cg_one_is_torch_sgd_nesterov():
    """With the coefficient on g set to 1 the rule is the textbook Nesterov step: torch.optim.SGD."""
    rng = np.random.default_rng(5)
    n, T, beta, eta = 40, 12, 0.9, 0.2
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=float(F32(eta)), momentum=float(F32(beta)), nesterov=True)
    o = single(theta0, eta_l=eta, beta_l=beta, cg_l=1.0)
    for k in range(T):
        p.grad = torch.tensor(G[k], dtype=torch.float64)
        opt.step()
        apply(o, 0, 0, G[k])
        np.testing.assert_allclose(o.get(O.THETA), p.detach().numpy(), rtol=1e-13, atol=1e-18)


def test_paper_rule_equals_g_plus_beta_squared_old_momentum():
    """The proof restates the applied direction as  grad + beta^2 m_old  (first display after the update
    rules in App. E); with cg = 1 - beta the oracle must take exactly that step."""
    rng = np.random.default_rng(6)
    n, beta, eta = 50, 0.9, 0.2
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    o = single(theta0, eta_l=eta, beta_l=beta)
    bf, ef = float(F32(beta)), float(F32(eta))
    for k in range(8):
        g = rng.normal(0, 1e-3, n).astype(F32)
        m_old, th_old = o.get(O.MOM), o.get(O.THETA)
        apply(o, 0, 0, g)
        # (1-beta) here is the fp32 value the oracle was given, so compare with that same number
        cg = float(F32(1) - F32(beta))
        expect = th_old - ef * ((cg + bf) * g.astype(np.float64) + bf * bf * m_old)
        np.testing.assert_allclose(o.get(O.THETA), expect, rtol=1e-13, atol=1e-18)
    assert abs((float(F32(1) - F32(beta)) + bf) - 1.0) < 1e-7       # (1-beta) + beta == 1: the coefficient on g


# ---------------------------------------------------------------- merge
@pytest.mark.parametrize("precision", [32, 64])
@pytest.mark.parametrize("form", BOTH_FORMS)
def test_merge_weight_one_and_zero_return_an_operand_exactly(precision, form):
    rng = np.random.default_rng(7)
    n = 300
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    for alpha in (1.0, 0.0):
        o = single(theta0, eta_l=0.3, beta_l=0.9, eta_g=0.15, beta_g=0.5, K=2, alpha=alpha,
                   precision=precision, form=form)
        for k in range(2):
            apply(o, 0, k, rng.normal(0, 1e-3, n).astype(F32))
        o.gps_receive(0)
        apply(o, 0, 0, rng.normal(0, 1e-3, n).astype(F32))         # lands while the Delta is in flight
        before = o.get(O.THETA)
        inbox = o.get(O.AUX)
        assert np.array_equal(inbox, o.get(O.GPS_THETA))
        o.arrive_global(0)
        info = o.lps_step(0)
        assert info.kind == 2 and info.t_last == info.t == 3
        after = o.get(O.THETA)
        assert np.array_equal(after, inbox if alpha == 1.0 else before)
        assert not np.any(o.get(O.AUX))                             # accumulation restarts from zero


def test_repeated_merges_contract_geometrically():
    """theta - Theta shrinks by (1 - alpha) per merge when nothing else moves (the merge of Alg. 1's LPS block)."""
    alpha = 0.25
    theta0 = np.array([8.0, -4.0, 0.5, 16.0], dtype=F32)
    g = np.array([1.0, 2.0, -3.0, 0.5], dtype=F32)
    o = single(theta0, eta_l=1.0, eta_g=0.0, K=1, alpha=alpha)
    apply(o, 0, 0, g)
    o.gps_receive(0)                                    # eta_g = 0: the global model stays theta0
    o.arrive_global(0); o.lps_step(0)
    o.set_rules(eta_l=0.0, beta_l=0.0, cg_l=1.0, eta_g=0.0, beta_g=0.0, cg_g=1.0, alpha=alpha)
    for n in range(2, 10):
        apply(o, 0, 0, g)                               # eta_l = 0: no movement, Delta = 0
        o.gps_receive(0)
        o.arrive_global(0); o.lps_step(0)
        np.testing.assert_allclose(o.get(O.THETA) - theta0, -((1 - alpha) ** n) * g.astype(np.float64), rtol=1e-14)
        assert np.array_equal(o.get(O.GPS_THETA), theta0.astype(np.float64))


def test_hierarchy_collapses_to_one_level():
    """1 LPS, beta_g = 0, eta_g = 1, alpha = 1, merge right after each GPS update: the GPS tracks the LPS,
    and the pair behaves as one momentum-SGD server (checked against the IIR closed form)."""
    rng = np.random.default_rng(8)
    T, n, beta, eta = 20, 16, 0.9, 0.2
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    bf, ef, cg = float(F32(beta)), float(F32(eta)), float(F32(1) - F32(beta))
    m_ref = scipy.signal.lfilter([1.0], [1.0, -bf], G.astype(np.float64), axis=0)
    theta_ref = theta0 - np.cumsum(ef * (cg * G.astype(np.float64) + bf * m_ref), axis=0)
    for form in BOTH_FORMS:
        o = single(theta0, eta_l=eta, beta_l=beta, eta_g=1.0, beta_g=0.0, K=1, alpha=1.0, form=form)
        for k in range(T):
            apply(o, 0, 0, G[k]); o.gps_receive(0); o.arrive_global(0); o.lps_step(0)
            np.testing.assert_allclose(o.get(O.THETA), theta_ref[k], rtol=1e-12, atol=1e-17)
            np.testing.assert_allclose(o.get(O.GPS_THETA), theta_ref[k], rtol=1e-12, atol=1e-17)


# ---------------------------------------------------------------- worked example (hand-derived from Alg. 1)
@pytest.mark.parametrize("precision", [32, 64])
@pytest.mark.parametrize("form", BOTH_FORMS)
def test_hand_derived_worked_example(precision, form):
    with open(os.path.join(HERE, "golden", "alg1_worked_example.json")) as f:
        ex = json.load(f)
    o = HalosOracle(np.array(ex["theta0"], dtype=F32), ex["n_lps"], eta_l=ex["eta_l"], beta_l=ex["beta_l"],
                    cg_l=ex["cg_l"], eta_g=ex["eta_g"], beta_g=ex["beta_g"], cg_g=ex["cg_g"], alpha=ex["alpha"],
                    K=ex["K"], precision=precision, form=form)
    for step in ex["script"]:
        l = step["lps"]
        if step["op"] == "delta":
            o.arrive_delta(l, step["worker"], np.array(step["g"], dtype=F32))
        elif step["op"] == "step":
            info = o.lps_step(l)
            e = step["expect"]
            assert (info.kind, info.t, info.t_last, info.sent) == (e["kind"], e["t"], e["t_last"], e["sent"]), step
            if "expect_theta" in step:
                assert np.array_equal(o.get(O.THETA, l), np.array(step["expect_theta"], dtype=np.float64))
        elif step["op"] == "gps":
            o.gps_receive(l)
            assert np.array_equal(o.get(O.GPS_THETA), np.array(step["expect_Theta"], dtype=np.float64))
        elif step["op"] == "global":
            o.arrive_global(l)
    fin = ex["final"]
    for l in range(ex["n_lps"]):
        assert np.array_equal(o.get(O.THETA, l), np.array(fin["theta"][l], dtype=np.float64))
        assert np.array_equal(o.get(O.AUX, l), np.array(fin["aux"][l], dtype=np.float64))
        c = o.counters(l)
        assert (c["t"], c["t_last"]) == (fin["t"][l], fin["t_last"][l])
    assert np.array_equal(o.get(O.GPS_THETA), np.array(fin["Theta"], dtype=np.float64))
    assert o.counters(0)["gps_updates"] == fin["gps_updates"]


def test_queue_is_first_in_first_out():
    """Deltas and returned global models share one queue and are handled in arrival order (Sec. 4.1 item 2).
    Hand-derived with beta = 0, eta = 1, alpha = 1/2: a delta that arrived BEFORE the global model is applied
    before the merge, so only half of it survives; with momentum, two queued deltas do not commute either."""
    theta0 = np.array([8.0, -4.0, 0.0, 16.0], dtype=F32)
    g1 = np.array([1.0, 2.0, 3.0, 4.0], dtype=F32)
    g2 = np.array([2.0, 0.0, -2.0, 4.0], dtype=F32)
    o = single(theta0, K=1, alpha=0.5)
    assert apply(o, 0, 0, g1).sent == 1
    o.gps_receive(0)                                       # Theta_1 = theta0 - g1
    o.arrive_delta(0, 1, g2)                               # arrives first ...
    o.arrive_global(0)                                     # ... the global model second
    assert [o.lps_step(0).kind, o.lps_step(0).kind] == [1, 2]
    assert np.array_equal(o.get(O.THETA), (theta0 - g1 - 0.5 * g2).astype(np.float64))
    # the other arrival order gives a different model: merge first, then the whole delta
    o = single(theta0, K=1, alpha=0.5)
    apply(o, 0, 0, g1); o.gps_receive(0)
    o.arrive_global(0)
    o.arrive_delta(0, 1, g2)
    assert [o.lps_step(0).kind, o.lps_step(0).kind] == [2, 1]
    assert np.array_equal(o.get(O.THETA), (theta0 - g1 - g2).astype(np.float64))
    # two queued deltas with momentum: m after both is beta*(g_first) + g_second
    o = single(theta0, beta_l=0.5, eta_l=0.25)
    o.arrive_delta(0, 0, g1); o.arrive_delta(0, 1, g2)
    assert (o.lps_step(0).worker, o.lps_step(0).worker) == (0, 1)
    assert np.array_equal(o.get(O.MOM), (0.5 * g1 + g2).astype(np.float64))


# ---------------------------------------------------------------- invariants on seeded traces
def _random_trace_run(precision, form, n=4096, subset=None, seed=11, dtype="f32", flat=True):
    import synth
    from oracle.replay import replay
    w = synth.get_workload("410m").scaled(synth.flat_layout(n), n_updates=96)
    tr = synth.make_trace(w, seed=seed)
    idx = torch.arange(n, dtype=torch.int64) if subset is None else torch.as_tensor(subset, dtype=torch.int64)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
    cache = {}

    def delta(slot):
        if slot not in cache:
            g = synth.normal_at(w.seed, 1 + slot, idx, synth.tensors.scale_f32(w.delta_sigma))
            cache[slot] = synth.to_bf16_bits(g).numpy() if dtype == "bf16" else g.numpy()
        return cache[slot]

    o = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha,
                    K=tr.k_initial, precision=precision, form=form)
    log = replay(o, tr.events, delta)
    return w, tr, o, log


def _all_state(o, n_lps):
    out = {}
    for l in range(n_lps):
        for name, what in (("theta", O.THETA), ("m", O.MOM), ("aux", O.AUX)):
            out[f"{name}{l}"] = (o.get(what, l), o.get(what + O.SCALE, l))
    out["Theta"] = (o.get(O.GPS_THETA), o.get(O.GPS_THETA + O.SCALE))
    out["M"] = (o.get(O.GPS_MOM), o.get(O.GPS_MOM + O.SCALE))
    return out


def test_snapshot_form_equals_accumulator_form():
    """Delta by subtraction (the Delta of Alg. 1's LPS block as written) and Delta as a running sum are the same quantity."""
    w, tr, a, log_a = _random_trace_run(64, FORM_LITERAL)
    _, _, b, log_b = _random_trace_run(64, FORM_ACCUMULATOR)
    assert log_a == log_b
    sa, sb = _all_state(a, w.n_lps), _all_state(b, w.n_lps)
    for k in sa:
        scale = np.maximum(sa[k][1], 1e-30)
        assert np.max(np.abs(sa[k][0] - sb[k][0]) / scale) < 1e-11, k


def test_step_log_matches_schedule_bookkeeping_and_counters():
    """t counts worker updates only; one Delta in flight per LPS; the GPS counter equals the number of
    Deltas received (the counters and tests of Alg. 1's GPS and LPS blocks).  The schedule generator keeps its own counters."""
    import synth
    w, tr, o, log = _random_trace_run(64, FORM_LITERAL)
    ev = tr.events
    steps = ev[ev["kind"] == synth.EV_LPS_STEP]
    assert len(steps) == len(log)
    for rec, (i, kind, t, t_last, sent, acc) in zip(steps, log):
        assert (kind, t, t_last, sent, acc) == (rec["exp_kind"], rec["exp_t"], rec["exp_t_last"], rec["exp_send"],
                                                 rec["exp_accumulate"])
    n_g = tr.count(synth.EV_GPS_MERGE)
    assert o.counters(0)["gps_updates"] == n_g
    for l in range(w.n_lps):
        mine = steps[steps["lps"] == l]
        c = o.counters(l)
        assert c["t"] == int((mine["exp_kind"] == 1).sum())
        assert int(mine["exp_send"].sum()) <= max(1, c["t"] // w.k_range[0])


@pytest.mark.parametrize("precision,form", [(64, FORM_LITERAL), (32, FORM_ACCUMULATOR)])
def test_elementwise_independence(precision, form):
    """Every step is elementwise, so replaying any subset of indices gives bit-identical values there.
    (This is what lets full-size GPU results be checked on sampled elements.)"""
    n = 4096
    subset = np.sort(np.random.default_rng(1).choice(n, 300, replace=False))
    w, _, full, _ = _random_trace_run(precision, form, n=n)
    _, _, part, _ = _random_trace_run(precision, form, n=n, subset=subset)
    sf, sp = _all_state(full, w.n_lps), _all_state(part, w.n_lps)
    for k in sf:
        assert np.array_equal(sf[k][0][subset], sp[k][0]), k


def test_fp32_accumulator_form_stays_within_1e5_of_fp64_reference():
    """fp32 arithmetic drifts from the fp64 reference by a few 2^-24 of each element's largest magnitude
    along the event sequence -- the error model behind the GPU parity tolerance."""
    w, tr, ref, _ = _random_trace_run(64, FORM_LITERAL, n=1 << 15)
    _, _, lo, _ = _random_trace_run(32, FORM_ACCUMULATOR, n=1 << 15)
    sr, sl = _all_state(ref, w.n_lps), _all_state(lo, w.n_lps)
    worst = 0.0
    for k in sr:
        x, scale = sr[k]
        err = np.abs(sl[k][0] - x) / np.maximum(np.maximum(np.abs(x), scale), 1e-30)
        worst = max(worst, float(err.max()))
    assert worst < 1e-5, worst
    assert worst > 0.0                     # they are different precisions: identical would mean a wiring mistake


def test_linearity_in_inputs():
    """All update rules are linear in (Theta_0, deltas): scaling every input by 2^k scales every state by 2^k
    exactly, and the response to a sum is the sum of responses (fp64, inputs with few mantissa bits)."""
    import synth
    from oracle.replay import replay
    n = 64
    w = synth.get_workload("tiny").scaled(synth.flat_layout(n), n_updates=24)
    tr = synth.make_trace(w, seed=5)
    rng = np.random.default_rng(2)

    def run(theta0, pool):
        o = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g,
                        alpha=w.alpha, K=tr.k_initial)
        replay(o, tr.events, lambda s: pool[s])
        return _all_state(o, w.n_lps)

    def inputs():
        return ((rng.integers(-64, 64, n) / 256.0).astype(F32),
                [(rng.integers(-64, 64, n) / 4096.0).astype(F32) for _ in range(w.pool_slots)])

    (xa, pa), (xb, pb) = inputs(), inputs()
    sa, sb = run(xa, pa), run(xb, pb)
    s4 = run(xa * 4, [p * 4 for p in pa])
    ssum = run(xa + xb, [p + q for p, q in zip(pa, pb)])
    for k in sa:
        assert np.array_equal(s4[k][0], 4 * sa[k][0]), k
        np.testing.assert_allclose(ssum[k][0], sa[k][0] + sb[k][0], rtol=0, atol=1e-13)


# ---------------------------------------------------------------- bf16 deltas
def test_bf16_upcast_matches_torch_for_every_bit_pattern():
    bits = torch.arange(0, 1 << 16, dtype=torch.int32).to(torch.int16)
    ref = bits.view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([O.bf16_to_f32(int(b) & 0xFFFF) for b in bits.tolist()], dtype=F32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert O.bf16_to_f32(0x3F80) == 1.0 and O.bf16_to_f32(0xC000) == -2.0


def test_bf16_delta_path_equals_f32_path_fed_prerounded_deltas():
    w, _, a, _ = _random_trace_run(64, FORM_LITERAL, dtype="bf16")
    import synth
    from oracle.replay import replay
    n = 4096
    idx = torch.arange(n, dtype=torch.int64)
    tr = synth.make_trace(w, seed=11)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()

    def delta(slot):
        g = synth.normal_at(w.seed, 1 + slot, idx, synth.tensors.scale_f32(w.delta_sigma))
        return g.to(torch.bfloat16).to(torch.float32).numpy()            # pre-rounded, passed as fp32

    b = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha,
                    K=tr.k_initial)
    replay(b, tr.events, delta)
    sa, sb = _all_state(a, w.n_lps), _all_state(b, w.n_lps)
    for k in sa:
        assert np.array_equal(sa[k][0], sb[k][0]), k


# ---------------------------------------------------------------- monitors
def test_norm_monitors_on_known_vectors():
    """|g|^2 of the last delta and |theta - Theta_i|^2 before the last merge (the quantities bounded by
    assumptions 4 and 5 of Sec. 4.2), on integer vectors where the sums are obvious."""
    theta0 = np.array([8.0, -4.0, 0.0, 16.0], dtype=F32)
    g1 = np.array([1.0, 2.0, 3.0, 4.0], dtype=F32)
    g2 = np.array([2.0, 0.0, -2.0, 4.0], dtype=F32)
    o = single(theta0, K=1, alpha=0.5)
    assert o.norms(0) == (0.0, 0.0)
    apply(o, 0, 0, g1)
    assert o.norms(0) == (30.0, 0.0)                                   # 1 + 4 + 9 + 16
    o.gps_receive(0)                                                   # Theta_1 = theta0 - g1
    apply(o, 0, 1, g2)                                                 # theta = theta0 - g1 - g2
    assert o.norms(0) == (24.0, 0.0)
    o.arrive_global(0); o.lps_step(0)
    assert o.norms(0) == (24.0, 24.0)                                  # theta - Theta_1 = -g2 before the merge


# ---------------------------------------------------------------- protocol violations
def test_protocol_violations_are_rejected():
    o = single(np.zeros(4, dtype=F32), K=1)
    with pytest.raises(O.OracleError):
        o.gps_receive(0)                       # nothing in flight
    with pytest.raises(O.OracleError):
        o.arrive_global(0)                     # nothing was sent back
    o.arrive_delta(0, 0, np.ones(4, dtype=F32))
    with pytest.raises(O.OracleError):
        o.arrive_delta(0, 0, np.ones(4, dtype=F32))   # same worker twice
    assert o.lps_step(0).sent == 1
    assert o.lps_step(0).kind == 0             # empty queue is not an error
    o.gps_receive(0)
    with pytest.raises(O.OracleError):
        o.gps_receive(0)                       # already consumed
