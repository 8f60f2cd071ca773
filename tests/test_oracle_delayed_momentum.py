"""Pins for the oracle's delayed Nesterov momentum (the optimizer the paper's runs use at both tiers, Sec. 5.1 and
the hyper-parameter table of App. D with its delays d_l, d_g).  As in test_oracle_pins.py nothing here re-types the
oracle's loop: each test compares it with a closed form, a library filter, or the oracle's own plain rule."""
import numpy as np
import pytest
import scipy.signal

import oracle as O
from oracle import HalosOracle, FORM_ACCUMULATOR, FORM_LITERAL
from test_oracle_pins import F32, apply, single, _random_trace_run, _all_state


def _delayed_reference(G, theta0, eta, beta, cg, d):
    """Closed form, vectorised over time: momentum is the cycle means filtered by 1/(1 - beta z^-1) and held between
    refreshes; the model is theta_0 minus eta times [ (cg/d) * running sum of g + beta * sum of the refreshed
    momenta so far ].  Returns per-step (m, theta, buffer)."""
    T = G.shape[0]
    Gd = G.astype(np.float64)
    n_cycles = T // d
    means = Gd[:n_cycles * d].reshape(n_cycles, d, -1).mean(axis=1)
    m_cycle = scipy.signal.lfilter([1.0], [1.0, -beta], means, axis=0) if n_cycles else means
    m_t = np.zeros_like(Gd)
    mom_sum = np.zeros_like(Gd)
    for t in range(T):
        k = (t + 1) // d                      # refreshes done after step t
        m_t[t] = m_cycle[k - 1] if k > 0 else 0.0
        mom_sum[t] = m_cycle[:k].sum(axis=0)
    theta_t = theta0 - eta * ((cg / d) * np.cumsum(Gd, axis=0) + beta * mom_sum)
    buf_t = np.stack([Gd[(t // d) * d:t + 1].sum(axis=0) if (t + 1) % d else np.zeros(G.shape[1]) for t in range(T)])
    return m_t, theta_t, buf_t


def test_delay_one_is_the_plain_rule_bit_for_bit():
    """d = 1: every update refreshes the momentum from a one-element mean, which is ModelUpdate of App. E."""
    for precision, form in ((32, FORM_ACCUMULATOR), (64, FORM_LITERAL)):
        w, tr, plain, log_a = _random_trace_run(precision, form, n=2048)
        import synth
        from oracle.replay import replay
        import torch
        idx = torch.arange(2048, dtype=torch.int64)
        theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
        o = HalosOracle(theta0, w.n_lps, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha,
                        K=tr.k_initial, precision=precision, form=form)
        for l in range(w.n_lps):
            o.set_delay(l, 1)
        o.set_delay(-1, 1)
        cache = {}

        def delta(slot):
            if slot not in cache:
                cache[slot] = synth.normal_at(w.seed, 1 + slot, idx, synth.tensors.scale_f32(w.delta_sigma)).numpy()
            return cache[slot]

        log_b = replay(o, tr.events, delta)
        assert log_a == log_b
        sa, sb = _all_state(plain, w.n_lps), _all_state(o, w.n_lps)
        for k in sa:
            assert np.array_equal(sa[k][0], sb[k][0]), k


@pytest.mark.parametrize("precision", [32, 64])
def test_without_momentum_the_delay_only_divides_the_rate(precision):
    """beta = 0: the momentum term vanishes and what is left is plain SGD at rate eta / d -- the property the paper
    states for this optimizer (App. D, note under the hyper-parameter table).  d a power of two and dyadic data make
    every operation exact."""
    d, eta = 4, 0.5
    rng = np.random.default_rng(5)
    G = (rng.integers(-64, 64, (11, 40)) / 1024.0).astype(F32)
    theta0 = (rng.integers(-500, 500, 40) / 32.0).astype(F32)
    o = single(theta0, eta_l=eta, beta_l=0.0, precision=precision)
    o.set_delay(0, d)
    plain = single(theta0, eta_l=eta / d, beta_l=0.0, precision=precision)
    for t in range(G.shape[0]):
        apply(o, 0, 0, G[t])
        apply(plain, 0, 0, G[t])
        expect = theta0 - (eta / d) * G[:t + 1].astype(np.float64).sum(axis=0)
        assert np.array_equal(o.get(O.THETA), expect)
        assert np.array_equal(o.get(O.THETA), plain.get(O.THETA))
        assert o.delay_seen(0) == (t + 1) % d


@pytest.mark.parametrize("d,beta,eta", [(6, 0.9, 3.2), (2, 0.5, 0.3), (16, 0.9, 0.2), (3, 0.0, 1.0)])
def test_delayed_momentum_is_a_filter_over_cycle_means(d, beta, eta):
    rng = np.random.default_rng(6)
    T, n = 50, 21
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    bf, ef = float(F32(beta)), float(F32(eta))
    cg = float(F32(1) - F32(beta))
    m_ref, theta_ref, buf_ref = _delayed_reference(G, theta0, ef, bf, cg, d)
    o = single(theta0, eta_l=eta, beta_l=beta)
    o.set_delay(0, d)
    for t in range(T):
        apply(o, 0, 0, G[t])
        np.testing.assert_allclose(o.get(O.MOM), m_ref[t], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.THETA), theta_ref[t], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.BUFFER), buf_ref[t], rtol=1e-12, atol=1e-18)


def test_constant_delta_closed_form_is_exact_in_fp32():
    """d = 4, beta = 0.5, eta = 0.25, cg = 0.5, g = k 2^-10: after c full cycles  m = g (1 - beta^c)/(1 - beta)  and
    theta = theta_0 - eta g [ c d (cg/d) + beta sum_{j<=c} (1 - beta^j)/(1 - beta) ], every operation exact."""
    d, beta, eta = 4, 0.5, 0.25
    g = (np.arange(-5, 6) / 1024.0).astype(F32)
    theta0 = np.linspace(-1, 1, 11).astype(F32)
    for precision in (32, 64):
        o = single(theta0, eta_l=eta, beta_l=beta, precision=precision, form=FORM_ACCUMULATOR)
        o.set_delay(0, d)
        gd = g.astype(np.float64)
        for c in range(1, 7):
            for _ in range(d):
                apply(o, 0, 0, g)
            m_closed = gd * (1 - beta ** c) / (1 - beta)
            mom_sum = sum((1 - beta ** j) / (1 - beta) for j in range(1, c + 1))
            th_closed = theta0 - eta * gd * (c * (1 - beta) + beta * mom_sum)
            assert np.array_equal(o.get(O.MOM), m_closed)
            assert np.array_equal(o.get(O.THETA), th_closed)
            assert np.array_equal(o.get(O.BUFFER), np.zeros(11))
            # the accumulated update is what was subtracted from the model
            assert np.array_equal(o.get(O.AUX), theta0.astype(np.float64) - o.get(O.THETA))


def test_gps_delayed_rule_is_a_filter_over_cycle_means():
    """1 LPS, K = 1, beta_l = 0, eta_l = 1, alpha = 0: every Delta is one worker delta, so the GPS model follows the
    delayed rule with (eta_g, beta_g, d_g) over that sequence."""
    rng = np.random.default_rng(7)
    T, n, d_g = 31, 17, 2
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    beta_g, eta_g = 0.5, 0.3
    bf, ef, cg = float(F32(beta_g)), float(F32(eta_g)), float(F32(1) - F32(beta_g))
    M_ref, Theta_ref, B_ref = _delayed_reference(G, theta0, ef, bf, cg, d_g)
    o = single(theta0, eta_g=eta_g, beta_g=beta_g, K=1, alpha=0.0, form=FORM_ACCUMULATOR)
    o.set_delay(-1, d_g)
    for t in range(T):
        assert apply(o, 0, 0, G[t]).sent == 1
        o.gps_receive(0)
        np.testing.assert_allclose(o.get(O.GPS_MOM), M_ref[t], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.GPS_THETA), Theta_ref[t], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.GPS_BUFFER), B_ref[t], rtol=1e-12, atol=1e-18)
        np.testing.assert_array_equal(o.get(O.AUX), o.get(O.GPS_THETA))
        o.arrive_global(0)
        assert o.lps_step(0).kind == 2
        assert o.delay_seen(-1) == (t + 1) % d_g
        assert o.delay_seen(0) == 0           # the LPS itself runs the plain rule here


def test_merge_leaves_the_cycle_alone():
    """The gradient buffer and the position in the cycle are optimizer state of the server: a merge in mid-cycle
    (the merge of Alg. 1's LPS block changes theta only) must not disturb them."""
    rng = np.random.default_rng(8)
    n, d = 9, 5
    G = rng.normal(0, 1e-3, (7, n)).astype(F32)
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    o = single(theta0, eta_l=0.2, beta_l=0.9, K=2, alpha=0.25, eta_g=0.15, beta_g=0.5)
    o.set_delay(0, d)
    apply(o, 0, 0, G[0])
    assert apply(o, 0, 0, G[1]).sent == 1
    o.gps_receive(0)
    apply(o, 0, 0, G[2])                       # third update of the cycle, while the Delta is away
    o.arrive_global(0)
    buf, seen, mom = o.get(O.BUFFER), o.delay_seen(0), o.get(O.MOM)
    assert seen == 3
    np.testing.assert_allclose(buf, G[:3].astype(np.float64).sum(axis=0), rtol=1e-12)
    assert o.lps_step(0).kind == 2
    assert np.array_equal(o.get(O.BUFFER), buf) and o.delay_seen(0) == seen and np.array_equal(o.get(O.MOM), mom)
    apply(o, 0, 0, G[3])
    apply(o, 0, 0, G[4])                       # fifth: refresh
    assert o.delay_seen(0) == 0
    np.testing.assert_allclose(o.get(O.MOM), G[:5].astype(np.float64).mean(axis=0), rtol=1e-12)


def test_delay_changes_only_between_cycles():
    o = single(np.zeros(4, dtype=F32))
    o.set_delay(0, 3)
    apply(o, 0, 0, np.ones(4, dtype=F32))
    with pytest.raises(O.OracleError):
        o.set_delay(0, 2)
    apply(o, 0, 0, np.ones(4, dtype=F32))
    apply(o, 0, 0, np.ones(4, dtype=F32))
    o.set_delay(0, 2)                           # cycle closed: allowed
    o.set_delay(0, 0)                           # and back to the plain rule


def test_fp32_delayed_rule_stays_within_1e5_of_fp64_reference():
    """Same bound as for the plain rule, on the error scales the oracle propagates."""
    import synth
    import torch
    from oracle.replay import replay
    n = 4096
    w = synth.get_workload("410m").scaled(synth.flat_layout(n), n_updates=160)
    tr = synth.make_trace(w, seed=21)
    idx = torch.arange(n, dtype=torch.int64)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
    cache = {}

    def delta(slot):
        if slot not in cache:
            cache[slot] = synth.normal_at(w.seed, 1 + slot, idx, synth.tensors.scale_f32(w.delta_sigma)).numpy()
        return cache[slot]

    states = []
    for precision, form in ((32, FORM_ACCUMULATOR), (64, FORM_LITERAL)):
        o = HalosOracle(theta0, w.n_lps, eta_l=3.2, beta_l=0.9, eta_g=0.3, beta_g=0.5, alpha=w.alpha,
                        K=tr.k_initial, precision=precision, form=form)
        for l in range(w.n_lps):
            o.set_delay(l, 16)
        o.set_delay(-1, 2)
        replay(o, tr.events, delta)
        st = _all_state(o, w.n_lps)
        for l in range(w.n_lps):
            st[f"buffer{l}"] = (o.get(O.BUFFER, l), o.get(O.BUFFER + O.SCALE, l))
        st["B"] = (o.get(O.GPS_BUFFER), o.get(O.GPS_BUFFER + O.SCALE))
        states.append(st)
    worst = 0.0
    for k in states[0]:
        scale = np.maximum(np.maximum(states[1][k][1], np.abs(states[1][k][0])), 1e-30)
        worst = max(worst, float(np.max(np.abs(states[0][k][0] - states[1][k][0]) / scale)))
    assert 0 < worst < 1e-5, worst
