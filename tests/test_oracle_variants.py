"""Pins for the comparison rules the oracle states next to Alg. 1: weighted arrivals (a caller-side staleness
scaling, Sec. 5.2), the averaged step over several deltas (the synchronous outer step of the Local-SGD methods of
Sec. 2), the single-tier server (the global server applying worker deltas itself, App. D's baseline column), and
half-precision deltas (the workers of Sec. 5.1 train in fp16); and this repository's own option of keeping the servers'
momentum in bfloat16.  Each is checked against a closed form, a library
routine, or a reduction to a rule that is pinned elsewhere; nothing re-types the oracle's loops."""
import numpy as np
import pytest
import scipy.signal
import torch

import oracle as O
from oracle import HalosOracle, FORM_ACCUMULATOR, FORM_LITERAL

F32 = np.float32


def single(theta0, **kw):
    base = dict(eta_l=1.0, beta_l=0.0, eta_g=1.0, beta_g=0.0, alpha=0.0, K=1 << 30)
    base.update(kw)
    return HalosOracle(np.asarray(theta0, dtype=F32), 1, **base)


# ---------------------------------------------------------------- half-precision deltas
def test_f16_upcast_matches_torch_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.float16).to(torch.float32).numpy()
    got = np.array([O.f16_to_f32(int(b)) for b in bits], dtype=F32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))      # signs of zero and subnormals included


def test_f16_delta_equals_the_same_delta_upcast_first():
    rng = np.random.default_rng(5)
    theta0 = rng.normal(0, 0.02, 300).astype(F32)
    g16 = rng.normal(0, 1e-3, (6, 300)).astype(np.float16)
    g16[0, :8] = np.array([0.0, -0.0, 6e-8, -6e-8, 6.1e-5, 65504.0, -65504.0, 1e-7], dtype=np.float16)   # zeros, subnormals, extremes
    for precision in (32, 64):
        a = single(theta0, eta_l=0.2, beta_l=0.9, precision=precision, form=FORM_ACCUMULATOR)
        b = single(theta0, eta_l=0.2, beta_l=0.9, precision=precision, form=FORM_ACCUMULATOR)
        for k in range(6):
            a.arrive_delta(0, 0, g16[k]); a.lps_step(0)
            b.arrive_delta(0, 0, g16[k].astype(F32)); b.lps_step(0)
        for what in (O.THETA, O.MOM, O.AUX):
            assert np.array_equal(a.get(what), b.get(what))


# ---------------------------------------------------------------- weighted arrivals
def test_weight_one_is_the_plain_arrival_bit_for_bit():
    rng = np.random.default_rng(6)
    theta0 = rng.normal(0, 0.02, 200).astype(F32)
    G = rng.normal(0, 1e-3, (10, 200)).astype(F32)
    for precision in (32, 64):
        a = single(theta0, eta_l=0.2, beta_l=0.9, K=4, precision=precision)
        b = single(theta0, eta_l=0.2, beta_l=0.9, K=4, precision=precision)
        for k in range(10):
            a.arrive_delta(0, 0, G[k]); b.arrive_delta(0, 0, G[k], weight=1.0)
            assert a.lps_step(0).sent == b.lps_step(0).sent
        for what in (O.THETA, O.MOM, O.AUX):
            assert np.array_equal(a.get(what), b.get(what))


def test_weighted_delta_is_the_delta_scaled_beforehand():
    """ModelUpdate(x, w g) by definition: with a dyadic weight the product is exact, so both routes agree bit for bit;
    and the closed form of the momentum after weighted arrivals is the filter of App. E over w_k g_k."""
    rng = np.random.default_rng(7)
    theta0 = rng.normal(0, 0.02, 64).astype(F32)
    G = (rng.integers(-512, 512, (8, 64)) / 4096.0).astype(F32)
    W = np.array([0.5, 0.25, 1.0, 0.0, 2.0, 0.125, 0.75, 1.5], dtype=F32)
    beta, eta = 0.5, 0.25
    for precision in (32, 64):
        a = single(theta0, eta_l=eta, beta_l=beta, precision=precision, form=FORM_ACCUMULATOR)
        b = single(theta0, eta_l=eta, beta_l=beta, precision=precision, form=FORM_ACCUMULATOR)
        for k in range(8):
            a.arrive_delta(0, 0, G[k], weight=float(W[k])); a.lps_step(0)
            b.arrive_delta(0, 0, (W[k] * G[k]).astype(F32)); b.lps_step(0)
            for what in (O.THETA, O.MOM, O.AUX):
                assert np.array_equal(a.get(what), b.get(what)), (precision, k, what)
    wg = (W[:, None].astype(np.float64) * G.astype(np.float64))
    m_ref = scipy.signal.lfilter([1.0], [1.0, -beta], wg, axis=0)
    theta_ref = theta0 - np.cumsum(eta * ((1 - beta) * wg + beta * m_ref), axis=0)
    np.testing.assert_allclose(a.get(O.MOM), m_ref[-1], rtol=1e-12, atol=1e-18)
    np.testing.assert_allclose(a.get(O.THETA), theta_ref[-1], rtol=1e-12, atol=1e-18)


def test_weight_zero_only_lets_the_momentum_coast():
    """w = 0: m <- beta m, theta <- theta - eta beta (beta m): the delta itself leaves no trace."""
    theta0 = np.array([1.0, -2.0, 0.5], dtype=F32)
    g1 = np.array([0.5, 0.25, -1.0], dtype=F32)
    junk = np.array([123.0, -77.0, 9.0], dtype=F32)
    o = single(theta0, eta_l=0.5, beta_l=0.5)
    o.arrive_delta(0, 0, g1); o.lps_step(0)
    th1, m1 = o.get(O.THETA).copy(), o.get(O.MOM).copy()
    o.arrive_delta(0, 0, junk, weight=0.0); o.lps_step(0)
    assert np.array_equal(o.get(O.MOM), 0.5 * m1)
    assert np.array_equal(o.get(O.THETA), th1 - 0.5 * (0.5 * (0.5 * m1)))


# ---------------------------------------------------------------- averaged step
@pytest.mark.parametrize("precision", [32, 64])
def test_average_of_one_is_the_plain_step_bit_for_bit(precision):
    rng = np.random.default_rng(8)
    theta0 = rng.normal(0, 0.02, 100).astype(F32)
    G = rng.normal(0, 1e-3, (7, 100)).astype(F32)
    a = single(theta0, eta_l=0.2, beta_l=0.9, K=3, precision=precision)
    b = single(theta0, eta_l=0.2, beta_l=0.9, K=3, precision=precision)
    for k in range(7):
        a.arrive_delta(0, 0, G[k]); b.arrive_delta(0, 0, G[k])
        ia, ib = a.lps_step(0), b.lps_step_average(0, 1)
        assert (ia.kind, ia.t, ia.t_last, ia.sent, ia.accumulated, ia.worker) == (ib.kind, ib.t, ib.t_last, ib.sent, ib.accumulated, ib.worker)
        if ia.sent:
            a.gps_receive(0); a.arrive_global(0); a.lps_step(0)
            b.gps_receive(0); b.arrive_global(0); b.lps_step(0)
    for what in (O.THETA, O.MOM, O.AUX, O.GPS_THETA, O.GPS_MOM):
        assert np.array_equal(a.get(what), b.get(what))


def test_average_is_one_update_with_the_mean():
    """n deltas averaged = ONE ModelUpdate with their mean: t advances by one, every sender's slot is free again,
    identical deltas average to themselves, and dyadic deltas give exactly the single update with (a + b + c + d)/4."""
    theta0 = np.array([8.0, -4.0, 0.0, 16.0], dtype=F32)
    a_, b_, c_, d_ = (np.array(v, dtype=F32) for v in ([1, 2, 3, 4], [2, 0, -2, 4], [4, 4, 4, 4], [1, 2, -1, 0]))
    for precision in (32, 64):
        o = single(theta0, eta_l=0.5, beta_l=0.5, K=2, precision=precision, form=FORM_ACCUMULATOR)
        for w, g in enumerate((a_, b_, c_, d_)):
            o.arrive_delta(0, w, g)
        info = o.lps_step_average(0, 4)
        assert (info.kind, info.t, info.t_last, info.sent, info.accumulated, info.worker) == (1, 1, 0, 0, 1, 3)
        assert o.counters(0)["queued"] == 0
        ref = single(theta0, eta_l=0.5, beta_l=0.5, K=2, precision=precision, form=FORM_ACCUMULATOR)
        ref.arrive_delta(0, 0, ((a_ + b_ + c_ + d_) / 4).astype(F32)); ref.lps_step(0)
        for what in (O.THETA, O.MOM, O.AUX):
            assert np.array_equal(o.get(what), ref.get(what))
        # all four workers may send again; the second averaged step completes the accumulation (K = 2 updates, not 8 deltas)
        for w in range(4):
            o.arrive_delta(0, w, a_)
        info = o.lps_step_average(0, 4)
        assert (info.t, info.sent) == (2, 1)
        ref.arrive_delta(0, 0, a_); assert ref.lps_step(0).sent == 1                 # four identical deltas average to one
        for what in (O.THETA, O.MOM, O.AUX):
            assert np.array_equal(o.get(what), ref.get(what))


def test_average_adds_in_arrival_order_and_uses_the_weights():
    """fp32: (2^24 + 1) - 2^24 added left to right is 0, not 1 -- the stated order is part of the definition (fp64 keeps the
    1).  Weights multiply each delta before it is added."""
    big = np.array([16777216.0], dtype=F32)
    one = np.array([1.0], dtype=F32)
    o32 = single([0.0], precision=32)
    o64 = single([0.0], precision=64)
    for o in (o32, o64):
        o.arrive_delta(0, 0, big); o.arrive_delta(0, 1, one); o.arrive_delta(0, 2, -big)
        o.lps_step_average(0, 3)
    assert o32.get(O.THETA)[0] == 0.0
    assert o64.get(O.THETA)[0] == -1.0 / 3.0 or abs(o64.get(O.THETA)[0] + 1.0 / 3.0) < 1e-15
    o = single([0.0, 0.0], precision=64)
    o.arrive_delta(0, 0, np.array([4.0, 8.0], dtype=F32), weight=0.5)
    o.arrive_delta(0, 1, np.array([2.0, -2.0], dtype=F32), weight=2.0)
    o.lps_step_average(0, 2)
    assert np.array_equal(o.get(O.THETA), -np.array([(2.0 + 4.0) / 2, (4.0 - 4.0) / 2]))


def test_average_refuses_what_is_not_there():
    o = single([0.0, 1.0], K=1)
    g = np.array([1.0, 1.0], dtype=F32)
    with pytest.raises(O.OracleError):
        o.lps_step_average(0, 1)                        # empty queue
    o.arrive_delta(0, 0, g)
    with pytest.raises(O.OracleError):
        o.lps_step_average(0, 2)                        # only one delta queued
    assert o.lps_step_average(0, 1).sent == 1
    o.gps_receive(0)
    o.arrive_delta(0, 0, g); o.arrive_global(0); o.arrive_delta(0, 1, g)
    with pytest.raises(O.OracleError):
        o.lps_step_average(0, 2)                        # a returned model sits between the two deltas
    assert o.counters(0)["queued"] == 3                 # nothing was consumed


# ---------------------------------------------------------------- single tier
@pytest.mark.parametrize("precision", [32, 64])
@pytest.mark.parametrize("delay", [1, 3])
def test_single_tier_server_is_the_same_rule_one_level_up(precision, delay):
    """The global server applying worker deltas itself = a lone local server with the same (eta, beta, cg, delay) fed the same
    deltas: same model, same momentum, bit for bit.  (The local rule is pinned against the filter closed form, the library
    optimizer and the delayed-rule pins elsewhere.)"""
    rng = np.random.default_rng(9)
    theta0 = rng.normal(0, 0.02, 150).astype(F32)
    G = rng.normal(0, 1e-3, (9, 150)).astype(F32)
    W = [1.0, 0.5, 1.0, 0.7071067811865476, 1.0, 1.0, 0.25, 1.0, 1.0]
    eta, beta = 0.15 * delay, 0.5
    top = single(theta0, eta_g=eta, beta_g=beta, precision=precision)
    low = single(theta0, eta_l=eta, beta_l=beta, precision=precision, form=FORM_ACCUMULATOR)
    if delay > 1:
        top.set_delay(-1, delay); low.set_delay(0, delay)
    for k in range(9):
        top.gps_apply_delta(G[k], weight=W[k])
        low.arrive_delta(0, 0, G[k], weight=W[k]); low.lps_step(0)
        assert np.array_equal(top.get(O.GPS_THETA), low.get(O.THETA)), k
        assert np.array_equal(top.get(O.GPS_MOM), low.get(O.MOM)), k
        assert top.delay_seen(-1) == low.delay_seen(0)
    assert top.counters(0)["gps_updates"] == 9
    assert np.array_equal(top.get(O.THETA), theta0.astype(np.float64))       # the local server took no part


def test_single_tier_server_matches_the_filter_closed_form():
    rng = np.random.default_rng(10)
    T, n, beta, eta = 25, 21, 0.9, 0.05
    theta0 = rng.normal(0, 0.02, n).astype(F32)
    G = rng.normal(0, 1e-3, (T, n)).astype(F32)
    bf, ef, cg = float(F32(beta)), float(F32(eta)), float(F32(1) - F32(beta))
    M_ref = scipy.signal.lfilter([1.0], [1.0, -bf], G.astype(np.float64), axis=0)
    Theta_ref = theta0 - np.cumsum(ef * (cg * G.astype(np.float64) + bf * M_ref), axis=0)
    o = single(theta0, eta_g=eta, beta_g=beta)
    for k in range(T):
        o.gps_apply_delta(G[k])
        np.testing.assert_allclose(o.get(O.GPS_MOM), M_ref[k], rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.get(O.GPS_THETA), Theta_ref[k], rtol=1e-12, atol=1e-18)


def test_single_tier_scales_bound_the_values():
    rng = np.random.default_rng(11)
    theta0 = rng.normal(0, 0.02, 64).astype(F32)
    o = single(theta0, eta_g=0.15, beta_g=0.5)
    seen = np.abs(theta0.astype(np.float64))
    for k in range(12):
        g = rng.normal(0, 1e-3, 64).astype(F32)
        o.gps_apply_delta(g)
        seen = np.maximum(seen, np.abs(g))
        for what in (O.GPS_THETA, O.GPS_MOM):
            v = np.abs(o.get(what)); seen = np.maximum(seen, v)
            assert np.all(o.get(what + O.SCALE) >= v)
    for what in (O.GPS_THETA, O.GPS_MOM):
        assert np.all(o.get(what + O.SCALE) <= seen * (1 + 1e-12))


# ---------------------------------------------------------------- no global momentum (Sec. 5.4)
def test_without_global_momentum_the_global_model_never_needs_M():
    """beta_g = 0: Theta_i = Theta_0 - eta_g cg_g (G_1 + ... + G_i), whatever the momentum array holds -- the closed form an
    implementation that keeps no M at all must reproduce (exact on dyadic inputs)."""
    theta0 = (np.arange(-8, 8) / 4.0).astype(F32)
    rng = np.random.default_rng(12)
    G = (rng.integers(-64, 64, (6, 16)) / 256.0).astype(F32)
    eta_g = 0.5
    o = single(theta0, eta_g=eta_g, beta_g=0.0, K=1, alpha=0.0, form=FORM_ACCUMULATOR)
    run = np.zeros(16)
    for k in range(6):
        o.arrive_delta(0, 0, G[k]); assert o.lps_step(0).sent == 1
        o.gps_receive(0); o.arrive_global(0); o.lps_step(0)
        run = run + G[k]                       # eta_l = 1, beta_l = 0: each accumulated update is the delta itself
        assert np.array_equal(o.get(O.GPS_THETA), theta0 - eta_g * 1.0 * run)
        assert np.array_equal(o.get(O.GPS_MOM), G[k].astype(np.float64))       # what M would hold: just the last update


# ---------------------------------------------------------------- momentum kept in bfloat16
def test_bf16_rounding_matches_torch():
    """binary32 -> bfloat16, nearest with ties to even: every upper half with the lower halves that decide a rounding
    (exact, just above, just below and at the tie, all ones), plus random patterns, against torch's conversion."""
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    pats = (hi[:, None] | lows[None, :]).ravel()
    pats = np.concatenate([pats, np.random.default_rng(31).integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)])
    vals = pats.view(F32)
    want = torch.from_numpy(vals.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.f32_to_bf16_array(vals)
    nan = np.isnan(vals)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x007F) != 0)       # a NaN stays a NaN
    # hand-checked ties at 1.0 (spacing 2^-7): 1 + 2^-8 lies between 0x3F80 (even) and 0x3F81 -> down;
    # 1 + 3 * 2^-8 between 0x3F81 and 0x3F82 (even) -> up; just above a tie always up; infinity by overflow
    assert O.f32_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert O.f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert O.f32_to_bf16(float(F32(1.0 + 2.0 ** -8 + 2.0 ** -23))) == 0x3F81
    assert O.f32_to_bf16(-(1.0 + 3 * 2.0 ** -8)) == 0xBF82
    assert O.f32_to_bf16(float(np.finfo(F32).max)) == 0x7F80


@pytest.mark.parametrize("precision", [32, 64])
def test_bf16_momentum_hand_example(precision):
    """One element, beta = 1, eta = 1, cg = 1, three deltas 1, 2^-8, 3 * 2^-8.  Momentum before rounding: 1, 1 + 2^-8,
    then (from the ROUNDED 1) 1 + 3 * 2^-8; in bfloat16: 1, 1 (tie to even), 1 + 2^-6 (tie to even, upwards).  Each step
    subtracts g + m with the rounded m: 2, then 1 + 2^-8, then 3 * 2^-8 + 1 + 2^-6."""
    o = single([8.0], eta_l=1.0, beta_l=1.0, cg_l=1.0, precision=precision, form=FORM_ACCUMULATOR, momentum_bf16=True)
    expect_m = [1.0, 1.0, 1.0 + 2.0 ** -6]
    steps = [2.0, 1.0 + 2.0 ** -8, 3 * 2.0 ** -8 + 1.0 + 2.0 ** -6]
    theta = 8.0
    for k, g in enumerate([1.0, 2.0 ** -8, 3 * 2.0 ** -8]):
        o.arrive_delta(0, 0, np.array([g], dtype=F32)); o.lps_step(0)
        theta -= steps[k]
        assert o.get(O.MOM)[0] == expect_m[k], k
        assert o.get(O.THETA)[0] == theta, k
    assert o.get(O.AUX)[0] == sum(steps)


@pytest.mark.parametrize("precision", [32, 64])
def test_bf16_momentum_changes_nothing_when_nothing_needs_rounding(precision):
    """With beta = 1/2 and deltas that are small multiples of 2^-6, four updates keep every momentum within bfloat16's
    eight significant bits: the option must then give the full-precision run bit for bit, on both tiers."""
    rng = np.random.default_rng(33)
    theta0 = rng.normal(0, 0.02, 64).astype(F32)
    G = (rng.integers(-3, 4, size=(4, 64)) * 2.0 ** -6).astype(F32)
    out = []
    for flag in (False, True):
        o = HalosOracle(theta0, 1, eta_l=0.25, beta_l=0.5, eta_g=0.5, beta_g=0.5, alpha=0.5, K=2, precision=precision,
                        form=FORM_ACCUMULATOR, momentum_bf16=flag)
        for k in range(4):
            o.arrive_delta(0, 0, G[k])
            if o.lps_step(0).sent:
                o.gps_receive(0); o.arrive_global(0); o.lps_step(0)
        out.append([o.get(w) for w in (O.THETA, O.MOM, O.AUX, O.GPS_THETA, O.GPS_MOM)])
    for a, b in zip(*out):
        assert np.array_equal(a, b)
    assert np.any(out[0][4] != 0)           # the global server did update


def test_bf16_momentum_is_rounded_on_both_tiers_and_only_the_momentum():
    """Random run: every momentum value (local and global, single tier too) is a bfloat16 value afterwards; models and
    accumulated updates are not confined to it; the run differs from the full-precision one."""
    rng = np.random.default_rng(34)
    theta0 = rng.normal(0, 0.02, 500).astype(F32)
    G = rng.normal(0, 1e-3, (12, 500)).astype(F32)
    runs = {}
    for flag in (False, True):
        o = HalosOracle(theta0, 1, eta_l=0.2, beta_l=0.9, eta_g=0.15, beta_g=0.5, alpha=0.25, K=3, precision=32,
                        form=FORM_ACCUMULATOR, momentum_bf16=flag)
        for k in range(13):                 # K = 3: the last update leaves an accumulation of one step open
            o.arrive_delta(0, 0, G[k % 12])
            if o.lps_step(0).sent:
                o.gps_receive(0); o.arrive_global(0); o.lps_step(0)
        two_tier_M = o.get(O.GPS_MOM).astype(F32)          # after updates that came through the local server only
        o.gps_apply_delta(G[0])
        runs[flag] = {w: o.get(w).astype(F32) for w in (O.THETA, O.MOM, O.AUX, O.GPS_THETA, O.GPS_MOM)}
        runs[flag]["two_tier_M"] = two_tier_M
    is_bf16 = lambda v: np.all((v.view(np.uint32) & 0xFFFF) == 0)
    r = runs[True]
    assert is_bf16(r[O.MOM]) and is_bf16(r["two_tier_M"]) and np.any(r["two_tier_M"] != 0) and is_bf16(r[O.GPS_MOM])
    assert not is_bf16(runs[False][O.MOM]) and not is_bf16(runs[False]["two_tier_M"]) and not is_bf16(runs[False][O.GPS_MOM])
    assert not is_bf16(r[O.THETA]) and not is_bf16(r[O.GPS_THETA]) and not is_bf16(r[O.AUX])
    assert not np.array_equal(r[O.THETA], runs[False][O.THETA])
    # the rounded momentum stays within half a bfloat16 spacing (2^-9 relative) of what one more exact update of the
    # previous rounded value would give; against the full-precision run it drifts by far less than its own size
    assert np.abs(r[O.MOM] - runs[False][O.MOM]).max() < 0.05 * np.abs(runs[False][O.MOM]).max()


def test_bf16_momentum_refuses_the_delayed_rule_and_unrepresentable_state():
    o = single([1.0], eta_l=0.2, beta_l=0.9)
    o.set_delay(0, 4)
    with pytest.raises(O.OracleError):
        o.set_momentum_bf16(True)
    o = single([1.0], eta_l=0.2, beta_l=0.9, momentum_bf16=True)
    with pytest.raises(O.OracleError):
        o.set_delay(0, 4)
    o = single([1.0], eta_l=0.2, beta_l=0.9)
    o.arrive_delta(0, 0, np.array([1.0 + 2.0 ** -20], dtype=F32)); o.lps_step(0)
    with pytest.raises(O.OracleError):
        o.set_momentum_bf16(True)            # the momentum now holds a value bfloat16 cannot
