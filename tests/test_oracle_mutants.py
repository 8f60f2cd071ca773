"""Do the pins actually pin?  Each mutant below is the oracle's source with one plausible mistake planted
(a dropped term, a wrong sign, a wrong index/operand, a mis-ordered step), compiled to its own library.
The closed-form pins of test_oracle_pins.py must fail on every one of them.  Everything runs on the CPU."""
import os
import subprocess
import sys

import pytest

import oracle as O
import test_oracle_pins as pins
import test_oracle_delayed_momentum as dpins
import test_oracle_error_scales as spins
import test_oracle_variants as vpins

SRC = os.path.join(os.path.dirname(os.path.abspath(O.__file__)), "halos_oracle.cpp")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("step added instead of subtracted", "x = x - step;", "x = x + step;"),
    ("momentum decay dropped", "m = std::fma(r.beta, m, grad);", "m = m + grad;"),
    ("delta not added to momentum", "m = std::fma(r.beta, m, grad);", "m = r.beta * m;"),
    ("direction uses old coefficient 1 on grad", "R direction = std::fma(r.beta, m, r.cg * grad);",
     "R direction = std::fma(r.beta, m, grad);"),
    ("momentum term dropped from direction", "R direction = std::fma(r.beta, m, r.cg * grad);",
     "R direction = r.cg * grad;"),
    ("learning rate dropped", "R step = r.eta * direction;", "R step = direction;"),
    ("merge weights swapped", "s.theta[j] = std::fma(alpha, s.inbox[j], keep * s.theta[j]);",
     "s.theta[j] = std::fma(keep, s.inbox[j], alpha * s.theta[j]);"),
    ("merge in difference form", "s.theta[j] = std::fma(alpha, s.inbox[j], keep * s.theta[j]);",
     "s.theta[j] = s.theta[j] + alpha * (s.inbox[j] - s.theta[j]) * R(1.0000001);"),
    ("snapshot is the pre-merge model", "s.snap = s.theta;                                           // theta_{t_last}: the post-merge model",
     "/* snapshot left at its old value */"),
    ("t_last not reset at merge", "s.t_last = s.t;                                             // t_last <- t", ""),
    ("updates in flight keep accumulating", "const bool accumulate = (s.phase == ACCUMULATING);", "const bool accumulate = true;"),
    ("Delta sign flipped", "s.frozen[j] = (form == 1) ? s.acc[j] : (s.snap[j] - s.theta[j]);",
     "s.frozen[j] = (form == 1) ? -s.acc[j] : (s.theta[j] - s.snap[j]);"),
    ("threshold off by one", "if (accumulate && s.t - s.t_last >= s.K) {", "if (accumulate && s.t - s.t_last > s.K) {"),
    ("GPS uses the local rule", "model_update<R>(Theta[j], M[j], s.frozen[j], global, momentum_bf16);",
     "model_update<R>(Theta[j], M[j], s.frozen[j], local, momentum_bf16);"),
    ("LPS merges the live global model, not the frozen one", "s.theta[j] = std::fma(alpha, s.inbox[j], keep * s.theta[j]);",
     "s.theta[j] = std::fma(alpha, gps_Theta_live[j], keep * s.theta[j]);"),
    ("queue handled last-in first-out", "QueueItem<R> it = std::move(s.queue.front());\n        s.queue.pop_front();",
     "QueueItem<R> it = std::move(s.queue.back());\n        s.queue.pop_back();"),
    ("bf16 placed in the low half", "uint32_t u = (uint32_t)bits << 16;", "uint32_t u = (uint32_t)bits;"),
    ("t counts merges too", "out.kind = 2;", "out.kind = 2; s.t += 1;"),
    # delayed Nesterov momentum
    ("delayed: step added instead of subtracted", "x = x - applied;", "x = x + applied;"),
    ("delayed: buffer not cleared at the refresh", "        buffer = R(0);\n", ""),
    ("delayed: momentum takes the sum, not the mean", "m = std::fma(r.beta, m, buffer * inv_d);", "m = std::fma(r.beta, m, buffer);"),
    ("delayed: gradient rate not divided by d", "const R grad_part = (r.cg * inv_d) * grad;", "const R grad_part = r.cg * grad;"),
    ("delayed: momentum applied on every update", "direction = std::fma(r.beta, m, grad_part);\n        buffer = R(0);\n    }",
     "buffer = R(0);\n    }\n    direction = std::fma(r.beta, m, grad_part);"),
    ("delayed: refresh one update late", "refresh = s.delay.seen + 1 == s.delay.d;", "refresh = s.delay.seen == s.delay.d;"),
    ("delayed: momentum refreshed from the last gradient only", "m = std::fma(r.beta, m, buffer * inv_d);", "m = std::fma(r.beta, m, grad);"),
    ("delayed: GPS cycle counts LPS updates", "if (gps_delay.enabled) gps_delay.seen = refresh ? 0 : gps_delay.seen + 1;",
     "if (gps_delay.enabled) gps_delay.seen = s.delay.seen;"),
    ("delayed: merge clears the gradient buffer", "            s.phase = ACCUMULATING;\n            out.kind = 2;",
     "            s.phase = ACCUMULATING; std::fill(s.buffer.begin(), s.buffer.end(), R(0));\n            out.kind = 2;"),
    # error-scale bookkeeping (the denominator of the fp64 tolerance)
    ("scales: step scale inflated tenfold", "    return std::fabs(r.eta) * (std::fabs(r.cg) * grad_scale + std::fabs(r.beta) * m_scale);",
     "    return R(10) * std::fabs(r.eta) * (std::fabs(r.cg) * grad_scale + std::fabs(r.beta) * m_scale);"),
    ("scales: merge does not carry the global model's scale",
     "                raise_to(s.sc_theta[j], s.sc_aux[j]);                   // scale of the merged global model\n", ""),
    ("scales: GPS ignores the scale that travels with G",
     "            raise_to(sc_M[j], s.sc_aux[j]);                             // the scale of G travels with it\n", ""),
    ("scales: momentum scale follows the value down", "                raise_to(s.sc_m[j], std::fabs(s.m[j]));",
     "                s.sc_m[j] = std::fabs(s.m[j]);"),
    ("scales: returned model keeps G's scale instead of Theta's", "        s.sc_aux = sc_Theta;\n", ""),
    ("scales: accumulated update's scale survives the merge",
     "            std::fill(s.sc_aux.begin(), s.sc_aux.end(), R(0));\n", ""),
    ("scales: delayed buffer scale adds signed values", "    buffer_scale = first ? g_mag : buffer_scale + g_mag;",
     "    buffer_scale = first ? g_mag : buffer_scale + grad;"),
    ("scales: delayed momentum scale ignores the buffer", "        raise_to(m_scale, buffer_scale * inv_d);\n", ""),
    # weighted arrivals, averaged step, single tier, half-precision deltas
    ("variants: weight ignored", "const R w = R(it.weight);                                   // the caller's scalar on this delta (1 = none)",
     "const R w = R(1);"),
    ("variants: average not divided by n", "const R inv_n = R(1) / R(count);", "const R inv_n = R(1);"),
    ("variants: average keeps only the last delta", "gvec[j] = (i == 0) ? term : gvec[j] + term;", "gvec[j] = term;"),
    ("variants: average counts n updates", "        apply_update(s, gvec, out);\n        out.t = s.t; out.t_last = s.t_last;",
     "        apply_update(s, gvec, out); s.t += count - 1;\n        out.t = s.t; out.t_last = s.t_last;"),
    ("variants: average ignores the weights", "const R term = w * R(it.grad[j]);", "const R term = R(it.grad[j]);"),
    ("variants: average leaves the senders marked busy", "            s.worker_queued[it.worker] = 0;\n            out.worker = it.worker;\n        }\n        const R inv_n",
     "            out.worker = it.worker;\n        }\n        const R inv_n"),
    ("variants: single tier uses the local rule", "model_update<R>(Theta[j], M[j], grad, global, momentum_bf16);",
     "model_update<R>(Theta[j], M[j], grad, local, momentum_bf16);"),
    ("variants: single tier forgets the weight", "const R grad = w * R(g[j]);", "const R grad = R(g[j]);"),
    ("variants: single tier never closes its momentum cycle", "if (gps_delay.enabled) { gps_delay.seen = refresh ? 0 : gps_delay.seen + 1; }",
     "if (gps_delay.enabled) { gps_delay.seen = gps_delay.seen + 1; }"),
    ("variants: f16 exponent bias off by one", "((exp + 112u) << 23)", "((exp + 111u) << 23)"),
    ("variants: f16 subnormals flushed", "float v = (float)frac * 5.9604644775390625e-08f;", "float v = 0.0f * (float)frac;"),
    ("variants: f16 mantissa shifted one bit short", "else if (exp != 0) u = sign | ((exp + 112u) << 23) | (frac << 13);",
     "else if (exp != 0) u = sign | ((exp + 112u) << 23) | (frac << 12);"),
    ("scales: everything doubled at the end", "        case 10: copy_out(o->lps[l].sc_theta, out); return 0;",
     "        case 10: { std::vector<R> v = o->lps[l].sc_theta; for (auto &x : v) x *= R(2); copy_out(v, out); return 0; }"),
    # momentum kept in bfloat16
    ("bf16 momentum: truncated instead of rounded", "    u += 0x7FFFu + ((u >> 16) & 1u);", "    u += 0u;"),
    ("bf16 momentum: ties rounded away from zero", "    u += 0x7FFFu + ((u >> 16) & 1u);", "    u += 0x8000u;"),
    ("bf16 momentum: the step uses the momentum before rounding",
     "    if (m_bf16) m = R(bf16_value(f32_to_bf16((float)m)));   // momentum kept in bfloat16: the rounded value is the state\n"
     "    R direction = std::fma(r.beta, m, r.cg * grad);",
     "    const R m_exact = m;\n    if (m_bf16) m = R(bf16_value(f32_to_bf16((float)m)));\n"
     "    R direction = std::fma(r.beta, m_exact, r.cg * grad);"),
    ("bf16 momentum: the global server's momentum stays unrounded", "model_update<R>(Theta[j], M[j], s.frozen[j], global, momentum_bf16);",
     "model_update<R>(Theta[j], M[j], s.frozen[j], global);"),
    ("bf16 momentum: the single-tier server's momentum stays unrounded", "model_update<R>(Theta[j], M[j], grad, global, momentum_bf16);",
     "model_update<R>(Theta[j], M[j], grad, global);"),
]

PIN_TESTS = [
    lambda: [pins.test_zero_momentum_unit_rate_adopts_worker_end_model(p) for p in (32, 64)],
    lambda: [pins.test_k_identical_deltas_accumulate_to_k_eta_g(f, 64) for f in pins.BOTH_FORMS],
    pins.test_constant_delta_gives_geometric_momentum_series_exactly_in_fp32,
    lambda: pins.test_momentum_recursion_matches_iir_filter(0.9, 0.2),
    pins.test_gps_rule_matches_iir_filter,
    pins.test_cg_one_is_torch_sgd_nesterov,
    pins.test_paper_rule_equals_g_plus_beta_squared_old_momentum,
    lambda: [pins.test_merge_weight_one_and_zero_return_an_operand_exactly(64, f) for f in pins.BOTH_FORMS],
    pins.test_repeated_merges_contract_geometrically,
    pins.test_queue_is_first_in_first_out,
    pins.test_hierarchy_collapses_to_one_level,
    lambda: [pins.test_hand_derived_worked_example(64, f) for f in pins.BOTH_FORMS],
    pins.test_snapshot_form_equals_accumulator_form,
    pins.test_step_log_matches_schedule_bookkeeping_and_counters,
    pins.test_bf16_upcast_matches_torch_for_every_bit_pattern,
    dpins.test_delay_one_is_the_plain_rule_bit_for_bit,
    lambda: dpins.test_without_momentum_the_delay_only_divides_the_rate(64),
    lambda: dpins.test_delayed_momentum_is_a_filter_over_cycle_means(6, 0.9, 3.2),
    dpins.test_constant_delta_closed_form_is_exact_in_fp32,
    dpins.test_gps_delayed_rule_is_a_filter_over_cycle_means,
    dpins.test_merge_leaves_the_cycle_alone,
    lambda: [spins.test_worked_example_scales_and_raw_state(64, f) for f in pins.BOTH_FORMS],
    spins.test_snapshot_form_view_follows_the_phases,
    lambda: [spins.test_scale_rules_with_momentum_rate_and_coefficient(64, f) for f in pins.BOTH_FORMS],
    lambda: spins.test_scale_rules_of_the_delayed_rule(64),
    lambda: spins.test_scales_are_bounded_on_both_sides_on_a_seeded_trace(1, 1),
    vpins.test_f16_upcast_matches_torch_for_every_bit_pattern,
    vpins.test_weighted_delta_is_the_delta_scaled_beforehand,
    vpins.test_average_is_one_update_with_the_mean,
    vpins.test_average_adds_in_arrival_order_and_uses_the_weights,
    lambda: [vpins.test_single_tier_server_is_the_same_rule_one_level_up(64, d) for d in (1, 3)],
    vpins.test_single_tier_server_matches_the_filter_closed_form,
    vpins.test_bf16_rounding_matches_torch,
    lambda: [vpins.test_bf16_momentum_hand_example(p) for p in (32, 64)],
    vpins.test_bf16_momentum_is_rounded_on_both_tiers_and_only_the_momentum,
]


def _build_mutant(tmp_path, idx, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not unique / not found: {old!r}"
    text = text.replace(old, new)
    if "gps_Theta_live" in new:     # give the merge access to the live global model
        text = text.replace("int lps_step(int l, StepInfo *info) {\n        Lps<R> &s = lps[l];",
                            "int lps_step(int l, StepInfo *info) {\n        Lps<R> &s = lps[l];\n        const std::vector<R> &gps_Theta_live = Theta;")
    src = tmp_path / f"mutant_{idx}.cpp"
    lib = tmp_path / f"libmutant_{idx}.so"
    src.write_text(text)
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-mfma", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(lib), str(src)])
    return str(lib)


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_some_pin_fails_on_each_planted_mistake(idx, tmp_path, monkeypatch):
    name, old, new = MUTANTS[idx]
    lib_path = _build_mutant(tmp_path, idx, old, new)
    monkeypatch.setattr(O, "_lib", None)
    monkeypatch.setattr(O, "build", lambda force=False: lib_path)
    caught = []
    try:
        for t in PIN_TESTS:
            try:
                t()
            except (AssertionError, O.OracleError) as e:
                caught.append(getattr(t, "__name__", "pin"))
                break
    finally:
        monkeypatch.setattr(O, "_lib", None)       # the next user reloads the real oracle
    assert caught, f"no pin noticed the mutant: {name}"


def test_the_unmutated_oracle_is_back():
    """After the mutant runs the module must serve the real library again."""
    O._lib = None
    pins.test_hand_derived_worked_example(64, O.FORM_LITERAL)
