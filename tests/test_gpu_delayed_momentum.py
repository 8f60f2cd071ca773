"""GPU parity of delayed Nesterov momentum (Sec. 5.1; App. D, delays d_l and d_g): the HIP path through the C ABI
against the CPU oracle on the same seeded inputs, gradient buffers included."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth
from oracle import FORM_ACCUMULATOR, FORM_LITERAL
from parity_util import REL_TOL, check_step_logs, compare_state, oracle_run, oracle_state, sample_indices
from test_gpu_parity import RAGGED, _cluster

pytestmark = pytest.mark.gpu


def _delayed(base, d_l, d_g, **kw):
    # rates as the paper's table gives them: the listed value is eta / d
    return replace(base, d_l=d_l, d_g=d_g, eta_l=0.2 * d_l, eta_g=0.15 * d_g, **kw)


def _parity(w, trace, fuse_pull=False, placement="plain", idx=None, batch=0):
    print(f"[parity] workload={w.name} n={w.layout.total} dtype={w.delta_dtype} d_l={w.d_l} d_g={w.d_g} "
          f"events={len(trace.events)} fuse_pull={fuse_pull} placement={placement}", flush=True)
    c = _cluster(w, trace, placement=placement)
    try:
        gpu_log, _ = c.replay(trace.events, fuse_pull=fuse_pull, batch=batch)
        torch.cuda.synchronize()
        if idx is None:
            gpu = {k: c.flat(k) for k in c.state_lists()}
        else:
            tidx = torch.from_numpy(idx)
            gpu = {k: c.gather(k, tidx) for k in c.state_lists()}
        from paper_2506_04531_amd import binding as B
        seen = [B.halos_lps_get_momentum_delay(h) for h in c.lps] + [B.halos_gps_get_momentum_delay(c.gps)]
    finally:
        c.close()
        del c
        torch.cuda.empty_cache()
    o32, log32 = oracle_run(w, trace, idx, 32, FORM_ACCUMULATOR)
    check_step_logs(trace, gpu_log, log32)
    # the position in the cycle is host state of the library: it must match the oracle's
    for l in range(w.n_lps):
        assert seen[l] == {"d": w.d_l, "seen": o32.delay_seen(l)}, (l, seen[l])
    assert seen[-1] == {"d": w.d_g, "seen": o32.delay_seen(-1)}
    ref32 = oracle_state(o32, w.n_lps)
    worst, n_diff, name = compare_state(gpu, ref32, bitwise=True)
    assert n_diff == 0, f"{n_diff} elements differ from the same-order fp32 oracle (worst {worst:.3g} in {name})"
    o64, log64 = oracle_run(w, trace, idx, 64, FORM_LITERAL)
    assert log64 == log32
    worst, _, name = compare_state(gpu, oracle_state(o64, w.n_lps), bitwise=False)
    n_buf = sum(1 for k in ref32 if k.startswith("buffer") or k == "B")
    print(f"[parity] {w.name}: bit-exact vs fp32 oracle ({n_buf} open gradient buffers compared); "
          f"max rel err vs fp64 reference {worst:.3g} ({name})", flush=True)
    assert worst <= REL_TOL, (worst, name)
    return n_buf


@pytest.mark.parametrize("d_l,d_g,dtype,fuse", [(16, 2, "f32", False), (16, 2, "bf16", True), (3, 2, "bf16", False),
                                               (2, 5, "f32", True), (1, 4, "f32", False), (4, 1, "bf16", True),
                                               (7, 3, "f32", True)])
def test_ragged_tensor_list_every_element(d_l, d_g, dtype, fuse):
    """Full tiles, ragged and scalar tails; first / inner / refresh updates at both tiers; delays that do and do not
    divide the accumulation count."""
    w = _delayed(synth.get_workload("410m").scaled(RAGGED, n_updates=128, name=f"dn{d_l}x{d_g}"), d_l, d_g,
                 delta_dtype=dtype)
    _parity(w, synth.make_trace(w, seed=31 + d_l), fuse_pull=fuse)


def test_open_cycles_are_compared():
    """A trace that stops in mid-cycle at most servers: the gradient buffers themselves are checked."""
    w = _delayed(synth.get_workload("160m").scaled(RAGGED, n_updates=75, name="dn-open"), 16, 5)
    assert _parity(w, synth.make_trace(w, seed=5)) >= 2


@pytest.mark.parametrize("recipe", ["1b-dn", "410m-dn", "paper-410m-dn"])
def test_scaled_down_workloads_every_element(recipe):
    base = synth.get_workload(recipe)
    lay = synth.gpt_layout(96, 2, vocab=1031, d_ff=768 if recipe.startswith("1b") else 384)
    w = base.scaled(lay, n_updates=min(base.n_updates, 160), name=recipe + "-small")
    _parity(w, synth.make_trace(w), fuse_pull=True)


def test_snapshot_form_with_delayed_momentum():
    """HALOS_FLAG_SNAPSHOT together with the delayed rule: bit-exact against the fp32 literal-form oracle."""
    from paper_2506_04531_amd import binding as B
    w = _delayed(synth.get_workload("410m").scaled(RAGGED, n_updates=120, name="dn-snap"), 4, 2)
    trace = synth.make_trace(w)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0], flags=B.FLAG_SNAPSHOT)
    c = _cluster(w, trace, hp=hp)
    try:
        gpu_log, _ = c.replay(trace.events, fuse_pull=True, batch=4)
        torch.cuda.synchronize()
        gpu = {k: c.flat(k) for k in c.state_lists()}
    finally:
        c.close()
    o32, log32 = oracle_run(w, trace, None, 32, FORM_LITERAL)
    check_step_logs(trace, gpu_log, log32)
    worst, n_diff, name = compare_state(gpu, oracle_state(o32, w.n_lps, snapshot_form=True), bitwise=True)
    assert n_diff == 0, (n_diff, worst, name)


@pytest.mark.parametrize("name", ["1b-dn", "paper-410m-dn"])
def test_full_size_workloads_on_sampled_elements(name):
    """Full benchmark sizes in the configuration bench.py times (state placed by HBM region, fused pulls, every merge
    in the pass of the update behind it)."""
    w = synth.get_workload(name)
    trace = synth.make_trace(w)
    idx = sample_indices(w.layout, 1 << 17, seed=6)
    _parity(w, trace, fuse_pull=True, placement="regions", idx=idx, batch=4)


def test_delay_one_is_the_plain_rule_and_errors():
    from paper_2506_04531_amd import binding as B
    n = 3 * 4096 + 5
    dev = "cuda:0"
    mk = lambda: [torch.zeros(n, device=dev)]
    Theta = [torch.randn(n, device=dev)]
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4)
    g = [torch.randn(n, device=dev) * 1e-3]

    def run(set_delay_one):
        Th, M, th, m, acc = [Theta[0].clone()], mk(), mk(), mk(), mk()
        gps = B.halos_gps_create([n], hp, Th, M)
        lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
        if set_delay_one:
            B.halos_lps_set_momentum_delay(lps, 1)            # no buffer needed
            B.halos_gps_set_momentum_delay(gps, 1, None)
        for _ in range(4):
            B.halos_lps_push_update(lps, 0, g, B.F32)
            B.halos_lps_step(lps)
        B.halos_gps_merge(gps, lps)
        torch.cuda.synchronize()
        out = [t[0].clone() for t in (Th, M, th, m, acc)]
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
        return out

    for a, b in zip(run(False), run(True)):
        assert torch.equal(a, b)

    Th, M, th, m, acc, buf = [Theta[0].clone()], mk(), mk(), mk(), mk(), mk()
    gps = B.halos_gps_create([n], hp, Th, M)
    lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
    try:
        for bad_d in (0, -3):
            with pytest.raises(B.HalosError) as e:
                B.halos_lps_set_momentum_delay(lps, bad_d, buf)
            assert e.value.status == B.EINVAL
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_set_momentum_delay(lps, 3, None)                      # d > 1 needs a buffer
        assert e.value.status == B.EINVAL
        try:        # too short: rejected unless torch happened to carve the tensor from a larger block
            B.halos_gps_set_momentum_delay(gps, 2, [torch.zeros(100, device=dev)])
            B.halos_gps_set_momentum_delay(gps, 1)
        except B.HalosError as err:
            assert err.status == B.EINVAL
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_set_momentum_delay(lps, 2, [torch.zeros(n + 4, device=dev)[1:]])    # misaligned
        assert e.value.status == B.EINVAL
        assert B.halos_lps_get_momentum_delay(lps) == {"d": 1, "seen": 0}
        B.halos_lps_set_momentum_delay(lps, 3, buf)
        B.halos_lps_push_update(lps, 0, g, B.F32)
        B.halos_lps_step(lps)
        assert B.halos_lps_get_momentum_delay(lps) == {"d": 3, "seen": 1}
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_set_momentum_delay(lps, 2, buf)                       # in mid-cycle
        assert e.value.status == B.ESTATE
        for _ in range(2):
            B.halos_lps_push_update(lps, 0, g, B.F32)
            B.halos_lps_step(lps)
        assert B.halos_lps_get_momentum_delay(lps) == {"d": 3, "seen": 0}
        B.halos_lps_set_momentum_delay(lps, 1)                                # between cycles: allowed
        torch.cuda.synchronize()
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)


def test_buffer_needs_no_initialisation():
    """The first update of a cycle overwrites the gradient buffer without reading it: garbage (even NaN) in it
    beforehand must not reach any state."""
    from paper_2506_04531_amd.harness import Cluster
    w = _delayed(synth.get_workload("tiny").scaled(RAGGED, n_updates=24, name="dn-nan"), 3, 2)
    trace = synth.make_trace(w, seed=2)
    c = Cluster(w, "cuda:0", k_initial=trace.k_initial)
    try:
        for ts in c.buffer + [c.gps_buffer]:
            for t in ts:
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        gpu_log, _ = c.replay(trace.events)
        torch.cuda.synchronize()
        gpu = {k: c.flat(k) for k in c.state_lists()}
    finally:
        c.close()
    o32, log32 = oracle_run(w, trace, None, 32, FORM_ACCUMULATOR)
    check_step_logs(trace, gpu_log, log32)
    worst, n_diff, name = compare_state(gpu, oracle_state(o32, w.n_lps), bitwise=True)
    assert n_diff == 0, (n_diff, worst, name)


@pytest.mark.parametrize("snapshot", [False, True])
def test_merges_ride_in_the_next_update_pass_under_a_momentum_delay(snapshot):
    """With a momentum delay, a replay that asks for batching holds each merge back and issues it with the update step
    that follows (halos_lps_step_batch: merge and one delayed update in one pass).  State, step log and handed-back models
    equal the step-by-step replay's and the oracle's, bit for bit."""
    from dataclasses import replace
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import Cluster
    from parity_util import check_step_logs, compare_state, oracle_run, oracle_state
    from test_gpu_parity import RAGGED
    w = replace(synth.get_workload("160m").scaled(RAGGED, n_updates=160, name="dn-mergebatch"), d_l=4, d_g=2, eta_l=0.8, eta_g=0.3)
    trace = synth.make_trace(w, seed=123)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0], flags=B.FLAG_SNAPSHOT if snapshot else 0)
    runs = []
    for batch in (0, 4):
        c = Cluster(w, "cuda:0", k_initial=trace.k_initial, hp=hp)
        try:
            log, tm = c.replay(trace.events, fuse_pull=True, batch=batch, timed=True)
            torch.cuda.synchronize()
            state = {k: c.flat(k) for k in c.state_lists()}
            for l, dst in enumerate(c.pull_dst):
                state[f"pull{l}"] = torch.cat([t.reshape(-1) for t in dst]).cpu().numpy()
            runs.append((log, state, tm))
        finally:
            c.close()
    merged = {k: len(v) for k, v in runs[1][2].items() if "_merge_" in k}
    print(f"[parity] {w.name} snapshot={snapshot}: passes that open with the merge {merged}", flush=True)
    assert sum(merged.values()) >= 5 and len(merged) >= 2         # at more than one position of the momentum cycle
    assert runs[0][0] == runs[1][0]
    for k in runs[0][1]:
        assert np.array_equal(runs[0][1][k].view(np.uint32), runs[1][1][k].view(np.uint32)), k
    o32, log32 = oracle_run(w, trace, None, 32, FORM_LITERAL if snapshot else FORM_ACCUMULATOR)
    check_step_logs(trace, runs[1][0], log32)
    gpu = {k: v for k, v in runs[1][1].items() if not k.startswith("pull")}
    worst, n_diff, name = compare_state(gpu, oracle_state(o32, w.n_lps, snapshot_form=snapshot), bitwise=True)
    assert n_diff == 0, (n_diff, worst, name)
