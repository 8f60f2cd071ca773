"""GPU parity of the variants next to the base path: IEEE-half deltas, weighted arrivals, the momentum-free global
server, merges that do not clear the third buffer, the single-tier server, and momentum kept in bfloat16 -- each
through the C ABI against the CPU oracle on the same seeded inputs."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle as O
import synth
from oracle import FORM_ACCUMULATOR, FORM_LITERAL, HalosOracle
from parity_util import REL_TOL, check_step_logs, compare_state, oracle_run, oracle_state
from test_gpu_parity import RAGGED, _cluster, _full_parity

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------- IEEE-half deltas
@pytest.mark.parametrize("layout", ["ragged", "gpt"])
def test_half_precision_deltas_every_element(layout):
    """fp16 deltas (many of them subnormal at these magnitudes) upcast in the update pass."""
    lay = RAGGED if layout == "ragged" else synth.gpt_layout(96, 2, vocab=1031)
    w = replace(synth.get_workload("160m").scaled(lay, n_updates=96, name="f16-" + layout), delta_dtype="f16")
    _full_parity(w, synth.make_trace(w, seed=71))


def test_every_half_bit_pattern_goes_through_the_update_exactly():
    """theta_0 = 0, beta = 0, eta = cg = 1: theta = -g, so the updated model shows the upcast of every one of the 65,536
    half patterns (NaNs and infinities replaced by zeros: they would poison the state by design)."""
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16).copy()
    h[~np.isfinite(h)] = 0.0
    n = h.size + 3                                       # not a multiple of the vector width: the scalar tail sees halves too
    g = torch.zeros(n, dtype=torch.float16, device=dev)
    g[:h.size] = torch.from_numpy(h).to(dev)
    Theta, M, th, m, acc = (torch.zeros(n, device=dev) for _ in range(5))
    hp = B.paper_hparams(1.0, 0.0, 1.0, 0.0, 0.0, 1 << 30, cg_l=1.0, cg_g=1.0)
    gps = B.halos_gps_create([n], hp, [Theta], [M])
    lps = B.halos_lps_create(gps, 0, 1, [th], [m], [acc])
    try:
        B.halos_lps_push_update(lps, 0, [g], B.F16)
        B.halos_lps_step(lps)
        torch.cuda.synchronize()
        got = th.cpu().numpy()[:h.size]
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
    want = np.array([O.f16_to_f32(int(b)) for b in h.view(np.uint16)], dtype=np.float32)
    o = HalosOracle(np.zeros(h.size, dtype=np.float32), 1, eta_l=1.0, beta_l=0.0, eta_g=1.0, beta_g=0.0, alpha=0.0,
                    K=1 << 30, cg_l=1.0, cg_g=1.0, precision=32, form=FORM_ACCUMULATOR)
    o.arrive_delta(0, 0, h); o.lps_step(0)
    ref = o.get(O.THETA).astype(np.float32)
    assert np.array_equal(ref, np.float32(0.0) - want)                 # the oracle's model is minus the upcast delta
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


# ---------------------------------------------------------------- weighted arrivals
@pytest.mark.parametrize("dtype,d_l", [("f32", 1), ("bf16", 1), ("f32", 4)])
def test_staleness_weighted_arrivals_every_element(dtype, d_l):
    """Every delta carries the weight (1 + staleness)^-0.5 (the caller's polynomial; halos_lps_push_update_weighted)."""
    base = synth.get_workload("410m").scaled(RAGGED, n_updates=96, name=f"weighted-{dtype}-d{d_l}")
    w = replace(base, delta_dtype=dtype, staleness_exponent=0.5, d_l=d_l, eta_l=0.2 * d_l)
    trace = synth.make_trace(w, seed=81)
    st = trace.events[trace.events["kind"] == synth.EV_ARRIVE_DELTA]["staleness"]
    assert st.max() > 0, "the schedule must produce stale arrivals for this test to mean anything"
    _full_parity(w, trace)


def test_weight_must_be_finite():
    from paper_2506_04531_amd import binding as B
    w = synth.get_workload("tiny").scaled(synth.flat_layout(5000), n_updates=4, name="badweight")
    trace = synth.make_trace(w)
    c = _cluster(w, trace)
    try:
        for bad in (float("nan"), float("inf")):
            with pytest.raises(B.HalosError) as e:
                B.halos_lps_push_update_weighted(c.lps[0], 0, c.pool[0], c.delta_dtype, 0, bad)
            assert e.value.status == B.EINVAL
            with pytest.raises(B.HalosError) as e:
                B.halos_gps_push_update(c.gps, c.pool[0], c.delta_dtype, bad)
            assert e.value.status == B.EINVAL
        assert B.halos_lps_get_counters(c.lps[0])["queued"] == 0
    finally:
        c.close()


# ---------------------------------------------------------------- momentum-free global server (Sec. 5.4)
@pytest.mark.parametrize("recipe", ["70m", "160m"])
def test_global_server_without_momentum_every_element(recipe):
    """HALOS_FLAG_GPS_NO_MOMENTUM: no M exists; everything else equals the general rule at beta_g = 0 (the oracle),
    compared numerically exactly (an exact zero may differ in sign)."""
    from paper_2506_04531_amd import binding as B
    base = synth.get_workload(recipe)
    lay = RAGGED if recipe == "70m" else synth.gpt_layout(96, 2, vocab=1031)
    w = replace(base.scaled(lay, n_updates=120, name=recipe + "-nomom"), beta_g=0.0)
    trace = synth.make_trace(w)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, 0.0, w.alpha, w.k_range[0], flags=B.FLAG_GPS_NO_MOMENTUM)
    c = _cluster(w, trace, hp=hp)
    try:
        assert c.M is None
        gpu_log, _ = c.replay(trace.events, fuse_pull=True)
        torch.cuda.synchronize()
        gpu = {k: c.flat(k) for k in c.state_lists()}
    finally:
        c.close()
    assert "M" not in gpu
    o32, log32 = oracle_run(w, trace, None, 32, FORM_ACCUMULATOR)
    check_step_logs(trace, gpu_log, log32)
    ref = oracle_state(o32, w.n_lps, with_scale=False)
    for k, v in gpu.items():
        r = ref[k][0].astype(np.float32)
        assert np.array_equal(v, r), k                       # numeric equality: +0 == -0, no NaN anywhere
    o64, _ = oracle_run(w, trace, None, 64, FORM_LITERAL)
    ref64 = {k: v for k, v in oracle_state(o64, w.n_lps).items() if k != "M"}
    worst, _, name = compare_state(gpu, ref64, bitwise=False)
    assert worst <= REL_TOL, (worst, name)


def test_momentum_free_server_refuses_what_needs_momentum():
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    n = 5000
    Theta, buf, g = (torch.zeros(n, device=dev) for _ in range(3))
    with pytest.raises(B.HalosError) as e:                   # the flag with beta_g != 0
        B.halos_gps_create([n], B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4, flags=B.FLAG_GPS_NO_MOMENTUM), [Theta], None)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.HalosError) as e:                   # deferring the clear makes no sense with a snapshot
        B.halos_gps_create([n], B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4, flags=B.FLAG_SNAPSHOT | B.FLAG_DEFER_CLEAR), [Theta], [buf])
    assert e.value.status == B.EINVAL
    gps = B.halos_gps_create([n], B.paper_hparams(0.2, 0.9, 0.15, 0.0, 0.25, 4, flags=B.FLAG_GPS_NO_MOMENTUM), [Theta], None)
    try:
        with pytest.raises(B.HalosError) as e:
            B.halos_gps_push_update(gps, [g], B.F32)
        assert e.value.status == B.ESTATE
        with pytest.raises(B.HalosError) as e:
            B.halos_gps_set_momentum_delay(gps, 2, [buf])
        assert e.value.status == B.ESTATE
        with pytest.raises(B.HalosError) as e:
            B.halos_set_hparams(gps, True, B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4))
        assert e.value.status == B.EINVAL
        B.halos_set_hparams(gps, True, B.paper_hparams(0.2, 0.9, 0.3, 0.0, 0.25, 4))       # the rate may change
    finally:
        B.halos_gps_destroy(gps)


# ---------------------------------------------------------------- merges that leave the third buffer alone
@pytest.mark.parametrize("recipe,dtype,d_l", [("410m", "f32", 1), ("160m", "bf16", 1), ("70m", "f32", 3)])
def test_deferred_clear_changes_no_result(recipe, dtype, d_l):
    """HALOS_FLAG_DEFER_CLEAR: the merge writes theta only and the next accumulating update stores 0 + its step.  Every
    array equals the oracle's bit for bit; the third buffer of a server that has merged and not updated since is
    unspecified and left out."""
    from paper_2506_04531_amd import binding as B
    base = synth.get_workload(recipe).scaled(RAGGED, n_updates=120, name=f"defer-{recipe}")
    w = replace(base, delta_dtype=dtype, d_l=d_l, eta_l=0.2 * d_l, max_link_delay=2, k_range=(2, 5))
    trace = synth.make_trace(w, seed=91)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0], flags=B.FLAG_DEFER_CLEAR)
    n_merges = int((trace.events["kind"] == synth.EV_ARRIVE_GLOBAL).sum())
    assert n_merges >= 4
    # stop right after a merge as well as at the end, so that both kinds of final state are seen
    ev = trace.events
    last_merge = max(i for i in range(len(ev)) if ev[i]["kind"] == synth.EV_LPS_STEP and ev[i]["exp_kind"] == 2)
    for cut in (last_merge + 1, len(ev)):
        c = _cluster(w, trace, hp=hp)
        try:
            gpu_log, _ = c.replay(ev[:cut], fuse_pull=True)
            torch.cuda.synchronize()
            gpu = {k: c.flat(k) for k in c.state_lists()}
            fresh = [B.halos_lps_get_counters(h) for h in c.lps]
        finally:
            c.close()
        o32, log32 = oracle_run(w, replace(trace, events=ev[:cut]), None, 32, FORM_ACCUMULATOR)
        assert gpu_log == log32
        ref = oracle_state(o32, w.n_lps)
        skipped = 0
        for l, cnt in enumerate(fresh):
            if cnt["phase"] == B.PHASE_ACCUMULATING and cnt["t"] == cnt["t_last"] and cnt["t"] > 0:
                ref.pop(f"aux{l}"); skipped += 1
        if cut == last_merge + 1:
            assert skipped >= 1
        worst, n_diff, name = compare_state(gpu, ref, bitwise=True)
        assert n_diff == 0, (cut, n_diff, worst, name)


# ---------------------------------------------------------------- single tier
@pytest.mark.parametrize("dtype,d_g", [("f32", 1), ("bf16", 1), ("f16", 1), ("f32", 3)])
def test_single_tier_server_every_element(dtype, d_g):
    """halos_gps_push_update: the global server applies worker deltas itself (weights included), against the oracle's
    gps_apply_delta, model and momentum (and the open gradient buffer) bit for bit."""
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import alloc_tensor_list, fill_delta_slot, fill_initial_model
    dev = torch.device("cuda:0")
    w = replace(synth.get_workload("70m").scaled(RAGGED, n_updates=1, name="single-tier"), delta_dtype=dtype, d_g=d_g,
                eta_g=0.05 * d_g, beta_g=0.9)
    numel = [int(x) for x in w.layout.numel]
    f32 = torch.float32
    Theta, M, Bf = (alloc_tensor_list(numel, f32, dev) for _ in range(3))
    fill_initial_model(w, Theta)
    ddt = {"f32": f32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    code = {"f32": B.F32, "bf16": B.BF16, "f16": B.F16}[dtype]
    pool = []
    for s in range(4):
        ts = alloc_tensor_list(numel, ddt, dev)
        fill_delta_slot(w, s, ts)
        pool.append(ts)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, 8)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    weights = [1.0, 0.5, float(np.float32(2 ** -0.5)), 1.0, 0.25, 1.0, 1.0, float(np.float32(3 ** -0.5))]
    try:
        if d_g > 1:
            B.halos_gps_set_momentum_delay(gps, d_g, Bf)
        for k, wt in enumerate(weights):
            B.halos_gps_push_update(gps, pool[k % 4], code, wt)
        torch.cuda.synchronize()
        assert B.halos_gps_get_counters(gps)["updates"] == len(weights)
        flat = lambda ts: torch.cat([t.reshape(-1) for t in ts]).cpu().numpy()
        gpu = {"Theta": flat(Theta), "M": flat(M), "B": flat(Bf)}
    finally:
        B.halos_gps_destroy(gps)
    idx = torch.arange(w.layout.total, dtype=torch.int64)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
    scale = torch.from_numpy(synth.delta_scales(w)[w.layout.tensor_of(idx.numpy())])
    o = HalosOracle(theta0, 1, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha, K=8,
                    precision=32, form=FORM_ACCUMULATOR)
    if d_g > 1:
        o.set_delay(-1, d_g)
    for k, wt in enumerate(weights):
        g = synth.normal_at(w.seed, 1 + k % 4, idx, scale)
        g = g.to(ddt).to(torch.float32).numpy()                     # what the 16-bit buffer holds, upcast (exact)
        o.gps_apply_delta(g, wt)
    for name, what in (("Theta", O.GPS_THETA), ("M", O.GPS_MOM)):
        ref = o.get(what).astype(np.float32)
        assert np.array_equal(gpu[name].view(np.uint32), ref.view(np.uint32)), name
    if o.delay_seen(-1) > 0:
        ref = o.get(O.GPS_BUFFER).astype(np.float32)
        assert np.array_equal(gpu["B"].view(np.uint32), ref.view(np.uint32))


# ---------------------------------------------------------------- several deltas in one pass
@pytest.mark.parametrize("dtype,flags", [("f32", 0), ("bf16", 0), ("f16", 0), ("f32", "snapshot"), ("bf16", "defer"), ("bf16", "bf16m")])
def test_averaged_step_every_element(dtype, flags):
    """halos_lps_step_average: n queued deltas (with weights) become one update with their mean, against the oracle's
    lps_step_average; rounds of 1..4 deltas, accumulation, GPS updates and merges in between."""
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import alloc_tensor_list, fill_delta_slot, fill_initial_model
    dev = torch.device("cuda:0")
    w = replace(synth.get_workload("70m").scaled(RAGGED, n_updates=1, name="avg"), delta_dtype=dtype)
    numel = [int(x) for x in w.layout.numel]
    f32 = torch.float32
    Theta, th, acc = (alloc_tensor_list(numel, f32, dev) for _ in range(3))
    M, m = (alloc_tensor_list(numel, torch.bfloat16 if flags == "bf16m" else f32, dev) for _ in range(2))
    fill_initial_model(w, Theta)
    ddt = {"f32": f32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    code = {"f32": B.F32, "bf16": B.BF16, "f16": B.F16}[dtype]
    pool = []
    for s in range(4):
        ts = alloc_tensor_list(numel, ddt, dev)
        fill_delta_slot(w, s, ts)
        pool.append(ts)
    fl = {0: 0, "snapshot": B.FLAG_SNAPSHOT, "defer": B.FLAG_DEFER_CLEAR, "bf16m": B.FLAG_BF16_MOMENTUM}[flags]
    K = 2
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, K, flags=fl)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 4, th, m, acc)
    idx = torch.arange(w.layout.total, dtype=torch.int64)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
    scale = torch.from_numpy(synth.delta_scales(w)[w.layout.tensor_of(idx.numpy())])
    host = []
    for s in range(4):
        g = synth.normal_at(w.seed, 1 + s, idx, scale)
        host.append(synth.to_bf16_bits(g).numpy() if dtype == "bf16" else synth.to_f16(g).numpy() if dtype == "f16" else g.numpy())
    o = HalosOracle(theta0, 1, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha, K=K,
                    precision=32, form=FORM_LITERAL if flags == "snapshot" else FORM_ACCUMULATOR, momentum_bf16=(flags == "bf16m"))
    flat = lambda ts: torch.cat([t.reshape(-1) for t in ts]).float().cpu().numpy()
    rounds = [(4, [1.0, 1.0, 1.0, 1.0]), (2, [0.5, 1.0]), (3, [1.0, 0.25, 0.70710677]), (1, [1.0]), (4, [1.0, 0.5, 1.0, 2.0]), (2, [1.0, 1.0])]
    try:
        for r, (n, ws) in enumerate(rounds):
            for k in range(n):
                B.halos_lps_push_update_weighted(lps, k, pool[(r + k) % 4], code, 0, ws[k])
                o.arrive_delta(0, k, host[(r + k) % 4], ws[k])
            gi = B.halos_lps_step_average(lps, n)
            oi = o.lps_step_average(0, n)
            assert (gi.kind, gi.t, gi.t_last, gi.delta_ready, gi.accumulated, gi.worker) == \
                   (oi.kind, oi.t, oi.t_last, oi.sent, oi.accumulated, oi.worker), r
            if gi.delta_ready:
                B.halos_gps_merge(gps, lps); o.gps_receive(0)
                if r % 2:                                      # merge now, or leave the returned model in flight for a round
                    B.halos_lps_push_global(lps); o.arrive_global(0)
                    assert B.halos_lps_step(lps).kind == 2 and o.lps_step(0).kind == 2
            elif B.halos_lps_get_counters(lps)["phase"] == B.PHASE_RETURNING:
                B.halos_lps_push_global(lps); o.arrive_global(0)
                assert B.halos_lps_step(lps).kind == 2 and o.lps_step(0).kind == 2
            torch.cuda.synchronize()
            gpu = {"Theta": flat(Theta), "M": flat(M), "theta0": flat(th), "m0": flat(m), "aux0": flat(acc)}
            ref = oracle_state(o, 1, with_scale=False, snapshot_form=(flags == "snapshot"))
            cnt = B.halos_lps_get_counters(lps)
            if flags == "defer" and cnt["phase"] == B.PHASE_ACCUMULATING and cnt["t"] == cnt["t_last"] and cnt["t"] > 0:
                ref.pop("aux0")
            worst, n_diff, name = compare_state(gpu, ref, bitwise=True)
            assert n_diff == 0, (r, n_diff, worst, name)
        # refusals: not enough deltas, a global model in the way, an end model
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_step_average(lps, 2)
        assert e.value.status == B.ESTATE
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_step_average(lps, 5)
        assert e.value.status == B.EINVAL
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)


@pytest.mark.parametrize("recipe,dtype,flags,weighted", [("160m", "bf16", 0, False), ("160m", "f32", "defer", True),
                                                         ("70m", "f16", 0, False), ("160m", "f32", "snapshot", False),
                                                         ("160m", "bf16", "bf16m", True)])
def test_batched_steps_equal_single_steps(recipe, dtype, flags, weighted):
    """halos_lps_step_batch on a bursty schedule (8 workers per server at uneven rates): wherever several deltas of one
    server wait, they go through one pass.  State, step log and every model handed back equal the step-by-step run's
    and the oracle's, bit for bit."""
    from paper_2506_04531_amd import binding as B
    base = synth.get_workload(recipe).scaled(RAGGED, n_updates=200, name=f"batch-{recipe}")
    w = replace(base, delta_dtype=dtype, n_lps=2, workers_per_lps=8, hetero_rates=True, staleness_exponent=0.5 if weighted else 0.0)
    trace = synth.make_trace(w, seed=97)
    fl = {0: 0, "snapshot": B.FLAG_SNAPSHOT, "defer": B.FLAG_DEFER_CLEAR, "bf16m": B.FLAG_BF16_MOMENTUM}[flags]
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0], flags=fl)
    runs = []
    for batch in (0, 4):
        c = _cluster(w, trace, hp=hp)
        try:
            log, tm = c.replay(trace.events, fuse_pull=True, batch=batch, timed=True)
            torch.cuda.synchronize()
            state = {k: c.flat(k) for k in c.state_lists()}
            for l, dst in enumerate(c.pull_dst):
                state[f"pull{l}"] = torch.cat([t.reshape(-1) for t in dst]).cpu().numpy()
            fresh = [B.halos_lps_get_counters(h) for h in c.lps]
            runs.append((log, state, tm))
        finally:
            c.close()
    batched = {k: len(v) for k, v in runs[1][2].items() if k.startswith("lps_update_batch")}
    print(f"[parity] {w.name}: batched launches {batched}", flush=True)
    assert sum(batched.values()) >= 5, "the schedule must produce bursts for this test to mean anything"
    assert sum(n for k, n in batched.items() if "_merge_" in k) >= 3, "some passes must open with a merge"
    assert runs[0][0] == runs[1][0]
    skip = {f"aux{l}" for l, cnt in enumerate(fresh)
            if flags == "defer" and cnt["phase"] == B.PHASE_ACCUMULATING and cnt["t"] == cnt["t_last"] and cnt["t"] > 0}
    for k in runs[0][1]:
        if k not in skip:
            assert np.array_equal(runs[0][1][k].view(np.uint32), runs[1][1][k].view(np.uint32)), k
    o32, log32 = oracle_run(w, trace, None, 32, FORM_LITERAL if flags == "snapshot" else FORM_ACCUMULATOR,
                            momentum_bf16=(flags == "bf16m"))
    check_step_logs(trace, runs[1][0], log32)
    ref = oracle_state(o32, w.n_lps, snapshot_form=(flags == "snapshot"))
    for k in skip:
        ref.pop(k)
    gpu = {k: v for k, v in runs[1][1].items() if not k.startswith("pull")}
    worst, n_diff, name = compare_state(gpu, ref, bitwise=True)
    assert n_diff == 0, (n_diff, worst, name)


def test_batch_call_on_a_single_item_is_the_ordinary_step():
    from paper_2506_04531_amd import binding as B
    w = synth.get_workload("tiny").scaled(synth.flat_layout(9000), n_updates=4, name="batch1")
    trace = synth.make_trace(w)
    c = _cluster(w, trace)
    try:
        h = c.lps[0]
        assert B.halos_lps_step_batch(h, 4, True) == []                       # empty queue
        B.halos_lps_push_update(h, 0, c.pool[0], c.delta_dtype)
        infos = B.halos_lps_step_batch(h, 4, True)
        assert len(infos) == 1 and (infos[0].kind, infos[0].t, infos[0].worker) == (1, 1, 0)
        B.halos_lps_push_update(h, 0, c.pool[0], c.delta_dtype)
        B.halos_lps_push_update(h, 1, c.pool[1], c.delta_dtype)
        infos = B.halos_lps_step_batch(h, 1, False)                            # asked for one: takes one
        assert len(infos) == 1 and infos[0].t == 2
        infos = B.halos_lps_step_batch(h, 4, False)
        assert len(infos) == 1 and infos[0].t == 3 and B.halos_lps_get_counters(h)["queued"] == 0
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_step_batch(h, 5, False)
        assert e.value.status == B.EINVAL
    finally:
        c.close()


@pytest.mark.parametrize("flags", [0, "snapshot", "defer", "bf16m", "delayed", "delayed+snapshot", "nopull"])
def test_batch_that_opens_with_the_merge_equals_the_steps_one_by_one(flags):
    """A returned global model at the head of the queue with deltas behind it: halos_lps_step_batch merges and updates in
    one pass.  Two identical clusters take the same items, one through the batch call and one step by step; state, counters
    and the models handed back must agree bit for bit, for K reached inside the batch and not."""
    from paper_2506_04531_amd import binding as B
    fl = {0: 0, "snapshot": B.FLAG_SNAPSHOT, "defer": B.FLAG_DEFER_CLEAR, "bf16m": B.FLAG_BF16_MOMENTUM, "delayed": 0,
          "delayed+snapshot": B.FLAG_SNAPSHOT, "nopull": 0}[flags]
    pull = flags != "nopull"                         # without the hand-back the batch still opens with the merge (plain rule only)
    delayed = str(flags).startswith("delayed")       # momentum delay 3: the merge shares a pass with ONE delta, the rest follow singly
    w = replace(synth.get_workload("160m").scaled(RAGGED, n_updates=8, name=f"mergebatch-{flags}"), n_lps=1, workers_per_lps=4,
                pool_slots=4, d_l=3 if delayed else 1, eta_l=0.6 if delayed else 0.2)
    trace = synth.make_trace(w)
    out = []
    for batched in (False, True):
        hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, 2, flags=fl)
        c = _cluster(w, trace, hp=hp)
        try:
            h = c.lps[0]
            log = []
            for rnd, (K, n_behind) in enumerate([(2, 3), (5, 2), (1, 1), (2, 3)]):
                B.halos_lps_set_threshold(h, 2)
                for k in range(2):                                              # two updates complete an accumulation
                    B.halos_lps_push_update(h, k, c.pool[(rnd + k) % 4], c.delta_dtype)
                    B.halos_lps_step_pull(h)
                B.halos_gps_merge(c.gps, h)
                B.halos_lps_push_global(h)
                for k in range(n_behind):                                       # deltas arrive behind the returned model
                    B.halos_lps_push_update(h, k, c.pool[(rnd + k + 1) % 4], c.delta_dtype)
                B.halos_lps_set_threshold(h, K)
                if batched:
                    infos = B.halos_lps_step_batch(h, 4, pull)
                    assert [i.kind for i in infos] == [2] + [1] * (1 if delayed else n_behind), (rnd, [i.kind for i in infos])
                    while B.halos_lps_get_counters(h)["queued"]:
                        infos += B.halos_lps_step_batch(h, 4, pull)
                else:
                    infos = [B.halos_lps_step(h)] + [(B.halos_lps_step_pull if pull else B.halos_lps_step)(h) for _ in range(n_behind)]
                log.append([(i.kind, i.worker, i.t, i.t_last, i.delta_ready, i.accumulated) for i in infos])
                cnt = B.halos_lps_get_counters(h)
                if cnt["phase"] == B.PHASE_SENT:                                # K was reached inside the batch: send it on
                    B.halos_gps_merge(c.gps, h); B.halos_lps_push_global(h); B.halos_lps_step(h)
                else:                                                           # finish the accumulation for the next round
                    while B.halos_lps_get_counters(h)["phase"] != B.PHASE_SENT:
                        B.halos_lps_set_threshold(h, 1)
                        B.halos_lps_push_update(h, 3, c.pool[rnd % 4], c.delta_dtype); B.halos_lps_step_pull(h)
                    B.halos_gps_merge(c.gps, h); B.halos_lps_push_global(h); B.halos_lps_step(h)
            torch.cuda.synchronize()
            state = {k: c.flat(k) for k in c.state_lists()}
            state["pull"] = torch.cat([t.reshape(-1) for t in c.pull_dst[0]]).cpu().numpy()
            fresh = B.halos_lps_get_counters(h)
            out.append((log, state, fresh))
        finally:
            c.close()
    assert out[0][0] == out[1][0]
    assert out[0][2] == out[1][2]
    for k in out[0][1]:
        if flags == "defer" and k == "aux0":
            continue                                                            # ends right after a merge: unspecified there
        assert np.array_equal(out[0][1][k].view(np.uint32), out[1][1][k].view(np.uint32)), k


# ---------------------------------------------------------------- the variants at full benchmark size
@pytest.mark.parametrize("name,variant", [("160m", "batch+defer"), ("70m", "nomom+f16"), ("410m", "weighted+snapshot"),
                                          ("160m", "bf16-momentum")])
def test_variants_at_full_size_on_sampled_elements(name, variant):
    """Full benchmark sizes, arena placement, fused pulls, the variants switched on; the oracle replays the sampled
    elements (random ones plus every tensor and tile boundary)."""
    from paper_2506_04531_amd import binding as B
    from parity_util import sample_indices
    w = synth.get_workload(name)
    flags, batch, form = 0, 0, FORM_ACCUMULATOR
    if variant == "bf16-momentum":
        flags, batch = B.FLAG_BF16_MOMENTUM, 4
    elif variant == "batch+defer":
        flags, batch = B.FLAG_DEFER_CLEAR, 4
    elif variant == "nomom+f16":
        w = replace(w, delta_dtype="f16", beta_g=0.0)
        flags = B.FLAG_GPS_NO_MOMENTUM
    else:
        w = replace(w, staleness_exponent=0.5)
        flags, form = B.FLAG_SNAPSHOT, FORM_LITERAL
    trace = synth.make_trace(w)
    idx = sample_indices(w.layout, 1 << 16, seed=7)
    print(f"[parity] workload={name} variant={variant} n={w.layout.total} sample={idx.size} events={len(trace.events)}", flush=True)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0], flags=flags)
    c = _cluster(w, trace, placement="regions", hp=hp)
    try:
        gpu_log, tm = c.replay(trace.events, fuse_pull=True, batch=batch, timed=True)
        torch.cuda.synchronize()
        gpu = {k: c.gather(k, torch.from_numpy(idx)) for k in c.state_lists()}
        fresh = [B.halos_lps_get_counters(h) for h in c.lps]
    finally:
        c.close()
        del c
        torch.cuda.empty_cache()
    if batch:
        assert any(k.startswith("lps_update_batch") for k in tm), "the full-size schedule must contain bursts"
    o32, log32 = oracle_run(w, trace, idx, 32, form, momentum_bf16=bool(flags & B.FLAG_BF16_MOMENTUM))
    check_step_logs(trace, gpu_log, log32)
    ref = oracle_state(o32, w.n_lps, snapshot_form=(form == FORM_LITERAL))
    if flags & B.FLAG_GPS_NO_MOMENTUM:
        ref.pop("M")
    if flags & B.FLAG_DEFER_CLEAR:
        for l, cnt in enumerate(fresh):
            if cnt["phase"] == B.PHASE_ACCUMULATING and cnt["t"] == cnt["t_last"] and cnt["t"] > 0:
                ref.pop(f"aux{l}")
    if flags & B.FLAG_GPS_NO_MOMENTUM:
        for k, v in gpu.items():
            assert np.array_equal(v, ref[k][0].astype(np.float32)), k          # numerically exact (sign of zero aside)
    else:
        worst, n_diff, wname = compare_state(gpu, ref, bitwise=True)
        assert n_diff == 0, (n_diff, worst, wname)


# ---------------------------------------------------------------- momentum kept in bfloat16
@pytest.mark.parametrize("recipe,dtype,mode", [("70m", "f32", "plain"), ("160m", "bf16", "pull"), ("410m", "f32", "pull+batch"),
                                               ("160m", "f16", "snapshot"), ("70m", "f32", "norms")])
def test_bf16_momentum_every_element(recipe, dtype, mode):
    """HALOS_FLAG_BF16_MOMENTUM: the momentum arrays of both tiers hold bfloat16 and every new momentum is rounded (nearest
    even) before it enters the step.  The rounding is decided on the fp32 value, so the reference is the fp32
    same-order oracle with the same option: every array bit for bit (the 16-bit momentum upcast exactly)."""
    from paper_2506_04531_amd import binding as B
    lay = RAGGED if recipe != "160m" else synth.gpt_layout(96, 2, vocab=1031)
    w = replace(synth.get_workload(recipe).scaled(lay, n_updates=120, name=f"{recipe}-bf16m-{mode}"), delta_dtype=dtype)
    trace = synth.make_trace(w, seed=91)
    flags = B.FLAG_BF16_MOMENTUM | (B.FLAG_SNAPSHOT if mode == "snapshot" else 0) | (B.FLAG_NORMS if mode == "norms" else 0)
    form = FORM_LITERAL if mode == "snapshot" else FORM_ACCUMULATOR
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, w.k_range[0], flags=flags)
    print(f"[parity] workload={w.name} n={w.layout.total} dtype={dtype} mode={mode} events={len(trace.events)}", flush=True)
    c = _cluster(w, trace, hp=hp)
    try:
        assert all(t.dtype == torch.bfloat16 for t in c.M) and all(t.dtype == torch.bfloat16 for ts in c.m for t in ts)
        gpu_log, _ = c.replay(trace.events, fuse_pull=(mode != "plain"), batch=4 if mode == "pull+batch" else 0)
        torch.cuda.synchronize()
        gpu = {k: c.flat(k) for k in c.state_lists()}
        norms = B.halos_lps_get_norms(c.lps[0]) if mode == "norms" else None
    finally:
        c.close()
    o32, log32 = oracle_run(w, trace, None, 32, form, momentum_bf16=True)
    check_step_logs(trace, gpu_log, log32)
    worst, n_diff, name = compare_state(gpu, oracle_state(o32, w.n_lps, snapshot_form=(mode == "snapshot")), bitwise=True)
    assert n_diff == 0, (n_diff, worst, name)
    assert np.any(gpu["M"] != 0) and np.any(gpu["m0"] != 0)
    if norms is not None:
        ref = o32.norms(0)
        assert abs(norms[0] - ref[0]) <= 1e-4 * ref[0] and abs(norms[1] - ref[1]) <= 1e-4 * max(ref[1], 1e-30)
    # for the record: how far the rounding moves the models from the full-precision fp64 reference
    o64, _ = oracle_run(w, trace, None, 64, FORM_LITERAL)
    ref64 = o64.get(O.GPS_THETA)
    dev_rel = float(np.sqrt(np.mean((gpu["Theta"] - ref64) ** 2)) / np.sqrt(np.mean(ref64 ** 2)))
    print(f"[parity] {w.name}: bit-exact vs the fp32 oracle with bfloat16 momentum; rms deviation of Theta from the "
          f"full-precision fp64 reference {dev_rel:.3g} of its rms", flush=True)
    assert dev_rel < 1e-3


def test_bf16_momentum_on_the_single_tier_server_and_with_end_models():
    """The global server applying worker deltas itself, and a local server forming the delta from the worker's end model,
    both with 16-bit momentum."""
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import alloc_tensor_list, fill_delta_slot, fill_initial_model
    dev = torch.device("cuda:0")
    w = replace(synth.get_workload("70m").scaled(RAGGED, n_updates=1, name="bf16m-single"), eta_g=0.05, beta_g=0.9)
    numel = [int(x) for x in w.layout.numel]
    f32, bf16 = torch.float32, torch.bfloat16
    Theta, th, acc, wm, end = (alloc_tensor_list(numel, f32, dev) for _ in range(5))
    M, m = alloc_tensor_list(numel, bf16, dev), alloc_tensor_list(numel, bf16, dev)
    fill_initial_model(w, Theta)
    pool = []
    for s in range(3):
        ts = alloc_tensor_list(numel, f32, dev)
        fill_delta_slot(w, s, ts)
        pool.append(ts)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, 8, flags=B.FLAG_BF16_MOMENTUM)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
    flat = lambda ts: torch.cat([t.reshape(-1) for t in ts]).float().cpu().numpy()
    try:
        B.halos_lps_set_worker_model(lps, 0, wm)
        B.halos_pull_model(lps, False, wm)                                  # the worker's start model
        for a, b, d in zip(end, wm, pool[2]):                               # its end model: start minus some progress
            a.copy_(b - d)
        B.halos_lps_push_end_model(lps, 0, end)
        B.halos_lps_step_pull(lps)
        for k in range(5):
            B.halos_gps_push_update(gps, pool[k % 3], B.F32, 1.0 if k != 2 else 0.5)
        torch.cuda.synchronize()
        gpu = {"Theta": flat(Theta), "M": flat(M), "theta0": flat(th), "m0": flat(m), "aux0": flat(acc), "wm": flat(wm)}
        end_host = flat(end)
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
    idx = torch.arange(w.layout.total, dtype=torch.int64)
    theta0 = synth.normal_at(w.seed, 0, idx, synth.tensors.scale_f32(w.init_sigma)).numpy()
    scale = torch.from_numpy(synth.delta_scales(w)[w.layout.tensor_of(idx.numpy())])
    deltas = [synth.normal_at(w.seed, 1 + s, idx, scale).numpy() for s in range(3)]
    o = HalosOracle(theta0, 1, eta_l=w.eta_l, beta_l=w.beta_l, eta_g=w.eta_g, beta_g=w.beta_g, alpha=w.alpha, K=8,
                    precision=32, form=FORM_ACCUMULATOR, momentum_bf16=True)
    g = theta0 - end_host                                                   # start - end, in fp32 like a worker would
    o.arrive_delta(0, 0, g); o.lps_step(0)
    for k in range(5):
        o.gps_apply_delta(deltas[k % 3], 1.0 if k != 2 else 0.5)
    for name, what in (("Theta", O.GPS_THETA), ("M", O.GPS_MOM), ("theta0", O.THETA), ("m0", O.MOM), ("aux0", O.AUX)):
        ref = o.get(what).astype(np.float32)
        assert np.array_equal(gpu[name].view(np.uint32), ref.view(np.uint32)), name
    assert np.array_equal(gpu["wm"].view(np.uint32), gpu["theta0"].view(np.uint32))     # the worker got the updated model back


def test_bf16_momentum_refuses_what_is_not_built_for_it():
    from paper_2506_04531_amd import binding as B
    w = synth.get_workload("tiny").scaled(synth.flat_layout(5000), n_updates=4, name="bf16m-refuse")
    trace = synth.make_trace(w)
    hp = B.paper_hparams(w.eta_l, w.beta_l, w.eta_g, w.beta_g, w.alpha, 4, flags=B.FLAG_BF16_MOMENTUM)
    c = _cluster(w, trace, hp=hp)
    try:
        buf = [torch.zeros(5000, device="cuda:0")]
        for call in (lambda: B.halos_lps_set_momentum_delay(c.lps[0], 4, buf), lambda: B.halos_gps_set_momentum_delay(c.gps, 2, buf)):
            with pytest.raises(B.HalosError) as e:
                call()
            assert e.value.status == B.ESTATE and "bfloat16" in str(e.value)
        B.halos_lps_set_momentum_delay(c.lps[0], 1, None)                   # delay 1 is the plain rule: fine
    finally:
        c.close()
