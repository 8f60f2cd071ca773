"""halos_lps_step_norms -- the step for callers that cannot allocate -- against halos_lps_step on a server created
under HALOS_FLAG_NORMS (whose partial sums live in a buffer of its own): same state, same monitors, bit for bit, on
calls in a row that share the GPU's fixed scratch array, the later ones with a smaller input than the first."""
import ctypes

import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def _server_pair(numel, K, seed):
    """Two independent GPS+LPS pairs over the same layout and the same initial model: `ref` created under the flag
    (steps with halos_lps_step, monitors read with halos_lps_get_norms), `dut` without it (steps with the new call)."""
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cpu").manual_seed(seed)
    theta0 = [(0.02 * torch.randn(n, generator=gen)).to(dev) for n in numel]
    out = {}
    for name, flags in (("ref", B.FLAG_NORMS), ("dut", 0)):
        hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, K, flags=flags)
        Theta = [t.clone() for t in theta0]
        M, th, m, acc = ([torch.empty_like(t) for t in theta0] for _ in range(4))
        gps = B.halos_gps_create(numel, hp, Theta, M)
        lps = B.halos_lps_create(gps, 0, 2, th, m, acc)
        out[name] = dict(gps=gps, lps=lps, Theta=Theta, M=M, theta=th, m=m, acc=acc)
    return out, gen


def _state(s):
    return torch.cat([t.reshape(-1) for k in ("Theta", "M", "theta", "m", "acc") for t in s[k]]).cpu().numpy()


def test_step_without_allocation_matches_the_flagged_step_on_successive_sizes():
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    big = [4096 * 300 + 17, 5, 4096 * 40, 0, 1023]         # 343 tiles: 343 partial sums per launch
    small = [4096 * 2 + 3, 7]                              # 4 tiles: the second call uses only the head of the array
    K = 2
    servers = []
    try:
        pairs = []
        for numel, seed in ((big, 1), (small, 2)):
            pair, gen = _server_pair(numel, K, seed)
            servers.append(pair)
            deltas = [[(1e-3 * torch.randn(n, generator=gen)).to(dev) for n in numel] for _ in range(3)]
            pairs.append((numel, pair, deltas))
        norms_dev = torch.full((2,), -1.0, dtype=torch.float64, device=dev)
        lib = B.load_library()

        def both_step(pair, expect_kind):
            ref, dut = pair["ref"], pair["dut"]
            info_r = B.halos_lps_step(ref["lps"])
            info_d = B.halos_lps_step_norms(dut["lps"], norms_dev)
            assert (info_r.kind, info_r.t, info_r.t_last, info_r.delta_ready, info_r.accumulated, info_r.worker) == \
                   (info_d.kind, info_d.t, info_d.t_last, info_d.delta_ready, info_d.accumulated, info_d.worker)
            assert info_d.kind == expect_kind
            want = B.halos_lps_get_norms(ref["lps"])
            torch.cuda.synchronize()
            got = norms_dev.cpu().numpy()
            return want, got

        # updates in a row: big layout, then small, then big again, then small -- the array keeps the last call's contents
        for rnd in range(2):
            for numel, pair, deltas in pairs:
                for s in ("ref", "dut"):
                    B.halos_lps_push_update(pair[s]["lps"], rnd % 2, deltas[rnd], B.F32)
                want, got = both_step(pair, 1)
                assert got[0] == want[0] and want[0] > 0.0, (numel[:1], rnd, got, want)
                ref_sum = sum(float((d.double() ** 2).sum()) for d in deltas[rnd])
                assert abs(got[0] - ref_sum) <= 1e-6 * ref_sum        # and it is the sum of squares of the delta
                assert np.array_equal(_state(pair["ref"]).view(np.uint32), _state(pair["dut"]).view(np.uint32))
        # K = 2 reached on both: GPS update, returned model, merge (the monitor of a merge goes to the second slot)
        before = norms_dev.cpu().numpy().copy()
        for numel, pair, deltas in pairs:
            for s in ("ref", "dut"):
                B.halos_gps_merge(pair[s]["gps"], pair[s]["lps"])
                B.halos_lps_push_global(pair[s]["lps"])
            want, got = both_step(pair, 2)
            assert got[1] == want[1] and want[1] > 0.0, (numel[:1], got, want)
            assert got[0] == before[0]                                 # a merge leaves the first slot alone
            assert np.array_equal(_state(pair["ref"]).view(np.uint32), _state(pair["dut"]).view(np.uint32))
        # an empty queue writes nothing and reports kind 0
        norms_dev.fill_(-7.0)
        info = B.halos_lps_step_norms(pairs[0][1]["dut"]["lps"], norms_dev)
        torch.cuda.synchronize()
        assert info.kind == 0 and norms_dev.cpu().tolist() == [-7.0, -7.0]
        # argument errors: null / misaligned / host pointer, and a launch shape whose partial sums do not fit
        dut = pairs[0][1]["dut"]["lps"]
        B.halos_lps_push_update(dut, 0, pairs[0][2][2], B.F32)
        for bad in (0, norms_dev.data_ptr() + 4):
            with pytest.raises(B.HalosError) as e:
                B.halos_lps_step_norms(dut, bad)
            assert e.value.status == B.EINVAL
        host = (ctypes.c_double * 2)()
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_step_norms(dut, ctypes.addressof(host))
        assert e.value.status == B.EINVAL
        assert B.halos_lps_get_counters(dut)["queued"] == 1            # nothing was consumed by the failed calls
        assert B.halos_lps_step_norms(dut, norms_dev).kind == 1
    finally:
        for pair in servers:
            for s in pair.values():
                B.halos_lps_destroy(s["lps"])
                B.halos_gps_destroy(s["gps"])


def test_too_many_partial_sums_are_rejected():
    """The fixed array holds 16384 partial sums: a layout with more than 384 tensors needs several launches per step, and
    at 64 workgroups per compute unit these no longer fit.  The call must refuse and leave everything as it was."""
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    numel = [4096 * 44] * 385                       # two launch ranges: 384 tensors (16896 tiles) and 1 tensor (44 tiles)
    tiles_first = 384 * 44
    need = min(tiles_first, 64 * n_cu) + min(44, 64 * n_cu)
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4)
    flat = torch.zeros(sum(numel), device=dev)
    views = list(flat.split(numel))
    mk = lambda: list(torch.zeros(sum(numel), device=dev).split(numel))
    Theta, M, th, m, acc, g = views, mk(), mk(), mk(), mk(), mk()
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
    norms_dev = torch.zeros(2, dtype=torch.float64, device=dev)
    try:
        B.halos_lps_push_update(lps, 0, g, B.F32)
        B.halos_set_launch_config(64, -1)
        if need > 16384:
            with pytest.raises(B.HalosError) as e:
                B.halos_lps_step_norms(lps, norms_dev)
            assert e.value.status == B.EINVAL and "16384" in e.value.message
            assert B.halos_lps_get_counters(lps)["queued"] == 1
        B.halos_set_launch_config(1, -1)
        assert B.halos_lps_step_norms(lps, norms_dev).kind == 1
        torch.cuda.synchronize()
        assert norms_dev.cpu().tolist() == [0.0, 0.0]
    finally:
        B.halos_set_launch_config(1, 1)             # back to the defaults
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
