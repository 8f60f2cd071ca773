"""Error behaviour of the C ABI on a real device: every misuse returns a status, leaves state untouched,
and no kernel is launched on bad operands."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture()
def small():
    from paper_2506_04531_amd import binding as B
    numel = [5000, 0, 37]
    dev = "cuda:0"
    mk = lambda dt=torch.float32: [torch.zeros(n, dtype=dt, device=dev) for n in numel]
    Theta = mk()
    for t in Theta:
        t.normal_(0, 0.02)
    M = [torch.full_like(t, 7.0) for t in Theta]              # create must zero it
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 2)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    th, m, acc = mk(), mk(), mk()
    for t in th + m + acc:
        t.fill_(3.0)                                          # create must overwrite all three
    lps = B.halos_lps_create(gps, 0, 2, th, m, acc)
    torch.cuda.synchronize()
    yield dict(B=B, numel=numel, Theta=Theta, M=M, th=th, m=m, acc=acc, gps=gps, lps=lps, mk=mk, hp=hp)
    B.halos_lps_destroy(lps)
    B.halos_gps_destroy(gps)


def _status(fn, *a):
    from paper_2506_04531_amd import binding as B
    try:
        fn(*a)
    except B.HalosError as e:
        return e.status
    return B.OK


def test_create_initialises_state(small):
    s = small
    for a, b in zip(s["th"], s["Theta"]):
        assert torch.equal(a, b)                               # Alg. 1, LPS initialisation: theta_0 <- Theta_0
    for t in s["m"] + s["acc"] + s["M"]:
        assert not t.any()
    c = s["B"].halos_lps_get_counters(s["lps"])
    assert (c["t"], c["t_last"], c["phase"], c["queued"]) == (0, 0, 0, 0)


def test_bad_arguments_are_einval(small):
    s, B = small, small["B"]
    g = s["mk"]()
    assert _status(B.halos_lps_push_update, s["lps"], 2, g, B.F32) == B.EINVAL          # worker out of range
    assert _status(B.halos_lps_push_update, s["lps"], -1, g, B.F32) == B.EINVAL
    assert _status(B.halos_lps_push_update, s["lps"], 0, g, 7) == B.EINVAL              # unknown dtype
    assert _status(B.halos_lps_push_update, s["lps"], 0, [None, None, None], B.F32) == B.EINVAL
    short = [torch.zeros(100, device="cuda:0"), None, torch.zeros(37, device="cuda:0")]
    # a 100-element tensor where 5000 are needed: rejected unless torch happened to carve it from a larger block
    st = _status(B.halos_lps_push_update, s["lps"], 0, short, B.F32)
    assert st in (B.EINVAL, B.OK)
    if st == B.OK:
        B.halos_lps_step(s["lps"])
    mis = [g[0].data_ptr() + 4, None, g[2].data_ptr()]
    assert _status(B.halos_lps_push_update, s["lps"], 1, mis, B.F32) == B.EINVAL        # not 16-byte aligned
    host = np.zeros(5000, dtype=np.float32)
    assert _status(B.halos_lps_push_update, s["lps"], 1, [host.ctypes.data & ~15, None, g[2].data_ptr()], B.F32) == B.EINVAL
    assert "tensor 0" in B.halos_last_error()
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 1.5, 2)                                   # alpha > 1
    assert _status(B.halos_set_hparams, s["lps"], False, hp) == B.EINVAL
    hp = B.paper_hparams(float("nan"), 0.9, 0.15, 0.5, 0.25, 2)
    assert _status(B.halos_set_hparams, s["gps"], True, hp) == B.EINVAL
    assert _status(B.halos_lps_set_threshold, s["lps"], 0) == B.EINVAL
    assert _status(B.halos_pull_model, s["lps"], True, g) == B.EINVAL                   # an LPS handle passed as GPS
    assert _status(B.halos_gps_create, [], s["hp"], [], []) == B.EINVAL
    assert _status(B.halos_gps_create, [-1], s["hp"], g[:1], g[:1]) == B.EINVAL
    assert _status(B.halos_lps_create, s["gps"], 0, 0, s["th"], s["m"], s["acc"]) == B.EINVAL


def test_protocol_violations_are_estate_and_change_nothing(small):
    s, B = small, small["B"]
    g = s["mk"]()
    for t in g:
        t.fill_(1.0 / 1024)
    snap = lambda: [t.clone() for t in s["th"] + s["m"] + s["acc"] + s["Theta"] + s["M"]]
    same = lambda a: all(torch.equal(x, y) for x, y in zip(a, s["th"] + s["m"] + s["acc"] + s["Theta"] + s["M"]))
    before = snap()
    assert _status(B.halos_gps_merge, s["gps"], s["lps"]) == B.ESTATE                   # nothing accumulated yet
    assert _status(B.halos_lps_push_global, s["lps"]) == B.ESTATE
    info = B.halos_lps_step(s["lps"])
    assert info.kind == 0                                                                # empty queue: OK, no-op
    torch.cuda.synchronize()
    assert same(before)
    B.halos_lps_push_update(s["lps"], 0, g, B.F32, 3)
    assert _status(B.halos_lps_push_update, s["lps"], 0, g, B.F32) == B.ESTATE          # same worker twice
    B.halos_lps_push_update(s["lps"], 1, g, B.F32, 5)
    assert B.halos_lps_get_counters(s["lps"])["max_staleness"] == 5
    assert B.halos_lps_step(s["lps"]).delta_ready == 0
    assert B.halos_lps_step(s["lps"]).delta_ready == 1                                   # K = 2
    assert _status(B.halos_lps_push_global, s["lps"]) == B.ESTATE                        # GPS has not run
    B.halos_gps_merge(s["gps"], s["lps"])
    assert _status(B.halos_gps_merge, s["gps"], s["lps"]) == B.ESTATE                    # already consumed
    torch.cuda.synchronize()
    mid = snap()
    B.halos_lps_push_global(s["lps"])
    assert _status(B.halos_lps_push_global, s["lps"]) == B.ESTATE
    torch.cuda.synchronize()
    assert same(mid)
    info = B.halos_lps_step(s["lps"])
    assert (info.kind, info.t, info.t_last) == (2, 2, 2)
    assert B.halos_gps_get_counters(s["gps"])["updates"] == 1
    torch.cuda.synchronize()
    assert not any(t.any() for t in s["acc"])


def test_merge_endpoints_exact_on_device(small):
    """alpha = 1 returns the global model bit for bit, alpha = 0 leaves the local model untouched."""
    s, B = small, small["B"]
    g = s["mk"]()
    for t in g:
        t.normal_(0, 1e-3)
    for alpha in (1.0, 0.0):
        hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, alpha, 1)
        B.halos_set_hparams(s["lps"], False, hp)
        B.halos_lps_push_update(s["lps"], 0, g, B.F32)
        assert B.halos_lps_step(s["lps"]).delta_ready == 1
        B.halos_gps_merge(s["gps"], s["lps"])
        B.halos_lps_push_update(s["lps"], 1, g, B.F32)                                   # applied while in flight
        assert B.halos_lps_step(s["lps"]).accumulated == 0
        torch.cuda.synchronize()
        local = [t.clone() for t in s["th"]]
        inbox = [t.clone() for t in s["acc"]]
        for a, b in zip(inbox, s["Theta"]):
            assert torch.equal(a, b)                                                     # the returned model is this Theta_i
        B.halos_lps_push_global(s["lps"])
        assert B.halos_lps_step(s["lps"]).kind == 2
        torch.cuda.synchronize()
        want = inbox if alpha == 1.0 else local
        for a, b in zip(s["th"], want):
            assert torch.equal(a, b)


def test_many_tensors_need_several_launch_ranges():
    """More tensors than fit one kernel-argument block: the call is split into launch ranges."""
    from paper_2506_04531_amd import binding as B
    n_t = 900
    numel = [17 + (i % 5) * 4099 for i in range(n_t)]
    dev = "cuda:0"
    mk = lambda: [torch.zeros(n, device=dev) for n in numel]
    Theta, M, th, m, acc, g, dst = mk(), mk(), mk(), mk(), mk(), mk(), mk()
    for i, t in enumerate(Theta):
        t.fill_(float(i))
    for i, t in enumerate(g):
        t.fill_(1.0 + i / 1024.0)
    hp = B.paper_hparams(1.0, 0.0, 1.0, 0.0, 0.5, 1)          # beta = 0, eta = 1: theta <- theta - g
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
    try:
        B.halos_lps_push_update(lps, 0, g, B.F32)
        B.halos_lps_step(lps)
        B.halos_pull_model(lps, False, dst)
        torch.cuda.synchronize()
        for i in range(n_t):
            expect = float(i) - (1.0 + i / 1024.0)
            assert torch.all(th[i] == expect) and torch.all(dst[i] == expect) and torch.all(acc[i] == 1.0 + i / 1024.0), i
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)


def test_hand_derived_worked_example_through_the_library():
    """The integer example derived by hand from Algorithm 1 (tests/golden) replayed through the C ABI: the GPU
    path is held to the paper-derived numbers directly, not only to the oracle."""
    import json
    import os
    from paper_2506_04531_amd import binding as B
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "alg1_worked_example.json")) as f:
        ex = json.load(f)
    dev = "cuda:0"
    n = len(ex["theta0"])
    T = lambda v: torch.tensor(v, dtype=torch.float32, device=dev)
    Theta, M = [T(ex["theta0"])], [torch.zeros(n, device=dev)]
    hp = B.paper_hparams(ex["eta_l"], ex["beta_l"], ex["eta_g"], ex["beta_g"], ex["alpha"], ex["K"],
                         cg_l=ex["cg_l"], cg_g=ex["cg_g"])
    gps = B.halos_gps_create([n], hp, Theta, M)
    state = [([torch.empty(n, device=dev)], [torch.empty(n, device=dev)], [torch.empty(n, device=dev)])
             for _ in range(ex["n_lps"])]
    lps = [B.halos_lps_create(gps, l, 2, *state[l]) for l in range(ex["n_lps"])]
    keep = []
    try:
        for step in ex["script"]:
            l = step["lps"]
            if step["op"] == "delta":
                g = [T(step["g"])]
                keep.append(g)
                B.halos_lps_push_update(lps[l], step["worker"], g, B.F32)
            elif step["op"] == "step":
                info = B.halos_lps_step(lps[l])
                e = step["expect"]
                assert (info.kind, info.t, info.t_last, info.delta_ready) == (e["kind"], e["t"], e["t_last"], e["sent"]), step
                if "expect_theta" in step:
                    torch.cuda.synchronize()
                    assert state[l][0][0].tolist() == step["expect_theta"]
            elif step["op"] == "gps":
                B.halos_gps_merge(gps, lps[l])
                torch.cuda.synchronize()
                assert Theta[0].tolist() == step["expect_Theta"]
            elif step["op"] == "global":
                B.halos_lps_push_global(lps[l])
        torch.cuda.synchronize()
        fin = ex["final"]
        for l in range(ex["n_lps"]):
            assert state[l][0][0].tolist() == fin["theta"][l]
            assert state[l][2][0].tolist() == fin["aux"][l]
            c = B.halos_lps_get_counters(lps[l])
            assert (c["t"], c["t_last"]) == (fin["t"][l], fin["t_last"][l])
        assert Theta[0].tolist() == fin["Theta"]
        assert B.halos_gps_get_counters(gps)["updates"] == fin["gps_updates"]
    finally:
        for h in lps:
            B.halos_lps_destroy(h)
        B.halos_gps_destroy(gps)


def test_plain_c_client_of_the_abi():
    """tests/host/abi_client.c: the boundary used from C with hipMalloc'ed memory, no Python in the loop."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "host", "abi_client")
    assert os.path.exists(exe), "abi_client is built by __graft_entry__.build()"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(res.stdout, res.stderr)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "all values as derived" in res.stdout


def test_gps_may_be_destroyed_before_its_local_servers():
    """The local servers launch with their GPS's layout tables: those must outlive a GPS handle that is destroyed first."""
    from paper_2506_04531_amd import binding as B
    n = 2 * 4096 + 3
    mk = lambda: [torch.zeros(n, device="cuda:0")]
    Theta, M, th, m, acc, dst = [torch.randn(n, device="cuda:0")], mk(), mk(), mk(), mk(), mk()
    g = [torch.full((n,), 0.5, device="cuda:0")]
    hp = B.paper_hparams(1.0, 0.0, 1.0, 0.0, 0.0, 1 << 20)
    gps = B.halos_gps_create([n], hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 1, th, m, acc)
    B.halos_gps_destroy(gps)
    assert _status(B.halos_gps_get_counters, gps) == B.EINVAL            # the handle is gone for the caller
    assert _status(B.halos_lps_create, gps, 1, 1, th, m, acc) == B.EINVAL
    B.halos_lps_push_update(lps, 0, g, B.F32)                             # ... but the local server still works
    assert B.halos_lps_step(lps).kind == 1
    B.halos_pull_model(lps, False, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst[0], Theta[0] - 0.5)
    B.halos_lps_destroy(lps)                                              # releases the GPS's tables too
    # destroyed handles are refused by every call (they are looked up in the registry of live handles, never dereferenced)
    assert _status(B.halos_lps_step, lps) == B.EINVAL
    assert _status(B.halos_lps_push_global, lps) == B.EINVAL
    assert _status(B.halos_lps_get_counters, lps) == B.EINVAL
    assert _status(B.halos_pull_model, gps, True, dst) == B.EINVAL
    B.halos_lps_destroy(lps)                                              # destroying twice is harmless
    B.halos_gps_destroy(gps)
    arena = B.halos_arena_create([1 << 20], max_walk_bytes=4 << 30)
    B.halos_arena_destroy(arena)
    assert _status(B.halos_arena_alloc, arena, 0, 256) == B.EINVAL
    B.halos_arena_destroy(arena)


def test_end_model_must_not_overlap_the_registered_start_model():
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    n = 9000
    Theta, M, th, m, acc, wm, end = (torch.zeros(n, device=dev) for _ in range(7))
    gps = B.halos_gps_create([n], B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4), [Theta], [M])
    lps = B.halos_lps_create(gps, 0, 1, [th], [m], [acc])
    try:
        B.halos_lps_set_worker_model(lps, 0, [wm])
        for bad in ([wm], [wm.data_ptr() + 4096]):                 # the buffer itself, and a view into it
            with pytest.raises(B.HalosError) as e:
                B.halos_lps_push_end_model(lps, 0, bad)
            assert e.value.status == B.EINVAL and "overlaps" in e.value.message
        assert B.halos_lps_get_counters(lps)["queued"] == 0
        B.halos_lps_push_end_model(lps, 0, [end])
        assert B.halos_lps_step_pull(lps).kind == 1
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)


def test_forget_buffers_makes_the_next_pointer_set_be_checked_again():
    """A pointer set is range-checked when a server first sees it.  After halos_forget_buffers the same addresses are
    checked again: here the second time they belong to an allocation that is too small."""
    from paper_2506_04531_amd import binding as B
    dev = torch.device("cuda:0")
    n = 1 << 20
    Theta, M, th, m, acc = (torch.zeros(n, device=dev) for _ in range(5))
    # an allocation of exactly known size: the arena gives a request above 2 GiB a device allocation of its own
    big_bytes = (2 << 30) + (64 << 20)
    arena = B.halos_arena_create([1 << 20], 4 << 30)
    big = B.halos_arena_alloc(arena, 0, big_bytes)
    gps = B.halos_gps_create([n], B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 4), [Theta], [M])
    lps = B.halos_lps_create(gps, 0, 1, [th], [m], [acc])
    try:
        tail = big + big_bytes - n * 4                               # the last n floats of the allocation: fits exactly
        torch.cuda.synchronize()
        B.halos_probe_streams([], [tail], n * 4, 1)                  # zero-fill them (the probe writes zeros)
        B.halos_lps_push_update(lps, 0, [tail], B.F32)
        assert B.halos_lps_step(lps).kind == 1
        short = tail + (2 << 20)                                      # n floats from here run 2 MiB past the allocation
        with pytest.raises(B.HalosError) as e:
            B.halos_lps_push_update(lps, 0, [short], B.F32)
        assert e.value.status == B.EINVAL
        B.halos_lps_push_update(lps, 0, [tail], B.F32)               # remembered: accepted without a new check
        assert B.halos_lps_step(lps).kind == 1
        B.halos_forget_buffers(lps, False)
        B.halos_forget_buffers(gps, True)
        B.halos_lps_push_update(lps, 0, [tail], B.F32)               # checked again, still fine
        assert B.halos_lps_step(lps).kind == 1
        with pytest.raises(B.HalosError):
            B.halos_forget_buffers(0, False)
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
        B.halos_arena_destroy(arena)


def test_many_tensors_through_the_multi_delta_passes():
    """More tensors than one launch range, zero-sized tensors among them, through halos_lps_step_batch (deltas only, and
    opening with a merge) and halos_lps_step_average: the per-worker device tables of delta pointers span all ranges.  beta = 0, eta = 1 and
    dyadic values make every expected number exact."""
    from paper_2506_04531_amd import binding as B
    n_t = 800
    numel = [0 if i % 97 == 5 else 9 + (i % 7) * 2051 for i in range(n_t)]
    dev = "cuda:0"
    mk = lambda fill=None: [torch.zeros(n, device=dev) if fill is None else torch.full((n,), fill(i), device=dev)
                            for i, n in enumerate(numel)]
    Theta, M, th, m, acc = mk(lambda i: float(i)), mk(), mk(), mk(), mk()
    g = [mk(lambda i, k=k: (k + 1) * 0.25 + i / 256.0) for k in range(3)]
    wm = [mk() for _ in range(3)]
    hp = B.paper_hparams(1.0, 0.0, 1.0, 0.0, 0.5, 1 << 30)
    gps = B.halos_gps_create(numel, hp, Theta, M)
    lps = B.halos_lps_create(gps, 0, 3, th, m, acc)
    try:
        for k in range(3):
            B.halos_lps_set_worker_model(lps, k, wm[k])
            B.halos_lps_push_update(lps, k, g[k], B.F32)
        infos = B.halos_lps_step_batch(lps, 4, True)
        assert [i.t for i in infos] == [1, 2, 3] and [i.worker for i in infos] == [0, 1, 2]
        torch.cuda.synchronize()
        for i in range(n_t):
            if numel[i] == 0:
                continue
            run = float(i)
            for k in range(3):
                run -= (k + 1) * 0.25 + i / 256.0
                assert torch.all(wm[k][i] == run), (i, k)            # each worker got the model right after ITS update
            assert torch.all(th[i] == run) and torch.all(acc[i] == float(i) - run), i
        # averaged step over the first two deltas: one update with their mean (0.375 + i/256; the factor 1/2 is exact)
        for k in range(2):
            B.halos_lps_push_update(lps, k, g[k], B.F32)
        info = B.halos_lps_step_average(lps, 2)
        assert (info.t, info.worker) == (4, 1)
        torch.cuda.synchronize()
        for i in range(n_t):
            if numel[i]:
                want = float(i) - 1.5 - 3 * (i / 256.0) - 0.375 - i / 256.0
                assert torch.all(th[i] == want), (i, float(th[i][0]), want)
        # a batch that opens with the merge: complete the accumulation, add one update while it is in flight, let the
        # global server answer, then take [returned model, delta, delta] in one call
        B.halos_lps_set_threshold(lps, 1)
        B.halos_lps_push_update(lps, 0, g[0], B.F32)
        assert B.halos_lps_step_batch(lps, 4, True)[0].delta_ready == 1
        B.halos_lps_push_update(lps, 2, g[2], B.F32)
        assert B.halos_lps_step_pull(lps).accumulated == 0
        B.halos_gps_merge(gps, lps)                                  # Theta <- Theta - G = the local model at the send
        B.halos_lps_push_global(lps)
        B.halos_lps_push_update(lps, 1, g[1], B.F32)
        B.halos_lps_push_update(lps, 2, g[2], B.F32)
        B.halos_lps_set_threshold(lps, 1 << 30)
        infos = B.halos_lps_step_batch(lps, 4, True)
        assert [i.kind for i in infos] == [2, 1, 1] and [i.worker for i in infos] == [-1, 1, 2]
        assert [i.t_last for i in infos] == [6, 6, 6] and [i.t for i in infos] == [6, 7, 8]
        torch.cuda.synchronize()
        for i in range(n_t):
            if numel[i]:
                sent = float(i) - 1.5 - 3 * (i / 256.0) - 0.375 - i / 256.0 - (0.25 + i / 256.0)      # model at the send = Theta_i
                merged = 0.5 * sent + 0.5 * (sent - (0.75 + i / 256.0))                                # alpha = 1/2
                after1 = merged - (0.5 + i / 256.0)
                after2 = after1 - (0.75 + i / 256.0)
                assert torch.all(Theta[i] == sent), i
                assert torch.all(wm[1][i] == after1) and torch.all(wm[2][i] == after2) and torch.all(th[i] == after2), i
                assert torch.all(acc[i] == 1.25 + 2 * (i / 256.0)), i                                  # restarted by the merge
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)


def test_create_and_destroy_give_back_what_they_took():
    """The library's own device allocations (tile table, pointer tables, norm scratch, arena slabs) are released by the
    destroy calls: after many create / use / destroy rounds the device has as much free memory as before."""
    from paper_2506_04531_amd import binding as B
    dev = "cuda:0"
    numel = [5000, 0, 12345, 4096]
    mk = lambda: [torch.zeros(n, device=dev) for n in numel]
    Theta, M, th, m, acc, g, wm = (mk() for _ in range(7))
    norms_out = torch.zeros(2, dtype=torch.float64, device=dev)

    def one_round(flags):
        hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 2, flags=flags)
        gps = B.halos_gps_create(numel, hp, Theta, M)
        lps = B.halos_lps_create(gps, 0, 2, th, m, acc)
        B.halos_lps_set_worker_model(lps, 0, wm)
        B.halos_lps_set_worker_model(lps, 1, wm)
        for k in range(2):
            B.halos_lps_push_update(lps, k, g, B.F32)
        assert len(B.halos_lps_step_batch(lps, 4, True)) == (1 if flags & B.FLAG_NORMS else 2)
        while B.halos_lps_get_counters(lps)["queued"]:
            B.halos_lps_step_pull(lps)
        B.halos_gps_merge(gps, lps)
        B.halos_lps_push_global(lps)
        B.halos_lps_step(lps)
        B.halos_gps_destroy(gps)            # retired first, released with its last local server
        B.halos_lps_destroy(lps)

    torch.cuda.synchronize()
    one_round(0)                             # warm: the runtime's own pools settle
    one_round(B.FLAG_NORMS)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for r in range(150):
        one_round(B.FLAG_NORMS if r % 2 else 0)
    arena = B.halos_arena_create([1 << 28, 1 << 28], max_walk_bytes=8 << 30)
    B.halos_arena_destroy(arena)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after >= free_before - (8 << 20), (free_before, free_after)


def test_a_layout_of_empty_tensors_runs_the_protocol_and_launches_nothing():
    """Degenerate input: every tensor of the layout has zero elements.  The protocol (queue, counters, send test, merge)
    still runs; there is nothing to compute."""
    from paper_2506_04531_amd import binding as B
    numel = [0, 0, 0]
    none = [None, None, None]
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 2)
    gps = B.halos_gps_create(numel, hp, none, none)
    lps = B.halos_lps_create(gps, 0, 2, none, none, none)
    try:
        B.halos_lps_set_worker_model(lps, 0, none)
        B.halos_lps_set_worker_model(lps, 1, none)
        B.halos_lps_push_update(lps, 0, none, B.BF16)
        B.halos_lps_push_update(lps, 1, none, B.BF16)
        infos = B.halos_lps_step_batch(lps, 4, True)
        assert [(i.kind, i.t, i.delta_ready) for i in infos] == [(1, 1, 0), (1, 2, 1)]
        B.halos_gps_merge(gps, lps)
        B.halos_lps_push_global(lps)
        B.halos_lps_push_update(lps, 0, none, B.BF16)
        infos = B.halos_lps_step_batch(lps, 4, True)
        assert [(i.kind, i.t, i.t_last) for i in infos] == [(2, 2, 2), (1, 3, 2)]
        B.halos_pull_model(lps, False, none)
        B.halos_pull_model(gps, True, none)
        torch.cuda.synchronize()
        assert B.halos_gps_get_counters(gps)["updates"] == 1
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)
