"""The event-loop calls of the library only launch kernels on the caller's stream (no allocation, no synchronisation,
no memset), so a caller may capture them into a HIP graph.  One full accumulation cycle -- K worker updates with the
model handed back, the GPS update, the merge -- brings the protocol back to where it started, so the captured graph
can be replayed; every replay must give exactly what the same cycle gives when issued call by call."""
import numpy as np
import pytest
import torch

from test_gpu_parity import RAGGED

pytestmark = pytest.mark.gpu


def _make(B, numel, theta0, K, n_workers, flags=0, delay=(1, 1)):
    from paper_2506_04531_amd.harness import alloc_tensor_list
    mk = lambda: alloc_tensor_list(numel, torch.float32, "cuda:0")
    s = dict(Theta=mk(), M=mk(), th=mk(), m=mk(), acc=mk(), wm=[mk() for _ in range(n_workers)], extra=[])
    for t, v in zip(s["Theta"], theta0):
        t.copy_(v)
    hp = B.paper_hparams(0.2 * delay[0], 0.9, 0.15 * delay[1], 0.5, 0.25, K, flags=flags)
    s["gps"] = B.halos_gps_create(numel, hp, s["Theta"], s["M"])
    s["lps"] = B.halos_lps_create(s["gps"], 0, n_workers, s["th"], s["m"], s["acc"])
    if delay[0] > 1:
        s["extra"].append(mk()); B.halos_lps_set_momentum_delay(s["lps"], delay[0], s["extra"][-1])
    if delay[1] > 1:
        s["extra"].append(mk()); B.halos_gps_set_momentum_delay(s["gps"], delay[1], s["extra"][-1])
    for k in range(n_workers):
        B.halos_lps_set_worker_model(s["lps"], k, s["wm"][k])
    return s


def _cycle(B, s, deltas, K):
    """K updates (worker k % n_workers, model handed back in the same pass), hand-over, GPS update, merge."""
    n_workers = len(s["wm"])
    for k in range(K):
        B.halos_lps_push_update(s["lps"], k % n_workers, deltas[k % len(deltas)], B.F32)
        info = B.halos_lps_step_pull(s["lps"])
    assert info.delta_ready == 1
    B.halos_gps_merge(s["gps"], s["lps"])
    B.halos_lps_push_global(s["lps"])
    assert B.halos_lps_step(s["lps"]).kind == 2


def _state(s):
    lists = [s["Theta"], s["M"], s["th"], s["m"], s["acc"]] + s["wm"]
    return [torch.cat([t.reshape(-1) for t in ts]).clone() for ts in lists]


@pytest.mark.parametrize("flags_name,delay", [("none", (1, 1)), ("norms", (1, 1)), ("none", (2, 1))])
def test_captured_cycle_replays_like_eager_calls(flags_name, delay):
    from paper_2506_04531_amd import binding as B
    numel = [int(x) for x in RAGGED.numel]
    K, n_workers = 4, 2          # K is a multiple of the local delay, so the momentum cycle closes with the protocol's
    gen = torch.Generator().manual_seed(5)
    theta0 = [torch.randn(n, generator=gen) * 0.02 for n in numel]
    deltas = [[(torch.randn(n, generator=gen) * 1e-3).to("cuda:0") for n in numel] for _ in range(3)]
    flags = B.FLAG_NORMS if flags_name == "norms" else 0
    a = _make(B, numel, theta0, K, n_workers, flags, delay)      # replayed from a graph
    b = _make(B, numel, theta0, K, n_workers, flags, delay)      # issued call by call
    try:
        _cycle(B, a, deltas, K)      # warm-up: pointer checks are cached by the library after the first use
        _cycle(B, b, deltas, K)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            _cycle(B, a, deltas, K)                               # recorded, not run
        torch.cuda.synchronize()
        for sa, sb in zip(_state(a), _state(b)):                  # capture alone changed nothing on the device
            assert torch.equal(sa, sb)
        for rep in range(3):
            graph.replay()
            _cycle(B, b, deltas, K)
            torch.cuda.synchronize()
            for i, (sa, sb) in enumerate(zip(_state(a), _state(b))):
                assert np.array_equal(sa.cpu().numpy().view(np.uint32), sb.cpu().numpy().view(np.uint32)), (rep, i)
            if flags:
                assert B.halos_lps_get_norms(a["lps"]) == B.halos_lps_get_norms(b["lps"])
            # eager work of the program itself between replays
            torch.cuda.synchronize()
    finally:
        for s in (a, b):
            B.halos_lps_destroy(s["lps"])
            B.halos_gps_destroy(s["gps"])


def _batched_cycle(B, s, deltas):
    """K = 2: two queued deltas in one pass (the second completes the accumulation), GPS update, the returned model
    merged in the pass of the next delta, one more update to complete the next accumulation, GPS update, merge."""
    lps, gps = s["lps"], s["gps"]
    B.halos_lps_push_update(lps, 0, deltas[0], B.F32)
    B.halos_lps_push_update(lps, 1, deltas[1], B.F32)
    infos = B.halos_lps_step_batch(lps, 4, True)
    assert [i.kind for i in infos] == [1, 1] and infos[1].delta_ready == 1
    B.halos_gps_merge(gps, lps)
    B.halos_lps_push_global(lps)
    B.halos_lps_push_update(lps, 0, deltas[2], B.F32)
    infos = B.halos_lps_step_batch(lps, 4, True)
    assert [i.kind for i in infos] == [2, 1]
    B.halos_lps_push_update(lps, 1, deltas[0], B.F32)
    assert B.halos_lps_step_pull(lps).delta_ready == 1
    B.halos_gps_merge(gps, lps)
    B.halos_lps_push_global(lps)
    assert B.halos_lps_step(lps).kind == 2


@pytest.mark.parametrize("flags_name", ["none", "bf16m"])
def test_captured_batched_cycle_replays_like_eager_calls(flags_name):
    """The batch call (queued deltas in one pass; a merge opening the pass of the delta behind it) rewrites its per-worker
    tables of delta pointers with a small kernel in stream order, so it can be captured too."""
    from paper_2506_04531_amd import binding as B
    from paper_2506_04531_amd.harness import alloc_tensor_list
    numel = [int(x) for x in RAGGED.numel]
    gen = torch.Generator().manual_seed(6)
    theta0 = [torch.randn(n, generator=gen) * 0.02 for n in numel]
    deltas = [[(torch.randn(n, generator=gen) * 1e-3).to("cuda:0") for n in numel] for _ in range(3)]
    flags = B.FLAG_BF16_MOMENTUM if flags_name == "bf16m" else 0

    def make():
        s = _make(B, numel, theta0, 2, 2, 0) if not flags else None
        if s is None:           # the same with 16-bit momentum arrays
            mk = lambda dt=torch.float32: alloc_tensor_list(numel, dt, "cuda:0")
            s = dict(Theta=mk(), M=mk(torch.bfloat16), th=mk(), m=mk(torch.bfloat16), acc=mk(), wm=[mk(), mk()], extra=[])
            for t, v in zip(s["Theta"], theta0):
                t.copy_(v)
            hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 2, flags=flags)
            s["gps"] = B.halos_gps_create(numel, hp, s["Theta"], s["M"])
            s["lps"] = B.halos_lps_create(s["gps"], 0, 2, s["th"], s["m"], s["acc"])
            for k in range(2):
                B.halos_lps_set_worker_model(s["lps"], k, s["wm"][k])
        return s

    a, b = make(), make()
    state = lambda s: [torch.cat([t.reshape(-1) for t in ts]).float().clone()
                       for ts in [s["Theta"], s["M"], s["th"], s["m"], s["acc"]] + s["wm"]]
    try:
        _batched_cycle(B, a, deltas)      # warm-up: pointer checks cached, delta tables in the state every cycle leaves them in
        _batched_cycle(B, b, deltas)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            _batched_cycle(B, a, deltas)
        torch.cuda.synchronize()
        for sa, sb in zip(state(a), state(b)):
            assert torch.equal(sa, sb)
        for rep in range(3):
            graph.replay()
            _batched_cycle(B, b, deltas)
            torch.cuda.synchronize()
            for i, (sa, sb) in enumerate(zip(state(a), state(b))):
                assert np.array_equal(sa.cpu().numpy().view(np.uint32), sb.cpu().numpy().view(np.uint32)), (rep, i)
    finally:
        for s in (a, b):
            B.halos_lps_destroy(s["lps"])
            B.halos_gps_destroy(s["gps"])
