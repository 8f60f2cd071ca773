"""Random call sequences, valid and invalid, through the library's host-side protocol state machine and through
the oracle's: the two were written independently and must agree on every outcome (CPU only)."""
import ctypes
import os
import random
import subprocess

import numpy as np
import pytest

import oracle as O
from oracle import HalosOracle

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("shim") / "libproto_shim.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-Wall", "-o", out,
                           os.path.join(HERE, "host", "proto_shim.cpp")])
    lib = ctypes.CDLL(out)
    lib.proto_new.restype = ctypes.c_void_p
    lib.proto_free.argtypes = [ctypes.c_void_p]
    lib.proto_set_K.argtypes = [ctypes.c_void_p, ctypes.c_int]
    lib.proto_push_delta.argtypes = [ctypes.c_void_p, ctypes.c_int]
    lib.proto_push_global.argtypes = [ctypes.c_void_p]
    lib.proto_step.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_longlong)]
    lib.proto_step_average.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_longlong)]
    lib.proto_consume.argtypes = [ctypes.c_void_p]
    lib.proto_phase.argtypes = [ctypes.c_void_p]
    lib.proto_queued.argtypes = [ctypes.c_void_p]
    lib.cycle_new.restype = ctypes.c_void_p
    for f in ("cycle_free", "cycle_set_d", "cycle_commit", "cycle_seen"):
        getattr(lib, f).argtypes = [ctypes.c_void_p] + ([ctypes.c_int] if f == "cycle_set_d" else [])
    return lib


@pytest.mark.parametrize("seed", range(12))
def test_random_sequences_agree_with_the_oracle(shim, seed):
    rng = random.Random(seed)
    n_workers = rng.randint(1, 4)
    K = rng.randint(1, 5)
    p = shim.proto_new(n_workers, K)
    cyc = shim.cycle_new()          # the local server's position in its delayed-momentum cycle
    o = HalosOracle(np.zeros(3, dtype=np.float32), 1, eta_l=0.1, beta_l=0.5, eta_g=0.1, beta_g=0.5, alpha=0.5, K=K)
    g = np.ones(3, dtype=np.float32)
    out = (ctypes.c_longlong * 6)()
    for _ in range(400):
        op = rng.choice(["delta", "delta", "delta", "step", "step", "step", "average", "global", "consume", "setK", "setD"])
        if op == "delta":
            w = rng.randint(0, n_workers - 1)
            rc = shim.proto_push_delta(p, w)
            try:
                o.arrive_delta(0, w, g)
                ok = True
            except O.OracleError:
                ok = False
            assert (rc == 0) == ok
        elif op == "global":
            rc = shim.proto_push_global(p)
            try:
                o.arrive_global(0)
                ok = True
            except O.OracleError:
                ok = False
            assert (rc == 0) == ok
        elif op == "consume":
            rc = shim.proto_consume(p)
            try:
                o.gps_receive(0)
                ok = True
            except O.OracleError:
                ok = False
            assert (rc == 0) == ok
        elif op == "setD":             # the momentum delay may change only between cycles
            d = rng.randint(1, 4)
            rc = shim.cycle_set_d(cyc, d)
            try:
                o.set_delay(0, d)
                ok = True
            except O.OracleError:
                ok = False
            assert (rc == 0) == ok
        elif op == "average":          # the first n queue items as one update with their mean: allowed only if all are deltas
            n = rng.randint(1, 4)
            rc = shim.proto_step_average(p, n, out)
            try:
                info = o.lps_step_average(0, n)
                ok = True
            except O.OracleError:
                ok = False
            assert (rc == 0) == ok
            if ok:
                kind, worker, acc, freezes, t, t_last = list(out)
                assert (kind, worker, acc, freezes, t, t_last) == (info.kind, info.worker, info.accumulated, info.sent, info.t, info.t_last)
                shim.cycle_commit(cyc)
                assert shim.cycle_seen(cyc) == o.delay_seen(0)
        elif op == "setK":
            k = rng.randint(1, 5)
            assert shim.proto_set_K(p, k) == 0
            o.set_K(0, k)
        else:
            shim.proto_step(p, out)
            info = o.lps_step(0)
            kind, worker, acc, freezes, t, t_last = list(out)
            assert (kind, t, t_last) == (info.kind, info.t, info.t_last)
            if kind == 1:
                assert (worker, acc, freezes) == (info.worker, info.accumulated, info.sent)
                shim.cycle_commit(cyc)
            assert shim.cycle_seen(cyc) == o.delay_seen(0)
        c = o.counters(0)
        assert (shim.proto_phase(p), shim.proto_queued(p)) == (c["phase"], c["queued"])
    shim.proto_free(p)
    shim.cycle_free(cyc)
