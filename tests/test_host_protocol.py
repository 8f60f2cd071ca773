"""Host logic of the library (queue, counters, accumulation threshold, one update in flight) on the CPU."""
import ctypes
import os
import subprocess

import pytest

import synth

HERE = os.path.dirname(os.path.abspath(__file__))
OK, BAD_ARG, BAD_STATE = 0, 1, 2


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("shim") / "libproto_shim.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-Wall", "-o", out,
                           os.path.join(HERE, "host", "proto_shim.cpp")])
    lib = ctypes.CDLL(out)
    lib.proto_new.restype = ctypes.c_void_p
    for f in ("proto_free", "proto_set_K", "proto_push_delta", "proto_push_global", "proto_step", "proto_consume",
              "proto_phase", "proto_queued"):
        getattr(lib, f).argtypes = [ctypes.c_void_p] + {"proto_set_K": [ctypes.c_int], "proto_push_delta": [ctypes.c_int],
                                                         "proto_step": [ctypes.POINTER(ctypes.c_longlong)]}.get(f, [])
    lib.proto_step_average.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_longlong)]
    lib.cycle_new.restype = ctypes.c_void_p
    for f in ("cycle_free", "cycle_set_d", "cycle_next", "cycle_commit", "cycle_seen", "cycle_d"):
        getattr(lib, f).argtypes = [ctypes.c_void_p] + ([ctypes.c_int] if f == "cycle_set_d" else [])
    return lib


def _step(lib, p):
    out = (ctypes.c_longlong * 6)()
    lib.proto_step(p, out)
    return list(out)


def test_threshold_and_single_update_in_flight(shim):
    p = shim.proto_new(2, 2)
    assert _step(shim, p)[0] == 0                                   # empty queue
    assert shim.proto_push_delta(p, 0) == OK
    assert shim.proto_push_delta(p, 0) == BAD_STATE                 # same worker twice
    assert shim.proto_push_delta(p, 2) == BAD_ARG and shim.proto_push_delta(p, -1) == BAD_ARG
    assert shim.proto_push_delta(p, 1) == OK
    assert shim.proto_queued(p) == 2
    assert _step(shim, p) == [1, 0, 1, 0, 1, 0]
    assert shim.proto_consume(p) == BAD_STATE                       # nothing frozen yet
    assert _step(shim, p) == [1, 1, 1, 1, 2, 0]                     # K = 2 reached: freezes
    assert shim.proto_phase(p) == 1
    assert shim.proto_push_global(p) == BAD_STATE                   # GPS has not answered
    shim.proto_push_delta(p, 0)
    assert _step(shim, p) == [1, 0, 0, 0, 3, 0]                     # in flight: applied but not accumulated
    assert shim.proto_consume(p) == OK and shim.proto_consume(p) == BAD_STATE
    assert shim.proto_push_global(p) == OK and shim.proto_push_global(p) == BAD_STATE
    shim.proto_push_delta(p, 1)
    assert _step(shim, p) == [2, -1, 0, 0, 3, 3]                    # merge comes first: it was queued first
    assert _step(shim, p) == [1, 1, 1, 0, 4, 3]
    assert shim.proto_set_K(p, 0) == BAD_ARG and shim.proto_set_K(p, 1) == OK
    shim.proto_push_delta(p, 0)
    assert _step(shim, p) == [1, 0, 1, 1, 5, 3]                     # lowered K is honoured (t - t_last = 2 >= 1)
    shim.proto_free(p)


@pytest.mark.parametrize("name", ["tiny", "70m", "160m", "410m", "1b", "paper-70m", "paper-410m"])
def test_protocol_follows_the_schedule_bookkeeping(shim, name):
    """Replaying a benchmark trace through the state machine reproduces the generator's expectations."""
    w = synth.get_workload(name)
    tr = synth.make_trace(w)
    ps = [shim.proto_new(w.workers_per_lps, k) for k in tr.k_initial]
    for ev in tr.events:
        p = ps[int(ev["lps"])]
        kind = int(ev["kind"])
        if kind == synth.EV_ARRIVE_DELTA:
            assert shim.proto_push_delta(p, int(ev["worker"])) == OK
        elif kind == synth.EV_ARRIVE_GLOBAL:
            assert shim.proto_push_global(p) == OK
        elif kind == synth.EV_GPS_MERGE:
            assert shim.proto_consume(p) == OK
        elif kind == synth.EV_LPS_STEP:
            shim.proto_set_K(p, int(ev["k_cur"]))
            k, worker, acc, freezes, t, t_last = _step(shim, p)
            assert (k, t, t_last) == (int(ev["exp_kind"]), int(ev["exp_t"]), int(ev["exp_t_last"]))
            if k == 1:
                assert (acc, freezes, worker) == (int(ev["exp_accumulate"]), int(ev["exp_send"]), int(ev["worker"]))
    for p in ps:
        shim.proto_free(p)


def test_momentum_cycle_positions(shim):
    """Delayed momentum (Sec. 5.1, App. D delays): the first update of a cycle restarts the buffer, the d-th refreshes
    the momentum; d = 1 refreshes every time; the delay changes only between cycles."""
    FIRST, INNER, REFRESH = 1, 2, 3
    c = shim.cycle_new()
    try:
        assert (shim.cycle_d(c), shim.cycle_seen(c)) == (1, 0)
        for _ in range(3):                                   # plain rule: every update is a refresh
            assert shim.cycle_next(c) == REFRESH
            shim.cycle_commit(c)
            assert shim.cycle_seen(c) == 0
        assert shim.cycle_set_d(c, 0) == BAD_ARG and shim.cycle_set_d(c, -2) == BAD_ARG
        assert shim.cycle_set_d(c, 4) == OK
        seq = []
        for _ in range(9):
            seq.append((shim.cycle_next(c), shim.cycle_seen(c)))
            shim.cycle_commit(c)
        assert seq == [(FIRST, 0), (INNER, 1), (INNER, 2), (REFRESH, 3), (FIRST, 0), (INNER, 1), (INNER, 2), (REFRESH, 3),
                       (FIRST, 0)]
        assert shim.cycle_seen(c) == 1
        assert shim.cycle_set_d(c, 2) == BAD_STATE and shim.cycle_d(c) == 4     # in mid-cycle
        for _ in range(3):
            shim.cycle_commit(c)
        assert shim.cycle_seen(c) == 0 and shim.cycle_set_d(c, 2) == OK
        assert [shim.cycle_next(c), shim.cycle_commit(c), shim.cycle_next(c)][::2] == [FIRST, REFRESH]
    finally:
        shim.cycle_free(c)


def test_averaged_step_counts_as_one_update(shim):
    """n deltas averaged: t advances by one, every sender may send again, the send test sees one update, and a queued
    global model is never stepped over."""
    p = shim.proto_new(4, 2)
    out = (ctypes.c_longlong * 6)()
    assert shim.proto_step_average(p, 1, out) == -1                 # empty queue
    for w in range(3):
        assert shim.proto_push_delta(p, w) == OK
    assert shim.proto_step_average(p, 4, out) == -1                 # only three queued
    assert shim.proto_step_average(p, 3, out) == 0
    assert list(out) == [1, 2, 1, 0, 1, 0]
    assert shim.proto_queued(p) == 0
    for w in range(4):
        assert shim.proto_push_delta(p, w) == OK                    # all senders free again
    assert shim.proto_step_average(p, 2, out) == 0
    assert list(out) == [1, 1, 1, 1, 2, 0]                          # second UPDATE reaches K = 2 (five deltas so far)
    assert shim.proto_phase(p) == 1
    assert shim.proto_consume(p) == OK and shim.proto_push_global(p) == OK
    assert shim.proto_push_delta(p, 0) == OK                        # queue: delta 2, delta 3, global, delta 0
    assert shim.proto_step_average(p, 3, out) == -1                 # the global model is third in line
    assert shim.proto_step_average(p, 2, out) == 0
    assert list(out) == [1, 3, 0, 0, 3, 0]                          # in flight: applied, not accumulated
    assert _step(shim, p) == [2, -1, 0, 0, 3, 3]
    assert shim.proto_step_average(p, 1, out) == 0 and list(out) == [1, 0, 1, 0, 4, 3]
    shim.proto_free(p)
