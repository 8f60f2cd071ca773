"""ctypes access to the plain CPU oracle (oracle/halos_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports or calls it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "halos_oracle.cpp")
_LIB = os.path.join(_HERE, "libhalos_oracle.so")

THETA, MOM, AUX, GPS_THETA, GPS_MOM = 0, 1, 2, 3, 4
SNAP, FROZEN, INBOX = 20, 21, 22   # raw state of an LPS: theta_{t_last}, the G it last froze, the model last returned
BUFFER, GPS_BUFFER = 6, 7   # gradient buffers of the delayed momentum (an LPS's, the GPS's)
SCALE = 10   # add to the ids above for the running max-magnitude of the same array

FORM_LITERAL = 0       # Delta by snapshot subtraction (the Delta of Algorithm 1's LPS block as written)
FORM_ACCUMULATOR = 1   # running sum of applied steps


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no contraction; -mfma only makes std::fma one instruction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-mfma", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC]
        subprocess.check_call(cmd)
    return _LIB


class StepInfo(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("sent", ctypes.c_int32), ("accumulated", ctypes.c_int32),
                ("worker", ctypes.c_int32), ("t", ctypes.c_int64), ("t_last", ctypes.c_int64)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        f32, i32, i64, vp = ctypes.c_float, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        lib.ho_create.restype = vp
        lib.ho_create.argtypes = [i64, i32, i32, i32, f32, f32, f32, f32, f32, f32, f32, vp, vp]
        lib.ho_destroy.argtypes = [vp]
        lib.ho_arrive_delta_f32.argtypes = [vp, i32, i32, vp]
        lib.ho_arrive_delta_bf16.argtypes = [vp, i32, i32, vp]
        lib.ho_arrive_delta_weighted.argtypes = [vp, i32, i32, vp, f32]
        lib.ho_arrive_delta_16.argtypes = [vp, i32, i32, vp, i32, f32]
        lib.ho_lps_step_average.argtypes = [vp, i32, i32, ctypes.POINTER(StepInfo)]
        lib.ho_gps_apply_delta.argtypes = [vp, vp, f32]
        lib.ho_f16_to_f32.restype = f32
        lib.ho_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.ho_arrive_global.argtypes = [vp, i32]
        lib.ho_lps_step.argtypes = [vp, i32, ctypes.POINTER(StepInfo)]
        lib.ho_gps_receive.argtypes = [vp, i32]
        lib.ho_set_K.argtypes = [vp, i32, i32]
        lib.ho_set_delay.argtypes = [vp, i32, i32]
        lib.ho_delay_seen.argtypes = [vp, i32]
        lib.ho_set_rules.argtypes = [vp, f32, f32, f32, f32, f32, f32, f32]
        lib.ho_get.argtypes = [vp, i32, i32, vp]
        lib.ho_counters.argtypes = [vp, i32] + [vp] * 5
        lib.ho_norms.argtypes = [vp, i32, vp]
        lib.ho_stopwatch.argtypes = [vp, vp, vp]
        lib.ho_bf16_to_f32.restype = f32
        lib.ho_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.ho_f32_to_bf16.restype = ctypes.c_uint16
        lib.ho_f32_to_bf16.argtypes = [f32]
        lib.ho_set_momentum_bf16.argtypes = [vp, i32]
        lib.ho_f32_to_bf16_array.argtypes = [vp, i64, vp]
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    pass


class HalosOracle:
    """One GPS and n_lps LPSs over a flat vector of n parameters.

    precision 64 is the reference; precision 32 with form=FORM_ACCUMULATOR
    performs the same fp32 operations, in the same order, as a one-pass fp32
    implementation and can be compared bit for bit.
    """

    def __init__(self, theta0: np.ndarray, n_lps: int, *, eta_l: float, beta_l: float, eta_g: float, beta_g: float,
                 alpha: float, K: Sequence[int] | int, cg_l: float | None = None, cg_g: float | None = None,
                 precision: int = 64, form: int = FORM_LITERAL, momentum_bf16: bool = False):
        lib = _load()
        theta0 = np.ascontiguousarray(theta0, dtype=np.float32)
        self.n = int(theta0.size)
        self.n_lps = int(n_lps)
        f = np.float32
        if cg_l is None:
            cg_l = f(1) - f(beta_l)       # the paper's (1 - beta), formed in fp32 like any fp32 caller would
        if cg_g is None:
            cg_g = f(1) - f(beta_g)
        Ks = np.full(n_lps, K, dtype=np.int32) if np.isscalar(K) else np.ascontiguousarray(K, dtype=np.int32)
        assert Ks.size == n_lps
        self._lib = lib
        self._h = lib.ho_create(self.n, n_lps, precision, form, f(eta_l), f(beta_l), f(cg_l), f(eta_g), f(beta_g),
                                f(cg_g), f(alpha), Ks.ctypes.data, theta0.ctypes.data)
        if not self._h:
            raise OracleError("ho_create failed")
        if momentum_bf16:
            self.set_momentum_bf16(True)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ho_destroy(self._h)
            self._h = None

    __del__ = close

    def _chk(self, rc, what):
        if rc != 0:
            raise OracleError(f"{what}: protocol violation (code {rc})")

    def arrive_delta(self, l: int, worker: int, g: np.ndarray, weight: float = 1.0):
        """g is the pseudo-gradient (start - end model): float32 values, IEEE half values (numpy float16), or raw
        bfloat16 bit patterns as uint16/int16.  weight: the caller's scalar on this delta (1 = a plain arrival)."""
        g = np.ascontiguousarray(g)
        assert g.size == self.n
        w = np.float32(weight)
        if g.dtype == np.float32:
            rc = self._lib.ho_arrive_delta_weighted(self._h, l, worker, g.ctypes.data, w)
        elif g.dtype == np.float16:
            rc = self._lib.ho_arrive_delta_16(self._h, l, worker, g.ctypes.data, 2, w)
        elif g.dtype in (np.uint16, np.int16):
            rc = self._lib.ho_arrive_delta_16(self._h, l, worker, g.ctypes.data, 1, w)
        else:
            raise TypeError(g.dtype)
        self._chk(rc, "arrive_delta")

    def lps_step_average(self, l: int, count: int) -> StepInfo:
        """The `count` deltas at the head of LPS l's queue, averaged in arrival order, applied as ONE update."""
        info = StepInfo()
        self._chk(self._lib.ho_lps_step_average(self._h, l, count, ctypes.byref(info)), "lps_step_average")
        return info

    def gps_apply_delta(self, g: np.ndarray, weight: float = 1.0):
        """Single tier: the GPS applies a worker's pseudo-gradient (float32 values) with its own rule."""
        g = np.ascontiguousarray(g, dtype=np.float32)
        assert g.size == self.n
        self._chk(self._lib.ho_gps_apply_delta(self._h, g.ctypes.data, np.float32(weight)), "gps_apply_delta")

    def arrive_global(self, l: int):
        self._chk(self._lib.ho_arrive_global(self._h, l), "arrive_global")

    def lps_step(self, l: int) -> StepInfo:
        info = StepInfo()
        self._chk(self._lib.ho_lps_step(self._h, l, ctypes.byref(info)), "lps_step")
        return info

    def gps_receive(self, l: int):
        self._chk(self._lib.ho_gps_receive(self._h, l), "gps_receive")

    def set_K(self, l: int, K: int):
        self._chk(self._lib.ho_set_K(self._h, l, K), "set_K")

    def set_delay(self, which: int, d: int):
        """Delayed Nesterov momentum with delay d >= 1 for LPS `which` (or the GPS if which < 0); d = 0 switches back
        to the plain rule.  Only between cycles."""
        self._chk(self._lib.ho_set_delay(self._h, which, d), "set_delay")

    def set_momentum_bf16(self, on: bool):
        """Keep every server's momentum in bfloat16 (rounded to nearest even whenever it is updated); an option of this
        repository, not of the paper.  Refused once a momentum holds a value bfloat16 cannot, or under the delayed rule."""
        self._chk(self._lib.ho_set_momentum_bf16(self._h, 1 if on else 0), "set_momentum_bf16")

    def delay_seen(self, which: int) -> int:
        return int(self._lib.ho_delay_seen(self._h, which))

    def set_rules(self, *, eta_l, beta_l, cg_l, eta_g, beta_g, cg_g, alpha):
        f = np.float32
        self._lib.ho_set_rules(self._h, f(eta_l), f(beta_l), f(cg_l), f(eta_g), f(beta_g), f(cg_g), f(alpha))

    def get(self, what: int, l: int = 0) -> np.ndarray:
        out = np.empty(self.n, dtype=np.float64)
        self._chk(self._lib.ho_get(self._h, what, l, out.ctypes.data), "get")
        return out

    def norms(self, l: int):
        """(sum of g^2 of the last applied delta, sum of (theta - Theta_i)^2 before the last merge), fp64."""
        out = (ctypes.c_double * 2)()
        self._lib.ho_norms(self._h, l, out)
        return float(out[0]), float(out[1])

    def stopwatch(self):
        """Seconds spent inside, and calls of, the oracle's own handlers: {"lps_update": (s, n), "gps_update": ..., "lps_merge": ...}."""
        sec, n = (ctypes.c_double * 3)(), (ctypes.c_int64 * 3)()
        self._lib.ho_stopwatch(self._h, sec, n)
        return {k: (float(sec[i]), int(n[i])) for i, k in enumerate(("lps_update", "gps_update", "lps_merge"))}

    def counters(self, l: int):
        t, tl, gu = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        ph, q = ctypes.c_int32(), ctypes.c_int32()
        self._lib.ho_counters(self._h, l, ctypes.byref(t), ctypes.byref(tl), ctypes.byref(ph), ctypes.byref(q),
                              ctypes.byref(gu))
        return {"t": t.value, "t_last": tl.value, "phase": ph.value, "queued": q.value, "gps_updates": gu.value}


def bf16_to_f32(bits: int) -> float:
    return float(_load().ho_bf16_to_f32(bits & 0xFFFF))


def f32_to_bf16(value: float) -> int:
    return int(_load().ho_f32_to_bf16(ctypes.c_float(value)))


def f32_to_bf16_array(values: np.ndarray) -> np.ndarray:
    v = np.ascontiguousarray(values, dtype=np.float32)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().ho_f32_to_bf16_array(v.ctypes.data, v.size, out.ctypes.data)
    return out


def f16_to_f32(bits: int) -> float:
    return float(_load().ho_f16_to_f32(bits & 0xFFFF))
