"""ctypes binding of include/halos.h: same names, argument marshalling only.

Tensor arguments are sequences of torch CUDA tensors (one per tensor of the
layout); the binding passes their data pointers.  `stream` defaults to
torch's current HIP stream.  Any status other than HALOS_OK raises HalosError
carrying the status code and the library's message.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

OK, EINVAL, ESTATE, ENOMEM, EHIP = 0, 1, 2, 3, 4
F32, BF16, F16 = 0, 1, 2
FLAG_NORMS = 1
FLAG_SNAPSHOT = 2
FLAG_GPS_NO_MOMENTUM = 4
FLAG_DEFER_CLEAR = 8
FLAG_BF16_MOMENTUM = 16
PHASE_ACCUMULATING, PHASE_SENT, PHASE_RETURNING, PHASE_QUEUED = 0, 1, 2, 3


class Rule(ctypes.Structure):
    _fields_ = [("eta", ctypes.c_float), ("beta", ctypes.c_float), ("cg", ctypes.c_float)]


class HParams(ctypes.Structure):
    _fields_ = [("local", Rule), ("glob", Rule), ("alpha", ctypes.c_float), ("K", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class _Layout(ctypes.Structure):
    _fields_ = [("n_tensors", ctypes.c_int32), ("numel", ctypes.POINTER(ctypes.c_int64))]


class StepInfo(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("delta_ready", ctypes.c_int32), ("accumulated", ctypes.c_int32),
                ("worker", ctypes.c_int32), ("t", ctypes.c_int64), ("t_last", ctypes.c_int64)]


class HalosError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"halos status {status}: {message}")
        self.status = status
        self.message = message


def paper_hparams(eta_l: float, beta_l: float, eta_g: float, beta_g: float, alpha: float, K: int,
                  cg_l: Optional[float] = None, cg_g: Optional[float] = None, flags: int = 0) -> HParams:
    """Hyper-parameter block with the paper's coefficient cg = 1 - beta (halos_paper_rule) unless given."""
    f = np.float32
    lib = load_library()
    hp = HParams()
    hp.local = lib.halos_paper_rule(f(eta_l), f(beta_l)) if cg_l is None else Rule(f(eta_l), f(beta_l), f(cg_l))
    hp.glob = lib.halos_paper_rule(f(eta_g), f(beta_g)) if cg_g is None else Rule(f(eta_g), f(beta_g), f(cg_g))
    hp.alpha = f(alpha)
    hp.K = int(K)
    hp.flags = int(flags)
    return hp


_lib = None


def load_library():
    """Load libhalos.so (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    from . import LIB_PATH, build
    if not os.path.exists(LIB_PATH):
        build()
    import torch  # noqa: F401  -- first, so that the process uses the one HIP runtime torch brings with it
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32
    P = ctypes.POINTER
    sigs = {
        "halos_gps_create": [P(_Layout), P(HParams), P(vp), P(vp), vp, P(vp)],
        "halos_lps_create": [vp, i32, i32, P(vp), P(vp), P(vp), vp, P(vp)],
        "halos_lps_push_update": [vp, i32, P(vp), i32, u32],
        "halos_lps_push_update_weighted": [vp, i32, P(vp), i32, u32, ctypes.c_float],
        "halos_gps_push_update": [vp, P(vp), i32, ctypes.c_float, vp],
        "halos_lps_push_end_model": [vp, i32, P(vp), u32],
        "halos_lps_push_global": [vp],
        "halos_lps_step": [vp, vp, P(StepInfo)],
        "halos_lps_step_pull": [vp, vp, P(StepInfo)],
        "halos_lps_step_norms": [vp, vp, P(StepInfo), vp],
        "halos_lps_step_average": [vp, i32, vp, P(StepInfo)],
        "halos_lps_step_batch": [vp, i32, i32, vp, P(StepInfo), P(i32)],
        "halos_lps_set_worker_model": [vp, i32, P(vp), vp],
        "halos_gps_merge": [vp, vp, vp],
        "halos_pull_model": [vp, i32, P(vp), vp],
        "halos_set_hparams": [vp, i32, P(HParams)],
        "halos_lps_set_threshold": [vp, i32],
        "halos_forget_buffers": [vp, i32],
        "halos_lps_get_counters": [vp, P(i64), P(i64), P(i32), P(i32), P(u32)],
        "halos_gps_get_counters": [vp, P(i64)],
        "halos_lps_get_norms": [vp, vp, P(ctypes.c_double)],
        "halos_lps_set_momentum_delay": [vp, i32, P(vp), vp],
        "halos_gps_set_momentum_delay": [vp, i32, P(vp), vp],
        "halos_lps_get_momentum_delay": [vp, P(i32), P(i32)],
        "halos_gps_get_momentum_delay": [vp, P(i32), P(i32)],
        "halos_set_launch_config": [i32, i32],
        "halos_arena_create": [i32, P(ctypes.c_uint64), ctypes.c_uint64, P(vp)],
        "halos_arena_alloc": [vp, i32, ctypes.c_uint64, P(vp)],
        "halos_arena_info": [vp, P(i32), P(ctypes.c_uint64), P(ctypes.c_double), P(i32), P(i32)],
        "halos_probe_pair": [vp, vp, ctypes.c_uint64, i32, vp, P(ctypes.c_double)],
        "halos_probe_streams": [P(vp), i32, P(vp), i32, ctypes.c_uint64, i32, i32, vp, P(ctypes.c_double)],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = ctypes.c_int
    lib.halos_lps_destroy.argtypes = [vp]
    lib.halos_lps_destroy.restype = None
    lib.halos_gps_destroy.argtypes = [vp]
    lib.halos_gps_destroy.restype = None
    lib.halos_arena_destroy.argtypes = [vp]
    lib.halos_arena_destroy.restype = None
    lib.halos_paper_rule.argtypes = [ctypes.c_float, ctypes.c_float]
    lib.halos_paper_rule.restype = Rule
    lib.halos_last_error.argtypes = []
    lib.halos_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def halos_last_error() -> str:
    return load_library().halos_last_error().decode()


def _check(status: int):
    if status != OK:
        raise HalosError(status, halos_last_error())


def _ptrs(tensors) -> ctypes.Array:
    """Host array of device pointers.  Accepts torch tensors or raw integer addresses (None -> NULL)."""
    if tensors is None or isinstance(tensors, ctypes.Array):
        return tensors
    arr = (ctypes.c_void_p * max(1, len(tensors)))()
    for i, t in enumerate(tensors):
        if t is None:
            arr[i] = None
        elif isinstance(t, int):
            arr[i] = t
        else:
            arr[i] = t.data_ptr() if t.numel() > 0 else None
    return arr


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def halos_gps_create(numel: Sequence[int], hp: HParams, Theta, M, stream=None) -> int:
    lib = load_library()
    n = len(numel)
    arr = (ctypes.c_int64 * max(1, n))(*[int(x) for x in numel])
    lay = _Layout(n, arr)
    out = ctypes.c_void_p()
    _check(lib.halos_gps_create(ctypes.byref(lay), ctypes.byref(hp), _ptrs(Theta), _ptrs(M), _stream(stream),
                                ctypes.byref(out)))
    return out.value


def halos_lps_create(gps: int, lps_id: int, n_workers: int, theta, m, acc, stream=None) -> int:
    lib = load_library()
    out = ctypes.c_void_p()
    _check(lib.halos_lps_create(gps, lps_id, n_workers, _ptrs(theta), _ptrs(m), _ptrs(acc), _stream(stream),
                                ctypes.byref(out)))
    return out.value


def halos_lps_push_update(lps: int, worker: int, g, dtype: int, staleness: int = 0) -> None:
    _check(load_library().halos_lps_push_update(lps, worker, _ptrs(g), dtype, staleness))


def halos_lps_push_update_weighted(lps: int, worker: int, g, dtype: int, staleness: int, weight: float) -> None:
    _check(load_library().halos_lps_push_update_weighted(lps, worker, _ptrs(g), dtype, staleness, weight))


def halos_gps_push_update(gps: int, g, dtype: int, weight: float = 1.0, stream=None) -> None:
    _check(load_library().halos_gps_push_update(gps, _ptrs(g), dtype, weight, _stream(stream)))


def halos_lps_push_end_model(lps: int, worker: int, end_model, staleness: int = 0) -> None:
    _check(load_library().halos_lps_push_end_model(lps, worker, _ptrs(end_model), staleness))


def halos_lps_push_global(lps: int) -> None:
    _check(load_library().halos_lps_push_global(lps))


def halos_lps_step(lps: int, stream=None) -> StepInfo:
    info = StepInfo()
    _check(load_library().halos_lps_step(lps, _stream(stream), ctypes.byref(info)))
    return info


def halos_lps_step_pull(lps: int, stream=None) -> StepInfo:
    info = StepInfo()
    _check(load_library().halos_lps_step_pull(lps, _stream(stream), ctypes.byref(info)))
    return info


def halos_lps_step_average(lps: int, count: int, stream=None) -> StepInfo:
    info = StepInfo()
    _check(load_library().halos_lps_step_average(lps, count, _stream(stream), ctypes.byref(info)))
    return info


def halos_lps_step_batch(lps: int, max_items: int, pull: bool = False, stream=None) -> list:
    """The StepInfo of every step taken (possibly none)."""
    infos = (StepInfo * 4)()
    n = ctypes.c_int32()
    _check(load_library().halos_lps_step_batch(lps, max_items, 1 if pull else 0, _stream(stream), infos, ctypes.byref(n)))
    out = []
    for i in range(n.value):
        c = StepInfo()
        ctypes.memmove(ctypes.byref(c), ctypes.byref(infos[i]), ctypes.sizeof(StepInfo))
        out.append(c)
    return out


def halos_lps_step_norms(lps: int, norms_out, stream=None) -> StepInfo:
    """norms_out: a torch CUDA tensor of two float64 (or a raw device address)."""
    info = StepInfo()
    p = norms_out if isinstance(norms_out, int) else norms_out.data_ptr()
    _check(load_library().halos_lps_step_norms(lps, _stream(stream), ctypes.byref(info), p))
    return info


def halos_lps_set_worker_model(lps: int, worker: int, model, stream=None) -> None:
    _check(load_library().halos_lps_set_worker_model(lps, worker, _ptrs(model), _stream(stream)))


def halos_gps_merge(gps: int, from_lps: int, stream=None) -> None:
    _check(load_library().halos_gps_merge(gps, from_lps, _stream(stream)))


def halos_pull_model(server: int, is_gps: bool, dst, stream=None) -> None:
    _check(load_library().halos_pull_model(server, 1 if is_gps else 0, _ptrs(dst), _stream(stream)))


def halos_set_hparams(server: int, is_gps: bool, hp: HParams) -> None:
    _check(load_library().halos_set_hparams(server, 1 if is_gps else 0, ctypes.byref(hp)))


def halos_forget_buffers(server: int, is_gps: bool) -> None:
    _check(load_library().halos_forget_buffers(server, 1 if is_gps else 0))


def halos_lps_set_threshold(lps: int, K: int) -> None:
    _check(load_library().halos_lps_set_threshold(lps, K))


def halos_lps_get_counters(lps: int) -> dict:
    t, tl = ctypes.c_int64(), ctypes.c_int64()
    ph, q, ms = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_uint32()
    _check(load_library().halos_lps_get_counters(lps, ctypes.byref(t), ctypes.byref(tl), ctypes.byref(ph),
                                                 ctypes.byref(q), ctypes.byref(ms)))
    return {"t": t.value, "t_last": tl.value, "phase": ph.value, "queued": q.value, "max_staleness": ms.value}


def halos_lps_get_norms(lps: int, stream=None) -> tuple:
    """(sum g^2 of the last update, sum (theta - Theta_i)^2 before the last merge)."""
    out = (ctypes.c_double * 2)()
    _check(load_library().halos_lps_get_norms(lps, _stream(stream), out))
    return float(out[0]), float(out[1])


def halos_gps_get_counters(gps: int) -> dict:
    u = ctypes.c_int64()
    _check(load_library().halos_gps_get_counters(gps, ctypes.byref(u)))
    return {"updates": u.value}


def halos_lps_set_momentum_delay(lps: int, d: int, buffer=None, stream=None) -> None:
    _check(load_library().halos_lps_set_momentum_delay(lps, d, _ptrs(buffer) if buffer is not None else None, _stream(stream)))


def halos_gps_set_momentum_delay(gps: int, d: int, buffer=None, stream=None) -> None:
    _check(load_library().halos_gps_set_momentum_delay(gps, d, _ptrs(buffer) if buffer is not None else None, _stream(stream)))


def halos_lps_get_momentum_delay(lps: int) -> dict:
    d, seen = ctypes.c_int32(), ctypes.c_int32()
    _check(load_library().halos_lps_get_momentum_delay(lps, ctypes.byref(d), ctypes.byref(seen)))
    return {"d": d.value, "seen": seen.value}


def halos_gps_get_momentum_delay(gps: int) -> dict:
    d, seen = ctypes.c_int32(), ctypes.c_int32()
    _check(load_library().halos_gps_get_momentum_delay(gps, ctypes.byref(d), ctypes.byref(seen)))
    return {"d": d.value, "seen": seen.value}


def halos_set_launch_config(blocks_per_cu: int = 0, nontemporal: int = -1) -> None:
    _check(load_library().halos_set_launch_config(blocks_per_cu, nontemporal))


def halos_probe_pair(a, b, nbytes: int, reps: int = 2, stream=None) -> float:
    """GB/s of a read-modify-write sweep over two device buffers (torch tensors or raw addresses)."""
    pa = a if isinstance(a, int) else a.data_ptr()
    pb = b if isinstance(b, int) else b.data_ptr()
    out = ctypes.c_double()
    _check(load_library().halos_probe_pair(pa, pb, int(nbytes), reps, _stream(stream), ctypes.byref(out)))
    return out.value


def halos_probe_streams(read_bufs, write_bufs, nbytes: int, reps: int = 2, unroll: int = 0, stream=None) -> float:
    """GB/s of a kernel that only reads `read_bufs` and only writes (zeros to) `write_bufs`: lists of torch tensors or
    raw addresses, up to four each.  unroll: 128-bit accesses per thread, stream and tile (0 = the update kernels' own)."""
    def arr(bufs):
        a = (ctypes.c_void_p * max(1, len(bufs)))()
        for i, b in enumerate(bufs):
            a[i] = b if isinstance(b, int) else b.data_ptr()
        return a
    out = ctypes.c_double()
    _check(load_library().halos_probe_streams(arr(read_bufs), len(read_bufs), arr(write_bufs), len(write_bufs),
                                              int(nbytes), reps, unroll, _stream(stream), ctypes.byref(out)))
    return out.value


def halos_arena_create(bytes_per_class: Sequence[int], max_walk_bytes: int = 0) -> int:
    n = len(bytes_per_class)
    arr = (ctypes.c_uint64 * max(1, n))(*[int(b) for b in bytes_per_class])
    out = ctypes.c_void_p()
    _check(load_library().halos_arena_create(n, arr, int(max_walk_bytes), ctypes.byref(out)))
    return out.value


def halos_arena_alloc(arena: int, cls: int, nbytes: int) -> int:
    """Raw device address of `nbytes` bytes in placement class `cls`."""
    out = ctypes.c_void_p()
    _check(load_library().halos_arena_alloc(arena, cls, int(nbytes), ctypes.byref(out)))
    return out.value


def halos_arena_info(arena: int, n_classes: int) -> dict:
    nr, walked, same = ctypes.c_int32(), ctypes.c_uint64(), ctypes.c_double()
    roc, soc = (ctypes.c_int32 * max(1, n_classes))(), (ctypes.c_int32 * max(1, n_classes))()
    _check(load_library().halos_arena_info(arena, ctypes.byref(nr), ctypes.byref(walked), ctypes.byref(same), roc, soc))
    return {"n_regions": nr.value, "walked_bytes": walked.value, "same_region_gbps": same.value,
            "region_of_class": list(roc)[:n_classes], "slabs_of_class": list(soc)[:n_classes]}


def halos_arena_destroy(arena: Optional[int]) -> None:
    if arena:
        load_library().halos_arena_destroy(arena)


def halos_lps_destroy(lps: Optional[int]) -> None:
    if lps:
        load_library().halos_lps_destroy(lps)


def halos_gps_destroy(gps: Optional[int]) -> None:
    if gps:
        load_library().halos_gps_destroy(gps)
