"""HALoS server-side update path for one MI355X (gfx950).

The work is done by hand-written HIP kernels behind the C ABI declared in
include/halos.h (built into paper_2506_04531_amd/libhalos.so).  This package
is the thin Python binding over that ABI: argument marshalling only.  There is
no CPU fallback: if the shared library is missing or no GPU is visible, calls
fail.
"""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libhalos.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "halos.h")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 instructions out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
]


def build(verbose: bool = False) -> str:
    """Compile the kernels and the C ABI for gfx950 (cross-compiles without a GPU)."""
    srcs = [os.path.join(_CSRC, "kernels.hip"), os.path.join(_CSRC, "halos.cpp"), os.path.join(_CSRC, "arena.cpp")]
    cmd = ["hipcc"] + HIPCC_FLAGS + ["-o", LIB_PATH] + srcs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    # clients of the ABI written in plain C (tests/host/*.c), linked against the library just built
    host_dir = os.path.join(os.path.dirname(_HERE), "tests", "host")
    for name in ("abi_client", "arena_client"):
        client_src = os.path.join(host_dir, name + ".c")
        if not os.path.exists(client_src):
            continue
        cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__", "-o",
               os.path.join(host_dir, name), client_src, "-L" + _HERE, "-lhalos", "-L/opt/rocm/lib", "-lamdhip64",
               "-Wl,-rpath,$ORIGIN/../../paper_2506_04531_amd", "-Wl,-rpath,/opt/rocm/lib"]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"gcc failed on {name}.c:\n" + res.stdout + res.stderr)
    return LIB_PATH


from .binding import (  # noqa: E402
    HalosError, HParams, Rule, StepInfo, F32, BF16,
    halos_gps_create, halos_lps_create, halos_lps_push_update, halos_lps_push_global, halos_lps_step,
    halos_lps_step_pull, halos_lps_set_worker_model, halos_lps_get_norms,
    halos_gps_merge, halos_pull_model, halos_set_hparams, halos_lps_set_threshold, halos_lps_get_counters,
    halos_gps_get_counters, halos_set_launch_config, halos_probe_pair, halos_lps_destroy, halos_gps_destroy, halos_last_error,
    load_library, paper_hparams,
)

__all__ = [
    "build", "LIB_PATH", "HEADER_PATH", "HalosError", "HParams", "Rule", "StepInfo", "F32", "BF16",
    "halos_gps_create", "halos_lps_create", "halos_lps_push_update", "halos_lps_push_global", "halos_lps_step",
    "halos_lps_step_pull", "halos_lps_set_worker_model", "halos_lps_get_norms",
    "halos_gps_merge", "halos_pull_model", "halos_set_hparams", "halos_lps_set_threshold",
    "halos_lps_get_counters", "halos_gps_get_counters", "halos_set_launch_config", "halos_probe_pair",
    "halos_lps_destroy",
    "halos_gps_destroy", "halos_last_error", "load_library", "paper_hparams",
]
