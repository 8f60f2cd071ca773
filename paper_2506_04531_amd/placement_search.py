"""Measure how the placement of the update pass's arrays over the HBM regions changes its speed.

    python -m paper_2506_04531_amd.placement_search [--elements 536870912] [--dtype f32|bf16]

Allocates slabs from every HBM region the RegionArena can find, then times the library's fused update pass
(halos_lps_step_pull: read delta, m, theta, third buffer; write m, theta, third buffer, worker model) for every
assignment of those five arrays to the regions, and prints the assignments grouped by pattern (regions renamed
X, Y, Z in order of first use, arrays in the order m, theta, third, delta, worker model).  This is how the
placement classes of harness.Cluster(placement="regions") were chosen; run it again on another device to re-derive
them.  Everything goes through the C ABI; PyTorch only holds the memory.
"""
from __future__ import annotations

import argparse
import itertools
from collections import defaultdict

import torch

from . import binding as B
from .harness import RegionArena


def _time_assignment(n, dtype, bufs, reps=3):
    """bufs: dict name -> 1-tensor list for delta, m, theta, third, model."""
    hp = B.paper_hparams(0.2, 0.9, 0.15, 0.5, 0.25, 1 << 30)
    gps = B.halos_gps_create([n], hp, bufs["Theta"], bufs["M"])
    lps = B.halos_lps_create(gps, 0, 1, bufs["theta"], bufs["m"], bufs["third"])
    try:
        B.halos_lps_set_worker_model(lps, 0, bufs["model"])
        B.halos_lps_push_update(lps, 0, bufs["delta"], dtype)
        B.halos_lps_step_pull(lps)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            B.halos_lps_push_update(lps, 0, bufs["delta"], dtype)
            B.halos_lps_step_pull(lps)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    finally:
        B.halos_lps_destroy(lps)
        B.halos_gps_destroy(gps)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--elements", type=int, default=1 << 29)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    args = ap.parse_args()
    n = args.elements
    dev = torch.device("cuda:0")
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    ddt = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    need = 7 * n * 4 + (1 << 30)
    arena = RegionArena(dev, [need, need, need], verbose=True)
    if arena.n_regions < 3:
        print(f"only {arena.n_regions} region(s) found: nothing to compare")
        return
    # per region: one buffer for each role (the GPS's two arrays always live in region 0; they are not touched by the timed pass)
    pool = []
    for r in range(3):
        pool.append({
            "delta": [arena.alloc(r, n, ddt).zero_()],
            "m": [arena.alloc(r, n, torch.float32)], "theta": [arena.alloc(r, n, torch.float32)],
            "third": [arena.alloc(r, n, torch.float32)], "model": [arena.alloc(r, n, torch.float32)],
        })
    gps_bufs = {"Theta": [arena.alloc(0, n, torch.float32).zero_()], "M": [arena.alloc(0, n, torch.float32)]}
    bytes_per_param = (4 if dtype == B.F32 else 2) + 28
    roles = ("m", "theta", "third", "delta", "model")
    groups = defaultdict(list)
    for assign in itertools.product(range(3), repeat=5):
        bufs = dict(gps_bufs)
        for role, r in zip(roles, assign):
            bufs[role] = pool[r][role]
        ms = _time_assignment(n, dtype, bufs)
        gbs = n * bytes_per_param / ms / 1e6
        rename, pat = {}, []
        for r in assign:
            if r not in rename:
                rename[r] = "XYZ"[len(rename)]
            pat.append(rename[r])
        groups["".join(pat)].append(gbs)
    print(f"update pass with fused pull, {n} elements per array, {args.dtype} delta, {bytes_per_param} B/parameter")
    print("pattern (m theta third delta model)   mean GB/s    min     max   assignments")
    for pat, v in sorted(groups.items(), key=lambda kv: -sum(kv[1]) / len(kv[1])):
        print(f"  {pat}                              {sum(v) / len(v):8.1f} {min(v):7.1f} {max(v):7.1f}   {len(v)}")


if __name__ == "__main__":
    main()
