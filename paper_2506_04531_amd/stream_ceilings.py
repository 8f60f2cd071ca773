"""Measure what this device's memory system delivers to plain streaming kernels, by HBM region.

    python -m paper_2506_04531_amd.stream_ceilings [--gib 1] [--reps 5]

Allocates a few buffers in each HBM region the RegionArena finds, then times halos_probe_streams (read some buffers,
write others, no arithmetic, the access pattern of the update kernels) for pure reads, pure writes, copies and the
stream mix of the update pass with fused pull (4 read, 4 written) under several placements.  The last block compares
the mix with the figure that the pure read and pure write rates predict, and with the 8 TB/s nominal peak: it is the
evidence for how much of the peak a kernel with this many written bytes can reach at all.
Everything goes through the C ABI; PyTorch only holds the memory.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as B
from .harness import RegionArena


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib", type=float, default=1.0, help="size of every buffer")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    nbytes = int(args.gib * (1 << 30)) // (1 << 14) * (1 << 14)
    n = nbytes // 4
    dev = torch.device("cuda:0")
    per_region = 8
    need = per_region * nbytes + (1 << 30)
    arena = RegionArena(dev, [need, need, need], verbose=True)
    if arena.n_regions < 3:
        print(f"only {arena.n_regions} region(s) found: placements below collapse onto fewer regions")
    X, Y, Z = ([arena.alloc(r, n, torch.float32).zero_() for _ in range(per_region)] for r in range(3))
    torch.cuda.synchronize()

    def run(reads, writes):
        return B.halos_probe_streams(reads, writes, nbytes, args.reps)

    rows = []
    rows.append(("1 read", run([X[0]], [])))
    rows.append(("2 reads, one region", run([X[0], X[1]], [])))
    rows.append(("4 reads, one region", run(X[:4], [])))
    rows.append(("4 reads over three regions", run([X[0], Y[0], Z[0], X[1]], [])))
    rows.append(("1 write", run([], [X[4]])))
    rows.append(("2 writes, one region", run([], [X[4], X[5]])))
    rows.append(("4 writes, one region", run([], X[4:8])))
    rows.append(("4 writes over three regions", run([], [X[4], Y[4], Z[4], X[5]])))
    rows.append(("copy (1 read, 1 write), one region", run([X[0]], [X[4]])))
    rows.append(("copy, two regions", run([X[0]], [Y[4]])))
    r4 = max(rows[2][1], rows[3][1])
    w4 = max(rows[6][1], rows[7][1])
    mixes = [
        ("4 reads + 4 writes, all in one region", X[:4], X[4:8]),
        ("4 reads + 4 writes, spread evenly (reads X Y Z X, writes X Y Z Y)", [X[0], Y[0], Z[0], X[1]], [X[4], Y[4], Z[4], Y[5]]),
        ("4 reads + 4 writes, as the benchmark places the update pass (reads X X X Y, writes X X Y Z)",
         [X[0], X[1], X[2], Y[0]], [X[4], X[5], Y[4], Z[4]]),
        ("4 reads + 4 writes, no region both read and written (reads X X X X, writes Y Z Y Z)", X[:4], [Y[4], Z[4], Y[5], Z[5]]),
    ]
    for name, rd, wr in mixes:
        rows.append((name, run(rd, wr)))
    print(f"\nbuffers of {nbytes / (1 << 30):.2f} GiB, {args.reps} timed sweeps each, GB/s = bytes moved / time")
    print(f"{'pattern':100s} {'GB/s':>8s} {'of 8 TB/s':>10s}")
    for name, v in rows:
        print(f"{name:100s} {v:8.0f} {v / 8000:10.1%}")
    # bytes of the update pass with fused pull and a bf16 delta: 14 read, 16 written per parameter
    pred = 30.0 / (14.0 / r4 + 16.0 / w4)
    print(f"\nbest 4-stream read rate {r4:.0f} GB/s, best 4-stream write rate {w4:.0f} GB/s")
    print(f"a pass that reads 14 and writes 16 bytes per parameter at those rates, if reads and writes did not disturb each "
          f"other: {pred:.0f} GB/s = {pred / 8000:.1%} of 8 TB/s; the mixes above show what is left of that when they do")


if __name__ == "__main__":
    main()
