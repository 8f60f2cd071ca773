"""Worker of the every-element full-size parity test: replay one workload's whole trace through the fp32 same-order
oracle on ONE contiguous chunk of the parameters and compare it, bit for bit, with the GPU state that the test saved.

    python tests/chunk_oracle_check.py WORKLOAD STATE_DIR LO HI

STATE_DIR holds one .npy file per state array (float32, all parameters, packed in layout order).  Prints one line:
"CHUNK lo hi differing_elements compared_elements".  CPU only; elements are independent, so a chunk is a full replay.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))


def main():
    name, state_dir, lo, hi = sys.argv[1], sys.argv[2], int(sys.argv[3]), int(sys.argv[4])
    import torch
    torch.set_num_threads(1)
    import synth
    from oracle import FORM_ACCUMULATOR
    from parity_util import oracle_run, oracle_state
    w = synth.get_workload(name)
    trace = synth.make_trace(w)
    idx = np.arange(lo, hi, dtype=np.int64)
    o, _log = oracle_run(w, trace, idx, 32, FORM_ACCUMULATOR)
    ref = oracle_state(o, w.n_lps, with_scale=False)
    n_diff = n_cmp = 0
    for k, (x_ref, _) in ref.items():
        gpu = np.load(os.path.join(state_dir, k + ".npy"), mmap_mode="r")[lo:hi]
        r32 = x_ref.astype(np.float32)
        n_diff += int((np.asarray(gpu).view(np.uint32) != r32.view(np.uint32)).sum())
        n_cmp += r32.size
    print(f"CHUNK {lo} {hi} {n_diff} {n_cmp}", flush=True)


if __name__ == "__main__":
    main()
