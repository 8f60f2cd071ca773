"""Host logic of the benchmark that the reported figures rest on: the algorithmic bytes per parameter that each kernel
label is charged with (the numerator of every GB/s figure and of the roofline fraction), and the refusal to run on more
than one GPU.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


# fp32 state: every array an event needs is read once and written once, 4 bytes each way; a 16-bit delta costs 2.
# S1 = delta + (m, theta, third) read and written; S3 = G, M, Theta read + M, Theta, returned model written; S4 = theta and
# returned model read + theta and third written; S5 = one read, one write.
@pytest.mark.parametrize("label,dtype,delayed,want", [
    ("lps_update_acc", "f32", False, 4 + 3 * 8),                 # 28
    ("lps_update_acc", "bf16", False, 2 + 3 * 8),                # 26
    ("lps_update_noacc", "f32", False, 4 + 2 * 8),               # 20: accumulated update in flight, third buffer untouched
    ("lps_update_noacc", "f16", False, 2 + 2 * 8),               # 18
    ("lps_update_acc_pull", "bf16", False, 26 + 4),              # the worker's model buffer written in the same pass
    ("lps_update_noacc_pull", "bf16", False, 18 + 4),
    ("lps_update_freeze_pull", "f32", False, 28 + 4),            # snapshot form: snapshot read, Delta written
    ("lps_update_restart_pull", "bf16", False, 30 - 4),          # third buffer written without being read
    ("gps_update", "f32", False, 24),
    ("gps_update_nomom", "f32", False, 16),
    ("lps_merge", "f32", False, 16),
    ("lps_merge_leave", "f32", False, 12),
    ("pull", "f32", False, 8),
    # delayed momentum: first = buffer written; inner = buffer read and written; refresh = buffer read, momentum read and written
    ("lps_update_acc_first_pull", "bf16", True, 2 + 8 + 8 + 4 + 4),
    ("lps_update_acc_pull", "bf16", True, 2 + 8 + 8 + 8 + 4),
    ("lps_update_acc_refresh_pull", "bf16", True, 2 + 8 + 8 + 12 + 4),
    ("gps_update_first", "f32", True, 16 + 4),
    ("gps_update_refresh", "f32", True, 16 + 12),
    # k deltas in one pass: k deltas read, k worker models written, momentum + model (+ third buffer) once
    ("lps_update_batch2_acc_pull", "bf16", False, 2 * 2 + 24 + 2 * 4),
    ("lps_update_batch3_noacc_pull", "f32", False, 3 * 4 + 16 + 3 * 4),
    ("lps_update_batch1_merge_pull", "bf16", False, 2 + 24 + 4),        # returned model read from, restarted sum written to, the third buffer
    ("lps_update_batch2_merge_pull", "f32", False, 2 * 4 + 24 + 2 * 4),
    ("lps_update_batch1_merge_first_pull", "bf16", True, 2 + 8 + 8 + 4 + 4),
    ("lps_update_batch1_merge_refresh_pull", "bf16", True, 2 + 8 + 8 + 12 + 4),
])
def test_bytes_charged_per_parameter(label, dtype, delayed, want):
    assert bench.bytes_per_param(label, dtype, delayed) == want


@pytest.mark.parametrize("label,dtype,want", [
    ("lps_update_acc_pull", "bf16", 26), ("lps_update_noacc_pull", "bf16", 18), ("gps_update", "f32", 20),
    ("lps_update_batch2_acc_pull", "bf16", 2 * 2 + 20 + 8), ("lps_merge", "f32", 16),
])
def test_bytes_with_16_bit_momentum(label, dtype, want):
    """The momentum's read and write cost 2 bytes each instead of 4; nothing else changes."""
    assert bench.bytes_per_param(label, dtype, False, 2) == want


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_stored_counter_traffic_is_keyed_by_the_kernel_source():
    """The counter-measured traffic in the benchmark line is reported only for the kernel source it was measured on."""
    table = bench.MEASURED_TRAFFIC
    assert len(table) == 1
    if bench.kernels_digest() not in table:
        pytest.skip("kernels.hip has changed since the counters under profiles/ were taken: the benchmark reports no traffic figure")
    per = table[bench.kernels_digest()]
    for key, measured in per.items():
        wl, label = key.split(":")
        algorithmic = bench.bytes_per_param(label, "bf16", wl.startswith("1b-dn"), 2 if wl.endswith("+bf16m") else 4)
        assert algorithmic <= measured <= 1.01 * algorithmic, (key, measured, algorithmic)
