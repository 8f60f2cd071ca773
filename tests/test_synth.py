"""The seeded input generators: determinism, shapes and distributions."""
import numpy as np
import torch

import synth
from synth.tensors import scale_f32


def test_layout_sizes_match_the_named_model_sizes():
    expect = {"tiny": (1 << 20, 1), "70m": (70_426_624, 76), "160m": (162_322_944, 148),
              "410m": (405_334_016, 292), "1b": (1_011_781_632, 196)}
    for name, (total, n_tensors) in expect.items():
        lay = synth.get_workload(name).layout
        assert lay.total == total and lay.n_tensors == n_tensors
        assert lay.offsets[-1] == total


def test_trace_is_deterministic_and_counts_updates():
    for name, w in synth.WORKLOADS.items():
        if w.schedule != "seeded":
            continue
        a, b = synth.make_trace(w), synth.make_trace(w)
        assert a.to_bytes() == b.to_bytes()
        assert a.n_update_steps == w.n_updates
        assert synth.make_trace(w, seed=w.seed + 1).to_bytes() != a.to_bytes()
        ev = a.events
        assert ev["staleness"].max() <= w.staleness_bound
        assert ev["slot"][ev["kind"] == synth.EV_ARRIVE_DELTA].max() < w.pool_slots
        # every merge step was preceded by exactly one GPS merge and one arrival of the global model
        assert a.n_merge_steps <= a.count(synth.EV_ARRIVE_GLOBAL) <= a.count(synth.EV_GPS_MERGE) <= int(ev["exp_send"].sum())


def test_trace_exercises_queueing_and_in_flight_updates():
    tr = synth.make_trace(synth.get_workload("410m"))
    ev = tr.events
    upd = ev[(ev["kind"] == synth.EV_LPS_STEP) & (ev["exp_kind"] == 1)]
    assert (upd["exp_accumulate"] == 0).any() and (upd["exp_accumulate"] == 1).any()
    ks = set(upd["k_cur"].tolist())
    assert min(ks) >= 2 and max(ks) <= 8 and len(ks) > 2
    # some delta waits behind another item: two arrivals for one LPS with no step of that LPS in between
    depth, deepest = {}, 0
    for r in ev:
        l = int(r["lps"])
        if r["kind"] in (synth.EV_ARRIVE_DELTA, synth.EV_ARRIVE_GLOBAL):
            depth[l] = depth.get(l, 0) + 1
            deepest = max(deepest, depth[l])
        elif r["kind"] == synth.EV_LPS_STEP:
            depth[l] = depth.get(l, 0) - 1
    assert deepest >= 2


def test_generator_subset_equals_full_and_is_seed_dependent():
    n = 10000
    idx = torch.arange(n, dtype=torch.int64)
    full = synth.normal_at(7, 3, idx, scale_f32(1e-3))
    pick = torch.tensor([0, 5, 77, 9999, 4096], dtype=torch.int64)
    assert torch.equal(synth.normal_at(7, 3, pick, scale_f32(1e-3)), full[pick])
    assert torch.equal(synth.normal_flat(7, 3, 100, 500, scale_f32(1e-3), chunk=128), full[100:600])
    assert not torch.equal(synth.normal_at(8, 3, idx, scale_f32(1e-3)), full)
    assert not torch.equal(synth.normal_at(7, 4, idx, scale_f32(1e-3)), full)


def test_generator_moments():
    idx = torch.arange(1 << 20, dtype=torch.int64)
    x = synth.normal_at(1, 1, idx, scale_f32(1e-3)).double()
    assert abs(x.mean().item()) < 5e-6
    assert abs(x.std().item() / 1e-3 - 1) < 5e-3
    kurt = ((x - x.mean()) ** 4).mean().item() / x.var().item() ** 2
    assert 2.7 < kurt < 3.0                      # Irwin-Hall n=8: 3 - 0.15
    # successive elements are uncorrelated
    assert abs((x[1:] * x[:-1]).mean().item()) / x.var().item() < 5e-3


def test_bf16_bits_are_round_to_nearest_even():
    x = torch.tensor([1.0, 1.00390625, 1.01171875, -2.0, 3.0e-5], dtype=torch.float32)
    bits = synth.to_bf16_bits(x).numpy().astype(np.uint16)
    # 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even; 1 + 3*2^-8 is a tie between 0x3F81 and 0x3F82 -> even
    assert bits[0] == 0x3F80 and bits[1] == 0x3F80 and bits[2] == 0x3F82 and bits[3] == 0xC000
