"""The paper's cluster model (App. A): duration formulas, tables, and the traces generated from them."""
import numpy as np
import pytest

import synth
from synth import paper_cluster as pc


def test_duration_formulas_against_hand_computed_values():
    # T = alpha + C / B : 70,426,624 fp32 parameters = 281,706,496 bytes over the slowest link (0.117 Gbps)
    c = 70_426_624 * 4
    assert pc.t_p2p(c, 0.117) == pytest.approx(281_706_496 * 8 / 0.117e9)
    assert 19.2 < pc.t_p2p(c, 0.117) < 19.3
    assert pc.t_p2p(c, 100.0) == pytest.approx(0.02253651968)
    assert pc.t_p2p(c, 100.0, alpha_s=0.5) == pytest.approx(0.52253651968)
    # T = 2 (N-1) C / (N B): 4 participants, 1 GB, 1 Gbps -> 2 * 3/4 * 8 s = 12 s
    assert pc.t_allreduce(4, 1e9, 1.0) == pytest.approx(12.0)
    assert pc.t_allreduce(1, 1e9, 1.0) == 0.0
    # T = H * T_profiled * S_fastest / S : 8 steps of 238.4 ms on a worker of speed 2.6 when the fastest is 10
    assert pc.t_compute(8, 238.4, 2.6, 10.0) == pytest.approx(8 * 0.2384 * 10 / 2.6)
    assert pc.t_compute(8, 238.4, 10.0, 10.0) == pytest.approx(1.9072)


def test_tables_are_the_printed_ones():
    bw = pc.BANDWIDTH_GBPS
    assert np.array_equal(bw, bw.T) and np.all(np.diag(bw) == 100.0)
    off = bw[~np.eye(4, dtype=bool)]
    assert off.min() == 0.117 and off.max() == 0.935                                 # "0.117 to 0.935 Gbps"
    s = pc.WORKER_SPEEDS
    assert s.shape == (4, 4) and s.max() == 10.0 and s.min() == 1.2 and np.all((s >= 1.0) & (s <= 10.0))
    assert pc.PROFILED_STEP_MS == {"70m": 238.4, "160m": 623.0, "410m": 1589.7}


def test_best_ring_maximises_the_slowest_link():
    slow, ring = pc.best_ring_bandwidth([0, 1, 2, 3])
    # brute force over the three distinct rings of four nodes
    cands = {(0, 1, 2, 3): min(0.537, 0.386, 0.127, 0.202), (0, 1, 3, 2): min(0.537, 0.117, 0.127, 0.935),
             (0, 2, 1, 3): min(0.935, 0.386, 0.117, 0.202)}
    assert slow == pytest.approx(max(cands.values())) == pytest.approx(0.127)
    assert pc.best_ring_bandwidth([2])[0] == 100.0
    assert pc.best_ring_bandwidth([0, 2])[0] == pytest.approx(0.935)


@pytest.mark.parametrize("name", ["paper-70m", "paper-160m", "paper-410m"])
def test_paper_trace_structure(name):
    w = synth.get_workload(name)
    a, b = synth.make_trace(w), synth.make_trace(w)
    assert a.to_bytes() == b.to_bytes()
    ev = a.events
    assert a.n_update_steps == w.n_updates
    assert np.all(np.diff(ev["time"]) >= 0)                                           # replay order is time order
    upd = ev[(ev["kind"] == synth.EV_LPS_STEP) & (ev["exp_kind"] == 1)]
    # every LPS sends after K = 32 accumulated updates, and updates keep landing while its update is in flight
    assert set(upd["k_cur"].tolist()) == {32}
    assert (upd["exp_accumulate"] == 0).any()
    # the region with the slowest link to the GPS (R-4, 0.202 Gbps to R-1) waits longest between send and merge
    wait = {}
    for l in range(4):
        mine = ev[ev["lps"] == l]
        sends = mine["time"][(mine["kind"] == synth.EV_LPS_STEP) & (mine["exp_send"] == 1)]
        merges = mine["time"][(mine["kind"] == synth.EV_LPS_STEP) & (mine["exp_kind"] == 2)]
        n = min(len(sends), len(merges))
        assert n >= 1
        wait[l] = float(np.mean(merges[:n] - sends[:n]))
    assert wait[3] == max(wait.values()) and wait[0] == min(wait.values())
    # round trip of the accumulated update and the returned model: two transfers over the LPS-GPS link
    c = w.layout.total * 4
    assert wait[3] >= 2 * pc.t_p2p(c, 0.202) * 1e6 - 2
    assert wait[0] >= 2 * pc.t_p2p(c, 100.0) * 1e6 - 2


def test_dynamic_local_updates_equalise_round_times():
    spec = pc.PaperClusterSpec(model="70m", n_params=70_426_624)
    tr = pc.make_paper_trace(spec, 64)
    r = tr.worker_period / 1e6
    assert r.max() / r.min() < 1.5                       # H scaled with speed: similar round times
    fixed = pc.make_paper_trace(pc.PaperClusterSpec(model="70m", n_params=70_426_624, dynamic_local_updates=False), 64)
    rf = fixed.worker_period / 1e6
    assert rf.max() / rf.min() == pytest.approx(10.0 / 1.2, rel=1e-3)     # fixed H: times inversely proportional to speed
    assert rf.min() == pytest.approx(1.9072, rel=1e-4)
