"""Pins for Algorithm 1 / Algorithm 2 of the oracle: hand-worked tiny cases and
the closed-form mass of a Zipf law."""
import json
import os

import numpy as np

from oracle import placement as pl
from paper_2510_20878_amd import workloads as wl


def test_alg1_split_by_hand():
    # 10 chunks; frequencies chosen so the descending order is 7,2,9,0,4,1,3,5,6,8
    af = [5, 3, 9, 3, 4, 1, 1, 12, 0, 7]
    assert pl.rank_order(af) == [7, 2, 9, 0, 4, 1, 3, 5, 6, 8]       # ties 1/3 and 5/6 by id
    # tau = 20 %, 30 % -> idx1 = 2, idx2 = 5
    cls = pl.classes_by_rank(af, [200_000, 300_000])
    assert [cls[c] for c in [7, 2]] == [0, 0]
    assert [cls[c] for c in [9, 0, 4]] == [1, 1, 1]
    assert [cls[c] for c in [1, 3, 5, 6, 8]] == [2] * 5


def test_alg1_paper_thresholds_floor(golden_dir):
    tau = json.load(open(os.path.join(golden_dir, "paper_values.json")))["alg1_thresholds_percent"]["tau"]
    ppm = [t * 10_000 for t in tau]
    # 2n = 38 units: floor(3.8) = 3 per class, the rest is coldest
    assert pl.split_points(38, ppm) == [3, 6, 9]
    cls = pl.classes_by_rank(list(range(38, 0, -1)), ppm)
    assert cls[:9] == [0, 0, 0, 1, 1, 1, 2, 2, 2] and set(cls[9:]) == {3}
    assert pl.split_points(1000, ppm) == [100, 200, 300]
    assert pl.split_points(5, [900_000, 900_000]) == [4, 5]          # clipped at n


def test_alg2_trace_by_hand(golden_dir):
    # 20 chunks, rank == id.  tau_GPU 10 %, tau_PIN 10 %, tau_PAGE 20 % -> lists
    # GPU {0,1}, PIN {2,3}, PAGE {4..7}, DISK {8..19}; capacities 2 / 2 / 2.
    sim = pl.TierSim(list(range(20)), [100_000, 100_000, 200_000], (2, 2, 2))
    assert sim.bounds == (2, 4, 8)
    D, G, P, A = sim.DISK, sim.GPU, sim.PIN, sim.PAGE
    assert sim.access(0) == (D, [(G, None)])          # disk -> GPU_LIST member goes to GPU
    assert sim.access(0) == (G, [])                   # now a GPU hit
    assert sim.access(2) == (D, [(P, None)])
    assert sim.access(9) == (D, [])                   # DISK_LIST member is not kept anywhere
    assert sim.access(9) == (D, [])
    assert sim.access(5) == (D, [(A, None)])
    assert sim.access(6) == (D, [(A, None)])
    assert sim.access(5) == (A, [])                   # refreshes 5: 6 is now least recent
    assert sim.access(7) == (D, [(A, 6)])             # LRU eviction of 6
    assert sim.resident(A) == [5, 7]
    assert sim.access(1) == (D, [(G, None)])
    assert sim.resident(G) == [0, 1]
    # a GPU_LIST chunk found in pinned memory is promoted; GPU is full -> evict LRU (0)
    sim.seed(P, [0])
    sim.q[G].d.pop(0)
    sim.seed(G, [3])                                  # GPU now holds 1 (older), 3
    assert sim.access(0) == (P, [(G, 1)])
    assert sim.resident(G) == [3, 0]
    assert 0 in sim.q[P]                              # inclusive: pinned copy stays


def test_alg2_two_tier_reduction():
    # everything pinned (unbounded), GPU capacity 3, GPU_LIST = ranks 0..4
    n = 50
    sim = pl.TierSim(list(range(n)), [100_000, 900_000, 0], (3, None, 0))
    sim.seed(sim.PIN, range(n))
    seq = [0, 1, 2, 3, 0, 7, 4, 1, 2, 2, 30, 0]
    got = [sim.access(c) for c in seq]
    G, P = sim.GPU, sim.PIN
    assert got == [
        (P, [(G, None)]), (P, [(G, None)]), (P, [(G, None)]),
        (P, [(G, 0)]),            # full: evicts 0
        (P, [(G, 1)]),            # 0 again: evicts 1
        (P, []),                  # rank 7 is not in GPU_LIST: served from pinned, not promoted
        (P, [(G, 2)]),
        (P, [(G, 3)]),
        (P, [(G, 0)]),
        (G, []),
        (P, []),
        (P, [(G, 4)]),
    ]


def test_zipf_mass_closed_form(golden_dir):
    hot = json.load(open(os.path.join(golden_dir, "paper_values.json")))["hot_fraction"]["fraction"]
    p = wl.zipf_pmf(100_000, 1.1)
    H = lambda n: float(np.sum(1.0 / np.arange(1, n + 1) ** 1.1))
    assert abs(p[:int(hot * 100_000)].sum() - H(1000) / H(100_000)) < 1e-12
    assert abs(p[:1000].sum() - 0.751) < 2e-3         # top 1 % of ids draw ~75 % of accesses
    assert abs(wl.zipf_pmf(10_000)[:2000].sum() - 0.895) < 3e-3
    req = wl.zipf_requests(100_000, 4000, 8, seed=4)
    assert req.shape == (4000, 8)
    assert all(len(set(r)) == 8 for r in req.tolist())
    share = float(np.mean(req < 1000))
    assert abs(share - 0.74) < 0.03                   # distinct-per-request trims the head a little


def test_floor_option_keeps_every_accessed_chunk_out_of_the_slow_tiers():
    """Hand-worked: 20 chunks, lists GPU {0,1}, PIN {2,3}, PAGE {4..7}, DISK the rest; queues of 2."""
    sim = pl.TierSim(list(range(20)), [100_000, 100_000, 200_000], (2, 2, 2))
    assert sim.access(12) == (pl.TierSim.DISK, [])                         # the algorithm leaves it on disk
    assert sim.access(12, floor=pl.TierSim.PIN) == (pl.TierSim.DISK, [(pl.TierSim.PIN, None)])
    assert sim.access(5, floor=pl.TierSim.PIN) == (pl.TierSim.DISK, [(pl.TierSim.PIN, None)])   # PAGE list -> pinned
    assert sim.access(0, floor=pl.TierSim.PIN) == (pl.TierSim.DISK, [(pl.TierSim.GPU, None)])   # faster lists unchanged
    assert sim.access(13, floor=pl.TierSim.PIN) == (pl.TierSim.DISK, [(pl.TierSim.PIN, 12)])    # LRU of the full queue
    assert sim.access(5, floor=pl.TierSim.PIN) == (pl.TierSim.PIN, [])
    assert sim.access(6, floor=pl.TierSim.PAGE) == (pl.TierSim.DISK, [(pl.TierSim.PAGE, None)])
    assert sim.resident(pl.TierSim.PIN) == [13, 5] and sim.resident(pl.TierSim.PAGE) == [6]
