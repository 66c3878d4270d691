"""Pins of the burst-parallel planner oracle (oracle/burst_plan.py) against things other than itself:
exhaustive enumeration, a hand-worked example, closed forms and invariants of Section 4.2."""
import itertools
import math

import numpy as np
import pytest

from oracle import burst_plan as bp


def random_tables(rng, L, G, scale_comm=1.0):
    """Costs on a 1/8 grid: every sum below is exact in fp64, so comparisons are equalities."""
    gpus = [1, 2, 4, 8, 16, 32][:G]
    comp = [[float(rng.integers(8, 200)) / 8 for _ in range(G)] for _ in range(L)]
    comm = [[[0.0 if (i == 0 or a == b) else scale_comm * float(rng.integers(0, 40)) / 8 for a in range(G)] for b in range(G)]
            for i in range(L)]
    sync = [[0.0 if a == 0 else float(rng.integers(0, 24)) / 8 for a in range(G)] for _ in range(L)]
    return gpus, comp, comm, sync


def path_time(plan, comp, comm, sync):
    t = 0.0
    for i, a in enumerate(plan):
        t += (comm[i][plan[i - 1]][a] if i > 0 else 0.0) + comp[i][a] + sync[i][a]
    return t


def test_hand_worked_two_layers():
    # two layers, one or two GPUs; numbers worked by hand (see the arithmetic in the comments)
    gpus = [1, 2]
    comp = [[10.0, 6.0], [8.0, 5.0]]
    comm = [[[0.0, 0.0], [0.0, 0.0]], [[0.0, 1.5], [1.5, 0.0]]]
    sync = [[0.0, 0.5], [0.0, 1.0]]
    r = bp.plan_chain(gpus, comp, comm, sync, math.inf)
    assert r["S"][1] == [10.0, 6.5] and r["T"][1] == [10.0, 6.5]
    # L2 on 1 GPU: from 2 GPUs 6.5 + 1.5 = 8 beats staying (10); on 2 GPUs: stay, 6.5 + 5 + 1
    assert r["S"][2] == [16.0, 12.5] and r["T"][2] == [9.5, 6.0]
    assert r["gpus"] == [2, 2] and r["time"] == 12.5
    amp = bp.amplification(gpus, comp, r["T"])
    assert amp == [[1.0, 1.3], [1.1875, 1.5]]
    # limit 1.25: L1 on 2 GPUs (amplification 1.3) may no longer precede L2, and L2 on 2 GPUs
    # (T = 1.5 + 5 + 1 = 7.5, amplification 1.875) is not an admissible end
    r = bp.plan_chain(gpus, comp, comm, sync, 1.25)
    assert r["S"][2] == [18.0, 17.5] and r["T"][2] == [8.0, 7.5]
    assert r["gpus"] == [1, 1] and r["time"] == 18.0


@pytest.mark.parametrize("seed", range(12))
def test_unlimited_amplification_is_the_shortest_path(seed):
    rng = np.random.default_rng(seed)
    L, G = int(rng.integers(1, 6)), int(rng.integers(1, 5))
    gpus, comp, comm, sync = random_tables(rng, L, G)
    r = bp.plan_chain(gpus, comp, comm, sync, math.inf)
    best_end = [math.inf] * G
    for plan in itertools.product(range(G), repeat=L):
        best_end[plan[-1]] = min(best_end[plan[-1]], path_time(plan, comp, comm, sync))
    assert r["S"][L] == best_end
    assert r["time"] == min(best_end)
    assert path_time(r["plan"], comp, comm, sync) == r["time"]


@pytest.mark.parametrize("seed", range(12))
def test_backtrace_is_consistent_under_a_limit(seed):
    rng = np.random.default_rng(100 + seed)
    L, G = int(rng.integers(2, 9)), int(rng.integers(2, 7))
    gpus, comp, comm, sync = random_tables(rng, L, G, scale_comm=0.25)
    limit = float(rng.choice([1.0, 1.25, 1.5, 2.0, 4.0]))
    r = bp.plan_chain(gpus, comp, comm, sync, limit)
    # the time reported is the sum along the plan, and S[i][g_i] is the partial sum
    assert path_time(r["plan"], comp, comm, sync) == r["time"]
    for i in range(1, L + 1):
        assert path_time(r["plan"][:i], comp, comm, sync) == r["S"][i][r["plan"][i - 1]]
    # one GPU everywhere is always considered first and only ever replaced by something no slower
    assert r["time"] <= sum(c[0] for c in comp)
    # a tighter limit never yields a faster plan than no limit
    assert r["time"] >= bp.plan_chain(gpus, comp, comm, sync, math.inf)["time"]


def test_no_communication_single_gpu_amplification_is_one():
    rng = np.random.default_rng(5)
    gpus, comp, _, _ = random_tables(rng, 6, 4)
    zero_comm = [[[0.0] * 4 for _ in range(4)] for _ in range(6)]
    zero_sync = [[0.0] * 4 for _ in range(6)]
    r = bp.plan_chain(gpus, comp, zero_comm, zero_sync, 2.0)
    amp = bp.amplification(gpus, comp, r["T"])
    assert all(row[0] == 1.0 for row in amp)
    assert r["S"][0] == [0.0] * 4


def test_perfect_scaling_bursts_every_layer_to_all_gpus():
    gpus = [1, 2, 4, 8]
    c1 = [64.0, 16.0, 40.0, 8.0, 24.0]
    comp = [[c / g for g in gpus] for c in c1]
    zero_comm = [[[0.0] * 4 for _ in range(4)] for _ in range(5)]
    zero_sync = [[0.0] * 4 for _ in range(5)]
    r = bp.plan_chain(gpus, comp, zero_comm, zero_sync, 1.0)   # amplification is exactly 1 everywhere
    assert r["gpus"] == [8] * 5 and r["time"] == sum(c1) / 8


def test_ties_take_the_later_gpu_count():
    gpus = [1, 2, 4]
    comp = [[3.0, 3.0, 3.0], [5.0, 5.0, 5.0]]
    zero_comm = [[[0.0] * 3 for _ in range(3)] for _ in range(2)]
    zero_sync = [[0.0] * 3 for _ in range(2)]
    r = bp.plan_chain(gpus, comp, zero_comm, zero_sync, math.inf)
    assert r["H"][2] == [2, 2, 2] and r["gpus"] == [4, 4]


def test_a_limit_below_one_falls_back_to_one_gpu():
    # nothing is admissible but the first candidate of every scan, which the algorithm always takes
    rng = np.random.default_rng(9)
    gpus, comp, comm, sync = random_tables(rng, 5, 4)
    r = bp.plan_chain(gpus, comp, comm, sync, 0.5)
    assert r["gpus"] == [1] * 5 and r["time"] == sum(c[0] for c in comp)


def test_cost_model_numbers():
    # 1200 bytes of activations, 100 B/s, 0.5 s delay: 1 -> 4 GPUs moves 1200 * (1 - 1/4) = 900 bytes per
    # GPU of the small set: 9 s + 0.5 s, forward and backward
    assert bp.comm_time(1200.0, 1, 4, 100.0, 0.5) == 19.0
    assert bp.comm_time(1200.0, 4, 1, 100.0, 0.5) == 19.0
    assert bp.comm_time(1200.0, 2, 4, 100.0, 0.5) == 2 * (300.0 / 100.0 + 0.5)
    assert bp.comm_time(1200.0, 4, 4, 100.0, 0.5) == 0.0
    # 800 bytes of gradients over 4 GPUs: two phases of 800 * 3/4 = 600 bytes
    assert bp.sync_time(800.0, 4, 100.0, 0.5) == 2 * (6.0 + 0.5)
    assert bp.sync_time(800.0, 1, 100.0, 0.5) == 0.0
    comm, sync = bp.cost_tables([1, 2, 4], [5000.0, 1200.0], [800.0, 400.0], 100.0, 0.5)
    assert comm[0] == [[0.0] * 3 for _ in range(3)]          # the network input is not redistributed
    assert comm[1][0][2] == 19.0 and comm[1][2][0] == 19.0 and comm[1][1][1] == 0.0
    assert sync[0][2] == 13.0 and sync[1][0] == 0.0
