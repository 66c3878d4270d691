"""Pins of the branch/join planner oracle (oracle/graph_plan.py) against things other than itself:
exhaustive enumeration where the reduction is exact, the chain planner on a flattened single-branch
block, a hand-worked block, and the plan's own time recomputed by an independent evaluator."""
import itertools
import math

import numpy as np
import pytest

from oracle import burst_plan as bp
from oracle import graph_plan as gp

INF = math.inf


def grid(rng, lo, hi):
    return float(rng.integers(lo, hi)) / 8      # 1/8 grid: every sum and max below is exact in fp64


def random_graph(rng, L, G, n_branches, move, allow_empty=True):
    """L main layers; layer `join` (>= 1) is fed by a block of n_branches branches."""
    gpus = [1, 2, 4, 8][:G]

    def table():
        return [[0.0 if a == b else grid(rng, 0, 24) for a in range(G)] for b in range(G)]

    layers = []
    join = int(rng.integers(1, L))
    for i in range(L):
        lay = {"comp": [grid(rng, 8, 120) for _ in range(G)], "sync": [0.0 if a == 0 else grid(rng, 0, 16) for a in range(G)],
               "comm": [[0.0] * G for _ in range(G)] if i == 0 else table(), "branches": []}
        if i == join:
            for k in range(n_branches):
                Lb = int(rng.integers(0 if (allow_empty and k > 0) else 1, 3))
                mv = [[move if move is not None else grid(rng, 0, 60) for _ in range(G)] for _ in range(G)]
                lay["branches"].append({"comp": [[grid(rng, 8, 120) for _ in range(G)] for _ in range(Lb)],
                                        "sync": [[0.0 if a == 0 else grid(rng, 0, 16) for a in range(G)] for _ in range(Lb)],
                                        "comm": [table() for _ in range(Lb)], "join": table(), "move": mv})
        layers.append(lay)
    return gpus, layers


def branch_time(br, g, plan, h):
    if not plan:
        return br["join"][g][h]
    t, prev = 0.0, g
    for l, a in enumerate(plan):
        t += br["comm"][l][prev][a] + br["comp"][l][a] + br["sync"][l][a]
        prev = a
    return t + br["join"][prev][h]


def block_cost(times, moves, lens):
    """Independent statement of the rule: the longest branch (first on ties), plus every other branch
    unless it has layers and fits beside the longest one after paying its move."""
    crit = times.index(max(times))
    total = times[crit]
    for k, t in enumerate(times):
        if k != crit and not (lens[k] > 0 and t + moves[k] <= times[crit]):
            total += t
    return total


def total_time(layers, main, branch_plans):
    t = 0.0
    for i, lay in enumerate(layers):
        a = main[i]
        if lay["branches"]:
            g = main[i - 1]
            times = [branch_time(br, g, branch_plans[k], a) for k, br in enumerate(lay["branches"])]
            t += block_cost(times, [br["move"][g][a] for br in lay["branches"]], [len(br["comp"]) for br in lay["branches"]])
        elif i > 0:
            t += lay["comm"][main[i - 1]][a]
        t += lay["comp"][a] + lay["sync"][a]
    return t


def brute_force(gpus, layers):
    G = len(gpus)
    (branches,) = [lay["branches"] for lay in layers if lay["branches"]]
    best = INF
    for main in itertools.product(range(G), repeat=len(layers)):
        for bp_ in itertools.product(*[list(itertools.product(range(G), repeat=len(br["comp"]))) for br in branches]):
            best = min(best, total_time(layers, main, bp_))
    return best


def plan_time(layers, r):
    (j,) = [i for i, lay in enumerate(layers) if lay["branches"]]
    return total_time(layers, r["plan"], r["blocks"][j]["plans"])


@pytest.mark.parametrize("seed", range(10))
def test_no_branch_can_move_block_is_the_sum(seed):
    rng = np.random.default_rng(seed)
    gpus, layers = random_graph(rng, int(rng.integers(2, 4)), int(rng.integers(2, 4)), int(rng.integers(2, 4)), move=INF)
    r = gp.plan_graph(gpus, layers, INF)
    assert r["time"] == brute_force(gpus, layers)
    assert plan_time(layers, r) == r["time"]
    assert not any(r["blocks"][i]["parallel"][k] for i in range(len(layers)) if r["blocks"][i] for k in range(len(r["blocks"][i]["parallel"])))


@pytest.mark.parametrize("seed", range(10))
def test_free_moves_block_is_the_longest_branch(seed):
    rng = np.random.default_rng(50 + seed)
    gpus, layers = random_graph(rng, int(rng.integers(2, 4)), int(rng.integers(2, 4)), int(rng.integers(2, 4)), move=0.0, allow_empty=False)
    r = gp.plan_graph(gpus, layers, INF)
    assert r["time"] == brute_force(gpus, layers)
    assert plan_time(layers, r) == r["time"]
    (blk,) = [b for b in r["blocks"] if b]
    assert sum(blk["parallel"]) == len(blk["parallel"]) - 1 and not blk["parallel"][blk["critical"]]


@pytest.mark.parametrize("seed", range(10))
def test_any_move_cost_plan_is_consistent_and_bounded(seed):
    rng = np.random.default_rng(90 + seed)
    gpus, layers = random_graph(rng, int(rng.integers(2, 4)), int(rng.integers(2, 4)), int(rng.integers(2, 4)), move=None)
    r = gp.plan_graph(gpus, layers, INF)
    assert plan_time(layers, r) == r["time"]             # the reported time is what the reported plan costs
    assert brute_force(gpus, layers) <= r["time"]        # the reduction picks each branch greedily: never below the optimum
    one = sum(lay["comp"][0] + sum(row[0] for br in lay["branches"] for row in br["comp"]) for lay in layers)
    assert r["time"] <= one                               # everything on one GPU costs no transfers and is always offered


@pytest.mark.parametrize("seed", range(8))
def test_single_branch_block_is_the_flattened_chain(seed):
    rng = np.random.default_rng(200 + seed)
    gpus, layers = random_graph(rng, 3, int(rng.integers(2, 5)), 1, move=INF, allow_empty=False)
    r = gp.plan_graph(gpus, layers, INF)
    comp, comm, sync = [], [], []
    for lay in layers:
        if lay["branches"]:
            (br,) = lay["branches"]
            comp += br["comp"]
            comm += br["comm"]
            sync += br["sync"]
            comm.append(br["join"])
        else:
            comm.append(lay["comm"])
        comp.append(lay["comp"])
        sync.append(lay["sync"])
    assert r["time"] == bp.plan_chain(gpus, comp, comm, sync, INF)["time"]


def hand_block():
    hop = [[0.0, 1.0], [1.0, 0.0]]
    half = [[0.5, 0.5], [0.5, 0.5]]
    X = {"comp": [[8.0, 4.0]], "sync": [[0.0, 0.0]], "comm": [hop], "join": hop, "move": half}
    Y = {"comp": [[3.0, 2.0]], "sync": [[0.0, 0.0]], "comm": [hop], "join": hop, "move": half}
    Z = {"comp": [], "sync": [], "comm": [], "join": [[0.0, 0.5], [0.5, 0.0]], "move": half}
    return [X, Y, Z]


def test_hand_worked_block():
    gpus = [1, 2]
    tr, info = gp.reduce_block(gpus, hand_block(), [6.0, 3.0], [0.0, 0.5], INF)
    # g=1,h=1: X via two GPUs 1+4+1 = 6 (one GPU: 8), Y on one GPU 3, Z 0; Y fits beside X (3+0.5 <= 6): 6
    # g=1,h=2: X 1+4 = 5, Y via two GPUs 1+2 = 3 (ties with nothing: one GPU costs 3+1), Z 0.5; Y moves: 5.5
    # g=2,h=1: X 4+1 = 5, Y 2+1 = 3, Z 0.5: 5.5;  g=2,h=2: X 4, Y 2, Z 0: 4
    assert tr == [[6.0, 5.5], [5.5, 4.0]]
    assert info[0][0]["plans"] == [[1], [0], []] and info[0][0]["extra"] == 1
    assert all(info[g][h]["parallel"] == [False, True, False] and info[g][h]["critical"] == 0 for g in range(2) for h in range(2))
    layers = [{"comp": [4.0, 2.0], "sync": [0.0, 0.5], "comm": [[0.0, 0.0], [0.0, 0.0]], "branches": []},
              {"comp": [6.0, 3.0], "sync": [0.0, 0.5], "comm": None, "branches": hand_block()}]
    r = gp.plan_graph(gpus, layers, INF)
    # S[1] = [4, 2.5]; joining layer on one GPU: min(4+6, 2.5+5.5) + 6 = 14; on two: min(4+5.5, 2.5+4) + 3.5 = 10
    assert r["S"][2] == [14.0, 10.0] and r["T"][2] == [11.5, 7.5]
    assert r["gpus"] == [2, 2] and r["time"] == 10.0 and r["blocks"][1]["extra"] == 2


def test_hand_worked_block_under_a_limit():
    # limit 1.5, g=2,h=2: X 4, Y 2 as before; moving Y would hold 2+2 GPUs for 4+3+0.5 = 7.5 against 17 of
    # one-GPU work: 30/17 = 1.76 > 1.5, so Y runs after X and the block costs 6
    tr, info = gp.reduce_block([1, 2], hand_block(), [6.0, 3.0], [0.0, 0.5], 1.5)
    assert tr[1][1] == 6.0 and info[1][1]["parallel"] == [False, False, False] and info[1][1]["extra"] == 0
    # g=1,h=1: moving Y (a one-GPU set) holds 1+1 GPUs for 6+6 = 12: 24/17 = 1.41 <= 1.5, so it still moves
    assert tr[0][0] == 6.0 and info[0][0]["parallel"] == [False, True, False]


def test_limits_only_ever_refuse_moves():
    for seed in range(8):
        rng = np.random.default_rng(300 + seed)
        gpus, layers = random_graph(rng, 3, 3, 3, move=None)
        free = gp.plan_graph(gpus, layers, INF)
        assert gp.plan_graph(gpus, layers, 1e12)["time"] == free["time"]
        floor = brute_force(gpus, layers)
        for limit in (1.0, 1.5, 2.0, 4.0):
            r = gp.plan_graph(gpus, layers, limit)
            # the same plan costed without a limit moves every branch that fits: never more than what is reported
            assert floor <= plan_time(layers, r) <= r["time"]
            (blk,) = [b for b in r["blocks"] if b]
            refused = sum(t for k, t in enumerate(blk["reach"]) if k != blk["critical"] and not blk["parallel"][k])
            assert r["time"] - plan_time(layers, r) <= refused
