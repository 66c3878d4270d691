"""dp_plan_graph (host-only C ABI) against the branch/join planner oracle: GPU counts, critical branches and
move decisions are integers and must agree exactly; both sides add the same fp64 terms in the same order, so
the tables agree bit for bit as well."""
import math

import numpy as np
import pytest

from oracle import graph_plan as orc


# Every test runs twice: unmarked (any host) and marked `gpu`, so that the run on the GPU machine also records the
# planner's parity (the library there is the one the kernels were built into).
@pytest.fixture(scope="module", params=["host", pytest.param("gpu_box", marks=pytest.mark.gpu)])
def dp(request):
    from paper_2112_10065_amd import binding
    return binding


def random_graph(rng, L, G, blocks_at, max_branches=4):
    gpus = sorted(set([1] + [int(v) for v in rng.integers(2, 65, G - 1)]))
    G = len(gpus)

    def table(hi):
        return [[0.0 if a == b else float(rng.uniform(0, hi)) for a in range(G)] for b in range(G)]

    def times(n):
        return [[float(rng.uniform(5e-6, 3e-3)) for _ in range(G)] for _ in range(n)]

    def syncs(n):
        return [[0.0 if a == 0 else float(rng.uniform(0, 3e-4)) for a in range(G)] for _ in range(n)]

    layers = []
    for i in range(L):
        lay = {"comp": times(1)[0], "sync": syncs(1)[0], "comm": [[0.0] * G for _ in range(G)] if i == 0 else table(4e-4), "branches": []}
        if i in blocks_at:
            for k in range(int(rng.integers(1, max_branches + 1))):
                Lb = int(rng.integers(0, 4)) if k > 0 else int(rng.integers(1, 4))
                lay["branches"].append({"comp": times(Lb), "sync": syncs(Lb), "comm": [table(4e-4) for _ in range(Lb)], "join": table(4e-4),
                                        "move": [[float(rng.uniform(0, 2e-3)) for _ in range(G)] for _ in range(G)]})
        layers.append(lay)
    return gpus, layers


def compare(got, want, gpus, layers):
    assert got["gpus"] == want["gpus"]
    assert got["time"] == want["time"]
    assert got["S"] == want["S"] and got["T"] == want["T"]
    for i, lay in enumerate(layers):
        if not lay["branches"]:
            assert got["blocks"][i] is None and want["blocks"][i] is None
            continue
        w = want["blocks"][i]
        assert got["blocks"][i]["critical"] == w["critical"]
        assert got["blocks"][i]["parallel"] == w["parallel"]
        assert got["blocks"][i]["gpus"] == [[gpus[a] for a in p] for p in w["plans"]]


@pytest.mark.parametrize("seed", range(40))
def test_graph_plan_matches_oracle(dp, seed):
    rng = np.random.default_rng(seed)
    L, G = int(rng.integers(2, 14)), int(rng.integers(1, 7))
    blocks_at = set(int(v) for v in rng.integers(1, L, int(rng.integers(1, 5))))
    gpus, layers = random_graph(rng, L, G, blocks_at)
    limit = [math.inf, 1.0, 1.2, 1.5, 2.0, 3.0, 6.0, 0.5][seed % 8]
    compare(dp.dp_plan_graph(gpus, layers, limit), orc.plan_graph(gpus, layers, limit), gpus, layers)


def test_without_blocks_it_is_the_chain_planner(dp):
    rng = np.random.default_rng(123)
    gpus, layers = random_graph(rng, 12, 5, set())
    g = dp.dp_plan_graph(gpus, layers, 1.5)
    c = dp.dp_plan_chain(gpus, [l["comp"] for l in layers], [l["comm"] for l in layers], [l["sync"] for l in layers], 1.5)
    assert g["gpus"] == c["gpus"] and g["time"] == c["time"] and g["S"] == c["S"] and g["T"] == c["T"]
    assert g["blocks"] == [None] * 12


def test_inception_shaped_module_chain(dp):
    """Eleven modules of four branches (1x1 | 1x1-3x3 | 1x1-3x3-3x3 | pool-1x1), each joined by a concatenation
    layer, between a stem and a classifier: the block structure of the paper's Inception workload, with
    synthetic time tables that fall sub-linearly with the per-GPU batch."""
    rng = np.random.default_rng(11)
    gpus = [1, 2, 4, 8]
    G = 4

    def comp_row(t1):
        return [t1 / g ** float(rng.uniform(0.5, 0.95)) for g in gpus]

    def hop(bytes_):
        return [[0.0 if a == b else 2 * (bytes_ * abs(1 / gpus[a] - 1 / gpus[b]) / 1.07e12 + 1e-5) for a in range(G)] for b in range(G)]

    def branch(depth):
        return {"comp": [comp_row(float(rng.uniform(2e-5, 2e-4))) for _ in range(depth)], "sync": None,
                "comm": [hop(4e6) for _ in range(depth)], "join": hop(4e6), "move": [[2 * (4e6 / 1.07e12 + 1e-5)] * G for _ in range(G)]}

    layers = [{"comp": comp_row(9e-4), "sync": None, "comm": None, "branches": []}]
    for _ in range(11):
        layers.append({"comp": comp_row(1e-5), "sync": None, "comm": None, "branches": [branch(1), branch(2), branch(3), branch(1)]})
    layers.append({"comp": comp_row(5e-5), "sync": None, "comm": hop(1e5), "branches": []})
    for limit in (math.inf, 2.0, 1.2):
        got = dp.dp_plan_graph(gpus, layers, limit)
        olayers = [dict(l, sync=[0.0] * G, comm=l["comm"] or [[0.0] * G for _ in range(G)],
                        branches=[dict(b, sync=[[0.0] * G for _ in b["comp"]]) for b in l["branches"]]) for l in layers]
        compare(got, orc.plan_graph(gpus, olayers, limit), gpus, layers)
        assert got["time"] <= sum(l["comp"][0] + sum(r[0] for b in l["branches"] for r in b["comp"]) for l in layers)


def test_bad_input_is_refused(dp):
    gpus = [1, 2]
    ok = {"comp": [1.0, 0.6], "sync": None, "comm": None, "branches": []}
    br = {"comp": [[1.0, 0.5]], "comm": None, "sync": None, "join": None, "move": None}
    with pytest.raises(dp.DpError) as e:      # a block needs a branching layer before it
        dp.dp_plan_graph(gpus, [dict(ok, branches=[br]), ok])
    assert e.value.status == dp.DP_ERR_BAD_DESC
    with pytest.raises(dp.DpError):           # negative move cost
        dp.dp_plan_graph(gpus, [ok, dict(ok, branches=[dict(br, move=[[0.0, -1.0], [0.0, 0.0]])])])
    with pytest.raises(dp.DpError):           # non-positive compute time
        dp.dp_plan_graph(gpus, [ok, dict(ok, branches=[dict(br, comp=[[0.0, 0.5]])])])
    r = dp.dp_plan_graph(gpus, [ok, dict(ok, branches=[br])])          # no move table: never moved, and a single branch is critical
    assert r["blocks"][1] == {"critical": 0, "parallel": [False], "gpus": [[2]]} and r["time"] == 0.6 + 0.5 + 0.6
