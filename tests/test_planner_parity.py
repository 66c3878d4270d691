"""dp_plan_chain / dp_plan_cost_tables (host-only C ABI) against the planner oracle: the GPU counts are
integers and must agree exactly; both sides add the same fp64 terms in the same order, so the tables agree
bit for bit as well."""
import math

import numpy as np
import pytest

from oracle import burst_plan as orc


# Every test runs twice: unmarked (any host) and marked `gpu`, so that the run on the GPU machine also records the
# planner's parity (the library there is the one the kernels were built into).
@pytest.fixture(scope="module", params=["host", pytest.param("gpu_box", marks=pytest.mark.gpu)])
def dp(request):
    from paper_2112_10065_amd import binding
    return binding


def tables(rng, L, G):
    gpus = sorted(set([1] + [int(v) for v in rng.integers(2, 65, G - 1)]))
    G = len(gpus)
    comp = [[float(rng.uniform(5e-6, 3e-3)) for _ in range(G)] for _ in range(L)]
    comm = [[[0.0 if a == b else float(rng.uniform(0, 4e-4)) for a in range(G)] for b in range(G)] for _ in range(L)]
    sync = [[0.0 if a == 0 else float(rng.uniform(0, 3e-4)) for a in range(G)] for _ in range(L)]
    return gpus, comp, comm, sync


@pytest.mark.parametrize("seed", range(40))
def test_plan_matches_oracle(dp, seed):
    rng = np.random.default_rng(seed)
    L, G = int(rng.integers(1, 40)), int(rng.integers(1, 8))
    gpus, comp, comm, sync = tables(rng, L, G)
    limit = [math.inf, 1.0, 1.1, 1.5, 2.0, 3.0, 0.5][seed % 7]
    want = orc.plan_chain(gpus, comp, comm, sync, limit)
    got = dp.dp_plan_chain(gpus, comp, comm, sync, limit)
    assert got["gpus"] == want["gpus"]
    assert got["time"] == want["time"]
    assert got["S"] == want["S"] and got["T"] == want["T"]


def test_null_tables_mean_zero_cost(dp):
    rng = np.random.default_rng(77)
    gpus, comp, _, _ = tables(rng, 9, 5)
    G = len(gpus)
    zc = [[[0.0] * G for _ in range(G)] for _ in range(9)]
    zs = [[0.0] * G for _ in range(9)]
    assert dp.dp_plan_chain(gpus, comp, None, None, 1.5) == dp.dp_plan_chain(gpus, comp, zc, zs, 1.5)
    assert dp.dp_plan_chain(gpus, comp, None, None, 1.5)["gpus"] == orc.plan_chain(gpus, comp, zc, zs, 1.5)["gpus"]


def test_vgg_shaped_chain(dp):
    """A 16-layer chain with the payload sizes of VGG-16 at global batch 32 and a synthetic time table of the
    measured shape (time falls sub-linearly with the per-GPU batch); costs from the closed-form model."""
    from paper_2112_10065_amd import workloads as W
    gpus = [1, 2, 4, 8, 16, 32]
    convs, fcs = W.vgg16_convs(), W.vgg16_linears()
    act = [32.0 * l.h * l.w * l.c * 2 for l in convs] + [32.0 * f.in_f * 2 for f in fcs]
    par = [4.0 * (l.k * l.r * l.s * l.c + l.k) for l in convs] + [4.0 * (f.in_f * f.out_f + f.out_f) for f in fcs]
    rng = np.random.default_rng(3)
    comp = []
    for i in range(16):
        t1 = float(rng.uniform(2e-4, 6e-4))
        comp.append([max(t1 / g ** 0.8, 4e-5) for g in gpus])
    for bw, delay in ((1.07e12, 1e-5), (5e10, 2e-5)):
        comm_o, sync_o = orc.cost_tables(gpus, act, par, bw, delay)
        comm_d, sync_d = dp.dp_plan_cost_tables(gpus, act, par, bw, delay)
        assert comm_d == comm_o and sync_d == sync_o
        for limit in (math.inf, 1.5, 2.0, 4.0):
            want = orc.plan_chain(gpus, comp, comm_o, sync_o, limit)
            got = dp.dp_plan_chain(gpus, comp, comm_d, sync_d, limit)
            assert got["gpus"] == want["gpus"] and got["time"] == want["time"]


def test_rejects_malformed_input(dp):
    comp = [[1.0, 0.6]]
    for bad in (lambda: dp.dp_plan_chain([2, 4], comp),            # first count must be 1
                lambda: dp.dp_plan_chain([1, 1], comp),            # not ascending
                lambda: dp.dp_plan_chain([1, 2], [[1.0, 0.0]]),    # comp must be positive
                lambda: dp.dp_plan_chain([1, 2], comp, [[[0.0, -1.0], [0.0, 0.0]]]),
                lambda: dp.dp_plan_chain([1, 2], comp, None, None, float("nan")),
                lambda: dp.dp_plan_cost_tables([1, 2], [1.0], [1.0], 0.0, 0.0)):
        with pytest.raises(dp.DpError) as e:
            bad()
        assert e.value.status == dp.DP_ERR_BAD_DESC
