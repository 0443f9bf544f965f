"""The benchmark's imbalance report (LPT on pairs and on tile counts from the
GPU balancer; index-order greedy, zigzag and contiguous splits computed by the
harness) against the oracle's balancers on the oracle's own tile map: per-rank
loads equal as integers, then the max/mean ratios."""
import numpy as np
import pytest

from oracle import balance as ob
from oracle import tilemap as ot
from paper_2503_11367_amd import workloads as wl

from gpu_util import DEV, fields

pytestmark = pytest.mark.gpu


def oracle_loads(w):
    f = fields(w.layout)
    cls, _, W = ot.tile_map_c(f[0], f[1], f[2], w.N_B, w.N_B)
    Wl = [int(x) for x in W]
    P, nB = w.P, len(Wl)
    out = {"lpt": ob.lpt(W, P)[1]}
    Wt = ot.tile_count_workload(cls)
    rob_t = ob.lpt(Wt, P)[0]
    lt = [0] * P
    for b, g in enumerate(rob_t):
        lt[int(g)] += Wl[b]
    out["lpt_tile_count"] = lt
    out["in_order"] = ob.in_order_greedy(W, P)[1]
    if nB % (2 * P) == 0:
        out["zigzag"] = ob.zigzag(W, P)[1]
    if nB % P == 0:
        out["contiguous"] = ob.contiguous(W, P)[1]
    return out, Wt


@pytest.mark.parametrize("c", [1, 3, 4, 5])
def test_report_matches_oracle(c):
    import bench
    w = wl.workload(c)
    rep = bench.imbalance_report(DEV, workloads=(c,), with_loads=True)[w.name]
    ref, Wt = oracle_loads(w)
    assert rep["tile_count_workloads"] == [int(x) for x in Wt]
    assert set(rep["loads"]) == set(ref)
    for name, load in ref.items():
        load = [int(x) for x in load]
        assert rep["loads"][name] == load, name
        assert rep[name] == pytest.approx(ob.imbalance(load), rel=1e-12), name


def test_pinned_values():
    """The tiny workload's hand-derived numbers: LPT loads (32832, 47136, 43040,
    40960), 47136 / 40992 for both LPT and zigzag; and the section 3.2.1 example
    vector 1,2,2,4,5,2,2,8 on four ranks under the index-order greedy of Alg. 1
    as printed: loads (6, 12, 4, 4)."""
    import bench
    rep = bench.imbalance_report(DEV, workloads=(1,), with_loads=True)["tiny"]
    assert rep["loads"]["lpt"] == [32832, 47136, 43040, 40960]
    assert rep["lpt"] == pytest.approx(47136 / 40992, rel=1e-12)
    assert rep["zigzag"] == pytest.approx(47136 / 40992, rel=1e-12)
    assert bench.in_order_greedy_loads([1, 2, 2, 4, 5, 2, 2, 8], 4) == [6, 12, 4, 4]
