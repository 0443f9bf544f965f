"""Pins for oracle/balance.py (CPU only)."""
import os

import numpy as np
import pytest

from oracle import balance as ob
from oracle import mask as om
from oracle import tilemap as ot
from paper_2503_11367_amd import workloads as wl


def paper_vector(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_example_workloads.txt")):
        if not line.startswith("#"):
            return [int(x) for x in line.split()]


def test_paper_example(golden_dir):
    """Section 3.2.1 example workloads 1,2,2,4,5,2,2,8 with G=4, traced by
    hand.  Visit order: b7(8) b4(5) b3(4) b1 b2 b5 b6 (2 each) b0(1)."""
    W = paper_vector(golden_dir)
    assert W == [1, 2, 2, 4, 5, 2, 2, 8] and sum(W) == 26
    rob, load, off, blocks = ob.lpt(W, 4)
    # b7->r0 (8); b4->r1 (5); b3->r2 (4); b1->r3 (2); b2->r3 (4, r3 was least);
    # b5: loads (8,5,4,4), tie r2/r3 -> lower id r2 (6); b6->r3 (6); b0->r1 (6).
    assert rob.tolist() == [1, 3, 3, 2, 1, 2, 3, 0]
    assert load.tolist() == [8, 6, 6, 6]
    assert int(load.max()) == ob.optimum_makespan(W, 4) == 8   # max item bounds OPT
    assert off.tolist() == [0, 1, 3, 5, 8]
    assert blocks.tolist() == [7, 0, 4, 3, 5, 1, 2, 6]
    # The listing as printed (no sort) co-locates b0 and b4 on rank 0, which is
    # what the section-3.2.2 narrative ("b1 and b5 assigned to GPU0", 1-based)
    # says.
    rob2, load2 = ob.in_order_greedy(W, 4)
    assert rob2[0] == 0 and rob2[4] == 0
    assert load2.tolist() == [6, 12, 4, 4]


def test_tiny_config_by_hand():
    """512-token layout, W from tests/golden/tiny_tilemap.txt, G=4, traced by
    hand.  Visit order b7,b6,b5,b1,b2,b3,b4,b0: b7->r0 (30752), b6->r1 (26656),
    b5->r2 (22560), b1->r3 (20480), b2->r3 (40960), b3->r2 (43040),
    b4->r1 (47136), b0->r0 (32832)."""
    W = [2080, 20480, 20480, 20480, 20480, 22560, 26656, 30752]
    rob, load, off, blocks = ob.lpt(W, 4)
    assert rob.tolist() == [0, 3, 3, 2, 1, 2, 1, 0]
    assert load.tolist() == [32832, 47136, 43040, 40960]
    assert abs(ob.imbalance(load) - 47136 / 40992) < 1e-12
    assert int(load.max()) == ob.optimum_makespan(W, 4)


@pytest.mark.parametrize("seed", range(12))
def test_lpt_vs_exhaustive_optimum(seed):
    rng = np.random.default_rng(seed)
    nB, P = int(rng.integers(3, 10)), int(rng.integers(2, 4))
    W = rng.integers(0, 50, size=nB).tolist()
    rob, load, off, blocks = ob.lpt(W, P)
    opt = ob.optimum_makespan(W, P)
    assert opt <= int(load.max())
    assert 3 * P * int(load.max()) <= (4 * P - 1) * opt      # LPT <= (4/3 - 1/(3P)) OPT
    assert int(load.sum()) == sum(W)


@pytest.mark.parametrize("seed", range(8))
def test_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    nB, P = int(rng.integers(1, 300)), int(rng.integers(1, 17))
    W = rng.integers(0, 2 ** 40, size=nB).tolist()
    rob, load, off, blocks = ob.lpt(W, P)
    assert int(load.sum()) == sum(W)
    # the bound quoted in section 3.2.1: sum t_i / G + t_max
    assert int(load.max()) * P <= sum(W) + P * max(W)
    assert int(load.max()) - int(load.min()) <= max(W)
    for g in range(P):
        mine = blocks[off[g]:off[g + 1]].tolist()
        assert mine == sorted(mine) and all(rob[b] == g for b in mine)
        assert sum(W[b] for b in mine) == int(load[g])
    assert sorted(blocks.tolist()) == list(range(nB))


def test_equal_weights_round_robin_and_p1():
    rob, load, _, _ = ob.lpt([5] * 12, 4)
    assert rob.tolist() == [0, 1, 2, 3] * 3 and load.tolist() == [15] * 4
    rob, load, off, blocks = ob.lpt([3, 1, 2], 1)
    assert rob.tolist() == [0, 0, 0] and load.tolist() == [6] and blocks.tolist() == [0, 1, 2]


def test_causal_zigzag_balanced_and_lpt_converges():
    """Section 2.2: for a causal mask the 2G-chunk zigzag split is balanced
    (up to the diagonal); section 3.2.1: LPT approaches perfect balance as the
    number of blocks grows."""
    lay = wl.Layout(4096, [], [0, 4096])
    sample, span, causal = om.token_fields(lay.S, lay.spans, lay.sample_off)[:3]
    _, _, W = ot.tile_map_c(sample, span, causal, 64, 64)
    _, zl = ob.zigzag(W, 4)
    assert ob.imbalance(zl) < 1.001
    _, cl = ob.contiguous(W, 4)
    assert ob.imbalance(cl) > 1.7
    _, ll, _, _ = ob.lpt(W, 4)
    assert ob.imbalance(ll) < 1.01
