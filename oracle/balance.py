"""Inter-GPU workload balancer (paper section 3.2.1, Alg. 1 and the
"weighted makespan minimization" paragraph): greedy Longest-Processing-Time-
First assignment of token blocks to G ranks, plus the exhaustive optimum of
the ILP for tiny inputs and two baseline splits.

Readings fixed here (the listing iterates blocks in index order, the text
says LPT and charges T log T to sorting in descending order; the heap is
pushed rank-first; ties are not discussed):
  * blocks are visited in order of (W descending, block index ascending);
  * the receiving rank is the one with (load ascending, rank id ascending);
  * each rank's block list is reported in ascending block index.

Pins: tests/test_oracle_balance.py -- the section-3.2.1 example vector
1,2,2,4,5,2,2,8 (tests/golden/paper_example_workloads.txt), the Graham bound
sum/G + t_max quoted in the same section, exhaustive optimum on tiny inputs
with LPT <= (4/3 - 1/(3G)) OPT, round-robin for equal workloads, conservation
of the total.
"""
import itertools

import numpy as np


def lpt(W, P):
    """Returns (rank_of_block[nB] int32, load[P] uint64, rank_off[P+1] int32,
    rank_blocks[nB] int32)."""
    W = [int(w) for w in W]
    nB = len(W)
    order = sorted(range(nB), key=lambda b: (-W[b], b))
    load = [0] * P
    rank_of_block = [0] * nB
    for b in order:
        g = min(range(P), key=lambda r: (load[r], r))
        rank_of_block[b] = g
        load[g] += W[b]
    rank_off = [0] * (P + 1)
    rank_blocks = []
    for g in range(P):
        mine = [b for b in range(nB) if rank_of_block[b] == g]
        rank_blocks += mine
        rank_off[g + 1] = len(rank_blocks)
    return (np.array(rank_of_block, dtype=np.int32), np.array(load, dtype=np.uint64),
            np.array(rank_off, dtype=np.int32), np.array(rank_blocks, dtype=np.int32))


def in_order_greedy(W, P):
    """Alg. 1 exactly as listed: no sort, blocks in index order."""
    load = [0] * P
    rank_of_block = []
    for w in W:
        g = min(range(P), key=lambda r: (load[r], r))
        rank_of_block.append(g)
        load[g] += int(w)
    return np.array(rank_of_block, dtype=np.int32), np.array(load, dtype=np.uint64)


def optimum_makespan(W, P):
    """Exhaustive minimum of the ILP objective C (max per-rank workload)."""
    W = [int(w) for w in W]
    best = sum(W)
    for assign in itertools.product(range(P), repeat=len(W)):
        load = [0] * P
        for w, g in zip(W, assign):
            load[g] += w
        best = min(best, max(load))
    return best


def zigzag(W, P):
    """Causal-LLM baseline split (section 2.2): 2P equal chunks, rank i takes
    chunk i and chunk 2P-1-i.  Requires len(W) % 2P == 0."""
    nB = len(W)
    assert nB % (2 * P) == 0
    c = nB // (2 * P)
    rank_of_block = np.zeros(nB, dtype=np.int32)
    for ch in range(2 * P):
        rank_of_block[ch * c:(ch + 1) * c] = ch if ch < P else 2 * P - 1 - ch
    load = np.zeros(P, dtype=np.uint64)
    for b in range(nB):
        load[rank_of_block[b]] += np.uint64(int(W[b]))
    return rank_of_block, load


def contiguous(W, P):
    nB = len(W)
    assert nB % P == 0
    rank_of_block = (np.arange(nB) // (nB // P)).astype(np.int32)
    load = np.zeros(P, dtype=np.uint64)
    for b in range(nB):
        load[rank_of_block[b]] += np.uint64(int(W[b]))
    return rank_of_block, load


def imbalance(load):
    """max / mean of the per-rank loads."""
    load = np.asarray(load, dtype=np.float64)
    return float(load.max() * load.size / load.sum())
