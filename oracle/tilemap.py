"""Tile map and per-block workloads (paper section 3.2.1: a block is skipped
when its mask block is all zeros; per-block workload counted row-wise).

  cnt[i,j] = #{(q,k) : q in q-tile i, k in k-tile j, vis(q,k)}
  cls[i,j] = EMPTY if cnt=0, FULL if cnt = tq*tk, else PARTIAL
  W[i]     = sum_j cnt[i,j]            (unmasked pairs of q-tile i)

The workload unit is unmasked (query,key) pairs (the ILP's W_i = row-wise sum
of the unmasked mask entries); Alg. 1's coarser "number of blocks to compute"
is `tile_count_workload`.

`tile_map` is the literal definition in NumPy, one strip of q rows at a time.
`tile_map_c` is the same double loop in plain C (oracle/tilemap_ref.c) for
the 128k-token case; tests pin it to `tile_map` and both to closed forms.

Pins: tests/test_oracle_mask.py -- hand-derived
values for the 512-token text/image/text layout (tests/golden/tiny_tilemap.txt),
lower-triangular FULL/PARTIAL/EMPTY pattern for all-text, closed-form totals.
"""
import ctypes
import os

import numpy as np

from .mask import visible

EMPTY, FULL, PARTIAL = 0, 1, 2


def tile_map(sample, span, causal, tq, tk, modality=None, attend=None, window=None):
    S = sample.shape[0]
    assert S % tq == 0 and S % tk == 0
    nq, nk = S // tq, S // tk
    cnt = np.zeros((nq, nk), dtype=np.uint32)
    k_idx = np.arange(S)
    for i in range(nq):
        q_idx = np.arange(i * tq, (i + 1) * tq)
        vis = visible(q_idx, k_idx, sample, span, causal, modality, attend, window)          # [tq, S]
        cnt[i] = vis.reshape(tq, nk, tk).sum(axis=(0, 2))
    cls = np.full((nq, nk), PARTIAL, dtype=np.uint8)
    cls[cnt == 0] = EMPTY
    cls[cnt == tq * tk] = FULL
    W = cnt.astype(np.uint64).sum(axis=1, dtype=np.uint64)
    return cls, cnt, W


def tile_count_workload(cls):
    """Alg. 1's literal workload: number of non-empty k-tiles per q-tile."""
    return (cls != EMPTY).sum(axis=1).astype(np.uint64)


_lib = None


def _load_c():
    global _lib
    if _lib is None:
        here = os.path.dirname(os.path.abspath(__file__))
        path = os.path.join(here, "libtilemap_ref.so")
        if not os.path.exists(path):
            raise RuntimeError("oracle/libtilemap_ref.so not built; run __graft_entry__.build()")
        _lib = ctypes.CDLL(path)
        _lib.tilemap_ref.restype = ctypes.c_int
        _lib.tilemap_ref.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int64, ctypes.c_int32,
                                                              ctypes.c_int32] + [ctypes.c_void_p] * 3
    return _lib


def tile_map_c(sample, span, causal, tq, tk, modality=None, attend=None, window=None):
    """Same result as tile_map, computed by the plain-C double loop."""
    lib = _load_c()
    S = sample.shape[0]
    assert S % tq == 0 and S % tk == 0
    nq, nk = S // tq, S // tk
    sa = np.ascontiguousarray(sample, dtype=np.int64)
    sp = np.ascontiguousarray(span, dtype=np.int64)
    ca = np.ascontiguousarray(causal, dtype=np.int64)
    mo = np.ascontiguousarray(np.zeros(S) if modality is None else modality, dtype=np.int64)
    at = np.ascontiguousarray(np.full(S, 0xFF) if attend is None else attend, dtype=np.int64)
    wi = np.ascontiguousarray(np.zeros(S) if window is None else window, dtype=np.int64)
    cls = np.zeros((nq, nk), dtype=np.uint8)
    cnt = np.zeros((nq, nk), dtype=np.uint32)
    W = np.zeros(nq, dtype=np.uint64)
    rc = lib.tilemap_ref(sa.ctypes.data, sp.ctypes.data, ca.ctypes.data, mo.ctypes.data, at.ctypes.data,
                         wi.ctypes.data, S, tq, tk,
                         cls.ctypes.data, cnt.ctypes.data, W.ctypes.data)
    assert rc == 0
    return cls, cnt, W
