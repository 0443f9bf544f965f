"""Masked-softmax attention forward and backward in float64 for one rank's
query rows against the full key/value sequence, with grouped-query heads.

The paper defers to the standard attention definition (section 3.2.2 cites
the online-softmax / FlashAttention line of kernels and section 4.3 states
"row-wise attention for local queries" over all gathered keys and values);
what those kernels compute is, for Q head h, KV head g = h // (Hq/Hkv),
local row i at global position q_i, scale = 1/sqrt(D):

  s_ik  = scale * <Q[i,h], K[k,g]>          for vis(q_i,k), else excluded
  LSE_i = log sum_k exp(s_ik)
  P_ik  = exp(s_ik - LSE_i)                 (0 where masked)
  O[i,h] = sum_k P_ik V[k,g]

  dV[k,g] = sum_{h in g} sum_i P_ik dO[i,h]
  dP_ik   = <dO[i,h], V[k,g]>
  Delta_i = <dO[i,h], O[i,h]>
  dS_ik   = P_ik (dP_ik - Delta_i)
  dQ[i,h] = scale * sum_k dS_ik K[k,g]
  dK[k,g] = scale * sum_{h in g} sum_i dS_ik Q[i,h]

with sums over i running over this rank's rows only.  A row with no visible
key gives O = 0, LSE = -inf and zero gradients.  Rows are independent, so the
code walks them in chunks purely to bound memory; there is no other blocking.

Pins: tests/test_oracle_attention.py -- all-text = causal softmax attention
via torch's CPU scaled_dot_product_attention, one all-covering span = unmasked
attention, packed samples = per-sample attention, probabilities sum to 1,
V constant => O constant, Q = 0 => mean of visible V rows, central finite
differences for dQ/dK/dV, sum_k dS_ik = 0 (seen from outside as sum_k dK[k,g] = 0
and as dQ = 0 when all keys are equal), union over ranks = full result,
torch autograd for the causal special case.
"""
import numpy as np

from .mask import visible


def _rows(blocks, N_B):
    blocks = np.asarray(blocks, dtype=np.int64)
    return (blocks[:, None] * N_B + np.arange(N_B)[None, :]).reshape(-1)


def rows_of_blocks(blocks, N_B):
    """Global token index of each local row: blocks[r // N_B]*N_B + r % N_B."""
    return _rows(blocks, N_B)


def probabilities(Qh, Kg, vis, scale):
    """P [n,S] and LSE [n] for one head and a chunk of rows."""
    s = scale * (Qh @ Kg.T)
    s = np.where(vis, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.where(vis, np.exp(s - m_safe), 0.0)
    l = e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        P = np.where(l > 0, e / l, 0.0)
        lse = np.where(l[:, 0] > 0, m_safe[:, 0] + np.log(l[:, 0]), -np.inf)
    return P, lse


def forward(Q_loc, K, V, rows, sample, span, causal, scale=None, chunk=512, modality=None, attend=None,
            window=None):
    """Q_loc [n,Hq,D], K,V [S,Hkv,D] float64; rows[n] global positions.
    Returns O [n,Hq,D] and LSE [Hq,n]."""
    n, Hq, D = Q_loc.shape
    S, Hkv, _ = K.shape
    rep = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    O = np.zeros((n, Hq, D), dtype=np.float64)
    LSE = np.zeros((Hq, n), dtype=np.float64)
    k_idx = np.arange(S)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        vis = visible(rows[a:b], k_idx, sample, span, causal, modality, attend, window)
        for h in range(Hq):
            g = h // rep
            P, lse = probabilities(Q_loc[a:b, h], K[:, g], vis, scale)
            O[a:b, h] = P @ V[:, g]
            LSE[h, a:b] = lse
    return O, LSE


def backward(Q_loc, K, V, dO, rows, sample, span, causal, scale=None, chunk=512, modality=None,
             attend=None, window=None):
    """Returns dQ [n,Hq,D], dK [S,Hkv,D], dV [S,Hkv,D] (this rank's partial
    sums), all float64."""
    n, Hq, D = Q_loc.shape
    S, Hkv, _ = K.shape
    rep = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    dQ = np.zeros_like(Q_loc, dtype=np.float64)
    dK = np.zeros_like(K, dtype=np.float64)
    dV = np.zeros_like(V, dtype=np.float64)
    k_idx = np.arange(S)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        vis = visible(rows[a:b], k_idx, sample, span, causal, modality, attend, window)
        for h in range(Hq):
            g = h // rep
            P, _ = probabilities(Q_loc[a:b, h], K[:, g], vis, scale)
            O = P @ V[:, g]
            dV[:, g] += P.T @ dO[a:b, h]
            dP = dO[a:b, h] @ V[:, g].T
            delta = (dO[a:b, h] * O).sum(axis=1, keepdims=True)
            dS = P * (dP - delta)
            dQ[a:b, h] = scale * (dS @ K[:, g])
            dK[:, g] += scale * (dS.T @ Q_loc[a:b, h])
    return dQ, dK, dV
