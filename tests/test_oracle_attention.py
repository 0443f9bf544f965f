"""Pins for oracle/attention.py (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import mask as om
from paper_2503_11367_amd import workloads as wl


def setup(lay, Hq, Hkv, D, seed, rows=None):
    rng = np.random.default_rng(seed)
    f = om.token_fields(lay.S, lay.spans, lay.sample_off, lay.noncausal, lay.deny, lay.nobidir)
    rows = np.arange(lay.S) if rows is None else rows
    Q = rng.standard_normal((len(rows), Hq, D))
    K = rng.standard_normal((lay.S, Hkv, D))
    V = rng.standard_normal((lay.S, Hkv, D))
    dO = rng.standard_normal((len(rows), Hq, D))
    return f, rows, Q, K, V, dO


def sdpa(Q, K, V, causal):
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]
    k = torch.from_numpy(K).permute(1, 0, 2)[None]
    v = torch.from_numpy(V).permute(1, 0, 2)[None]
    rep = q.shape[1] // k.shape[1]
    k = k.repeat_interleave(rep, dim=1)
    v = v.repeat_interleave(rep, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=causal)
    return o[0].permute(1, 0, 2).numpy()


def test_all_text_equals_causal_sdpa():
    lay = wl.Layout(96, [], [0, 96])
    f, rows, Q, K, V, _ = setup(lay, 4, 2, 16, 0)
    O, _ = oa.forward(Q, K, V, rows, f[0], f[1], f[2], chunk=40)
    assert np.allclose(O, sdpa(Q, K, V, True), atol=1e-12)


def test_shared_question_equals_causal_sdpa_per_answer():
    """Rows of answer a (and of the question) equal plain causal attention over
    the concatenation [question, answer a]."""
    nq, answers = 11, [7, 13, 5]
    lay = wl.layout_shared_question(nq, answers)
    f, rows, Q, K, V, _ = setup(lay, 4, 2, 16, 3)
    O, _ = oa.forward(Q, K, V, rows, f[0], f[1], f[2], modality=f[3], attend=f[4], chunk=16)
    pos = nq
    for n in answers:
        sel = np.r_[0:nq, pos:pos + n]
        ref = sdpa(Q[sel], K[sel], V[sel], True)
        assert np.allclose(O[sel], ref, atol=1e-12)
        pos += n


def test_lambda_equals_sdpa_with_the_band_mask():
    """Sinks plus sliding window: the library routine with the boolean mask
    written from the pattern's description (no mask predicate involved)."""
    L, n_sink, W = 90, 3, 12
    lay = wl.layout_lambda([L], n_sink, W)
    f, rows, Q, K, V, _ = setup(lay, 4, 2, 16, 5)
    win = om.token_windows(lay.S, lay.spans, lay.window)
    O, _ = oa.forward(Q, K, V, rows, f[0], f[1], f[2], modality=f[3], attend=f[4], window=win, chunk=32)
    pos = np.arange(L)
    band = (pos[None, :] <= pos[:, None]) & ((pos[None, :] < n_sink) | (pos[:, None] - pos[None, :] < W))
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]
    k = torch.from_numpy(K).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    v = torch.from_numpy(V).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=torch.from_numpy(band))
    assert np.allclose(O, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_single_span_equals_full_sdpa():
    lay = wl.Layout(64, [(0, 64, wl.IMAGE)], [0, 64])
    f, rows, Q, K, V, _ = setup(lay, 2, 2, 8, 1)
    O, _ = oa.forward(Q, K, V, rows, f[0], f[1], f[2])
    assert np.allclose(O, sdpa(Q, K, V, False), atol=1e-12)


def test_packed_equals_separate():
    lay = wl.Layout(90, [(40, 20, wl.IMAGE)], [0, 30, 90])
    f, rows, Q, K, V, _ = setup(lay, 2, 1, 8, 2)
    O, LSE = oa.forward(Q, K, V, rows, f[0], f[1], f[2])
    layA = wl.Layout(30, [], [0, 30])
    layB = wl.Layout(60, [(10, 20, wl.IMAGE)], [0, 60])
    fA = om.token_fields(30, layA.spans, layA.sample_off)
    fB = om.token_fields(60, layB.spans, layB.sample_off)
    OA, LA = oa.forward(Q[:30], K[:30], V[:30], np.arange(30), fA[0], fA[1], fA[2])
    OB, LB = oa.forward(Q[30:], K[30:], V[30:], np.arange(60), fB[0], fB[1], fB[2])
    assert np.allclose(O, np.concatenate([OA, OB]), atol=1e-12)
    assert np.allclose(LSE, np.concatenate([LA, LB], axis=1), atol=1e-12)


def test_probabilities_sum_to_one_and_lse():
    lay = wl.layout_random(3, 128, n_samples=2)
    f, rows, Q, K, V, _ = setup(lay, 1, 1, 8, 3)
    vis = om.visible(rows, np.arange(lay.S), f[0], f[1], f[2])
    P, lse = oa.probabilities(Q[:, 0], K[:, 0], vis, 0.3)
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-13)
    assert (P[~vis] == 0).all()
    s = 0.3 * Q[:, 0] @ K[:, 0].T
    ref = np.array([np.log(np.exp(s[i][vis[i]]).sum()) for i in range(lay.S)])
    assert np.allclose(lse, ref, atol=1e-12)


def test_constant_v_and_zero_q_read_back_the_mask():
    lay = wl.layout_random(5, 96, n_samples=2, noncausal_prob=0.5)
    f, rows, Q, K, V, _ = setup(lay, 2, 1, 8, 4)
    Vc = np.full_like(V, 0.75)
    O, _ = oa.forward(Q, K, Vc, rows, f[0], f[1], f[2])
    assert np.allclose(O, 0.75, atol=1e-13)
    # Q = 0: uniform probabilities over the visible set; with V = identity
    # columns O[i] is the indicator of the visible set divided by its size.
    S = lay.S
    Vi = np.eye(S)[:, None, :]
    O, LSE = oa.forward(np.zeros((S, 2, S)), np.zeros((S, 1, S)), Vi, rows, f[0], f[1], f[2])
    vis = om.visible(rows, np.arange(S), f[0], f[1], f[2])
    assert np.allclose(O[:, 0], vis / vis.sum(axis=1, keepdims=True), atol=1e-13)
    assert np.allclose(LSE[1], np.log(vis.sum(axis=1)), atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv():
    lay = wl.layout_random(6, 64)
    f, rows, Q, K, V, dO = setup(lay, 4, 2, 8, 5)
    O1, _ = oa.forward(Q, K, V, rows, f[0], f[1], f[2])
    Kr, Vr = np.repeat(K, 2, axis=1), np.repeat(V, 2, axis=1)
    O2, _ = oa.forward(Q, Kr, Vr, rows, f[0], f[1], f[2])
    assert np.allclose(O1, O2, atol=1e-13)
    dQ1, dK1, dV1 = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2])
    dQ2, dK2, dV2 = oa.backward(Q, Kr, Vr, dO, rows, f[0], f[1], f[2])
    assert np.allclose(dQ1, dQ2, atol=1e-12)
    assert np.allclose(dK1, dK2.reshape(64, 2, 2, 8).sum(axis=2), atol=1e-12)
    assert np.allclose(dV1, dV2.reshape(64, 2, 2, 8).sum(axis=2), atol=1e-12)


def test_rank_shares_union_to_full():
    lay = wl.layout_random(8, 128, n_samples=2)
    f, rows, Q, K, V, dO = setup(lay, 2, 1, 8, 6)
    O, LSE = oa.forward(Q, K, V, rows, f[0], f[1], f[2])
    dQ, dK, dV = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2])
    shares = [[0, 5, 6], [1, 2], [3, 4, 7]]           # blocks of 16 tokens
    dKs, dVs = np.zeros_like(dK), np.zeros_like(dV)
    for blocks in shares:
        r = oa.rows_of_blocks(blocks, 16)
        assert r.tolist() == [b * 16 + i for b in blocks for i in range(16)]
        o, l = oa.forward(Q[r], K, V, r, f[0], f[1], f[2])
        assert np.allclose(o, O[r], atol=1e-13) and np.allclose(l, LSE[:, r], atol=1e-13)
        dq, dk, dv = oa.backward(Q[r], K, V, dO[r], r, f[0], f[1], f[2])
        assert np.allclose(dq, dQ[r], atol=1e-12)
        dKs += dk
        dVs += dv
    assert np.allclose(dKs, dK, atol=1e-12) and np.allclose(dVs, dV, atol=1e-12)


def test_backward_matches_finite_differences():
    lay = wl.layout_random(9, 48, n_samples=2, noncausal_prob=0.5)
    blocks = [0, 2]
    rows = oa.rows_of_blocks(blocks, 16)
    f, rows, Q, K, V, dO = setup(lay, 4, 2, 8, 7, rows=rows)
    dQ, dK, dV = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2])

    def loss(Q_, K_, V_):
        O, _ = oa.forward(Q_, K_, V_, rows, f[0], f[1], f[2])
        return float((O * dO).sum())

    rng = np.random.default_rng(0)
    eps = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, n)) for n in X.shape)
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - G[idx]) < 1e-6 * max(1.0, abs(fd)), (name, idx, fd, G[idx])


def test_backward_causal_matches_autograd():
    lay = wl.Layout(40, [], [0, 40])
    f, rows, Q, K, V, dO = setup(lay, 4, 2, 8, 8)
    dQ, dK, dV = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2])
    q = torch.from_numpy(Q).requires_grad_()
    k = torch.from_numpy(K).requires_grad_()
    v = torch.from_numpy(V).requires_grad_()
    kk = k.repeat_interleave(2, dim=1)
    vv = v.repeat_interleave(2, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(
        q.permute(1, 0, 2)[None], kk.permute(1, 0, 2)[None], vv.permute(1, 0, 2)[None], is_causal=True)
    (o[0].permute(1, 0, 2) * torch.from_numpy(dO)).sum().backward()
    assert np.allclose(dQ, q.grad.numpy(), atol=1e-12)
    assert np.allclose(dK, k.grad.numpy(), atol=1e-12)
    assert np.allclose(dV, v.grad.numpy(), atol=1e-12)


def test_dv_column_sums_property():
    """Rows of P sum to one, so sum_k dV[k,g] = sum over the group's heads and
    rows of dO -- a size-independent identity used at full scale on the GPU."""
    lay = wl.layout_random(12, 80)
    f, rows, Q, K, V, dO = setup(lay, 4, 2, 8, 9)
    dQ, dK, dV = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2])
    assert np.allclose(dV.sum(axis=0), dO.reshape(80, 2, 2, 8).sum(axis=(0, 2)), atol=1e-12)


def test_ds_rows_sum_to_zero():
    """sum_k dS_ik = sum_k P_ik dP_ik - Delta_i = 0 for every row, whatever the mask.
    Seen from outside: sum_k dK[k,g] = scale sum_i (sum_k dS_ik) Q_i = 0, and when all
    keys of a head are the same vector dQ = scale (sum_k dS_ik) K = 0."""
    lay = wl.layout_random(13, 96, n_samples=2, noncausal_prob=0.3)
    f, rows, Q, K, V, dO = setup(lay, 4, 2, 8, 10, rows=oa.rows_of_blocks([1, 4, 5], 16))
    dQ, dK, dV = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2])
    assert np.abs(dK).max() > 1e-2
    assert np.allclose(dK.sum(axis=0), 0.0, atol=1e-12)
    K_same = np.broadcast_to(K[:1], K.shape).copy()
    dQ2, dK2, _ = oa.backward(Q, K_same, V, dO, rows, f[0], f[1], f[2])
    assert np.allclose(dQ2, 0.0, atol=1e-12) and np.abs(dK2).max() > 1e-3
