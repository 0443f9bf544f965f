"""GPU parity, attention backward (through the C ABI) against the float64
oracle: relative L2 error below 1e-2 on dQ, dK, dV (bf16 in/out, fp32
accumulation).  The GPU backward consumes the GPU forward's O and LSE, as in
training; the oracle recomputes its own forward in float64."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import balance as ob
from oracle import tilemap as ot
from paper_2503_11367_amd import binding as mb
from paper_2503_11367_amd import workloads as wl

from gpu_util import (DEV, bf16_to_f64, f64, fields, gpu_bits, make_tensors, max_abs, rel_l2, windows)

pytestmark = pytest.mark.gpu

TOL = 1e-2


def gpu_fwd_bwd(lay, blocks, block, t):
    bits = gpu_bits(lay)
    bl = torch.tensor(blocks, dtype=torch.int32, device=DEV)
    o, lse = mb.fwd(t["q"], t["k"], t["v"], bits, bl, block)
    dq, dk, dv = mb.bwd(t["q"], t["k"], t["v"], bits, bl, block, o, lse, t["do"])
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


def run_case(lay, blocks, block, Hq, Hkv, D, seed):
    f = fields(lay)
    n_loc = len(blocks) * block
    t = make_tensors(seed, n_loc, lay.S, Hq, Hkv, D)
    o, lse, dq, dk, dv = gpu_fwd_bwd(lay, blocks, block, t)
    rows = oa.rows_of_blocks(blocks, block)
    Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
    dq_ref, dk_ref, dv_ref = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2], modality=f[3], attend=f[4],
                                         window=windows(lay))
    for name, got, ref in (("dq", dq, dq_ref), ("dk", dk, dk_ref), ("dv", dv, dv_ref)):
        g = bf16_to_f64(got)
        assert np.isfinite(g).all(), name
        assert rel_l2(g, ref) < TOL, (name, rel_l2(g, ref))
    # keys that no row of the share sees get exactly zero
    from oracle import mask as om
    seen = om.visible(rows, np.arange(lay.S), f[0], f[1], f[2], f[3], f[4], windows(lay)).any(axis=0)
    assert (bf16_to_f64(dk)[~seen] == 0).all() and (bf16_to_f64(dv)[~seen] == 0).all()


@pytest.mark.parametrize("seed", range(3))
def test_attend_sets(seed):
    lay = wl.layout_random(70 + seed, S=1024, n_samples=1 + seed % 2, max_spans=6, noncausal_prob=0.2,
                           deny_prob=0.8)
    assert any(lay.deny)
    blocks = list(range(lay.S // 64)) if seed != 1 else list(range(1, lay.S // 64, 2))
    run_case(lay, blocks, 64, Hq=2 + 2 * (seed % 2), Hkv=2, D=[128, 64, 128][seed], seed=60 + seed)


def test_lambda_and_windowed_spans():
    """Attention sinks plus a sliding window (section 5.5's lambda pattern) and
    windows on bidirectional image spans."""
    run_case(wl.layout_lambda([2048], 4, 300), list(range(16)), 128, Hq=4, Hkv=2, D=128, seed=94)
    run_case(wl.layout_lambda([700, 324, 1024], 16, 256), [15, 3, 8, 9], 128, Hq=2, Hkv=1, D=64, seed=95)
    lay = wl.layout_random(71, S=1024, n_samples=2, max_spans=6)
    lay.window = [37 * (j + 1) for j in range(len(lay.spans))]
    run_case(lay, list(range(8)), 128, Hq=2, Hkv=1, D=128, seed=97)


def test_long_key_lists_cut_into_slices():
    """Sinks that every later row attends make one k-tile's list of query tiles
    far longer than the others: the key-outer pass cuts long lists into slices
    (separate workgroups, partial sums added in a fixed order).  Here the sink
    tile has 64 entries and is cut into 8 slices, the band tiles into 2."""
    run_case(wl.layout_lambda([4096], 32, 512), list(range(32)), 128, Hq=1, Hkv=1, D=64, seed=98)
    # a share that is not the whole sequence, two heads per group
    run_case(wl.layout_lambda([2048, 2048], 8, 200), list(range(3, 32)), 128, Hq=2, Hkv=1, D=128, seed=99)


def test_lambda_8k_sampled():
    """8192 tokens, 8 / 2 heads, 32 sinks, window 256: dQ of sampled rows, the
    column sums of dV, and dK / dV of one 64-key block inside the band, which
    only the next 64 + 256 rows see (the oracle on exactly those rows)."""
    S, n_sink, W, Hq, Hkv, D = 8192, 32, 256, 8, 2, 128
    lay = wl.layout_lambda([S], n_sink, W)
    f, win = fields(lay), windows(lay)
    blocks = list(range(S // 128))
    t = make_tensors(77, S, S, Hq, Hkv, D)
    _, _, dq, dk, dv = gpu_fwd_bwd(lay, blocks, 128, t)
    Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
    rows = np.arange(S)
    sel = np.sort(np.random.default_rng(2).choice(S, size=24, replace=False))
    for h in (0, 7):
        g = h // (Hq // Hkv)
        dq_ref, _, _ = oa.backward(Q[sel][:, h:h + 1], K[:, g:g + 1], V[:, g:g + 1], dO[sel][:, h:h + 1],
                                   rows[sel], f[0], f[1], f[2], modality=f[3], attend=f[4], window=win)
        assert rel_l2(bf16_to_f64(dq[torch.from_numpy(sel).to(DEV)][:, h:h + 1]), dq_ref) < TOL
    dv_sum = dv.float().sum(dim=0).cpu().numpy().astype(np.float64)
    ref = dO.reshape(S, Hkv, Hq // Hkv, D).sum(axis=(0, 2))
    assert np.abs(dv_sum - ref).max() < 2e-2 * np.abs(ref).max() + 0.5
    k0, g = 5000, 1
    seers = np.arange(k0, k0 + 64 + W)                 # every row that sees a key of the block
    hs = slice(g * (Hq // Hkv), (g + 1) * (Hq // Hkv))
    _, dk_ref, dv_ref = oa.backward(Q[seers][:, hs], K[:, g:g + 1], V[:, g:g + 1], dO[seers][:, hs], seers,
                                    f[0], f[1], f[2], modality=f[3], attend=f[4], window=win)
    blk = slice(k0, k0 + 64)
    assert rel_l2(bf16_to_f64(dk[blk, g:g + 1]), dk_ref[blk]) < TOL
    assert rel_l2(bf16_to_f64(dv[blk, g:g + 1]), dv_ref[blk]) < TOL


def test_many_short_spans():
    """Nearly every key (and row) starts a new run of mask fields."""
    run_case(wl.layout_short_spans(18), list(range(8)), 128, Hq=2, Hkv=1, D=128, seed=93)


def test_shared_question_and_block_causal():
    """Two patterns named in section 5.5: answers that see the question and
    themselves only (spans without the bidirectional term), and blocks that are
    bidirectional inside and causal across (block length not a tile multiple)."""
    run_case(wl.layout_shared_question(200, [130, 64, 257, 100], n_tail=145), list(range(7)), 128,
             Hq=4, Hkv=2, D=128, seed=81)
    run_case(wl.layout_shared_question(64, [128] * 7, n_tail=64), [7, 2, 12, 5], 64, Hq=2, Hkv=1, D=64, seed=82)
    run_case(wl.layout_block_causal(1024, 96), list(range(8)), 128, Hq=2, Hkv=2, D=128, seed=83)


def test_tiny_every_rank_share():
    w = wl.workload(1)
    f = fields(w.layout)
    _, _, W = ot.tile_map(f[0], f[1], f[2], w.N_B, w.N_B)
    _, _, off, rb = ob.lpt(W, w.P)
    for g in range(w.P):
        run_case(w.layout, rb[off[g]:off[g + 1]].tolist(), w.N_B, w.Hq, w.Hkv, w.D, seed=11 + g)
    run_case(w.layout, list(range(8)), w.N_B, w.Hq, w.Hkv, w.D, seed=10)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("seed", range(4))
def test_random_layouts(seed, D):
    lay = wl.layout_random(40 + seed, S=1024, n_samples=1 + seed % 3, noncausal_prob=0.25 * (seed % 2))
    block = [16, 32, 64, 128][seed % 4]
    rng = np.random.default_rng(seed)
    nb = lay.S // block
    take = int(rng.integers(1, nb + 1))
    blocks = np.sort(rng.choice(nb, size=take, replace=False)).tolist()
    run_case(lay, blocks, block, Hq=4, Hkv=2, D=D, seed=20 + seed)


@pytest.mark.parametrize("block", [48, 80, 240])
def test_block_size_not_a_power_of_two(block):
    """Blocks of 48, 80 and 240 tokens (multiples of 16 that divide S = 1920): the
    64-row steps of the key-outer pass and the 128-row q-tiles of the dQ pass straddle
    the blocks of the share."""
    lay = wl.layout_random(130 + block, S=1920, n_samples=2, max_spans=5)
    nb = lay.S // block
    rng = np.random.default_rng(block)
    blocks = rng.permutation(nb)[: max(3, nb // 2)].tolist()
    run_case(lay, blocks, block, Hq=4, Hkv=2, D=128, seed=150 + block)
    run_case(lay, sorted(blocks)[:3], block, Hq=2, Hkv=2, D=64, seed=151 + block)


def test_special_masks():
    run_case(wl.Layout(512, [], [0, 512]), list(range(4)), 128, 2, 1, 128, seed=41)
    run_case(wl.Layout(512, [(0, 512, 1)], [0, 512]), list(range(4)), 128, 2, 1, 128, seed=42)
    run_case(wl.Layout(768, [(300, 100, 2)], [0, 200, 768]), [4, 1, 5], 128, 2, 2, 64, seed=43)


def test_empty_share():
    """A rank that received no block (more ranks than blocks): forward does
    nothing, backward overwrites its partial dK, dV with zeros."""
    lay = wl.Layout(512, [(100, 200, 1)], [0, 512])
    t = make_tensors(5, 0, lay.S, 4, 2, 128)
    bits = gpu_bits(lay)
    bl = torch.zeros(0, dtype=torch.int32, device=DEV)
    o, lse = mb.fwd(t["q"], t["k"], t["v"], bits, bl, 64)
    assert o.shape == (0, 4, 128) and lse.shape == (4, 0)
    dk = torch.full_like(t["k"], 3.0)
    dv = torch.full_like(t["v"], -2.0)
    dq = torch.empty_like(t["q"])
    mb.bwd(t["q"], t["k"], t["v"], bits, bl, 64, o, lse, t["do"], out=(dq, dk, dv))
    torch.cuda.synchronize()
    assert (dk == 0).all() and (dv == 0).all()


def test_rank_partials_sum_to_full():
    """Summing the ranks' partial dK/dV reproduces the single-rank result."""
    w = wl.workload(1)
    lay = w.layout
    f = fields(lay)
    t = make_tensors(77, lay.S, lay.S, 2, 1, 64)
    _, _, dq_full, dk_full, dv_full = gpu_fwd_bwd(lay, list(range(8)), 64, t)
    _, _, W = ot.tile_map(f[0], f[1], f[2], 64, 64)
    _, _, off, rb = ob.lpt(W, 4)
    dk_sum = np.zeros((lay.S, 1, 64))
    dv_sum = np.zeros((lay.S, 1, 64))
    for g in range(4):
        blocks = rb[off[g]:off[g + 1]].tolist()
        rows = oa.rows_of_blocks(blocks, 64)
        tt = dict(t)
        tt["q"] = t["q"][torch.from_numpy(rows).to(DEV)].contiguous()
        tt["do"] = t["do"][torch.from_numpy(rows).to(DEV)].contiguous()
        _, _, dq, dk, dv = gpu_fwd_bwd(lay, blocks, 64, tt)
        assert rel_l2(bf16_to_f64(dq), bf16_to_f64(dq_full)[rows]) < 2e-3
        dk_sum += bf16_to_f64(dk)
        dv_sum += bf16_to_f64(dv)
    assert rel_l2(dk_sum, bf16_to_f64(dk_full)) < 1e-2
    assert rel_l2(dv_sum, bf16_to_f64(dv_full)) < 1e-2


def group_check(w, blocks, t, outs, g, sel_rows=None):
    """Oracle backward for the Q heads of KV group g on the whole share."""
    f = fields(w.layout)
    rep = w.Hq // w.Hkv
    hs = slice(g * rep, (g + 1) * rep)
    rows = oa.rows_of_blocks(blocks, w.N_B)
    Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
    dq_ref, dk_ref, dv_ref = oa.backward(Q[:, hs], K[:, g:g + 1], V[:, g:g + 1], dO[:, hs], rows,
                                         f[0], f[1], f[2])
    _, _, dq, dk, dv = outs
    assert rel_l2(bf16_to_f64(dq[:, hs]), dq_ref) < TOL
    assert rel_l2(bf16_to_f64(dk[:, g:g + 1]), dk_ref) < TOL
    assert rel_l2(bf16_to_f64(dv[:, g:g + 1]), dv_ref) < TOL


def sampled_dq_and_dv_sums(w, blocks, t, outs, n_rows=24, heads=(0, 5)):
    """Size-independent checks: dQ of sampled rows (each row needs only its own
    softmax), and sum_k dV[k,g] = sum over the group's heads and rows of dO."""
    f = fields(w.layout)
    rep = w.Hq // w.Hkv
    n_loc = len(blocks) * w.N_B
    rows = oa.rows_of_blocks(blocks, w.N_B)
    _, _, dq, dk, dv = outs
    Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
    sel = np.sort(np.random.default_rng(1).choice(n_loc, size=n_rows, replace=False))
    for h in heads:
        g = h // rep
        dq_ref, _, _ = oa.backward(Q[sel][:, h:h + 1], K[:, g:g + 1], V[:, g:g + 1],
                                   dO[sel][:, h:h + 1], rows[sel], f[0], f[1], f[2])
        assert rel_l2(bf16_to_f64(dq[torch.from_numpy(sel).to(DEV)][:, h:h + 1]), dq_ref) < TOL
    dv_sum = dv.float().sum(dim=0).cpu().numpy().astype(np.float64)
    ref = dO.reshape(n_loc, w.Hkv, rep, w.D).sum(axis=(0, 2))
    assert np.abs(dv_sum - ref).max() < 2e-2 * np.abs(ref).max() + 0.5


def test_workload2_full_sequence():
    w = wl.workload(2)
    blocks = list(range(w.layout.S // w.N_B))
    t = make_tensors(w.tensor_seed, w.layout.S, w.layout.S, w.Hq, w.Hkv, w.D)
    outs = gpu_fwd_bwd(w.layout, blocks, w.N_B, t)
    group_check(w, blocks, t, outs, g=5)
    sampled_dq_and_dv_sums(w, blocks, t, outs, heads=(0, 13, 31))


def test_large_share_keeps_its_own_preparation():
    """Shares whose head-major copies of Q and dO exceed 128 MiB (here 8192 rows x 48 heads x
    128: 192 MiB) take the backward's other launch order: the inputs of the key-outer pass
    come from a preparation of their own and the query-outer pass runs last.  Whole KV
    group against the oracle, element by element (also the only full-size case with six
    query heads per KV head)."""
    w2 = wl.workload(2)
    w = wl.Workload("vlm_8k_48_heads", w2.layout, 48, 8, 128, w2.N_B, 1, 2102)
    blocks = list(range(w.layout.S // w.N_B))
    t = make_tensors(w.tensor_seed, w.layout.S, w.layout.S, w.Hq, w.Hkv, w.D)
    outs = gpu_fwd_bwd(w.layout, blocks, w.N_B, t)
    group_check(w, blocks, t, outs, g=2)


def key_range_check(w, blocks, t, outs, g, k_lo, k_hi, max_rows):
    """dK and dV of the keys [k_lo, k_hi) of KV head g, element by element: the
    oracle runs on exactly the share's rows that see any of these keys (the
    other rows contribute nothing to them), for all query heads of the group.
    Returns the two relative L2 errors."""
    from oracle import mask as om
    f = fields(w.layout)
    rep = w.Hq // w.Hkv
    hs = slice(g * rep, (g + 1) * rep)
    rows = oa.rows_of_blocks(blocks, w.N_B)
    seers = np.flatnonzero(om.visible(rows, np.arange(k_lo, k_hi), f[0], f[1], f[2]).any(axis=1))
    assert 0 < seers.size <= max_rows, seers.size
    Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
    _, dk_ref, dv_ref = oa.backward(Q[seers][:, hs], K[:, g:g + 1], V[:, g:g + 1], dO[seers][:, hs],
                                    rows[seers], f[0], f[1], f[2], chunk=256)
    _, _, _, dk, dv = outs
    ks = slice(k_lo, k_hi)
    e_k = rel_l2(bf16_to_f64(dk[ks, g:g + 1]), dk_ref[ks])
    e_v = rel_l2(bf16_to_f64(dv[ks, g:g + 1]), dv_ref[ks])
    assert e_k < TOL and e_v < TOL, (k_lo, k_hi, seers.size, e_k, e_v)
    return seers.size


def heaviest_share(w):
    f = fields(w.layout)
    _, _, W = ot.tile_map_c(f[0], f[1], f[2], w.N_B, w.N_B)
    _, load, off, rb = ob.lpt(W, w.P)
    g = int(np.argmax(load))
    return rb[off[g]:off[g + 1]].tolist()


def test_workload3_heaviest_rank_one_group():
    w = wl.workload(3)
    blocks = heaviest_share(w)
    t = make_tensors(w.tensor_seed, len(blocks) * w.N_B, w.layout.S, w.Hq, w.Hkv, w.D)
    outs = gpu_fwd_bwd(w.layout, blocks, w.N_B, t)
    sampled_dq_and_dv_sums(w, blocks, t, outs, heads=(1, w.Hq - 2))
    group_check(w, blocks, t, outs, g=2)


def test_workload5_packed_samples_element_wise():
    """64 / 8 heads (the only shape with eight query heads per KV head): dK and
    dV of every key of two packed samples, one KV group each, against the oracle
    on exactly the share's rows of that sample (rows of other samples see none
    of its keys)."""
    w = wl.workload(5)
    blocks = heaviest_share(w)
    t = make_tensors(w.tensor_seed, len(blocks) * w.N_B, w.layout.S, w.Hq, w.Hkv, w.D)
    outs = gpu_fwd_bwd(w.layout, blocks, w.N_B, t)
    sampled_dq_and_dv_sums(w, blocks, t, outs, heads=(1, w.Hq - 2))
    rows = oa.rows_of_blocks(blocks, w.N_B)
    off = np.asarray(w.layout.sample_off)
    per_sample = np.histogram(rows, bins=off)[0]
    # the sample with the most rows of the share among those the oracle finishes in seconds,
    # and the one with the fewest (at least one block)
    ok = np.flatnonzero((per_sample >= w.N_B) & (per_sample <= 1280))
    big = int(ok[np.argmax(per_sample[ok])])
    small = int(ok[np.argmin(per_sample[ok])])
    assert big != small
    for smp, g in ((big, 3), (small, 6)):
        n = key_range_check(w, blocks, t, outs, g, int(off[smp]), int(off[smp + 1]), max_rows=1280)
        assert n == per_sample[smp]


def test_workload4_sampled():
    """131072 keys, 16384 rows: dQ of sampled rows, column sums of dV, and dK / dV
    element by element on two 128-key blocks -- one in late text, one inside an
    image span -- for a whole KV group (oracle on the share's rows that see
    them)."""
    from oracle import mask as om
    w = wl.workload(4)
    f = fields(w.layout)
    blocks = heaviest_share(w)
    t = make_tensors(w.tensor_seed, len(blocks) * w.N_B, w.layout.S, w.Hq, w.Hkv, w.D)
    outs = gpu_fwd_bwd(w.layout, blocks, w.N_B, t)
    sampled_dq_and_dv_sums(w, blocks, t, outs, n_rows=12, heads=(3, 30))
    rows = oa.rows_of_blocks(blocks, w.N_B)
    span_of = f[1]

    def latest_block(in_span):
        """Last 128-key block wholly inside a span (or wholly text) that between 384 and
        1536 rows of the share see."""
        for k0 in range(w.layout.S - 128, -1, -128):
            ids = span_of[k0:k0 + 128]
            if (ids != 0).all() != in_span or (ids == 0).all() == in_span or len(set(ids.tolist())) != 1:
                continue
            n = int(om.visible(rows, np.arange(k0, k0 + 128), f[0], f[1], f[2]).any(axis=1).sum())
            if 384 <= n <= 1536:
                return k0
        raise AssertionError("no such block")

    for in_span, g in ((False, 1), (True, 6)):
        k0 = latest_block(in_span)
        key_range_check(w, blocks, t, outs, g, k0, k0 + 128, max_rows=1536)


def test_row_that_sees_no_key():
    """Hand-built mask words (the encoder never produces such a token): one
    token without the causal bit and outside every span sees nothing, not even
    itself.  Forward: O = 0, LSE = -inf; backward: dQ = 0 for that row, finite
    dK / dV that match the oracle."""
    from oracle import mask as om
    S, block, Hq, Hkv, D = 512, 64, 4, 2, 128
    lay = wl.Layout(S, [(100, 150, 1)], [0, 300, S])
    sample, span, causal, modality, attend = fields(lay)
    blind = [77, 301, 448]                 # text tokens: span id 0
    causal = causal.copy()
    causal[blind] = 0
    words = om.encode(sample, span, causal, modality, attend)
    bits = torch.from_numpy(words.view(np.int64)).to(DEV)
    blocks = list(range(S // block))
    bl = torch.tensor(blocks, dtype=torch.int32, device=DEV)
    t = make_tensors(123, S, S, Hq, Hkv, D)
    o, lse = mb.fwd(t["q"], t["k"], t["v"], bits, bl, block)
    dq, dk, dv = mb.bwd(t["q"], t["k"], t["v"], bits, bl, block, o, lse, t["do"])
    torch.cuda.synchronize()
    assert (o[blind] == 0).all() and torch.isneginf(lse[:, blind]).all()
    assert (dq[blind] == 0).all()
    rows = np.arange(S)
    Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
    o_ref, lse_ref = oa.forward(Q, K, V, rows, sample, span, causal, modality=modality, attend=attend)
    dq_ref, dk_ref, dv_ref = oa.backward(Q, K, V, dO, rows, sample, span, causal, modality=modality,
                                         attend=attend)
    assert np.isneginf(lse_ref[:, blind]).all() and (dq_ref[blind] == 0).all()
    seeing = np.setdiff1d(rows, blind)
    assert max_abs(bf16_to_f64(o), o_ref) < 2e-2 and rel_l2(bf16_to_f64(o), o_ref) < 5e-3
    assert np.abs(lse.cpu().numpy().astype(np.float64)[:, seeing] - lse_ref[:, seeing]).max() < 4.5e-3
    for name, got, ref in (("dq", dq, dq_ref), ("dk", dk, dk_ref), ("dv", dv, dv_ref)):
        gg = bf16_to_f64(got)
        assert np.isfinite(gg).all(), name
        assert rel_l2(gg, ref) < TOL, (name, rel_l2(gg, ref))


def test_bad_block_index_leaves_outputs_untouched():
    """A block index outside [0, S/block) raises the status word (first int32 of
    the workspace); dq, dk, dv keep what they held."""
    lay = wl.Layout(512, [(100, 200, 1)], [0, 512])
    t = make_tensors(6, 128, lay.S, 2, 1, 64)
    bits = gpu_bits(lay)
    o, lse = mb.fwd(t["q"], t["k"], t["v"], bits, torch.tensor([1, 2], dtype=torch.int32, device=DEV), 64)
    ws = torch.zeros(mb.workspace_size(mb.OP_BWD, lay.S, 2, 64, 2, 1, 64), dtype=torch.uint8, device=DEV)
    for bad in ([1, 8], [-1, 2]):
        dq = torch.full_like(t["q"], 5.0)
        dk = torch.full_like(t["k"], 3.0)
        dv = torch.full_like(t["v"], -2.0)
        mb.bwd(t["q"], t["k"], t["v"], bits, torch.tensor(bad, dtype=torch.int32, device=DEV), 64, o, lse,
               t["do"], ws=ws, out=(dq, dk, dv))
        torch.cuda.synchronize()
        assert int(ws[:4].view(torch.int32)[0]) != 0
        assert (dq == 5.0).all() and (dk == 3.0).all() and (dv == -2.0).all()
    dq, dk, dv = mb.bwd(t["q"], t["k"], t["v"], bits, torch.tensor([1, 2], dtype=torch.int32, device=DEV), 64,
                        o, lse, t["do"], ws=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32)[0]) == 0 and torch.isfinite(dq.float()).all()
