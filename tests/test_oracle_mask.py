"""Pins for oracle/mask.py and oracle/tilemap.py (CPU only)."""
import os

import numpy as np
import pytest

from oracle import mask as om
from oracle import tilemap as ot
from paper_2503_11367_amd import workloads as wl


def fields(lay):
    return om.token_fields(lay.S, lay.spans, lay.sample_off, lay.noncausal, lay.deny, lay.nobidir)


def windows(lay):
    return om.token_windows(lay.S, lay.spans, lay.window) if any(lay.window) else None


def dense(lay):
    sample, span, causal, modality, attend = fields(lay)
    idx = np.arange(lay.S)
    if any(lay.deny) or any(lay.nobidir) or any(lay.window):
        return om.visible(idx, idx, sample, span, causal, modality, attend, windows(lay))
    return om.visible(idx, idx, sample, span, causal)


def closed_form_pairs(lay):
    """sum over samples L(L+1)/2 + sum over spans n(n-1)/2 (causal bit set)."""
    tot = 0
    for a, b in zip(lay.sample_off[:-1], lay.sample_off[1:]):
        L = b - a
        tot += L * (L + 1) // 2
    for _, n, _ in lay.spans:
        tot += n * (n - 1) // 2
    return tot


def test_all_text_is_lower_triangle():
    lay = wl.Layout(96, [], [0, 96])
    assert np.array_equal(dense(lay), np.tril(np.ones((96, 96), dtype=bool)))


def test_single_span_is_full():
    lay = wl.Layout(80, [(0, 80, wl.IMAGE)], [0, 80])
    assert dense(lay).all()


def test_packed_is_block_diagonal():
    lay = wl.Layout(100, [], [0, 30, 100])
    v = dense(lay)
    assert not v[30:, :30].any() and not v[:30, 30:].any()
    assert np.array_equal(v[:30, :30], np.tril(np.ones((30, 30), dtype=bool)))
    assert np.array_equal(v[30:, 30:], np.tril(np.ones((70, 70), dtype=bool)))


def test_span_rows_by_hand():
    # text[0:2] image[2:5] text[5:7]
    lay = wl.Layout(7, [(2, 3, wl.IMAGE)], [0, 7])
    expect = np.array([
        [1, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 1, 1, 0, 0],
        [1, 1, 1, 1, 1, 0, 0],
        [1, 1, 1, 1, 1, 0, 0],
        [1, 1, 1, 1, 1, 1, 0],
        [1, 1, 1, 1, 1, 1, 1]], dtype=bool)
    assert np.array_equal(dense(lay), expect)


def test_paper_bitfield_example():
    """Section 4.2: t2,t3 come from encoder A and carry no causal bit, so they
    attend only to encoder-A tokens; t4,t5 are text with the causal bit and
    attend to every earlier token whatever its modality."""
    lay = wl.Layout(6, [(2, 2, wl.IMAGE)], [0, 6], noncausal=[1])
    v = dense(lay)
    assert v[2].tolist() == [False, False, True, True, False, False]
    assert v[3].tolist() == [False, False, True, True, False, False]
    assert v[4].tolist() == [True, True, True, True, True, False]
    assert v[5].tolist() == [True] * 6
    sample, span, causal, modality, attend = fields(lay)
    bits = om.encode(sample, span, causal, modality)
    assert (int(bits[2]) >> 63) == 0 and (int(bits[4]) >> 63) == 1
    assert (int(bits[2]) >> 8) & 0xF == wl.IMAGE and (int(bits[4]) >> 8) & 0xF == wl.TEXT
    assert int(bits[4]) & 0xFF == 0xFF        # text attends all modalities


def test_word_written_out_bit_by_bit():
    """One token with every field set, against the word typed out from the layout
    (attend-set bits 0-7, modality 8-11, span id 12-27, sample id 28-43, look-back
    window 44-59, causal bit 63): sample 3, span 5, modality 2, window 7, causal,
    attends everything  ->  0x8000_7000_3000_52FF."""
    one = lambda x: np.array([x], dtype=np.int64)
    w = om.encode(one(3), one(5), one(1), one(2), attend=one(0xFF), window=one(7))
    assert int(w[0]) == 0x80007000300052FF
    # every field alone lands where the layout says, and nowhere else
    assert int(om.encode(one(0), one(0), one(0), one(0), attend=one(0))[0]) == 0
    assert int(om.encode(one(1), one(0), one(0), one(0), attend=one(0))[0]) == 1 << 28
    assert int(om.encode(one(0), one(1), one(0), one(0), attend=one(0))[0]) == 1 << 12
    assert int(om.encode(one(0), one(0), one(0), one(1), attend=one(0))[0]) == 1 << 8
    assert int(om.encode(one(0), one(0), one(0), one(0), attend=one(0), window=one(1))[0]) == 1 << 44
    assert int(om.encode(one(0xFFFF), one(0), one(0), one(0), attend=one(0))[0]) == 0xFFFF << 28
    assert int(om.encode(one(0), one(0xFFFF), one(0), one(0), attend=one(0))[0]) == 0xFFFF << 12
    assert int(om.encode(one(0), one(0), one(0), one(0), attend=one(0), window=one(0xFFFF))[0]) == 0xFFFF << 44
    # a packed layout through the layout expansion: token 70 is in sample 1, span 2 (audio)
    lay = wl.Layout(128, [(10, 20, wl.IMAGE), (64, 16, wl.AUDIO)], [0, 50, 128])
    f = fields(lay)
    assert int(om.encode(*f)[70]) == (1 << 63) | (1 << 28) | (2 << 12) | (wl.AUDIO << 8) | 0xFF


def test_attend_set_rows_by_hand():
    """text[0:2] audio[2:4] text[4:5] image[5:8] text[8:9]; the image span does not
    attend audio: its rows lose the two audio columns, nothing else changes
    (text rows still see the audio tokens, the span still sees itself)."""
    lay = wl.Layout(9, [(2, 2, wl.AUDIO), (5, 3, wl.IMAGE)], [0, 9], deny=[0, 1 << wl.AUDIO])
    expect = np.array([
        [1, 0, 0, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0, 0, 0],
        [1, 1, 1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 1, 1, 0, 0, 0, 0],
        [1, 1, 0, 0, 1, 1, 1, 1, 0],
        [1, 1, 0, 0, 1, 1, 1, 1, 0],
        [1, 1, 0, 0, 1, 1, 1, 1, 0],
        [1, 1, 1, 1, 1, 1, 1, 1, 1]], dtype=bool)
    assert np.array_equal(dense(lay), expect)
    bits = om.encode(*fields(lay))
    assert int(bits[5]) & 0xFF == 0xFF & ~(1 << wl.AUDIO) and int(bits[2]) & 0xFF == 0xFF


def test_denying_own_modality_keeps_the_span_itself():
    """A span that denies its own modality still sees its own tokens (same-span
    term) but not an earlier span of that modality."""
    lay = wl.Layout(8, [(1, 2, wl.IMAGE), (4, 3, wl.IMAGE)], [0, 8], deny=[0, 1 << wl.IMAGE])
    v = dense(lay)
    assert v[5].tolist() == [True, False, False, True, True, True, True, False]


def test_shared_question_rows_by_hand():
    """question[0:2], answers [2:4] and [4:7], trailing text [7:8]: an answer sees
    the question and its own earlier tokens, never the other answer; the
    trailing text sees everything before it."""
    lay = wl.layout_shared_question(2, [2, 3], n_tail=1)
    expect = np.array([
        [1, 0, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0, 0],
        [1, 1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 1, 0, 0, 0, 0],
        [1, 1, 0, 0, 1, 0, 0, 0],
        [1, 1, 0, 0, 1, 1, 0, 0],
        [1, 1, 0, 0, 1, 1, 1, 0],
        [1, 1, 1, 1, 1, 1, 1, 1]], dtype=bool)
    assert np.array_equal(dense(lay), expect)
    sample, span, causal, modality, attend = fields(lay)
    assert not span.any() and modality.tolist() == [0, 0, 1, 1, 2, 2, 2, 0]
    assert attend[2] == 0b00000011 and attend[4] == 0b00000101 and attend[7] == 0xFF


@pytest.mark.parametrize("nq,answers", [(5, [3]), (17, [9, 1, 30]), (64, [40] * 7)])
def test_shared_question_pair_count(nq, answers):
    """pairs = nq(nq+1)/2 + sum over answers of n*nq + n(n+1)/2."""
    lay = wl.layout_shared_question(nq, answers)
    want = nq * (nq + 1) // 2 + sum(n * nq + n * (n + 1) // 2 for n in answers)
    assert int(dense(lay).sum()) == want


def test_lambda_rows_by_hand():
    """7 tokens, 2 sinks, window 3: every token sees the sinks before it and the
    last three tokens up to itself."""
    lay = wl.layout_lambda([7], 2, 3)
    expect = np.array([
        [1, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 0, 0, 0, 0],
        [1, 1, 1, 1, 0, 0, 0],
        [1, 1, 1, 1, 1, 0, 0],
        [1, 1, 0, 1, 1, 1, 0],
        [1, 1, 0, 0, 1, 1, 1]], dtype=bool)
    assert np.array_equal(dense(lay), expect)
    assert windows(lay).tolist() == [0, 0, 3, 3, 3, 3, 3]


def lambda_pairs(sample_lens, n_sink, window):
    """per sample: s(s+1)/2 among the sinks, then body token i (0-based) sees the
    s sinks and min(i+1, W) body tokens."""
    tot = 0
    for L in sample_lens:
        tot += n_sink * (n_sink + 1) // 2
        tot += sum(n_sink + min(i + 1, window) for i in range(L - n_sink))
    return tot


@pytest.mark.parametrize("lens,n_sink,window", [([40], 4, 8), ([33, 70, 25], 3, 16), ([64, 64], 1, 1),
                                                 ([50], 5, 200)])
def test_lambda_pair_count_and_shape(lens, n_sink, window):
    lay = wl.layout_lambda(lens, n_sink, window)
    v = dense(lay)
    assert int(v.sum()) == lambda_pairs(lens, n_sink, window)
    # the same mask from its description: sinks or the band, inside a sample, never ahead
    pos = np.arange(lay.S)
    start = np.repeat(lay.sample_off[:-1], np.diff(lay.sample_off))
    q, k = pos[:, None], pos[None, :]
    want = (start[:, None] == start[None, :]) & (k <= q) & ((k - start[None, :] < n_sink) | (q - k < window))
    assert np.array_equal(v, want)


def test_window_not_shorter_than_the_sample_is_no_window():
    a = wl.layout_lambda([48, 30], 2, 48)
    b = wl.layout_lambda([48, 30], 2, 0)
    assert np.array_equal(dense(a), dense(b))
    pos = np.arange(78)
    smp = (pos >= 48).astype(int)
    assert np.array_equal(dense(b), (smp[:, None] == smp[None, :]) & (pos[None, :] <= pos[:, None]))


def test_window_limits_only_the_own_modality_and_not_the_own_span():
    """image span [2:6] with window 2 (bidirectional) after two text tokens: its
    tokens still see the whole span and all earlier text; a second image span
    [8:10] with window 2 loses the first span's tokens, which are more than one
    position back, but keeps the text."""
    lay = wl.Layout(10, [(2, 4, wl.IMAGE), (8, 2, wl.IMAGE)], [0, 10], window=[2, 2])
    v = dense(lay)
    assert v[3].tolist() == [True, True, True, True, True, True, False, False, False, False]
    assert v[8].tolist() == [True, True, False, False, False, False, True, True, True, True]
    assert v[9].tolist() == [True, True, False, False, False, False, True, True, True, True]
    assert v[7].tolist() == [True] * 8 + [False] * 2          # text is not limited


def test_tile_map_with_windows():
    lay = wl.layout_lambda([300, 212], 7, 40)
    f = fields(lay)
    w = windows(lay)
    a = ot.tile_map(f[0], f[1], f[2], 64, 32, f[3], f[4], w)
    b = ot.tile_map_c(f[0], f[1], f[2], 64, 32, f[3], f[4], w)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert int(a[2].sum()) == lambda_pairs([300, 212], 7, 40)
    # far below the band and to the right of the sinks' columns the tiles are empty
    assert a[0][4, 1] == ot.EMPTY and a[0][4, 0] == ot.PARTIAL


def test_window_field_round_trip():
    lay = wl.layout_lambda([100, 60], 4, 65535)
    bits = om.encode(*fields(lay), window=windows(lay))
    assert np.array_equal(om.decode_window(bits), windows(lay))
    for x, y in zip(om.decode(bits), fields(lay)):
        assert np.array_equal(x, y)
    assert lay.span_flags() == [2, 2 | (65535 << 16) - (1 << 32), 2, 2 | (65535 << 16) - (1 << 32)]


def test_block_causal_is_block_lower_triangle():
    lay = wl.layout_block_causal(40, 16)        # ragged last block of 8
    v = dense(lay)
    blk = np.arange(40) // 16
    assert np.array_equal(v, blk[:, None] >= blk[None, :])


@pytest.mark.parametrize("seed", range(6))
def test_attend_set_pair_count(seed):
    """Pairs under the attend-set predicate = pairs of the plain predicate minus
    the backward pairs (query in a span, earlier key of a denied modality, same
    sample, different span), counted here by an explicit loop over spans."""
    lay = wl.layout_random(30 + seed, S=320, n_samples=1 + seed % 3, deny_prob=0.6)
    sample, span, causal, modality, attend = fields(lay)
    idx = np.arange(lay.S)
    plain = int(om.visible(idx, idx, sample, span, causal).sum())
    lost = 0
    for j, (start, n, _) in enumerate(lay.spans):
        if not lay.deny[j]:
            continue
        s0 = max(a for a in lay.sample_off if a <= start)        # the span's sample starts here
        for k in range(s0, start):                                # keys before the span, same sample
            if (lay.deny[j] >> int(modality[k])) & 1:
                lost += n                                         # every token of the span loses key k
    assert any(lay.deny) or lost == 0
    assert int(dense(lay).sum()) == plain - lost


def test_tile_map_c_with_attend_sets():
    lay = wl.layout_random(44, S=512, n_samples=2, deny_prob=0.7)
    f = fields(lay)
    a = ot.tile_map(f[0], f[1], f[2], 64, 32, f[3], f[4])
    b = ot.tile_map_c(f[0], f[1], f[2], 64, 32, f[3], f[4])
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert int(a[2].sum()) == int(dense(lay).sum())


def test_encode_decode_round_trip():
    lay = wl.layout_packed(seed=7, S=4096, n_samples=5, span_lo=40, span_hi=300)
    lay.deny = [(i % 3) << 1 for i in range(len(lay.spans))]
    f = fields(lay)
    bits = om.encode(*f)
    assert bits.dtype == np.uint64
    for a, b in zip(om.decode(bits), f):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("seed", range(6))
def test_total_pairs_closed_form_random(seed):
    lay = wl.layout_random(seed, S=384, n_samples=1 + seed % 3)
    assert int(dense(lay).sum()) == closed_form_pairs(lay)


def test_tiny_golden(golden_dir):
    W, rows = None, []
    for line in open(os.path.join(golden_dir, "tiny_tilemap.txt")):
        if line.startswith("W "):
            W = [int(x) for x in line.split()[1:]]
        elif line.startswith("C "):
            rows.append(line.split()[1])
    lay = wl.layout_tiny()
    sample, span, causal = fields(lay)[:3]
    cls, cnt, Wo = ot.tile_map(sample, span, causal, 64, 64)
    assert Wo.tolist() == W and sum(W) == 163968 == closed_form_pairs(lay)
    sym = {ot.EMPTY: "E", ot.FULL: "F", ot.PARTIAL: "P"}
    assert ["".join(sym[c] for c in r) for r in cls.tolist()] == rows
    assert (cnt[cls == ot.PARTIAL] == 2080).all()
    assert ot.tile_count_workload(cls).tolist() == [1, 5, 5, 5, 5, 6, 7, 8]


def test_all_text_tile_classes():
    lay = wl.Layout(256, [], [0, 256])
    sample, span, causal = fields(lay)[:3]
    cls, cnt, W = ot.tile_map(sample, span, causal, 32, 32)
    for i in range(8):
        for j in range(8):
            want = ot.FULL if j < i else (ot.PARTIAL if j == i else ot.EMPTY)
            assert cls[i, j] == want
    assert (np.diag(cnt) == 32 * 33 // 2).all()


def test_rect_tiles_and_dense_agree():
    lay = wl.layout_random(11, S=512, n_samples=2)
    sample, span, causal = fields(lay)[:3]
    v = dense(lay)
    cls, cnt, W = ot.tile_map(sample, span, causal, 128, 64)
    ref = v.reshape(4, 128, 8, 64).sum(axis=(1, 3))
    assert np.array_equal(cnt, ref)
    assert np.array_equal(W, v.sum(axis=1).reshape(4, 128).sum(axis=1))


@pytest.mark.parametrize("seed", range(4))
def test_c_tilemap_matches_numpy(seed):
    lay = wl.layout_random(100 + seed, S=1024, n_samples=1 + seed, noncausal_prob=0.3)
    f = fields(lay)
    a = ot.tile_map(f[0], f[1], f[2], 64, 128)
    b = ot.tile_map_c(f[0], f[1], f[2], 64, 128)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("c", [2, 3, 4, 5])
def test_workload_totals_closed_form(c):
    w = wl.workload(c)
    sample, span, causal = fields(w.layout)[:3]
    cls, cnt, W = ot.tile_map_c(sample, span, causal, w.N_B, w.N_B)
    assert int(W.sum()) == closed_form_pairs(w.layout)
    if c == 2:
        assert int(W.sum()) == 35653632
    if c == 3:
        assert int(W.sum()) == 553961064
    if c == 4:
        # 131072 * 131073 / 2 + 24 * 4096 * 4095 / 2; beyond 2^32, so the workloads are 64-bit
        assert int(W.sum()) == 8791277568
