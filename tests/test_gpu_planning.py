"""GPU parity, integer stages: mask encode, tile map, balancer -- bit-exact
against the oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from oracle import balance as ob
from oracle import tilemap as ot
from paper_2503_11367_amd import binding as mb
from paper_2503_11367_amd import workloads as wl

from gpu_util import DEV, fields, gpu_bits, oracle_bits, to_np_u64, windows

pytestmark = pytest.mark.gpu


def layouts_small():
    out = [wl.layout_tiny(), wl.Layout(256, [], [0, 256]), wl.Layout(256, [(0, 256, 1)], [0, 256])]
    for seed in range(6):
        out.append(wl.layout_random(seed, S=1024, n_samples=1 + seed % 4, noncausal_prob=0.3))
    out.append(wl.layout_packed(seed=3, S=4096, n_samples=6, span_lo=30, span_hi=400))
    return out


def layouts_attend():
    """Layouts whose spans deny some modalities (attend-set generalisation)."""
    out = [wl.Layout(9 * 64, [(128, 128, wl.AUDIO), (320, 192, wl.IMAGE)], [0, 576], deny=[0, 1 << wl.AUDIO])]
    # "prepended" family (App. C): all modality tokens first, then the text; the audio
    # encoder's tokens do not attend the image tokens before them
    out.append(wl.Layout(1024, [(0, 300, wl.IMAGE), (300, 150, wl.AUDIO)], [0, 1024], deny=[0, 1 << wl.IMAGE]))
    # shared question (section 5.5): answers attend the question and themselves only
    out.append(wl.layout_shared_question(200, [130, 64, 257, 100], n_tail=145))
    out.append(wl.layout_shared_question(64, [128] * 7, n_tail=64))
    for seed in range(1, 5):
        out.append(wl.layout_random(60 + seed, S=1024, n_samples=1 + seed % 3, max_spans=6,
                                    noncausal_prob=0.2, deny_prob=0.7))
    return out


@pytest.mark.parametrize("idx", range(10))
def test_encode_small(idx):
    lay = layouts_small()[idx]
    assert np.array_equal(to_np_u64(gpu_bits(lay)), oracle_bits(lay))


def test_encode_long_lists():
    """More spans / samples than travel inside the kernel arguments: the lists
    are staged through the workspace."""
    for seed, ns in ((3, 80), (4, 200), (5, 30)):
        lay = wl.layout_random(seed, S=8192, n_samples=ns, max_spans=4, noncausal_prob=0.2, deny_prob=0.2)
        assert ns > 64 or len(lay.spans) > 64 or seed == 5
        assert np.array_equal(to_np_u64(gpu_bits(lay)), oracle_bits(lay))


def test_encode_reads_host_lists_before_it_returns():
    """The host span / offset arrays may be changed or freed as soon as the call
    returns, also on the long-list path (pinned host memory included, where an
    asynchronous copy would still be reading): here they are overwritten with
    garbage right after the call, before the stream is synchronised."""
    import ctypes
    lay = wl.layout_random(4, S=8192, n_samples=200, max_spans=4, noncausal_prob=0.2, deny_prob=0.2)
    n, ns = len(lay.spans), len(lay.sample_off) - 1
    assert n > 64 and ns > 64
    # both lists inside one pinned host buffer: spans (24 bytes each) first, then the offsets
    pinned = torch.empty(n * 24 + (ns + 1) * 8, dtype=torch.uint8, pin_memory=True)
    base = pinned.data_ptr()
    spans = (mb.Span * n).from_address(base)
    off = (ctypes.c_int64 * (ns + 1)).from_address(base + n * 24)
    for i, ((st, ln, mod), fl) in enumerate(zip(lay.spans, lay.span_flags())):
        spans[i] = mb.Span(int(st), int(ln), int(mod), int(fl))
    off[:] = [int(x) for x in lay.sample_off]
    bits = torch.zeros(lay.S, dtype=torch.int64, device=DEV)
    ws = torch.empty(mb.workspace_size(mb.OP_ENCODE, lay.S, n, ns), dtype=torch.uint8, device=DEV)
    # a long-running kernel ahead on the stream, so the encode kernels cannot have run yet
    a = torch.randn(4096, 4096, device=DEV)
    for _ in range(8):
        a = a @ a
        a = a / a.norm()
    rc = mb.lib().mmattn_mask_encode(base, n, base + n * 24, ns, lay.S, bits.data_ptr(), ws.data_ptr(),
                                     ws.numel(), torch.cuda.current_stream().cuda_stream)
    pinned.fill_(0xEE)
    assert rc == 0
    torch.cuda.synchronize()
    assert np.array_equal(to_np_u64(bits), oracle_bits(lay))


@pytest.mark.parametrize("c", [1, 2, 3, 4, 5])
def test_encode_workloads(c):
    lay = wl.workload(c).layout
    assert np.array_equal(to_np_u64(gpu_bits(lay)), oracle_bits(lay))


def check_tile_map(lay, tq, tk, use_c):
    f = fields(lay)
    bits = torch.from_numpy(oracle_bits(lay).view(np.int64)).to(DEV)      # oracle-encoded input
    cls, cnt, rp = mb.tile_map(bits, tq, tk)
    ref = (ot.tile_map_c if use_c else ot.tile_map)(f[0], f[1], f[2], tq, tk, f[3], f[4], windows(lay))
    assert np.array_equal(cls.cpu().numpy(), ref[0])
    assert np.array_equal(cnt.cpu().numpy().view(np.uint32), ref[1])
    assert np.array_equal(rp.cpu().numpy().view(np.uint64), ref[2])


@pytest.mark.parametrize("idx", range(10))
@pytest.mark.parametrize("tile", [(64, 64), (128, 64), (16, 256), (256, 32)])
def test_tile_map_small(idx, tile):
    lay = layouts_small()[idx]
    if lay.S % tile[0] or lay.S % tile[1]:
        pytest.skip("tile does not divide S")
    check_tile_map(lay, tile[0], tile[1], use_c=False)


@pytest.mark.parametrize("idx", range(8))
def test_encode_and_tile_map_with_attend_sets(idx):
    lay = layouts_attend()[idx]
    assert any(lay.deny)
    assert np.array_equal(to_np_u64(gpu_bits(lay)), oracle_bits(lay))
    for tile in ((64, 64), (128, 64), (64, 128)):
        if lay.S % tile[0] == 0 and lay.S % tile[1] == 0:
            check_tile_map(lay, tile[0], tile[1], use_c=False)


@pytest.mark.parametrize("tile", [(48, 48), (80, 80), (240, 240), (48, 128), (640, 16)])
def test_tile_map_tiles_not_powers_of_two(tile):
    """The public tile map with tq = tk = N_B for block sizes such as 48, 80 and
    240 (S = 1920), and with unequal tile sides."""
    for seed in (131, 132):
        lay = wl.layout_random(seed, S=1920, n_samples=3, max_spans=5, noncausal_prob=0.2)
        check_tile_map(lay, tile[0], tile[1], use_c=False)


def test_tile_map_many_short_runs():
    """Hundreds of 1-3 token spans of alternating modality: nearly every key
    starts a new run of equal mask fields."""
    rng = np.random.default_rng(17)
    spans, deny, pos = [], [], 1
    while pos + 8 < 1024:
        n = int(rng.integers(1, 4))
        spans.append((pos, n, 1 + len(spans) % 3))
        deny.append(int(rng.integers(0, 2)) << int(rng.integers(0, 4)))
        pos += n + int(rng.integers(0, 3))
    lay = wl.Layout(1024, spans, [0, 500, 1024] if not any(s <= 500 < s + n for s, n, _ in spans) else [0, 1024],
                    deny=deny)
    assert len(spans) > 250
    assert np.array_equal(to_np_u64(gpu_bits(lay)), oracle_bits(lay))
    for tile in ((64, 64), (128, 32), (16, 128)):
        check_tile_map(lay, tile[0], tile[1], use_c=False)


def layouts_window():
    """Look-back windows: attention sinks plus a sliding window (the lambda
    pattern of section 5.5) in one sample and packed, window shorter and longer
    than a tile, the largest window, and windows on ordinary image spans."""
    out = [wl.layout_lambda([1024], 4, 100), wl.layout_lambda([700, 324, 1024], 16, 256),
           wl.layout_lambda([2048], 64, 1), wl.layout_lambda([4096], 1, 65535),
           wl.layout_lambda([3000, 1096], 130, 777)]
    lay = wl.layout_random(71, S=1024, n_samples=2, max_spans=6)
    lay.window = [37 * (j + 1) for j in range(len(lay.spans))]
    out.append(lay)
    return out


@pytest.mark.parametrize("idx", range(6))
def test_encode_and_tile_map_with_windows(idx):
    lay = layouts_window()[idx]
    assert any(lay.window)
    assert np.array_equal(to_np_u64(gpu_bits(lay)), oracle_bits(lay))
    for tile in ((64, 64), (128, 64), (64, 128), (16, 256)):
        check_tile_map(lay, tile[0], tile[1], use_c=lay.S > 2048)


def test_lambda_tile_map_is_a_band():
    """8192 tokens, 64 sinks, window 1024: below the band only the sinks' column
    of tiles is left, so a q-tile has at most 1 + 1024/64 + 1 active k-tiles."""
    lay = wl.layout_lambda([8192], 64, 1024)
    check_tile_map(lay, 128, 64, use_c=True)
    bits = gpu_bits(lay)
    cls, _, _ = mb.tile_map(bits, 128, 64)
    active = (cls.cpu().numpy() != 0).sum(axis=1)
    assert active.max() <= 1 + 1024 // 64 + 2 and active[-1] == 1 + 1024 // 64 + 2


def test_tile_map_block_causal():
    for blk in (96, 128, 50):
        lay = wl.layout_block_causal(1024 if blk != 50 else 1000 + 24, blk)
        check_tile_map(lay, 128, 64, use_c=False)


@pytest.mark.parametrize("c", [1, 2, 3, 4, 5])
def test_tile_map_workloads(c):
    w = wl.workload(c)
    check_tile_map(w.layout, w.N_B, w.N_B, use_c=True)
    if c in (2, 3):
        check_tile_map(w.layout, 128, 64, use_c=True)


def check_balance(W, P):
    Wt = torch.from_numpy(np.asarray(W, dtype=np.uint64).view(np.int64)).to(DEV)
    rob, load, off, blocks = mb.balance(Wt, P)
    ref = ob.lpt(W, P)
    assert np.array_equal(rob.cpu().numpy(), ref[0])
    assert np.array_equal(load.cpu().numpy().view(np.uint64), ref[1])
    assert np.array_equal(off.cpu().numpy(), ref[2])
    assert np.array_equal(blocks.cpu().numpy(), ref[3])


def test_balance_paper_example_and_edges():
    check_balance([1, 2, 2, 4, 5, 2, 2, 8], 4)
    check_balance([7], 1)
    check_balance([7], 5)                     # more ranks than blocks
    check_balance([0, 0, 0, 0], 2)            # all-zero workloads
    check_balance([5] * 12, 4)                # all ties
    check_balance([2 ** 63, 2 ** 62, 2 ** 62, 1], 2)     # needs full 64-bit loads


def test_balance_maximum_sizes():
    """MMATTN_MAX_BLOCKS blocks over MMATTN_MAX_RANKS ranks, many ties."""
    rng = np.random.default_rng(99)
    check_balance(rng.integers(0, 50, size=16384).tolist(), 1024)
    check_balance(rng.integers(0, 2 ** 50, size=16384).tolist(), 1023)


@pytest.mark.parametrize("seed", range(8))
def test_balance_random(seed):
    rng = np.random.default_rng(seed)
    nB = int(rng.integers(1, 2500))
    P = int(rng.choice([1, 2, 3, 8, 63, 64, 65, 200, 1024]))
    hi = int(rng.choice([4, 1000, 2 ** 40]))
    check_balance(rng.integers(0, hi, size=nB).tolist(), P)


@pytest.mark.parametrize("c", [1, 2, 3, 4, 5])
def test_balance_workloads_end_to_end(c):
    """encode -> tile map -> balance, all on the GPU, against the oracle chain."""
    w = wl.workload(c)
    f = fields(w.layout)
    bits = gpu_bits(w.layout)
    _, _, rp = mb.tile_map(bits, w.N_B, w.N_B)
    rob, load, off, blocks = mb.balance(rp, w.P)
    _, _, Wref = ot.tile_map_c(f[0], f[1], f[2], w.N_B, w.N_B)
    ref = ob.lpt(Wref, w.P)
    assert np.array_equal(rob.cpu().numpy(), ref[0])
    assert np.array_equal(load.cpu().numpy().view(np.uint64), ref[1])
    assert np.array_equal(blocks.cpu().numpy(), ref[3])
    assert int(load.sum().item()) == int(Wref.sum())


@pytest.mark.parametrize("batch", range(3))
def test_plan_chain_random_shapes(batch):
    """encode -> tile map -> balance on randomly drawn layouts, with tile sides any
    divisor of S (odd ones included) and 1 to 64 ranks: every array bit for bit."""
    rng = np.random.default_rng(700 + batch)
    for case in range(25):
        S = int(rng.choice([64, 128, 192, 256, 480, 960, 1024, 1920, 4096, 6144]))
        kind = int(rng.integers(0, 4))
        seed = int(rng.integers(0, 100000))
        if kind == 0:
            lay = wl.layout_random(seed, S=S, n_samples=int(rng.integers(1, min(40, S // 4))), max_spans=6,
                                   noncausal_prob=0.3, deny_prob=0.3)
        elif kind == 1:
            lay = wl.layout_random(seed, S=S, n_samples=1, max_spans=12, noncausal_prob=0.1)
        elif kind == 2:
            lay = wl.layout_lambda([S], int(rng.integers(1, 20)), int(rng.integers(1, S)))
        else:
            lay = wl.layout_block_causal(S, int(rng.choice([b for b in (16, 32, 48, 64, 96) if S % b == 0])))
        divs = [d for d in range(8, S + 1) if S % d == 0 and S // d <= 4096]
        tq, tk = int(rng.choice(divs)), int(rng.choice(divs))
        P = int(rng.choice([1, 2, 3, 4, 8, 17, 64]))
        what = dict(batch=batch, case=case, S=S, kind=kind, seed=seed, tq=tq, tk=tk, P=P)
        f = fields(lay)
        bits = gpu_bits(lay)
        assert np.array_equal(to_np_u64(bits), oracle_bits(lay)), what
        cls, cnt, rp = mb.tile_map(bits, tq, tk)
        ref = ot.tile_map(f[0], f[1], f[2], tq, tk, f[3], f[4], windows(lay))
        assert np.array_equal(cls.cpu().numpy(), ref[0]), what
        assert np.array_equal(cnt.cpu().numpy().view(np.uint32), ref[1]), what
        assert np.array_equal(rp.cpu().numpy().view(np.uint64), ref[2]), what
        rob, load, off, rb = mb.balance(rp, P)
        r2 = ob.lpt(ref[2], P)
        assert np.array_equal(rob.cpu().numpy(), r2[0]), what
        assert np.array_equal(load.cpu().numpy().view(np.uint64), r2[1]), what
        assert np.array_equal(off.cpu().numpy(), r2[2]) and np.array_equal(rb.cpu().numpy(), r2[3]), what
