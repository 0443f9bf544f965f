"""The C-ABI library loads, exports every symbol the header declares, and
rejects bad arguments on the host before any GPU work (CPU only)."""
import ctypes
import os
import re

import pytest

from paper_2503_11367_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # non-null, 256-aligned, never dereferenced on an error path


def header_symbols():
    text = open(os.path.join(ROOT, "include", "mmattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmattn_[a-z_]+)\s*\(", text)))


def test_exports_match_header():
    L = mb.lib()
    syms = header_symbols()
    assert set(syms) >= {"mmattn_mask_encode", "mmattn_tile_map", "mmattn_balance", "mmattn_fwd",
                         "mmattn_bwd", "mmattn_workspace_size", "mmattn_version"}
    for s in syms:
        assert hasattr(L, s), s
    assert b"gfx950" in L.mmattn_version()


def spans_arr(items):
    arr = (mb.Span * max(len(items), 1))()
    for i, it in enumerate(items):
        arr[i] = mb.Span(*it)
    return arr


def encode_rc(spans, offs, S, bits=FAKE, ws=FAKE, ws_bytes=1 << 20):
    arr = spans_arr(spans)
    off = (ctypes.c_int64 * len(offs))(*offs)
    return mb.lib().mmattn_mask_encode(ctypes.addressof(arr) if spans else 0, len(spans),
                                       ctypes.addressof(off), len(offs) - 1, S, bits, ws, ws_bytes, 0)


def test_encode_validation():
    assert encode_rc([], [0, 64], 64, bits=0) == -1
    assert encode_rc([], [0, 64], 0) == -2
    assert encode_rc([], [0, 32], 64) == -5                      # last offset != S
    assert encode_rc([], [0, 40, 40, 64], 64) == -5              # empty sample
    assert encode_rc([(8, 8, 1, 0), (12, 4, 1, 0)], [0, 64], 64) == -5      # overlap
    assert encode_rc([(20, 8, 1, 0), (4, 4, 1, 0)], [0, 64], 64) == -5      # unsorted
    assert encode_rc([(60, 8, 1, 0)], [0, 64], 64) == -5                    # past the end
    assert encode_rc([(28, 8, 1, 0)], [0, 32, 64], 64) == -5                # crosses samples
    assert encode_rc([(8, 8, 0, 0)], [0, 64], 64) == -5                     # modality 0 is text
    assert encode_rc([(8, 8, 8, 0)], [0, 64], 64) == -5                     # one attend bit per modality
    assert encode_rc([(8, 8, 1, 4)], [0, 64], 64) == -5                     # unknown flag bit
    assert encode_rc([(8, 8, 1, 2 | 1)], [0, 64], 64) == -5                 # no bidirectional term, no causal bit
    assert encode_rc([(8, 8, 1, 2 | (2 << 8))], [0, 64], 64) == -5          # ... or own modality denied
    assert encode_rc([(8, 8, 1, 0)], [0, 64], 64, ws=0) == -4
    # a look-back window (flags bits 16-31, here the largest) passes the layout checks
    assert encode_rc([(8, 8, 1, 2 | (0xFFFF << 16) - (1 << 32))], [0, 64], 64, ws=0) == -4
    assert encode_rc([(8, 8, 1, 4 | (100 << 16))], [0, 64], 64, ws=0) == -5
    assert encode_rc([(8, 8, 1, 0)], [0, 64], 64, ws_bytes=8) == -4
    assert encode_rc([(8, 8, 1, 0)], [0, 64], 64, ws=FAKE + 8) == -4        # misaligned


def test_tile_map_validation():
    f = mb.lib().mmattn_tile_map
    assert f(0, 512, 64, 64, FAKE, FAKE, FAKE, 0) == -1
    assert f(FAKE, 512, 64, 64, FAKE, 0, FAKE, 0) == -1
    assert f(FAKE, 500, 64, 64, FAKE, FAKE, FAKE, 0) == -2
    assert f(FAKE, 512, 0, 64, FAKE, FAKE, FAKE, 0) == -2
    assert f(FAKE, 512, 64, 48, FAKE, FAKE, FAKE, 0) == -2
    assert f(FAKE, 1 << 20, 8, 64, FAKE, FAKE, FAKE, 0) == -3     # too many q-tiles


def test_balance_validation():
    f = mb.lib().mmattn_balance
    assert f(0, 8, 2, FAKE, FAKE, FAKE, FAKE, 0) == -1
    assert f(FAKE, 0, 2, FAKE, FAKE, FAKE, FAKE, 0) == -2
    assert f(FAKE, 8, 0, FAKE, FAKE, FAKE, FAKE, 0) == -2
    assert f(FAKE, 1 << 20, 2, FAKE, FAKE, FAKE, FAKE, 0) == -3
    assert f(FAKE, 8, 5000, FAKE, FAKE, FAKE, FAKE, 0) == -3


def fwd_rc(q=FAKE, k=FAKE, v=FAKE, bits=FAKE, blocks=FAKE, n_blocks=4, block=128, S=1024, Hq=4,
           Hkv=2, D=128, scale=0.1, dtype=0, o=FAKE, lse=FAKE, ws=FAKE, ws_bytes=1 << 30):
    return mb.lib().mmattn_fwd(q, k, v, bits, blocks, n_blocks, block, S, Hq, Hkv, D, scale, dtype,
                               o, lse, ws, ws_bytes, 0)


def test_fwd_validation():
    assert fwd_rc(q=0) == -1 and fwd_rc(o=0) == -1 and fwd_rc(blocks=0) == -1
    assert fwd_rc(Hq=3) == -2                 # Hq % Hkv
    assert fwd_rc(S=1000) == -2               # S % block
    assert fwd_rc(n_blocks=9) == -2           # more blocks than the sequence has
    assert fwd_rc(scale=0.0) == -2
    assert fwd_rc(D=96) == -3
    assert fwd_rc(dtype=1) == -3
    assert fwd_rc(block=8, S=1024) == -3      # block % 16
    assert fwd_rc(S=1 << 23, n_blocks=(65535 * 64) // 128 + 1) == -3      # share too long for one launch
    assert fwd_rc(q=FAKE + 2) == -2           # alignment
    assert fwd_rc(ws=0) == -4
    assert fwd_rc(ws_bytes=16) == -4
    # an empty share is valid, needs no per-row buffers and launches nothing
    assert fwd_rc(n_blocks=0, q=0, blocks=0, o=0, lse=0, ws=0, ws_bytes=0) == 0
    assert fwd_rc(n_blocks=0, k=0) == -1 and fwd_rc(n_blocks=-1) == -2


def test_fwd_heads_validation():
    f = mb.lib().mmattn_fwd_heads

    def rc(begin, count, n_blocks=4, ws_bytes=1 << 30):
        return f(FAKE, FAKE, FAKE, FAKE, FAKE, n_blocks, 128, 1024, 8, 4, 128, 0.1, 0, begin, count, 0,
                 FAKE, FAKE, FAKE, ws_bytes, 0)
    assert rc(-1, 1) == -2 and rc(0, 0) == -2 and rc(3, 2) == -2 and rc(4, 1) == -2
    assert rc(0, 5) == -2
    assert rc(1, 2, ws_bytes=64) == -4
    assert rc(1, 2, n_blocks=0) == 0              # empty share: nothing to do
    # one workspace serves every window, and is at least the whole-launch one
    w_all = mb.workspace_size(mb.OP_FWD, 1024, 4, 128, 8, 4, 128)
    w_win = mb.workspace_size(mb.OP_FWD_HEADS, 1024, 4, 128, 8, 4, 128)
    assert w_win >= w_all > 0


def test_fwd_staged_validation():
    f = mb.lib().mmattn_fwd_staged

    def rc(hps=1, k_src=FAKE, copy=FAKE, stream=0, ws_bytes=1 << 30):
        return f(FAKE, k_src, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 128, 1024, 8, 4, 128, 0.1, 0, hps,
                 FAKE, FAKE, FAKE, ws_bytes, copy, stream)
    assert rc(k_src=0) == -1
    assert rc(hps=0) == -2 and rc(hps=3) == -2
    assert rc(copy=0, stream=0) == -2             # the two streams must differ
    assert rc(ws_bytes=64) == -4


def test_bwd_validation():
    f = mb.lib().mmattn_bwd
    args = [FAKE, FAKE, FAKE, FAKE, FAKE, 4, 128, 1024, 4, 2, 128, 0.1, 0,
            FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, 0]
    bad = list(args); bad[15] = 0
    assert f(*bad) == -1
    bad = list(args); bad[8] = 3
    assert f(*bad) == -2
    bad = list(args); bad[20] = 16
    assert f(*bad) == -4


def test_workspace_size_monotone():
    a = mb.workspace_size(mb.OP_FWD, 8192, 64, 128, 32, 8, 128)
    b = mb.workspace_size(mb.OP_FWD, 16384, 128, 128, 32, 8, 128)
    assert 0 < a < b
    assert mb.workspace_size(mb.OP_TILE_MAP, 8192, 0, 0) == 0
    assert mb.workspace_size(mb.OP_ENCODE, 8192, 4, 1) >= 4 * 24 + 16
