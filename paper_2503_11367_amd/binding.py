"""Thin ctypes binding over libmmattn.so (include/mmattn.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and the current stream.  There is no
fallback: if the library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MMATTN_LIB", os.path.join(_HERE, "libmmattn.so"))

OK = 0
ERR_NAMES = {0: "OK", -1: "ERR_NULL", -2: "ERR_SHAPE", -3: "ERR_UNSUPPORTED",
             -4: "ERR_WORKSPACE", -5: "ERR_LAYOUT", -6: "ERR_HIP"}
OP_ENCODE, OP_TILE_MAP, OP_BALANCE, OP_FWD, OP_BWD, OP_FWD_HEADS = range(6)
TILE_EMPTY, TILE_FULL, TILE_PARTIAL = 0, 1, 2
SPAN_NONCAUSAL = 1
SPAN_NOBIDIR = 2
SPAN_DENY_SHIFT = 8       # flags bits 8-15: modalities the span's tokens do not attend
SPAN_WINDOW_SHIFT = 16    # flags bits 16-31: look-back window over the own modality, tokens
BF16 = 0


class Span(ctypes.Structure):
    _fields_ = [("start", ctypes.c_int64), ("len", ctypes.c_int64),
                ("modality", ctypes.c_int32), ("flags", ctypes.c_int32)]


class MMAttnError(RuntimeError):
    def __init__(self, call: str, rc: int):
        super().__init__(f"{call} failed: {ERR_NAMES.get(rc, rc)} ({rc})")
        self.rc = rc


_lib = None
_vp, _i32, _i64, _sz, _f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t,
                               ctypes.c_float)


def lib() -> ctypes.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2503_11367_amd.build` (no CPU fallback exists)")
        L = ctypes.CDLL(LIB_PATH)
        L.mmattn_version.restype = ctypes.c_char_p
        L.mmattn_workspace_size.restype = _sz
        L.mmattn_workspace_size.argtypes = [ctypes.c_int, _i64, _i32, _i32, _i32, _i32, _i32]
        L.mmattn_mask_encode.restype = ctypes.c_int
        L.mmattn_mask_encode.argtypes = [_vp, _i32, _vp, _i32, _i64, _vp, _vp, _sz, _vp]
        L.mmattn_tile_map.restype = ctypes.c_int
        L.mmattn_tile_map.argtypes = [_vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]
        L.mmattn_balance.restype = ctypes.c_int
        L.mmattn_balance.argtypes = [_vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
        L.mmattn_fwd.restype = ctypes.c_int
        L.mmattn_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i32, _i32, _i32, _f32,
                                 ctypes.c_int, _vp, _vp, _vp, _sz, _vp]
        L.mmattn_fwd_static.restype = ctypes.c_int
        L.mmattn_fwd_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i32, _i32, _i32, _f32,
                                        ctypes.c_int, _vp, _vp, _vp]
        L.mmattn_fwd_heads.restype = ctypes.c_int
        L.mmattn_fwd_heads.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i32, _i32, _i32, _f32,
                                       ctypes.c_int, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]
        L.mmattn_fwd_staged.restype = ctypes.c_int
        L.mmattn_fwd_staged.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i32, _i32,
                                        _i32, _f32, ctypes.c_int, _i32, _vp, _vp, _vp, _sz, _vp, _vp]
        L.mmattn_bwd.restype = ctypes.c_int
        L.mmattn_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i32, _i32, _i32, _f32,
                                 ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.mmattn_mfma_ceiling.restype = ctypes.c_int
        L.mmattn_mfma_ceiling.argtypes = [ctypes.c_int32, ctypes.c_int32, _vp, ctypes.c_size_t,
                                          ctypes.POINTER(ctypes.c_double), _vp]
        L.mmattn_stage_events.restype = ctypes.c_int
        L.mmattn_stage_events.argtypes = [ctypes.c_int, _vp, _vp]
        _lib = L
    return _lib


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.data_ptr()


def _check(call: str, rc: int):
    if rc != OK:
        raise MMAttnError(call, rc)


def workspace_size(op: int, S: int, n_blocks: int, block: int, Hq: int = 0, Hkv: int = 0,
                   D: int = 0) -> int:
    return int(lib().mmattn_workspace_size(op, S, n_blocks, block, Hq, Hkv, D))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def mask_encode(spans: Sequence[Tuple[int, int, int]], sample_off: Sequence[int], S: int,
                device="cuda", flags: Optional[Sequence[int]] = None, stream=None,
                bits: Optional[torch.Tensor] = None) -> torch.Tensor:
    """mmattn_mask_encode.  spans: (start, len, modality); flags: per-span flag
    words of the C ABI (SPAN_* bits, deny mask, look-back window; a window above
    32767 makes the 32-bit word negative); returns int64[S] holding the 64-bit
    words."""
    n = len(spans)
    arr = (Span * max(n, 1))()
    for i, (st, ln, mod) in enumerate(spans):
        arr[i] = Span(int(st), int(ln), int(mod), int(flags[i]) if flags else 0)
    off = (ctypes.c_int64 * len(sample_off))(*[int(x) for x in sample_off])
    if bits is None:
        bits = torch.empty(S, dtype=torch.int64, device=device)
    ws = _workspace(workspace_size(OP_ENCODE, S, n, len(sample_off) - 1), bits.device)
    rc = lib().mmattn_mask_encode(ctypes.addressof(arr) if n else 0, n, ctypes.addressof(off),
                                  len(sample_off) - 1, S, _ptr(bits), _ptr(ws), ws.numel(),
                                  _stream(stream))
    _check("mmattn_mask_encode", rc)
    return bits


def tile_map(bits: torch.Tensor, tq: int, tk: int, stream=None, want_cls=True, want_rowpairs=True):
    """mmattn_tile_map -> (cls uint8 [nq,nk], cnt int32-view-of-uint32 [nq,nk],
    rowpairs int64-view-of-uint64 [nq])."""
    S = bits.numel()
    nq, nk = max(S // max(tq, 1), 0), max(S // max(tk, 1), 0)
    dev = bits.device
    cls = torch.empty((nq, nk), dtype=torch.uint8, device=dev) if want_cls else None
    cnt = torch.empty((nq, nk), dtype=torch.int32, device=dev)
    rp = torch.empty(nq, dtype=torch.int64, device=dev) if want_rowpairs else None
    rc = lib().mmattn_tile_map(_ptr(bits), S, tq, tk, _ptr(cls), _ptr(cnt), _ptr(rp),
                               _stream(stream))
    _check("mmattn_tile_map", rc)
    return cls, cnt, rp


def balance(W: torch.Tensor, P: int, stream=None, host: bool = False):
    """mmattn_balance -> (rank_of_block int32[nB], load int64[P], rank_off
    int32[P+1], rank_blocks int32[nB]).  load and rank_off share one
    allocation; with host=True two more items follow, their host copies
    (uint64 / int32 numpy arrays) fetched with a single device-to-host copy."""
    nB = W.numel()
    dev = W.device
    Pn = max(P, 1)
    rob = torch.empty(nB, dtype=torch.int32, device=dev)
    both = torch.empty(8 * Pn + 4 * (Pn + 1), dtype=torch.uint8, device=dev)
    load = both[:8 * Pn].view(torch.int64)
    off = both[8 * Pn:].view(torch.int32)
    blocks = torch.empty(nB, dtype=torch.int32, device=dev)
    rc = lib().mmattn_balance(_ptr(W), nB, P, _ptr(rob), _ptr(load), _ptr(off), _ptr(blocks),
                              _stream(stream))
    _check("mmattn_balance", rc)
    if not host:
        return rob, load, off, blocks
    h = both.cpu().numpy()
    return rob, load, off, blocks, h[:8 * Pn].view("<u8"), h[8 * Pn:].view("<i4")


def fwd(q_loc: torch.Tensor, k: torch.Tensor, v: torch.Tensor, bits: torch.Tensor,
        blocks: torch.Tensor, block: int, scale: Optional[float] = None, stream=None,
        ws: Optional[torch.Tensor] = None, out=None):
    """mmattn_fwd.  q_loc [n_loc,Hq,D], k/v [S,Hkv,D] bf16; blocks int32.
    Returns (o_loc bf16 [n_loc,Hq,D], lse fp32 [Hq,n_loc])."""
    n_loc, Hq, D = q_loc.shape
    S, Hkv, _ = k.shape
    n_blocks = blocks.numel()
    scale = float(D) ** -0.5 if scale is None else float(scale)
    if out is None:
        o = torch.empty_like(q_loc)
        lse = torch.empty((Hq, n_loc), dtype=torch.float32, device=q_loc.device)
    else:
        o, lse = out
    if ws is None:
        ws = _workspace(workspace_size(OP_FWD, S, n_blocks, block, Hq, Hkv, D), q_loc.device)
    rc = lib().mmattn_fwd(_ptr(q_loc), _ptr(k), _ptr(v), _ptr(bits), _ptr(blocks), n_blocks, block,
                          S, Hq, Hkv, D, scale, BF16, _ptr(o), _ptr(lse), _ptr(ws), ws.numel(),
                          _stream(stream))
    _check("mmattn_fwd", rc)
    return o, lse


STATIC_SCRATCH_BYTES = 32 << 20


def fwd_static(q_loc, k, v, bits, blocks, block: int, out, scale: Optional[float] = None, stream=None):
    """mmattn_fwd_static: the forward on the library's own per-GPU scratch array;
    `out` = (o_loc, lse) must be given, nothing is allocated here or in the call."""
    n_loc, Hq, D = q_loc.shape
    S, Hkv, _ = k.shape
    scale = float(D) ** -0.5 if scale is None else float(scale)
    o, lse = out
    rc = lib().mmattn_fwd_static(_ptr(q_loc), _ptr(k), _ptr(v), _ptr(bits), _ptr(blocks), blocks.numel(),
                                 block, S, Hq, Hkv, D, scale, BF16, _ptr(o), _ptr(lse), _stream(stream))
    _check("mmattn_fwd_static", rc)
    return o, lse


def fwd_heads(q_loc, k, v, bits, blocks, block: int, kv_head_begin: int, kv_head_count: int,
              plan_ready: bool, out, ws: torch.Tensor, scale: Optional[float] = None, stream=None):
    """mmattn_fwd_heads: the forward for a window of KV heads, written into the
    window's heads of out = (o_loc, lse); ws from workspace_size(OP_FWD_HEADS, ...)."""
    n_loc, Hq, D = q_loc.shape
    S, Hkv, _ = k.shape
    scale = float(D) ** -0.5 if scale is None else float(scale)
    o, lse = out
    rc = lib().mmattn_fwd_heads(_ptr(q_loc), _ptr(k), _ptr(v), _ptr(bits), _ptr(blocks), blocks.numel(),
                                block, S, Hq, Hkv, D, scale, BF16, kv_head_begin, kv_head_count,
                                int(bool(plan_ready)), _ptr(o), _ptr(lse), _ptr(ws), ws.numel(),
                                _stream(stream))
    _check("mmattn_fwd_heads", rc)
    return o, lse


def fwd_staged(q_loc, k_src, v_src, k_stage, v_stage, bits, blocks, block: int, heads_per_stage: int,
               copy_stream, out=None, ws: Optional[torch.Tensor] = None, scale: Optional[float] = None,
               stream=None):
    """mmattn_fwd_staged: forward with K/V copied window by window on copy_stream
    while the windows already copied are attended on `stream`."""
    n_loc, Hq, D = q_loc.shape
    S, Hkv, _ = k_src.shape
    scale = float(D) ** -0.5 if scale is None else float(scale)
    if out is None:
        out = (torch.empty_like(q_loc), torch.empty((Hq, n_loc), dtype=torch.float32, device=q_loc.device))
    if ws is None:
        ws = _workspace(workspace_size(OP_FWD_HEADS, S, blocks.numel(), block, Hq, Hkv, D), q_loc.device)
    rc = lib().mmattn_fwd_staged(_ptr(q_loc), _ptr(k_src), _ptr(v_src), _ptr(k_stage), _ptr(v_stage),
                                 _ptr(bits), _ptr(blocks), blocks.numel(), block, S, Hq, Hkv, D, scale,
                                 BF16, heads_per_stage, _ptr(out[0]), _ptr(out[1]), _ptr(ws), ws.numel(),
                                 _stream(copy_stream), _stream(stream))
    _check("mmattn_fwd_staged", rc)
    for t in (k_src, v_src, k_stage, v_stage):
        t.record_stream(copy_stream)
    return out


def bwd(q_loc, k, v, bits, blocks, block: int, o_loc, lse, do_loc, scale: Optional[float] = None,
        stream=None, ws: Optional[torch.Tensor] = None, out=None):
    """mmattn_bwd -> (dq_loc [n_loc,Hq,D], dk [S,Hkv,D], dv [S,Hkv,D]) bf16."""
    n_loc, Hq, D = q_loc.shape
    S, Hkv, _ = k.shape
    n_blocks = blocks.numel()
    scale = float(D) ** -0.5 if scale is None else float(scale)
    if out is None:
        dq, dk, dv = torch.empty_like(q_loc), torch.empty_like(k), torch.empty_like(v)
    else:
        dq, dk, dv = out
    if ws is None:
        ws = _workspace(workspace_size(OP_BWD, S, n_blocks, block, Hq, Hkv, D), q_loc.device)
    rc = lib().mmattn_bwd(_ptr(q_loc), _ptr(k), _ptr(v), _ptr(bits), _ptr(blocks), n_blocks, block,
                          S, Hq, Hkv, D, scale, BF16, _ptr(o_loc), _ptr(lse), _ptr(do_loc),
                          _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), ws.numel(), _stream(stream))
    _check("mmattn_bwd", rc)
    return dq, dk, dv


STAGE_FWD, STAGE_DKV, STAGE_DQ, STAGE_DKV_REDUCE = 0, 1, 2, 3


def mfma_ceiling(iters: int, random_operands: bool, sink: torch.Tensor, stream=None) -> float:
    """mmattn_mfma_ceiling: enqueues the matrix-pipe-only kernel; returns its flop count."""
    fl = ctypes.c_double(0.0)
    rc = lib().mmattn_mfma_ceiling(int(iters), int(bool(random_operands)), _ptr(sink),
                                   sink.numel() * sink.element_size(), ctypes.byref(fl), _stream(stream))
    _check("mmattn_mfma_ceiling", rc)
    return fl.value


def stage_events(stage: int, ev_start: int, ev_stop: int):
    """mmattn_stage_events: raw hipEvent_t handles (0, 0 clears)."""
    _check("mmattn_stage_events", lib().mmattn_stage_events(stage, ev_start, ev_stop))


def bf16_from_bits(bits_u16: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 patterns (host) -> bf16 tensor on the device."""
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16))
    return t.to(device).view(torch.bfloat16)
