"""Helpers shared by the GPU parity tests (inputs, oracle glue, error norms)."""
import numpy as np
import torch

from oracle import mask as om
from paper_2503_11367_amd import binding as mb
from paper_2503_11367_amd import workloads as wl

DEV = "cuda"


def fields(lay):
    return om.token_fields(lay.S, lay.spans, lay.sample_off, lay.noncausal, lay.deny, lay.nobidir)


def windows(lay):
    """Per-token look-back windows, or None when the layout has none (the
    oracle's functions take it as the keyword `window`)."""
    return om.token_windows(lay.S, lay.spans, lay.window) if any(lay.window) else None


def gpu_bits(lay):
    return mb.mask_encode(lay.spans, lay.sample_off, lay.S, device=DEV, flags=lay.span_flags())


def oracle_bits(lay):
    return om.encode(*fields(lay), window=windows(lay))


def to_np_u64(t):
    return t.cpu().numpy().view(np.uint64)


def make_tensors(seed, n_loc, S, Hq, Hkv, D):
    """bf16-rounded N(0,1) tensors: uint16 patterns on the host plus their
    float64 widenings (oracle inputs) and bf16 device copies (GPU inputs)."""
    out = {}
    for i, (name, shape) in enumerate((("q", (n_loc, Hq, D)), ("k", (S, Hkv, D)),
                                       ("v", (S, Hkv, D)), ("do", (n_loc, Hq, D)))):
        b = wl.normal_bf16(seed * 10 + i, shape)
        out[name + "_bits"] = b
        out[name] = mb.bf16_from_bits(b, DEV)
    return out


def f64(bits_u16):
    return wl.bf16_bits_to_f32(bits_u16).astype(np.float64)


def bf16_to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def rel_l2(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def max_abs(a, b):
    return float(np.abs(a - b).max())
