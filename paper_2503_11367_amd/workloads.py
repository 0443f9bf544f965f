"""Seeded synthetic workloads: modality layouts and Q/K/V/dO tensors.

This module only *describes inputs*: where the bidirectional image/audio spans
and the packed-sample boundaries lie, and which random numbers fill the
tensors.  It contains none of the method's arithmetic (no mask predicate, no
tile counting, no balancing, no attention) and is the one module that both
the tests' oracle side and the GPU side draw their inputs from.

The layouts follow the three mask families of the paper's App. C (modality
tokens embedded among text, several embedded spans, multimodal packing) with
random placement and fixed per-modality token counts, and the five workload
shapes this repository is measured on.  Nothing here comes from a dataset.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

TEXT, IMAGE, AUDIO = 0, 1, 2


@dataclass
class Layout:
    """A sequence layout: bidirectional spans + packed-sample offsets."""
    S: int
    spans: List[Tuple[int, int, int]]          # (start, len, modality), sorted, disjoint
    sample_off: List[int]                      # n_samples+1 offsets, [0]=0, [-1]=S
    noncausal: List[int] = field(default_factory=list)   # per-span flag (0 = causal bit set)
    deny: List[int] = field(default_factory=list)        # per-span mask of modalities NOT attended
    nobidir: List[int] = field(default_factory=list)     # per-span flag (1 = no bidirectional term)
    window: List[int] = field(default_factory=list)      # per-span look-back window over the own modality (0 = none)

    def __post_init__(self):
        if not self.noncausal:
            self.noncausal = [0] * len(self.spans)
        if not self.deny:
            self.deny = [0] * len(self.spans)
        if not self.nobidir:
            self.nobidir = [0] * len(self.spans)
        if not self.window:
            self.window = [0] * len(self.spans)

    def span_flags(self) -> List[int]:
        """Per-span flag words of the C ABI: bit 0 non-causal, bit 1 no
        bidirectional term, bits 8-15 deny mask, bits 16-31 look-back window
        (as a signed 32-bit value, the type of the flags field)."""
        out = []
        for n, u, d, w in zip(self.noncausal, self.nobidir, self.deny, self.window):
            f = int(n) | (int(u) << 1) | (int(d) << 8) | (int(w) << 16)
            out.append(f - (1 << 32) if f >= (1 << 31) else f)
        return out


@dataclass
class Workload:
    name: str
    layout: Layout
    Hq: int
    Hkv: int
    D: int
    N_B: int          # balancer block size (tokens)
    P: int            # virtual CP ranks
    tensor_seed: int


def _composition(rng: np.random.Generator, total: int, parts: int, first_min: int = 0) -> List[int]:
    """Uniform random composition of `total` into `parts` non-negative integers
    (stars and bars); the first part is at least `first_min`."""
    total -= first_min
    cuts = np.sort(rng.integers(0, total + 1, size=parts - 1))
    edges = np.concatenate(([0], cuts, [total]))
    out = np.diff(edges).astype(np.int64).tolist()
    out[0] += first_min
    return out


def _interleave(gaps: List[int], span_lens: List[Tuple[int, int]], base: int = 0):
    """text gap, span, text gap, span, ..., text gap  ->  span tuples."""
    assert len(gaps) == len(span_lens) + 1
    pos = base + gaps[0]
    spans = []
    for (n, mod), g in zip(span_lens, gaps[1:]):
        spans.append((pos, n, mod))
        pos += n + g
    return spans, pos


def layout_tiny() -> Layout:
    """S=512: text[0:64], one image span [64:320], text[320:512]."""
    return Layout(512, [(64, 256, IMAGE)], [0, 512])


def layout_vlm(seed: int = 1002) -> Layout:
    """S=8192: T I T I T I T I with four 1024-token image spans; text lengths
    are integers in [256,1792] summing to 4096 (three drawn uniformly, the
    fourth is the remainder; redraw until the fourth is in range)."""
    rng = np.random.default_rng(seed)
    while True:
        t = rng.integers(256, 1793, size=3).tolist()
        last = 4096 - sum(t)
        if 256 <= last <= 1792:
            t.append(int(last))
            break
    spans, pos = [], 0
    for n_text in t:
        pos += n_text
        spans.append((pos, 1024, IMAGE))
        pos += 1024
    assert pos == 8192
    return Layout(8192, spans, [0, 8192])


def layout_vision_audio(seed: int = 1003) -> Layout:
    """S=32768: six 2048-token image spans and four 1500-token audio spans in
    seeded random order; the 14480 text tokens are a uniform random
    composition into the 11 gaps, the first gap holding at least one token."""
    rng = np.random.default_rng(seed)
    span_lens = [(2048, IMAGE)] * 6 + [(1500, AUDIO)] * 4
    order = rng.permutation(len(span_lens))
    span_lens = [span_lens[i] for i in order]
    n_text = 32768 - 6 * 2048 - 4 * 1500
    gaps = _composition(rng, n_text, len(span_lens) + 1, first_min=1)
    spans, pos = _interleave(gaps, span_lens)
    assert pos == 32768
    return Layout(32768, spans, [0, 32768])


def layout_long(seed: int = 1004) -> Layout:
    """S=131072: 24 image spans of 4096 tokens at seeded random offsets; the
    32768 text tokens are a random composition into 25 gaps (first >= 1)."""
    rng = np.random.default_rng(seed)
    span_lens = [(4096, IMAGE)] * 24
    gaps = _composition(rng, 131072 - 24 * 4096, 25, first_min=1)
    spans, pos = _interleave(gaps, span_lens)
    assert pos == 131072
    return Layout(131072, spans, [0, 131072])


def layout_packed(seed: int = 1005, S: int = 65536, n_samples: int = 16,
                  min_len: int = 64, span_lo: int = 576, span_hi: int = 2304) -> Layout:
    """Multimodal packing: `n_samples` samples whose lengths are a Dirichlet(1)
    draw scaled to sum to S (each at least `min_len`, largest-remainder
    rounding); each sample holds 1-3 image spans of span_lo..span_hi tokens,
    trailing spans dropped until they fit with at least one leading text
    token; the text of a sample is a random composition into its gaps."""
    rng = np.random.default_rng(seed)
    w = rng.dirichlet(np.ones(n_samples))
    free = S - n_samples * min_len
    raw = w * free
    lens = np.floor(raw).astype(np.int64)
    rem = free - int(lens.sum())
    order = np.argsort(-(raw - lens), kind="stable")
    lens[order[:rem]] += 1
    lens += min_len
    assert int(lens.sum()) == S
    spans, offs, pos = [], [0], 0
    for L in lens.tolist():
        n_sp = int(rng.integers(1, 4))
        sl = rng.integers(span_lo, span_hi + 1, size=n_sp).tolist()
        while sl and sum(sl) > L - 1:
            sl.pop()
        gaps = _composition(rng, L - sum(sl), len(sl) + 1, first_min=1)
        sp, end = _interleave(gaps, [(n, IMAGE) for n in sl], base=pos)
        assert end == pos + L
        spans += sp
        pos += L
        offs.append(pos)
    return Layout(S, spans, offs)


def layout_random(seed: int, S: int, n_samples: int = 1, max_spans: int = 4,
                  noncausal_prob: float = 0.0, deny_prob: float = 0.0) -> Layout:
    """Small randomised layout for parity sweeps: ragged, tile-unaligned spans."""
    rng = np.random.default_rng(seed)
    if n_samples > 1:
        cuts = np.sort(rng.choice(np.arange(1, S), size=n_samples - 1, replace=False)).tolist()
    else:
        cuts = []
    offs = [0] + cuts + [S]
    spans, nc, dn = [], [], []
    for a, b in zip(offs[:-1], offs[1:]):
        L = b - a
        n_sp = int(rng.integers(0, max_spans + 1))
        sl = []
        for _ in range(n_sp):
            n = int(rng.integers(1, max(2, L // 2)))
            if sum(sl) + n <= L - 1:
                sl.append(n)
        gaps = _composition(rng, L - sum(sl), len(sl) + 1, first_min=1 if L > sum(sl) else 0)
        sp, _ = _interleave(gaps, [(n, int(rng.integers(1, 3))) for n in sl], base=a)
        spans += sp
        nc += [int(rng.random() < noncausal_prob) for _ in sp]
        if deny_prob > 0.0:
            # a denied set drawn from {text, image, audio}: bits 0..2
            dn += [int(rng.integers(1, 8)) if rng.random() < deny_prob else 0 for _ in sp]
        else:
            dn += [0 for _ in sp]
    return Layout(S, spans, offs, nc, dn)


def layout_shared_question(n_question: int, answer_lens: List[int], n_tail: int = 0) -> Layout:
    """One question followed by up to seven answers and optional trailing text
    (the "shared question" pattern of the paper's comparison with DCP): answer
    a is a span of modality a without the bidirectional term whose tokens
    attend the text modality and their own, i.e. the question and the earlier
    tokens of the same answer, never another answer."""
    assert 1 <= len(answer_lens) <= 7
    spans, deny, pos = [], [], n_question
    for a, n in enumerate(answer_lens, start=1):
        spans.append((pos, n, a))
        deny.append(0xFE & ~(1 << a))
        pos += n
    S = pos + n_tail
    return Layout(S, spans, [0, S], deny=deny, nobidir=[1] * len(spans))


def layout_lambda(sample_lens: List[int], n_sink: int, window: int) -> Layout:
    """Attention sinks plus a sliding window (the "lambda" pattern of the
    paper's comparison with DCP), per packed sample: the first n_sink tokens
    are a span of modality 1, the rest a span of modality 2 with the look-back
    window; neither has the bidirectional term.  A token then sees its
    sample's sinks and the last `window` tokens up to itself."""
    spans, win, off = [], [], [0]
    for L in sample_lens:
        assert L > n_sink >= 1
        spans += [(off[-1], n_sink, 1), (off[-1] + n_sink, L - n_sink, 2)]
        win += [0, window]
        off.append(off[-1] + L)
    return Layout(off[-1], spans, off, nobidir=[1] * len(spans), window=win)


def layout_short_spans(seed: int, S: int = 1024) -> Layout:
    """Hundreds of spans of 1-3 tokens with alternating modalities, random deny
    masks and 0-2 text tokens between them: nearly every key starts a new run of
    equal mask fields."""
    rng = np.random.default_rng(seed)
    spans, deny, pos = [], [], 1
    while pos + 8 < S:
        n = int(rng.integers(1, 4))
        spans.append((pos, n, 1 + len(spans) % 3))
        deny.append(int(rng.integers(0, 2)) << int(rng.integers(0, 4)))
        pos += n + int(rng.integers(0, 3))
    return Layout(S, spans, [0, S], deny=deny)


def layout_block_causal(S: int, block: int) -> Layout:
    """Causal blockwise pattern read from its name: bidirectional inside each
    block of `block` tokens, causal across blocks (every block is a span)."""
    spans = [(a, min(block, S - a), IMAGE) for a in range(0, S, block)]
    return Layout(S, spans, [0, S])


def workload(c: int) -> Workload:
    """The five measured workloads (1-based)."""
    if c == 1:
        return Workload("tiny", layout_tiny(), 1, 1, 64, 64, 4, 2001)
    if c == 2:
        return Workload("vlm_8k", layout_vlm(), 32, 8, 128, 128, 1, 2002)
    if c == 3:
        return Workload("vision_audio_32k", layout_vision_audio(), 32, 8, 128, 128, 4, 2003)
    if c == 4:
        return Workload("long_128k", layout_long(), 32, 8, 128, 128, 8, 2004)
    if c == 5:
        return Workload("packed_64k", layout_packed(), 64, 8, 128, 128, 8, 2005)
    raise ValueError(f"no workload {c}")


# ---------------------------------------------------------------- tensors ---

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def normal_bf16(seed: int, shape) -> np.ndarray:
    """N(0,1) drawn in fp32 then rounded once to bf16; returns uint16 patterns.
    Both the oracle (after widening to fp64) and the GPU see these values."""
    rng = np.random.default_rng(seed)
    return f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))
