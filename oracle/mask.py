"""Mask predicate and 64-bit per-token bitfield (paper section 4.2, bitfield
attention mask; App. C mask families).

Per token t the layout gives
  sample(t)  index of the packed sample holding t (App. C, multimodal packing)
  span(t)    0 for text, else the 1-based id of the bidirectional span
  causal(t)  1 if the token attends to all of its previous tokens (the
             bitfield's most-significant "causal" bit, section 4.2)
  modality(t) 0 text / 1 image / 2 audio ...
and the predicate is
  vis(q,k) = [sample(q)=sample(k)] and
             ( [causal(q) and k<=q]  or  [span(q)!=0 and span(q)=span(k)] ).
Text is causal, a modality span is bidirectional within itself (and causal
to what precedes it when its causal bit is set), packed samples never see
each other.

Generalisation with the attend-set of section 4.2 (the word records which
modalities the token attends to): a span may be given a `deny` mask of
modalities its tokens do not attend; its attend-set is then all ones minus
those bits and the backward-looking term becomes
  [causal(q) and k<=q and attend(q) has bit modality(k)].
Tokens of the own span stay visible (same-span term).  With no deny masks
every attend-set is all ones and the predicate is the one above.

A span may also be marked `nobidir`: its tokens carry the modality and the
attend-set but span id 0, so only the backward-looking term applies to them.
This expresses the "shared question" pattern of the paper's comparison with
DCP (section 5.5 and its appendix): answers are nobidir spans of distinct modalities that attend
the text modality (the question) and their own.

A span may carry a look-back `window` W: among the earlier keys of the
span's own modality its tokens see only those with q - k < W (keys of other
modalities and the own-span term are not limited).  The "lambda" pattern of
the same comparison (a few leading sink tokens every later token keeps
attending, plus a sliding window) is then two nobidir spans per sample: the
sinks with one modality, the rest with another modality and the window.  The
paper names the pattern without giving its encoding; the window field
(bits 44-59 of the word) is this build's extension of the bitfield.

Word layout (LSB first, section 4.2: low bits = LLM and modality encoders,
bit 63 = causal bit):
  bits 0-7   attend-set, bit m set = may attend modality m   (all set here)
  bits 8-11  own modality index
  bits 12-27 span id (0 = none)
  bits 28-43 sample id
  bits 44-59 look-back window over keys of the own modality (0 = unlimited)
  bit 63     causal bit

Pins: tests/test_oracle_mask.py -- closed-form pair totals
sum L(L+1)/2 + sum n(n-1)/2, all-text = lower triangle, one span covering
everything = all ones, packed = block diagonal, the section-4.2 worked example
(encoder tokens without the causal bit see only their own encoder's tokens;
text tokens see every earlier token), encode/decode round trip; for the
attend-set generalisation a mask written out by hand and the pair count
(P1 count minus the denied backward pairs, counted by a separate loop); for
nobidir spans a shared-question mask written out by hand and its closed-form
pair count; for windows a lambda mask written out by hand, its closed-form
pair count, the mask built from the pattern's description, and window >=
length = no window; tests/test_oracle_attention.py checks that every
answer's rows equal plain causal attention over [question, that answer] and
that the lambda pattern equals the library routine with a band mask.
"""
import numpy as np

ATTEND_ALL = 0xFF
CAUSAL_BIT = 63


def token_fields(S, spans, sample_off, noncausal=None, deny=None, nobidir=None):
    """Expand a layout into per-token arrays (sample, span, causal, modality,
    attend).

    spans: iterable of (start, len, modality) in increasing start order.
    sample_off: n_samples+1 offsets with [0]=0 and [-1]=S.
    noncausal: optional per-span flag; 1 clears the causal bit of that span.
    deny: optional per-span 8-bit mask of modalities the span's tokens do not
          attend (cleared from their attend-set).
    nobidir: optional per-span flag; 1 leaves the span id of its tokens at 0
          (no bidirectional term; modality and attend-set still apply).
    """
    sample = np.zeros(S, dtype=np.int64)
    span = np.zeros(S, dtype=np.int64)
    causal = np.ones(S, dtype=np.int64)
    modality = np.zeros(S, dtype=np.int64)
    attend = np.full(S, ATTEND_ALL, dtype=np.int64)
    for i in range(len(sample_off) - 1):
        sample[sample_off[i]:sample_off[i + 1]] = i
    for j, (start, n, mod) in enumerate(spans):
        if nobidir is None or not nobidir[j]:
            span[start:start + n] = j + 1
        modality[start:start + n] = mod
        if noncausal is not None and noncausal[j]:
            causal[start:start + n] = 0
        if deny is not None and deny[j]:
            attend[start:start + n] = ATTEND_ALL & ~int(deny[j])
    return sample, span, causal, modality, attend


def token_windows(S, spans, window):
    """Per-token look-back window (0 = unlimited) from per-span windows."""
    w = np.zeros(S, dtype=np.int64)
    for (start, n, _mod), wj in zip(spans, window):
        w[start:start + n] = int(wj)
    return w


def visible(q_idx, k_idx, sample, span, causal, modality=None, attend=None, window=None):
    """Boolean matrix vis[q,k] for global token index arrays q_idx, k_idx.
    Without modality/attend every attend-set is taken as all ones; without
    window no token's look-back is limited."""
    q = np.asarray(q_idx)[:, None]
    k = np.asarray(k_idx)[None, :]
    same_sample = sample[q] == sample[k]
    back = (causal[q] == 1) & (k <= q)
    if attend is not None:
        back &= ((attend[q] >> modality[k]) & 1) == 1
    if window is not None:
        back &= (window[q] == 0) | (modality[q] != modality[k]) | (q - k < window[q])
    same_span = (span[q] != 0) & (span[q] == span[k])
    return same_sample & (back | same_span)


def encode(sample, span, causal, modality, attend=None, window=None):
    """Per-token 64-bit word from the fields, as uint64."""
    if attend is None:
        w = np.full(sample.shape, ATTEND_ALL, dtype=np.uint64)
    else:
        w = attend.astype(np.uint64)
    w |= modality.astype(np.uint64) << np.uint64(8)
    w |= span.astype(np.uint64) << np.uint64(12)
    w |= sample.astype(np.uint64) << np.uint64(28)
    if window is not None:
        w |= window.astype(np.uint64) << np.uint64(44)
    w |= causal.astype(np.uint64) << np.uint64(CAUSAL_BIT)
    return w


def decode(bits):
    """Inverse of encode: (sample, span, causal, modality, attend)."""
    b = np.asarray(bits, dtype=np.uint64)
    attend = (b & np.uint64(0xFF)).astype(np.int64)
    modality = ((b >> np.uint64(8)) & np.uint64(0xF)).astype(np.int64)
    span = ((b >> np.uint64(12)) & np.uint64(0xFFFF)).astype(np.int64)
    sample = ((b >> np.uint64(28)) & np.uint64(0xFFFF)).astype(np.int64)
    causal = ((b >> np.uint64(CAUSAL_BIT)) & np.uint64(1)).astype(np.int64)
    return sample, span, causal, modality, attend


def decode_window(bits):
    """The look-back window field of each word."""
    b = np.asarray(bits, dtype=np.uint64)
    return ((b >> np.uint64(44)) & np.uint64(0xFFFF)).astype(np.int64)
