"""GPU parity on randomly drawn small problems: sequence lengths that are
multiples of 128 but not powers of two, block sizes any multiple of 16 that
divides S, ragged and unsorted shares, 1 to 8 query heads per KV head (odd
counts included), both head dims, four mask families, three softmax scales.
Forward and backward through the C ABI against the float64 oracle, the usual
tolerances (O max-abs 2e-2 and relative L2 5e-3, LSE 4.5e-3, gradients
relative L2 1e-2)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2503_11367_amd import binding as mb
from paper_2503_11367_amd import workloads as wl

from gpu_util import DEV, bf16_to_f64, f64, fields, gpu_bits, make_tensors, max_abs, rel_l2, windows

pytestmark = pytest.mark.gpu


def draw(rng):
    S = int(rng.choice([128, 256, 384, 640, 896, 1024, 1536, 1920, 2048, 3072]))
    block = int(rng.choice([b for b in range(16, min(S, 512) + 1, 16) if S % b == 0]))
    nb = S // block
    take = int(rng.integers(1, min(nb, max(1, 1536 // block)) + 1))
    blocks = rng.permutation(nb)[:take].tolist()
    if rng.random() < 0.5:
        blocks = sorted(blocks)
    Hkv = int(rng.choice([1, 2, 3, 8]))
    Hq = Hkv * int(rng.choice([1, 2, 3, 4, 8]))
    if Hq > 16:
        Hq, Hkv = 16, 2
    D = int(rng.choice([64, 128]))
    kind = int(rng.integers(0, 4))
    seed = int(rng.integers(0, 100000))
    if kind == 0:
        lay = wl.layout_random(seed, S=S, n_samples=int(rng.integers(1, 5)), max_spans=6, noncausal_prob=0.2)
    elif kind == 1:
        lay = wl.layout_random(seed, S=S, n_samples=int(rng.integers(1, 3)), max_spans=8, noncausal_prob=0.3,
                               deny_prob=0.6)
    elif kind == 2:
        lay = wl.layout_lambda([S], int(rng.integers(1, 40)), int(rng.integers(1, S)))
    else:
        lay = wl.layout_block_causal(S, int(rng.choice([b for b in (32, 48, 64, 96, 128, 256) if b <= S])))
    scale = [None, 0.5 / np.sqrt(D), 3.0 / np.sqrt(D)][int(rng.integers(0, 3))]
    return lay, blocks, block, Hq, Hkv, D, seed, scale


@pytest.mark.parametrize("batch", range(4))
def test_random_shapes(batch):
    rng = np.random.default_rng(900 + batch)
    for case in range(12):
        lay, blocks, block, Hq, Hkv, D, seed, scale = draw(rng)
        what = dict(batch=batch, case=case, S=lay.S, block=block, blocks=blocks, Hq=Hq, Hkv=Hkv, D=D, scale=scale)
        f = fields(lay)
        t = make_tensors(seed, len(blocks) * block, lay.S, Hq, Hkv, D)
        bits = gpu_bits(lay)
        bl = torch.tensor(blocks, dtype=torch.int32, device=DEV)
        o, lse = mb.fwd(t["q"], t["k"], t["v"], bits, bl, block, scale=scale)
        dq, dk, dv = mb.bwd(t["q"], t["k"], t["v"], bits, bl, block, o, lse, t["do"], scale=scale)
        torch.cuda.synchronize()
        rows = oa.rows_of_blocks(blocks, block)
        Q, K, V, dO = f64(t["q_bits"]), f64(t["k_bits"]), f64(t["v_bits"]), f64(t["do_bits"])
        kw = dict(modality=f[3], attend=f[4], window=windows(lay), scale=scale)
        o_ref, lse_ref = oa.forward(Q, K, V, rows, f[0], f[1], f[2], **kw)
        dq_ref, dk_ref, dv_ref = oa.backward(Q, K, V, dO, rows, f[0], f[1], f[2], **kw)
        o_gpu, lse_gpu = bf16_to_f64(o), lse.cpu().numpy().astype(np.float64)
        assert np.isfinite(o_gpu).all(), what
        # a row that sees no key (non-causal span tokens can be such rows): LSE = -inf on both sides
        assert np.array_equal(np.isneginf(lse_gpu), np.isneginf(lse_ref)), what
        fin = np.isfinite(lse_ref)
        assert max_abs(o_gpu, o_ref) < 2e-2 and rel_l2(o_gpu, o_ref) < 5e-3, what
        assert not fin.any() or max_abs(lse_gpu[fin], lse_ref[fin]) < 4.5e-3, what
        for name, got, ref in (("dq", dq, dq_ref), ("dk", dk, dk_ref), ("dv", dv, dv_ref)):
            g = bf16_to_f64(got)
            assert np.isfinite(g).all(), (name, what)
            assert rel_l2(g, ref) < 1e-2, (name, rel_l2(g, ref), what)
