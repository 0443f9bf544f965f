"""mmattn_fwd_static, the forward for callers that cannot allocate: it must
give exactly what mmattn_fwd gives (same kernels, same plan, the library's own
per-GPU scratch array in place of the caller's workspace), also on a second
call with a smaller input that finds the first call's leftovers in the array."""
import pytest

from paper_2503_11367_amd import binding as mb

FAKE = 0x1000          # non-null, aligned, never dereferenced on an error path


def test_too_large_share_is_rejected_on_the_host():
    # two q-tiles of 8 heads against 8192 keys are cut into 64 list slices whose fp32 partial
    # results need 67 MiB: more than the static array holds
    S, nb, block, Hq, Hkv, D = 8192, 2, 128, 8, 8, 128
    assert mb.workspace_size(mb.OP_FWD, S, nb, block, Hq, Hkv, D) > mb.STATIC_SCRATCH_BYTES
    rc = mb.lib().mmattn_fwd_static(FAKE, FAKE, FAKE, FAKE, FAKE, nb, block, S, Hq, Hkv, D, 0.1, mb.BF16,
                                    FAKE, FAKE, 0)
    assert rc == -4
    # argument checks come first, as in mmattn_fwd
    assert mb.lib().mmattn_fwd_static(FAKE, 0, FAKE, FAKE, FAKE, nb, block, S, Hq, Hkv, D, 0.1, mb.BF16,
                                      FAKE, FAKE, 0) == -1
    assert mb.lib().mmattn_fwd_static(FAKE, FAKE, FAKE, FAKE, FAKE, nb, block, S, Hq, Hkv, 96, 0.1,
                                      mb.BF16, FAKE, FAKE, 0) == -3
    # an empty share needs no scratch at all
    assert mb.lib().mmattn_fwd_static(0, FAKE, FAKE, FAKE, 0, 0, block, S, Hq, Hkv, D, 0.1, mb.BF16,
                                      0, 0, 0) == 0


@pytest.mark.gpu
def test_two_calls_in_a_row_match_the_workspace_entry_point():
    import torch
    from paper_2503_11367_amd import workloads as wl
    from gpu_util import DEV, gpu_bits, make_tensors

    cases = [
        # 16 q-tiles x 32 head pairs: lists not cut, the scratch holds the plan only
        (wl.layout_random(30, S=2048, n_samples=1, max_spans=3), list(range(16)), 128, 64, 16, 128, 300),
        # few work items: every q-tile's list is cut into slices, 16 MiB of partial results in the scratch
        (wl.layout_random(31, S=1024, n_samples=2, max_spans=5), list(range(8)), 128, 4, 2, 128, 301),
        # smaller share, other head shape, unsorted block list; its slices land on the leftovers
        (wl.layout_random(32, S=1024, n_samples=1, max_spans=3), [5, 1, 6], 128, 2, 1, 64, 302),
    ]
    results = []
    for lay, blocks, block, Hq, Hkv, D, seed in cases:
        n_loc = len(blocks) * block
        t = make_tensors(seed, n_loc, lay.S, Hq, Hkv, D)
        bits = gpu_bits(lay)
        bl = torch.tensor(blocks, dtype=torch.int32, device=DEV)
        need = mb.workspace_size(mb.OP_FWD, lay.S, len(blocks), block, Hq, Hkv, D)
        assert need <= mb.STATIC_SCRATCH_BYTES
        ref = mb.fwd(t["q"], t["k"], t["v"], bits, bl, block)
        out = (torch.full_like(t["q"], float("nan")),
               torch.full((Hq, n_loc), float("nan"), dtype=torch.float32, device=DEV))
        results.append((t, bits, bl, block, ref, out))
    # the static calls back to back on one stream, each smaller than the one before
    for t, bits, bl, block, ref, out in results:
        mb.fwd_static(t["q"], t["k"], t["v"], bits, bl, block, out)
    torch.cuda.synchronize()
    for t, bits, bl, block, ref, out in results:
        assert torch.equal(out[0].view(torch.int16), ref[0].view(torch.int16))
        assert torch.equal(out[1].view(torch.int32), ref[1].view(torch.int32))
