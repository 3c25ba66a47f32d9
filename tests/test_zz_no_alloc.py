"""The entry point that allocates nothing (mixaq_block_forward_static) against mixaq_block_forward:
same bits, two calls in a row on one GPU's static scratch, the second on a smaller map."""
import numpy as np
import pytest
import torch

from paper_2507_19131_amd import synth

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    import gpu_harness as gh
    from paper_2507_19131_amd import binding as M
    dev = torch.device("cuda:0")
    cases = [synth.BlockSpec(2, 61, 75, 96, 3, shift=3), synth.BlockSpec(1, 26, 33, 128, 4, shift=0)]   # the second is smaller
    blocks, outs = [], []
    try:
        for i, spec in enumerate(cases):
            inp = synth.make_block_inputs(spec, 700 + i)
            x = torch.from_numpy(synth.make_feature_map(spec, 700 + i, blobs=True)).to(dev)
            gb = gh.GpuBlock(inp)
            blocks.append(gb)
            k = M.mixaq_keep_count(spec.nW, 0.4)
            _, perm = gb.score_select(x, k)
            y_ref = gb.forward(x, perm, k)                                  # caller's workspace
            y_ref2 = gb.forward(x, None, k)
            torch.cuda.synchronize()
            outs.append((gb, x, perm, k, y_ref, y_ref2))
        # the static calls run back to back, nothing else in between
        got = []
        for gb, x, perm, k, _, _ in outs:
            print("static call", gb.spec.H, gb.spec.W, gb.spec.C, flush=True)
            y = torch.full_like(x, float("nan"))
            M.mixaq_block_forward_static(gb.blk, x, perm, k, y)
            y2 = torch.full_like(x, float("nan"))
            M.mixaq_block_forward_static(gb.blk, x, None, k, y2)            # scores and list live in the static scratch too
            got.append((y, y2))
        torch.cuda.synchronize()
        for (gb, x, perm, k, y_ref, y_ref2), (y, y2) in zip(outs, got):
            assert not torch.isnan(y).any() and torch.equal(y, y_ref)
            assert torch.equal(y2, y_ref2) and torch.equal(y2, y_ref)
        # limits: a map whose scratch exceeds the static array, and a block on the seven-kernel path
        big = synth.BlockSpec(4, 256, 256, 128, 4)
        inp = synth.make_block_inputs(big, 702)
        sh, br = M.to_device(inp)
        blk = M.mixaq_block_create(M.make_desc(big), sh, br)
        try:
            xb = torch.zeros((4, 256, 256, 128), device=dev)
            with pytest.raises(M.MixaqError) as e:
                M.mixaq_block_forward_static(blk, xb, None, 10, torch.empty_like(xb))
            assert e.value.code == -4 and "static scratch" in str(e.value)
        finally:
            M.mixaq_block_destroy(blk)
        gb = blocks[1]
        M.mixaq_block_set_fused(gb.blk, 0)
        with pytest.raises(M.MixaqError) as e:
            M.mixaq_block_forward_static(gb.blk, outs[1][1], None, 3, torch.empty_like(outs[1][1]))
        assert e.value.code == -2
    finally:
        for gb in blocks:
            gb.close()
