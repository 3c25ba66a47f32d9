"""Runs one block on the GPU through the C ABI and on the CPU oracle, for the parity tests."""
import numpy as np
import torch

import oracle_api as O
from paper_2507_19131_amd import binding as M
from paper_2507_19131_amd import synth

INT_TAPS = ("a_qkv_in", "acc_qkv", "qkv", "acc_s", "p", "acc_o", "a_proj_in", "acc_proj", "a_fc1_in", "acc_fc1",
            "a_fc2_in", "acc_fc2")
FLOAT_TAPS = ("h", "y_win")


class GpuBlock:
    """A created block plus its workspace, destroyed on exit."""

    def __init__(self, inp, shift=None, fused=None):
        self.spec = inp.spec
        self.desc = M.make_desc(inp.spec, shift)
        self.shared, self.branches = M.to_device(inp)
        self.blk = M.mixaq_block_create(self.desc, self.shared, self.branches)
        if fused is not None:
            M.mixaq_block_set_fused(self.blk, fused)
        self.ws = M.alloc_workspace(self.blk)

    def close(self):
        if self.blk is not None:
            M.mixaq_block_destroy(self.blk)
            self.blk = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def score_select(self, x, k_high, reverse=0):
        spec = self.spec
        scores = torch.empty((spec.B, spec.nW), dtype=torch.float64, device=x.device)
        perm = torch.empty((spec.B, spec.nW), dtype=torch.int32, device=x.device)
        M.mixaq_score_windows(self.blk, x, scores)
        M.mixaq_select_windows(scores, spec.B, spec.nW, k_high, reverse, perm)
        return scores, perm

    def forward(self, x, perm, k_high, taps=None):
        y = torch.full_like(x, float("nan"))
        if taps is None:
            M.mixaq_block_forward(self.blk, x, perm, k_high, y, self.ws)
        else:
            M.mixaq_block_forward_taps(self.blk, x, perm, k_high, y, self.ws, taps)
        return y


def _forward_pruned(self, x, perm, k_high, k_low):
    y = torch.full_like(x, float("nan"))
    M.mixaq_block_forward_pruned(self.blk, x, perm, k_high, k_low, y, self.ws)
    return y


GpuBlock.forward_pruned = _forward_pruned


def compare_block(inp, x_np, k_high, shift=None, perm_np=None, taps="all", fused=None):
    """Oracle vs GPU on one block: returns a dict of mismatch counts / errors; asserts nothing."""
    spec = inp.spec
    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_np).to(dev)
    res = {}
    with GpuBlock(inp, shift, fused) as gb:
        g_scores, g_perm = gb.score_select(x, k_high)
        o_scores = O.score_windows(inp, x_np, shift)
        o_perm = O.select_windows(o_scores, k_high)
        res["score_rel_err"] = float(np.max(np.abs(g_scores.cpu().numpy() - o_scores) / np.maximum(np.abs(o_scores), 1e-300)))
        res["perm_mismatch"] = int((g_perm.cpu().numpy() != o_perm).sum())
        perm_use = o_perm if perm_np is None else perm_np
        perm_t = torch.from_numpy(np.ascontiguousarray(perm_use, dtype=np.int32)).to(dev)
        gt = M.alloc_taps(spec, taps) if taps else None
        y = gb.forward(x, perm_t, k_high, gt)
        torch.cuda.synchronize()
        y_np = y.cpu().numpy()
        oy, ot = O.block_forward(inp, x_np, perm_use, k_high, shift, want_taps=taps if taps else ())
        for n in INT_TAPS:
            if gt and n in gt:
                res[n] = int((gt[n].cpu().numpy() != ot[n]).sum())
        rms = float(np.sqrt(np.mean(oy.astype(np.float64) ** 2)))
        for n in FLOAT_TAPS:
            if gt and n in gt:
                res[n + "_maxabs"] = float(np.max(np.abs(gt[n].cpu().numpy().astype(np.float64) - ot[n])))
        res["y_nan"] = int(np.isnan(y_np).sum())
        res["y_maxabs"] = float(np.nanmax(np.abs(y_np.astype(np.float64) - oy)))
        res["y_rms"] = rms
        res["y_bit_identical"] = bool(np.array_equal(y_np, oy))
        # internal score+select path (perm = NULL)
        if perm_np is None:
            y2 = gb.forward(x, None, k_high)
            torch.cuda.synchronize()
            res["y_internal_select_equal"] = bool(torch.equal(y, y2))
    return res


def assert_parity(res):
    """Bit-exact selection, codes and accumulators; floats within 1e-3 x RMS of the oracle output."""
    assert res["perm_mismatch"] == 0, res
    assert res["score_rel_err"] <= 1e-12, res
    for n in INT_TAPS:
        if n in res:
            assert res[n] == 0, (n, res)
    assert res["y_nan"] == 0, res
    tol = 1e-3 * res["y_rms"]
    assert res["y_maxabs"] <= tol, res
    for n in FLOAT_TAPS:
        if n + "_maxabs" in res:
            assert res[n + "_maxabs"] <= tol, res
    if "y_internal_select_equal" in res:
        assert res["y_internal_select_equal"], res
