"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from paper_2507_19131_amd import synth

pytestmark = pytest.mark.gpu

gh = pytest.importorskip("gpu_harness") if torch.cuda.is_available() else None
if torch.cuda.is_available():
    from paper_2507_19131_amd import binding as M

def _case(B, H, W, C, heads, shift, keep, seed, blobs=False, outliers=False, bits=(8, 4), wbits=8, ranges=None, mode=0,
          mlp_ratio=4, **block_kw):
    spec = synth.BlockSpec(B, H, W, C, heads, shift=shift, act_bits_high=bits[0], act_bits_low=bits[1],
                           weight_bits=wbits, score_mode=mode, mlp_ratio=mlp_ratio)
    inp = synth.make_block_inputs(spec, seed, ranges=ranges, **block_kw)
    x = synth.make_feature_map(spec, seed, blobs=blobs, outlier_channels=outliers)
    return spec, inp, x, M.mixaq_keep_count(spec.nW, keep)


SMALL = [
    # B, H, W, C, heads, shift, keep, seed, kwargs
    (1, 56, 56, 96, 3, 0, 0.5, 1001, {}),                                             # config 1
    (2, 26, 33, 96, 3, 3, 0.4, 11, dict(blobs=True)),                                 # padded + shifted + batch
    (2, 20, 27, 128, 4, 3, 0.4, 12, dict(outliers=True, ranges={"a_qkv_in": (-12.0, 13.5), "a_fc1_in": (-11.0, 10.0)})),
    (1, 14, 21, 192, 6, 3, 0.5, 13, dict(mode=1)),
    (2, 20, 28, 256, 8, 0, 0.3, 14, {}),
    (2, 50, 84, 384, 12, 3, 0.25, 1003, {}),                                          # config 3 block
    (1, 25, 42, 768, 24, 3, 0.5, 1004, dict(bits=(4, 2), wbits=4)),                   # config 4 stage 4
    (1, 30, 30, 96, 3, 3, 0.0, 15, {}),                                               # everything low
    (1, 30, 30, 96, 3, 3, 1.0, 16, {}),                                               # everything high
    (3, 15, 16, 96, 3, 0, 0.11, 17, dict(blobs=True)),                                # one high window per image
    (1, 28, 35, 96, 3, 3, 0.5, 18, dict(bits=(6, 3))),                                # odd bit widths
    (2, 21, 21, 128, 4, 3, 0.6, 19, dict(bits=(5, 2), wbits=4)),                      # 2-bit low branch, 4-bit weights
    (1, 7, 7, 96, 3, 0, 1.0, 20, {}),                                                 # a single window
    (1, 5, 6, 96, 3, 0, 0.0, 24, {}),                                                 # a map smaller than one window
    (2, 3, 20, 128, 4, 0, 0.5, 25, {}),                                               # one row of windows, mostly padding
    (3, 98, 98, 192, 6, 3, 0.5, 26, {}),                                              # 588 windows at six heads: one wave per head
    (2, 84, 91, 128, 4, 3, 0.5, 28, dict(bits=(8, 2))),                               # 312 windows at four heads: one wave per head, codes four per byte
    (2, 21, 28, 512, 16, 3, 0.4, 29, dict(bits=(7, 3))),                              # sixteen heads (FC2 with K = 2048), seven kernels
    (1, 14, 21, 1024, 32, 3, 0.5, 27, {}),                                            # the widest supported block (FC2 with K = 4096)
]


# both implementations where both exist: the fused kernels cover C <= 384, the seven-kernel path every width
BLOCK_CASES = [case + (fused,) for case in SMALL for fused in (True, False) if not (fused and case[3] > 384)]


@pytest.mark.parametrize("B,H,W,C,heads,shift,keep,seed,kw,fused", BLOCK_CASES)
def test_block_matches_oracle(B, H, W, C, heads, shift, keep, seed, kw, fused):
    """fused: the window and token kernels (C <= 384); otherwise the seven-kernel path."""
    spec, inp, x, k = _case(B, H, W, C, heads, shift, keep, seed, **kw)
    print("case", B, H, W, C, heads, shift, keep, seed, kw, "fused", fused, flush=True)
    res = gh.compare_block(inp, x, k, fused=fused)
    print(res, flush=True)
    gh.assert_parity(res)


BIAS_CASES = [(C, heads, bits, wbits, shift, fused)
              for (C, heads, bits, wbits) in [(96, 3, (8, 4), 8), (384, 12, (8, 4), 8), (768, 24, (4, 2), 4)]
              for shift in (0, 3) for fused in (True, False) if not (fused and C > 384)]


@pytest.mark.parametrize("C,heads,bits,wbits,shift,fused", BIAS_CASES)
def test_independent_biases_per_branch(C, heads, bits, wbits, shift, fused):
    """PTQ variant (Sec. 4.3, PTQ setup): the low branch has biases of its own, visibly different from the
    high branch's; every tap must follow the bias of the row's branch (both implementations up to C = 384, the
    seven-kernel path, the only one there, at C = 768)."""
    spec, inp, x, k = _case(2, 20, 27, C, heads, shift, 0.4, 51, blobs=True, bits=bits, wbits=wbits,
                            per_branch_bias=True, bias_std=0.1)
    for n in ("b_qkv", "b_proj", "b_fc1", "b_fc2"):
        assert not np.array_equal(getattr(inp.branches[0], n), getattr(inp.branches[1], n))
    print("independent biases", C, shift, "fused", fused, flush=True)
    res = gh.compare_block(inp, x, k, fused=fused)
    print(res, flush=True)
    gh.assert_parity(res)


@pytest.mark.parametrize("C,heads,mlp_ratio", [(96, 3, 3), (96, 3, 1), (192, 6, 3), (128, 4, 2), (96, 3, 8), (768, 24, 7)])
def test_other_mlp_ratios(C, heads, mlp_ratio):
    """FFN widths other than 4C run the seven-kernel path; hidden sizes that are not a whole number of
    ring turns of the GEMM (9 or 3 slabs of 32) included, and K = 5376, which goes through LDS in seven chunks of 768."""
    spec, inp, x, k = _case(2, 20, 27, C, heads, 3, 0.5, 52, blobs=True, mlp_ratio=mlp_ratio)
    print("mlp_ratio", mlp_ratio, "C", C, flush=True)
    res = gh.compare_block(inp, x, k)
    print(res, flush=True)
    gh.assert_parity(res)


def test_long_k_on_a_few_hundred_row_tiles():
    """FC2 with K = 3072 on 111 64-row tiles: the GEMM keeps the whole K of a 32-row tile in LDS (222 tiles)."""
    spec, inp, x, k = _case(2, 50, 60, 384, 12, 3, 0.5, 54, blobs=True, mlp_ratio=8)
    assert spec.B * spec.nW * 49 > 64 * 64
    print("long K on many tiles", flush=True)
    res = gh.compare_block(inp, x, k)
    print(res, flush=True)
    gh.assert_parity(res)


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("score_mode,value", [(0, float("nan")), (1, float("inf"))])
def test_window_whose_score_is_not_a_number(score_mode, value, fused):
    """A NaN in the map (or an Inf under the scoring LayerNorm) gives a NaN score: that window is ranked last,
    the list stays a permutation, every kernel exits normally and all other windows match the oracle."""
    import oracle_api as O
    spec, inp, x, k = _case(2, 28, 35, 96, 3, 0, 0.5, 53, blobs=True, mode=score_mode)
    x = x.copy()
    x[1, 9, 16, 5] = value                                 # window (1, 2) of image 1
    bad_w = 1 * 5 + 2
    dev = torch.device("cuda:0")
    xt = torch.from_numpy(x).to(dev)
    print("NaN score case", score_mode, value, "fused", fused, flush=True)
    with gh.GpuBlock(inp, fused=fused) as gb:
        scores, perm = gb.score_select(xt, k)
        y = gb.forward(xt, perm, k)
        y2 = gb.forward(xt, None, k)                       # selection inside the call
        torch.cuda.synchronize()
    o_scores = O.score_windows(inp, x)
    assert np.isnan(o_scores[1, bad_w]) and np.isnan(o_scores).sum() == 1
    g_scores = scores.cpu().numpy()
    assert np.array_equal(np.isnan(g_scores), np.isnan(o_scores))
    o_perm = O.select_windows(o_scores, k)
    assert np.array_equal(perm.cpu().numpy(), o_perm) and o_perm[1, -1] == bad_w
    oy, _ = O.block_forward(inp, x, o_perm, k)
    yn = y.cpu().numpy()
    other = np.ones(yn.shape, dtype=bool)
    other[1, 7:14, 14:21] = False
    assert np.array_equal(yn[other], oy[other])
    assert np.array_equal(np.isnan(yn), np.isnan(oy))
    fin = ~np.isnan(oy)
    assert np.array_equal(yn[fin], oy[fin])
    assert np.array_equal(np.isnan(y2.cpu().numpy()), np.isnan(oy)) and torch.equal(torch.nan_to_num(y), torch.nan_to_num(y2))


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("shift", [0, 3])
def test_config2_full_size(shift, fused):
    """Swin-T stage 1 at detection scale, the size the benchmark times."""
    spec, inp, x, k = _case(1, 200, 336, 96, 3, shift, 0.5, 1002, blobs=True)
    print("config 2 shift", shift, "fused", fused, flush=True)
    res = gh.compare_block(inp, x, k, fused=fused)
    print(res, flush=True)
    gh.assert_parity(res)


def test_maximum_window_count():
    """4096 windows per image is the most the selection handles (448x448 map, shifted); more is refused."""
    spec, inp, x, k = _case(1, 448, 448, 96, 3, 3, 0.5, 23, blobs=True)
    assert spec.nW == 4096
    print("maximum window count", flush=True)
    res = gh.compare_block(inp, x, k, taps=("a_proj_in", "a_fc2_in"))
    print(res, flush=True)
    gh.assert_parity(res)
    sh, br = M.to_device(inp)
    with pytest.raises(M.MixaqError) as e:
        M.mixaq_block_create(M.make_desc(synth.BlockSpec(1, 455, 448, 96, 3)), sh, br)
    assert e.value.code == -2


def test_order_invariance_and_reverse_selection():
    spec, inp, x, k = _case(2, 26, 33, 96, 3, 3, 0.4, 21, blobs=True)
    dev = torch.device("cuda:0")
    xt = torch.from_numpy(x).to(dev)
    import oracle_api as O
    with gh.GpuBlock(inp) as gb:
        scores, perm = gb.score_select(xt, k)
        y0 = gb.forward(xt, perm, k)
        rng = np.random.default_rng(0)
        p2 = perm.cpu().numpy().copy()
        for b in range(2):
            p2[b, :k] = rng.permutation(p2[b, :k])
            p2[b, k:] = rng.permutation(p2[b, k:])
        y1 = gb.forward(xt, torch.from_numpy(p2).to(dev), k)
        torch.cuda.synchronize()
        assert torch.equal(y0, y1)
        _, rperm = gb.score_select(xt, k, reverse=1)
        assert np.array_equal(rperm.cpu().numpy(), O.select_windows(scores.cpu().numpy(), k, 1))


def test_error_paths_do_not_launch():
    spec, inp, x, k = _case(1, 14, 14, 96, 3, 0, 0.5, 22)
    sh, br = M.to_device(inp)
    d = M.make_desc(spec)
    d.act_bits_low = 9
    with pytest.raises(M.MixaqError) as e:
        M.mixaq_block_create(d, sh, br)
    assert e.value.code == -3
    d = M.make_desc(spec)
    d.C = 100
    with pytest.raises(M.MixaqError) as e:
        M.mixaq_block_create(d, sh, br)
    assert e.value.code == -2
    d = M.make_desc(spec, shift=3)
    d.H = 7
    with pytest.raises(M.MixaqError):
        M.mixaq_block_create(d, sh, br)
    with gh.GpuBlock(inp) as gb:
        xt = torch.from_numpy(x).cuda()
        y = torch.empty_like(xt)
        small = torch.empty(1024, dtype=torch.uint8, device="cuda")
        with pytest.raises(M.MixaqError) as e:
            M.mixaq_block_forward(gb.blk, xt, None, k, y, small)
        assert e.value.code == -4
        with pytest.raises(M.MixaqError) as e:
            M.mixaq_block_forward(gb.blk, xt, None, 99, y, gb.ws)
        assert e.value.code == -2
        with pytest.raises(M.MixaqError) as e:
            M.mixaq_block_forward(gb.blk, xt, None, k, xt, gb.ws)
        assert e.value.code == -2
        # the stage call: x, y and tmp must be three separate maps; blocks of another shape are refused
        scores = torch.empty((1, spec.nW), dtype=torch.float64, device="cuda")
        perm = torch.empty((1, spec.nW), dtype=torch.int32, device="cuda")
        tmp = torch.empty_like(xt)
        for bad in ((xt, xt, tmp), (xt, y, y), (xt, y, xt)):
            with pytest.raises(M.MixaqError) as e:
                M.mixaq_stage_forward([gb.blk, gb.blk], bad[0], [k], None, bad[1], bad[2], scores, perm, gb.ws)
            assert e.value.code == -2
        with pytest.raises(M.MixaqError) as e:
            M.mixaq_stage_forward([gb.blk, gb.blk], xt, [spec.nW + 1], None, y, tmp, scores, perm, gb.ws)
        assert e.value.code == -2
        M.mixaq_stage_forward([gb.blk, gb.blk], xt, [k], None, y, tmp, scores, perm, gb.ws)      # and the good call still runs
        torch.cuda.synchronize()


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("shift,kh_frac,kl_frac", [(0, 0.3, 0.4), (3, 0.25, 0.5), (3, 0.0, 0.0), (0, 0.5, 0.0)])
def test_activation_pruning_matches_oracle(shift, kh_frac, kl_frac, fused):
    """Three-way split (Sec. 3.4): high, low, pruned windows; pruned features are forwarded."""
    import oracle_api as O
    spec, inp, x, _ = _case(2, 26, 33, 96, 3, shift, 0.5, 31, blobs=True)
    nW = spec.nW
    kh, kl = int(kh_frac * nW), int(kl_frac * nW)
    print("pruning case shift", shift, "k_high", kh, "k_low", kl, "fused", fused, flush=True)
    dev = torch.device("cuda:0")
    xt = torch.from_numpy(x).to(dev)
    with gh.GpuBlock(inp, fused=fused) as gb:
        scores = torch.empty((2, nW), dtype=torch.float64, device=dev)
        perm = torch.empty((2, nW), dtype=torch.int32, device=dev)
        M.mixaq_score_windows(gb.blk, xt, scores)
        M.mixaq_select_windows3(scores, 2, nW, kh, kl, 0, perm)
        y = torch.full_like(xt, float("nan"))
        M.mixaq_block_forward_pruned(gb.blk, xt, perm, kh, kl, y, gb.ws)
        y2 = torch.full_like(xt, float("nan"))
        M.mixaq_block_forward_pruned(gb.blk, xt, None, kh, kl, y2, gb.ws)          # internal three-way selection
        torch.cuda.synchronize()
    o_perm = O.select_windows(O.score_windows(inp, x), kh, k_low=kl)
    assert np.array_equal(perm.cpu().numpy(), o_perm)
    oy, _ = O.block_forward(inp, x, o_perm, kh, k_low=kl)
    assert np.array_equal(y.cpu().numpy(), oy)
    assert torch.equal(y, y2)


@pytest.mark.parametrize("C,heads", [(96, 3), (128, 4), (384, 12), (768, 24)])
@pytest.mark.parametrize("shift,kh_frac,kl_frac", [(0, 0.5, -1), (3, 0.25, 0.5), (3, 0.0, 0.0)])
def test_forward_from_scores_matches_oracle(C, heads, shift, kh_frac, kl_frac):
    """The selection taken inside the first kernel from the stage's scores (fused path) or by the
    select kernel (seven-kernel path, C = 768) gives the oracle's block output."""
    import oracle_api as O
    spec, inp, x, _ = _case(2, 26, 33, C, heads, shift, 0.5, 41, blobs=True)
    nW = spec.nW
    kh = int(kh_frac * nW)
    kl = -1 if kl_frac < 0 else int(kl_frac * nW)
    print("scored case", C, shift, kh, kl, flush=True)
    dev = torch.device("cuda:0")
    xt = torch.from_numpy(x).to(dev)
    with gh.GpuBlock(inp) as gb:
        scores = torch.empty((2, nW), dtype=torch.float64, device=dev)
        M.mixaq_score_windows(gb.blk, xt, scores)
        y = torch.full_like(xt, float("nan"))
        perm_out = torch.full((2, nW), -1, dtype=torch.int32, device=dev)
        M.mixaq_block_forward_scored(gb.blk, xt, scores, kh, kl, y, gb.ws, perm_out=perm_out)
        torch.cuda.synchronize()
    o_perm = O.select_windows(O.score_windows(inp, x), kh, k_low=None if kl < 0 else kl)
    assert np.array_equal(perm_out.cpu().numpy(), o_perm)
    oy, _ = O.block_forward(inp, x, o_perm, kh, k_low=None if kl < 0 else kl)
    assert np.array_equal(y.cpu().numpy(), oy)


@pytest.mark.parametrize("B,H,W,C,heads", [(1, 84, 84, 384, 12), (1, 161, 165, 192, 6), (3, 50, 57, 256, 8)])
def test_forward_from_scores_past_the_small_map_forms(B, H, W, C, heads):
    """The in-kernel selection in the kernel forms of larger maps: one twelve-head workgroup per window (more than
    128 windows at C = 384), one wave per head at C = 192 (more than 512 windows), eight heads; shifted block, pruning."""
    import oracle_api as O
    spec, inp, x, _ = _case(B, H, W, C, heads, 3, 0.5, 43, blobs=True)
    nW = spec.nW
    kh, kl = int(0.4 * nW), int(0.45 * nW)
    print("scored case", C, B * nW, "windows", flush=True)
    dev = torch.device("cuda:0")
    xt = torch.from_numpy(x).to(dev)
    with gh.GpuBlock(inp) as gb:
        scores = torch.empty((B, nW), dtype=torch.float64, device=dev)
        M.mixaq_score_windows(gb.blk, xt, scores)
        y = torch.full_like(xt, float("nan"))
        perm_out = torch.full((B, nW), -1, dtype=torch.int32, device=dev)
        M.mixaq_block_forward_scored(gb.blk, xt, scores, kh, kl, y, gb.ws, perm_out=perm_out)
        torch.cuda.synchronize()
    o_perm = O.select_windows(O.score_windows(inp, x), kh, k_low=kl)
    assert np.array_equal(perm_out.cpu().numpy(), o_perm)
    oy, _ = O.block_forward(inp, x, o_perm, kh, k_low=kl, threads=16)
    assert np.array_equal(y.cpu().numpy(), oy)


def test_equal_scores_are_ordered_by_window_index():
    """Windows with exactly equal scores (here: windows that are zero everywhere, and two copies of one
    window) must be ranked by their index on both sides; the block output follows."""
    spec, inp, x, _ = _case(2, 35, 42, 96, 3, 3, 0.5, 61, blobs=True)
    x = x.copy()
    x[:, 7:21, 14:35, :] = 0.0                       # six whole windows of the un-shifted grid, score 0
    x[:, 28:35, 0:7, :] = x[:, 0:7, 0:7, :]          # window 20 repeats window 0
    for k in (3, 12, 26):                            # the cut falls before, inside and after the tied windows
        print("tie case k_high", k, flush=True)
        res = gh.compare_block(inp, x, k, taps=("a_proj_in",))
        print(res, flush=True)
        gh.assert_parity(res)
        assert res["y_internal_select_equal"]


@pytest.mark.parametrize("case", range(8))
def test_random_shapes_and_precisions(case):
    """Seeded random draws of batch, map size (padding in both directions), width, shift, keep ratio and bit
    widths: every tap and the output against the oracle."""
    rng = np.random.default_rng(9000 + case)
    C, heads = [(96, 3), (128, 4), (192, 6), (256, 8)][int(rng.integers(0, 4))]
    B = int(rng.integers(1, 4))
    H, W = int(rng.integers(14, 40)), int(rng.integers(14, 40))
    shift = int(rng.integers(0, 2)) * 3
    keep = float(rng.choice([0.0, 0.2, 0.5, 0.8, 1.0]))
    hi = int(rng.integers(4, 9))
    lo = int(rng.integers(2, hi + 1))
    wbits = int(rng.choice([4, 8]))
    spec, inp, x, k = _case(B, H, W, C, heads, shift, keep, 9100 + case, blobs=bool(rng.integers(0, 2)), bits=(hi, lo), wbits=wbits,
                            mode=int(rng.integers(0, 2)))
    print("random case", case, B, H, W, C, shift, keep, hi, lo, wbits, flush=True)
    res = gh.compare_block(inp, x, k)
    print(res, flush=True)
    gh.assert_parity(res)


def test_random_sweep_of_small_blocks():
    """Forty more seeded draws in one test, wider than the cases above: maps from 7x7 up, C = 384 too, either
    implementation, shared or independent biases, outlier channels.  (A one-off run of 1800 such draws during
    development found no mismatch.)"""
    for case in range(40):
        rng = np.random.default_rng(31000 + case)
        C, heads = [(96, 3), (128, 4), (192, 6), (256, 8), (384, 12)][int(rng.choice([0, 0, 1, 2, 3, 4]))]
        B = int(rng.integers(1, 4))
        H, W = int(rng.integers(7, 46)), int(rng.integers(7, 46))
        shift = int(rng.integers(0, 2)) * 3
        if (H + 6) // 7 * 7 < 14 or (W + 6) // 7 * 7 < 14:
            shift = 0                                  # a shifted block needs a padded map of at least 14x14
        keep = float(rng.choice([0.0, 0.2, 0.5, 0.8, 1.0]))
        hi = int(rng.integers(4, 9))
        lo = int(rng.integers(2, hi + 1))
        fused = bool(rng.integers(0, 4) != 0)
        spec, inp, x, k = _case(B, H, W, C, heads, shift, keep, 31100 + case, blobs=bool(rng.integers(0, 2)),
                                outliers=bool(rng.integers(0, 3) == 0), bits=(hi, lo), wbits=int(rng.choice([4, 8])),
                                mode=int(rng.integers(0, 2)), per_branch_bias=bool(rng.integers(0, 2)))
        print("sweep case", case, B, H, W, C, shift, keep, hi, lo, "fused", fused, flush=True)
        res = gh.compare_block(inp, x, k, fused=fused)
        gh.assert_parity(res)


@pytest.mark.parametrize("kind", ["zeros", "constant_tokens", "huge", "denormal", "one_hot"])
def test_degenerate_inputs(kind):
    """Inputs at the edges of the float arithmetic: zero variance (rstd = 1/sqrt(eps)), saturated quantizers,
    binary32 denormals, a single non-zero channel."""
    spec, inp, x, k = _case(1, 21, 30, 96, 3, 3, 0.5, 71)
    rng = np.random.default_rng(72)
    if kind == "zeros":
        x = np.zeros_like(x)
    elif kind == "constant_tokens":
        x = np.repeat(rng.standard_normal(x.shape[:3] + (1,)).astype(np.float32), 96, axis=3)
    elif kind == "huge":
        x = (x * np.float32(3e4)).astype(np.float32)
    elif kind == "denormal":
        x = (x.astype(np.float64) * 1e-39).astype(np.float32)
        assert np.any((x != 0) & (np.abs(x) < 1.1754944e-38))
    else:
        x = np.zeros_like(x)
        x[..., 5] = rng.standard_normal(x.shape[:3]).astype(np.float32) * 10
    print("degenerate input", kind, flush=True)
    res = gh.compare_block(inp, np.ascontiguousarray(x), k)
    print(res, flush=True)
    assert res["perm_mismatch"] == 0 and res["y_nan"] == 0
    for n in gh.INT_TAPS:
        assert res[n] == 0, (n, res)
    assert res["y_bit_identical"], res
