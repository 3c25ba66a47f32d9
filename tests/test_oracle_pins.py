"""Pins of the CPU oracle to things other than itself (all run without a GPU).

Each test names what fixes the expected value: a library routine, a closed
form, brute force, exact rational arithmetic, or a separately written block.
"""
import ctypes as C
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import ndtr

import oracle_api as O
from float_swin_ref import float_block, sqnr_db
from paper_2507_19131_amd import synth

L = O.lib()


def _arr_fn(fn, v):
    v = np.ascontiguousarray(v, dtype=np.float32)
    out = np.empty_like(v)
    fn(v.ctypes.data_as(O._FP), out.ctypes.data_as(O._FP), C.c_int64(v.size))
    return out


# ---------------------------------------------------------------- scalar arithmetic
def test_exp2_pinned_against_libm():
    y = np.linspace(-100.0, 0.0, 2_000_001).astype(np.float32)
    got = _arr_fn(L.orc_exp2_array, y).astype(np.float64)
    ref = np.exp2(y.astype(np.float64))
    assert np.max(np.abs(got / ref - 1.0)) <= 3e-7
    assert L.orc_exp2(0.0) == pytest.approx(1.0, abs=2e-7)
    # below the clamp the value of -100 is held (absolute error < 1e-30)
    assert L.orc_exp2(-1000.0) == L.orc_exp2(-100.0) < 1e-30
    # exact powers of two scale exactly
    assert L.orc_exp2(-3.0) == L.orc_exp2(0.0) / 8.0


def test_gelu_pinned_against_erf_form():
    x = np.linspace(-12.0, 12.0, 2_400_001).astype(np.float32)
    got = _arr_fn(L.orc_gelu_array, x).astype(np.float64)
    ref = x.astype(np.float64) * ndtr(x.astype(np.float64))
    assert np.max(np.abs(got - ref)) <= 5e-7          # half an ulp of the result at |x| >= 4 is 2.4e-7
    near = np.abs(x) <= 1.0
    assert np.max(np.abs(got[near] - ref[near])) <= 1.2e-7
    assert L.orc_gelu(0.0) == 0.0
    big = np.array([20.0, 1e3, 1e6, -20.0, -1e3, -1e6], dtype=np.float32)
    g = _arr_fn(L.orc_gelu_array, big)
    assert np.all(np.abs(g[:3] - big[:3]) <= 1e-6) and np.all(np.abs(g[3:]) <= 1e-6)


def _q_exact(v, scale, z, bits):
    """Exact rational evaluation of the quantizer definition."""
    inv = np.float32(1.0) / np.float32(scale)
    t = Fraction(float(np.float32(v))) * Fraction(float(inv)) + z
    fl = t.numerator // t.denominator
    fr = t - fl
    n = fl + 1 if fr > Fraction(1, 2) else fl if fr < Fraction(1, 2) else (fl if fl % 2 == 0 else fl + 1)
    return int(min(max(n, -(1 << (bits - 1))), (1 << (bits - 1)) - 1))


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantizer_roundtrip_and_exact_rounding(bits):
    rng = np.random.default_rng(bits)
    qmin, qmax = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    for scale, z in ((0.0371, 0), (0.0033, -3 if bits > 2 else -1), (1.7, qmin), (2.0 ** -6, 1)):
        scale = float(np.float32(scale))
        lo, hi = scale * (qmin - z), scale * (qmax - z)
        v = rng.uniform(lo, hi, size=4000).astype(np.float32)
        v = v[(v >= np.float32(lo)) & (v <= np.float32(hi))]
        q = np.array([L.orc_quantize(float(t), scale, z, bits) for t in v])
        assert q.min() >= qmin and q.max() <= qmax
        back = scale * (q - z)
        assert np.max(np.abs(v.astype(np.float64) - back)) <= scale / 2 * (1 + 2.0 ** -20)
        for t in v[:300]:
            assert L.orc_quantize(float(t), scale, z, bits) == _q_exact(t, scale, z, bits)
        # outside the clip range the code saturates
        assert L.orc_quantize(float(hi + 10 * scale), scale, z, bits) == qmax
        assert L.orc_quantize(float(lo - 10 * scale), scale, z, bits) == qmin
        assert L.orc_quantize(1e30, scale, z, bits) == qmax and L.orc_quantize(-1e30, scale, z, bits) == qmin
    # ties go to the even integer (scale 2^-6 makes v/scale exact)
    s = 2.0 ** -6
    assert L.orc_quantize(0.5 * s, s, 0, 8) == 0 and L.orc_quantize(1.5 * s, s, 0, 8) == 2
    assert L.orc_quantize(2.5 * s, s, 0, 8) == 2 and L.orc_quantize(-0.5 * s, s, 0, 8) == 0
    assert L.orc_quantize(2.5 * s, s, 1, 8) == 4       # the zero point is inside the rounding: 3.5 -> 4
    assert L.orc_quantize(1.5 * s, s, 1, 8) == 2 and L.orc_quantize(-1.5 * s, s, 3, 8) == 2


def test_layernorm_against_numpy():
    rng = np.random.default_rng(5)
    for Cc in (96, 128, 384):
        x = (rng.standard_normal(Cc) * rng.uniform(0.1, 30) + rng.uniform(-5, 5)).astype(np.float32)
        g = rng.uniform(0.3, 2, Cc).astype(np.float32)
        b = rng.standard_normal(Cc).astype(np.float32)
        y = np.empty(Cc, dtype=np.float32)
        L.orc_layernorm_token(x.ctypes.data_as(O._FP), Cc, g.ctypes.data_as(O._FP), b.ctypes.data_as(O._FP),
                              C.c_float(1e-5), y.ctypes.data_as(O._FP))
        xd = x.astype(np.float64)
        ref = (xd - xd.mean()) / np.sqrt(xd.var() + 1e-5) * g + b
        assert np.max(np.abs(y - ref)) <= 4e-6 * max(1.0, np.abs(ref).max())


def test_keep_count_values():
    # 0.4*1369 = 547.6 -> 548, 0.4*361 = 144.4 -> 144 (round half up of keep*nW)
    for nW, keep, k in ((1369, 0.4, 548), (361, 0.4, 144), (1392, 0.5, 696), (96, 0.25, 24), (96, 0.75, 72),
                        (64, 0.5, 32), (5, 0.5, 3), (10, 0.0, 0), (10, 1.0, 10)):
        assert O.keep_count(nW, keep) == k
    # round half up, per image, clamped: exact rational arithmetic on a sweep (ties at keep*nW = n + 1/2 included)
    for nW in (1, 2, 3, 5, 24, 49, 96, 361, 1369, 1392, 4096):
        for num in range(0, 21):
            want = (Fraction(num, 20) * nW + Fraction(1, 2)).__floor__()
            assert O.keep_count(nW, num / 20) == min(max(want, 0), nW), (nW, num)


# ---------------------------------------------------------------- geometry
SIZES = [(200, 336), (256, 256), (128, 128), (25, 42), (14, 14), (9, 30)]


@pytest.mark.parametrize("H,W", SIZES)
@pytest.mark.parametrize("shift", [0, 3])
def test_gather_is_pad_roll_partition(H, W, shift):
    """Window gather == numpy pad + roll(-s) + reshape partition; scatter inverts it."""
    spec = synth.BlockSpec(2, H, W, 4, 1, shift=shift)
    rng = np.random.default_rng(H * 1000 + W + shift)
    x = rng.standard_normal((2, H, W, 4)).astype(np.float32)
    nW = O.num_windows(spec)
    assert nW == spec.nW == (-(-H // 7)) * (-(-W // 7))
    perm = np.stack([rng.permutation(nW) for _ in range(2)]).astype(np.int32)
    win, valid = O.gather_windows(spec, x, perm)
    xp = np.zeros((2, spec.Hp, spec.Wp, 4), dtype=np.float32)
    xp[:, :H, :W] = x
    vp = np.zeros((2, spec.Hp, spec.Wp), dtype=np.uint8)
    vp[:, :H, :W] = 1
    xr, vr = np.roll(xp, (-shift, -shift), axis=(1, 2)), np.roll(vp, (-shift, -shift), axis=(1, 2))
    part = xr.reshape(2, spec.Hp // 7, 7, spec.Wp // 7, 7, 4).transpose(0, 1, 3, 2, 4, 5).reshape(2, nW, 49, 4)
    vpart = vr.reshape(2, spec.Hp // 7, 7, spec.Wp // 7, 7).transpose(0, 1, 3, 2, 4).reshape(2, nW, 49)
    exp = np.stack([part[b, perm[b]] for b in range(2)]).reshape(2 * nW, 49, 4)
    expv = np.stack([vpart[b, perm[b]] for b in range(2)]).reshape(2 * nW, 49)
    assert np.array_equal(win, exp) and np.array_equal(valid, expv)
    back = O.scatter_windows(spec, win, perm)
    assert np.array_equal(back, x)


def _swin_region_mask(Hp, Wp, ws, s):
    """Mask from region labels, the way the Swin reference builds it: [nW,49,49] bool (True = masked)."""
    img = np.zeros((Hp, Wp), dtype=np.int64)
    cnt = 0
    for hs in (slice(0, -ws), slice(-ws, -s), slice(-s, None)):
        for wsl in (slice(0, -ws), slice(-ws, -s), slice(-s, None)):
            img[hs, wsl] = cnt
            cnt += 1
    mw = img.reshape(Hp // ws, ws, Wp // ws, ws).transpose(0, 2, 1, 3).reshape(-1, ws * ws)
    return mw[:, :, None] != mw[:, None, :]


@pytest.mark.parametrize("H,W", [(14, 14), (14, 21), (21, 28), (26, 33), (9, 30)])
def test_shift_mask_matches_region_labelling(H, W):
    spec = synth.BlockSpec(1, H, W, 4, 1, shift=3)
    d = O.make_desc(spec)
    ref = _swin_region_mask(spec.Hp, spec.Wp, 7, 3)
    got = np.zeros_like(ref)
    for w in range(spec.nW):
        for i in range(49):
            for j in range(49):
                got[w, i, j] = L.orc_mask_pair(C.byref(d), w, i, j)
    assert np.array_equal(got, ref)
    d0 = O.make_desc(spec, shift=0)
    assert all(L.orc_mask_pair(C.byref(d0), w, i, 48 - i) == 0 for w in range(spec.nW) for i in range(49))


# ---------------------------------------------------------------- score / select
def test_score_modes_against_numpy_and_closed_form():
    spec = synth.BlockSpec(2, 20, 30, 32, 1, score_mode=0)
    inp = synth.make_block_inputs(spec, 3)
    x = synth.make_feature_map(spec, 3, blobs=True)
    xp = np.zeros((2, spec.Hp, spec.Wp, 32))
    xp[:, :20, :30] = x
    ref = (xp ** 2).reshape(2, spec.Hp // 7, 7, spec.Wp // 7, 7, 32).sum(axis=(2, 4, 5)).reshape(2, -1)
    got = O.score_windows(inp, x)
    assert np.allclose(got, ref, rtol=1e-13, atol=0)
    # the score ignores the block's shift (un-shifted grid of the stage input)
    assert np.array_equal(got, O.score_windows(inp, x, shift=3))
    # mode 1 with gamma = 1, beta = 0: every token contributes C*var/(var+eps)
    spec1 = synth.BlockSpec(2, 20, 30, 32, 1, score_mode=1)
    inp1 = synth.make_block_inputs(spec1, 3)
    inp1.shared.score_gamma = np.ones(32, dtype=np.float32)
    inp1.shared.score_beta = np.zeros(32, dtype=np.float32)
    var = xp.var(axis=-1)
    contrib = 32 * var / (var + 1e-5)
    contrib[:, 20:, :] = 0
    contrib[:, :, 30:] = 0
    ref1 = contrib.reshape(2, spec.Hp // 7, 7, spec.Wp // 7, 7).sum(axis=(2, 4)).reshape(2, -1)
    assert np.allclose(O.score_windows(inp1, x), ref1, rtol=2e-6)


def test_selection_against_sort():
    rng = np.random.default_rng(11)
    for nW, k in ((1, 0), (1, 1), (17, 5), (96, 48), (360, 180), (50, 0), (50, 50)):
        sc = rng.standard_normal((3, nW))
        sc[1, ::3] = sc[1, 0]                       # ties
        sc[2] = 0.0                                 # all equal
        for reverse in (0, 1):
            perm = O.select_windows(sc, k, reverse)
            for b in range(3):
                key = sc[b] if reverse else -sc[b]
                order = np.lexsort((np.arange(nW), key))          # (score desc, index asc)
                assert np.array_equal(perm[b], order)
                assert np.array_equal(np.sort(perm[b]), np.arange(nW))
                if k and k < nW:                                  # every high score >= every low score
                    hi, lo = sc[b][perm[b, :k]], sc[b][perm[b, k:]]
                    assert (hi.min() <= lo.max()) if reverse else (hi.min() >= lo.max())


# ---------------------------------------------------------------- whole block
def _setup(H, W, Cc, heads, shift, seed, Bn=1, blobs=True, bits=(8, 4), wbits=8, **block_kw):
    spec = synth.BlockSpec(Bn, H, W, Cc, heads, shift=shift, act_bits_high=bits[0], act_bits_low=bits[1], weight_bits=wbits)
    return spec, synth.make_block_inputs(spec, seed, **block_kw), synth.make_feature_map(spec, seed, blobs=blobs)


@pytest.mark.parametrize("H,W,shift", [(28, 35, 0), (26, 33, 3), (14, 14, 3)])
@pytest.mark.parametrize("bits", [(8, 4), (4, 2)])
def test_keep_one_and_zero_equal_uniform_block(H, W, shift, bits):
    """keep 1.0 == uniform high-bit block, keep 0 == uniform low-bit block (separately written)."""
    spec, inp, x = _setup(H, W, 64, 2, shift, 21, Bn=2, bits=bits, wbits=bits[0])
    nW = spec.nW
    y_hi, _ = O.block_forward(inp, x, None, nW)
    y_lo, _ = O.block_forward(inp, x, None, 0)
    assert np.array_equal(y_hi, O.uniform_block(inp, x, 0))
    assert np.array_equal(y_lo, O.uniform_block(inp, x, 1))
    assert not np.array_equal(y_hi, y_lo)


def test_output_invariant_to_window_order():
    spec, inp, x = _setup(26, 33, 64, 2, 3, 22, Bn=2)
    nW, k = spec.nW, 7
    sc = O.score_windows(inp, x)
    perm = O.select_windows(sc, k)
    y0, _ = O.block_forward(inp, x, perm, k)
    rng = np.random.default_rng(0)
    perm2 = perm.copy()
    for b in range(2):
        perm2[b, :k] = rng.permutation(perm[b, :k])
        perm2[b, k:] = rng.permutation(perm[b, k:])
    y1, _ = O.block_forward(inp, x, perm2, k, threads=3)
    assert np.array_equal(y0, y1)
    y2, _ = O.block_forward(inp, x, None, k, threads=1)      # internal score+select == explicit
    assert np.array_equal(y0, y2)


@pytest.mark.parametrize("H,W,Cc,heads,shift", [(28, 35, 96, 3, 0), (26, 33, 96, 3, 3), (21, 21, 128, 4, 3)])
def test_close_to_float_swin_block(H, W, Cc, heads, shift):
    """The 8-bit block tracks a float Swin block (dense masked attention, libm erf)
    written separately; more low-bit windows can only lower the SQNR."""
    spec, inp, x = _setup(H, W, Cc, heads, shift, 7)
    nW = spec.nW
    sc = O.score_windows(inp, x)
    sq = []
    for k in (nW, nW // 2, 0):
        perm = O.select_windows(sc, k)
        y, _ = O.block_forward(inp, x, perm, k)
        brw = np.ones((1, nW), dtype=int)
        brw[0, perm[0, :k]] = 0
        yf = float_block(inp, x, brw)
        sq.append(sqnr_db(yf - x, y - x))          # on the block's own contribution
    assert sq[0] >= 28.0, sq
    assert sq[0] > sq[1] > sq[2] >= 5.0, sq


def test_per_branch_biases_follow_the_windows_branch():
    """PTQ variant (Sec. 4.3, PTQ setup): biases independent per branch.  With large, distinct biases the
    block tracks the float block that gives every window the biases of ITS branch, and is far from the
    float blocks a bias mix-up would produce (both branches reading the high set, the low set, or swapped)."""
    wide = {"a_q": (-4.0, 4.0), "a_k": (-4.0, 4.0), "a_v": (-4.0, 4.0), "a_proj_in": (-3.0, 3.0), "a_fc2_in": (-0.17, 4.0)}
    spec, inp, x = _setup(21, 28, 64, 2, 3, 27, bits=(8, 8), per_branch_bias=True, bias_std=0.5, ranges=wide)
    nW = spec.nW
    k = nW // 2
    perm = O.select_windows(O.score_windows(inp, x), k)
    y, _ = O.block_forward(inp, x, perm, k)
    brw = np.ones((1, nW), dtype=int)
    brw[0, perm[0, :k]] = 0
    good = sqnr_db(float_block(inp, x, brw) - x, y - x)
    import copy
    names = ("b_qkv", "b_proj", "b_fc1", "b_fc2")
    bad = []
    for mix in ("both_high", "both_low", "swapped"):
        wrong = copy.deepcopy(inp)
        for n in names:
            hi, lo = getattr(inp.branches[0], n), getattr(inp.branches[1], n)
            setattr(wrong.branches[0], n, lo if mix != "both_high" else hi)
            setattr(wrong.branches[1], n, hi if mix != "both_low" else lo)
        bad.append(sqnr_db(float_block(wrong, x, brw) - x, y - x))
    assert good >= 40.0, (good, bad)
    assert max(bad) <= 10.0, (good, bad)
    # one layer at a time: moving a single bias of the low branch to the high branch's values is seen
    for n in names:
        wrong = copy.deepcopy(inp)
        setattr(wrong.branches[1], n, getattr(inp.branches[0], n))
        assert sqnr_db(float_block(wrong, x, brw) - x, y - x) <= 25.0, n


def test_selection_with_scores_that_are_not_numbers():
    """A NaN score is ranked as the least important value in both directions; the list stays a permutation
    and the other windows keep their order."""
    rng = np.random.default_rng(12)
    sc = rng.standard_normal((2, 23))
    sc[0, [4, 17]] = np.nan
    sc[1, 0] = np.nan
    sc[1, 5] = np.inf
    for reverse in (0, 1):
        perm = O.select_windows(sc, 7, reverse)
        for b in range(2):
            assert np.array_equal(np.sort(perm[b]), np.arange(23))
            nan_idx = np.flatnonzero(np.isnan(sc[b]))
            assert np.array_equal(perm[b, 23 - len(nan_idx):], nan_idx)            # last, by index
            rest = perm[b, :23 - len(nan_idx)]
            key = sc[b][rest] if reverse else -sc[b][rest]
            assert np.all(np.diff(key) >= 0)
    # a NaN in the map: the quantizers saturate on it, so it survives only along the residual path, in place
    spec, inp, x = _setup(21, 21, 32, 1, 0, 28)
    x = x.copy()
    x[0, 8, 9, 3] = np.nan                                  # inside window 4 of the 3x3 grid
    s = O.score_windows(inp, x)
    assert np.isnan(s[0, 4]) and np.isnan(s).sum() == 1
    perm = O.select_windows(s, 4)
    assert perm[0, -1] == 4
    y, _ = O.block_forward(inp, x, perm, 4)
    assert np.array_equal(np.argwhere(np.isnan(y)), [[0, 8, 9, 3]])
    clean = x.copy()
    clean[0, 8, 9, 3] = 0.0
    yc, _ = O.block_forward(inp, clean, perm, 4)
    other = np.ones(y.shape, dtype=bool)
    other[0, 7:14, 7:14] = False                            # the other windows do not see it
    assert np.array_equal(y[other], yc[other])


def _rn32(fr):
    """Round a Fraction to the nearest binary32 (ties to even)."""
    f = np.float32(float(fr))                      # double rounding is repaired below
    cands = [f, np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))]
    best = min(cands, key=lambda c: (abs(Fraction(float(c)) - fr), int(np.float32(c).view(np.uint32)) & 1))
    return np.float32(best)


@pytest.mark.parametrize("per_branch_bias", [False, True])
def test_taps_stage_by_stage(per_branch_bias):
    """Every integer stage recomputed from the previous tap with int64 numpy;
    float->code stages re-evaluated exactly (rational arithmetic) on samples.  With per_branch_bias the
    low branch has biases of its own (Sec. 4.3, PTQ setup): each sample takes the bias of ITS branch."""
    spec, inp, x = _setup(19, 24, 64, 2, 3, 23, Bn=2, per_branch_bias=per_branch_bias, bias_std=0.05)
    if per_branch_bias:
        for n in ("b_qkv", "b_proj", "b_fc1", "b_fc2"):
            assert not np.array_equal(getattr(inp.branches[0], n), getattr(inp.branches[1], n))
    nW, k = spec.nW, 5
    perm = O.select_windows(O.score_windows(inp, x), k)
    y, t = O.block_forward(inp, x, perm, k, want_taps="all")
    S, Cc, nh, hd = 2 * nW, 64, 2, 32
    sh = inp.shared
    br_of_slot = np.array([0 if (g % nW) < k else 1 for g in range(S)])
    qp = lambda name: np.array([inp.branches[b].q[name] for b in br_of_slot])      # [S,2]
    i64 = lambda a: a.astype(np.int64)
    # int GEMMs with zero-point identity sum((a-z)w) = sum(aw) - z*sum(w)
    z = qp("a_qkv_in")[:, 1].astype(np.int64)[:, None, None]
    assert np.array_equal(i64(t["acc_qkv"]), (i64(t["a_qkv_in"]) - z) @ i64(sh.w_qkv).T)
    z = qp("a_proj_in")[:, 1].astype(np.int64)[:, None, None]
    assert np.array_equal(i64(t["acc_proj"]), (i64(t["a_proj_in"]) - z) @ i64(sh.w_proj).T)
    z = qp("a_fc1_in")[:, 1].astype(np.int64)[:, None, None]
    assert np.array_equal(i64(t["acc_fc1"]), (i64(t["a_fc1_in"]) - z) @ i64(sh.w_fc1).T)
    z = qp("a_fc2_in")[:, 1].astype(np.int64)[:, None, None]
    assert np.array_equal(i64(t["acc_fc2"]), (i64(t["a_fc2_in"]) - z) @ i64(sh.w_fc2).T)
    # attention integer products; channel n = which*C + head*hd + dim
    qkv = i64(t["qkv"]).reshape(S, 49, 3, nh, hd)
    s_ref = np.einsum("sihd,sjhd->shij", qkv[:, :, 0], qkv[:, :, 1])
    assert np.array_equal(i64(t["acc_s"]), s_ref)
    zp = qp("a_p")[:, 1].astype(np.int64)[:, None, None, None]
    o_ref = np.einsum("shij,sjhd->sihd", i64(t["p"]) - zp, qkv[:, :, 2]).reshape(S, 49, Cc)
    assert np.array_equal(i64(t["acc_o"]), o_ref)
    # |acc| bound: K <= 3072 and |a|,|w| <= 128 (+ zero-point shift <= 255) keeps int32 safe
    assert 3072 * 255 * 128 < 2 ** 31
    # y is the scatter of y_win; h - shortcut etc. sampled exactly
    assert np.array_equal(O.scatter_windows(spec, t["y_win"], perm), y)
    rng = np.random.default_rng(1)
    f32 = lambda v: Fraction(float(np.float32(v)))
    shortcut, _ = O.gather_windows(spec, x, perm)          # the gather is pinned to numpy pad/roll/reshape above
    for _ in range(400):
        g, tok = rng.integers(S), rng.integers(49)
        b = inp.branches[br_of_slot[g]]
        bits = spec.act_bits_high if br_of_slot[g] == 0 else spec.act_bits_low
        # qkv epilogue: f = fma(acc, s_a*s_w, bias) -> code
        n = rng.integers(3 * Cc)
        m = np.float32(b.q["a_qkv_in"][0]) * sh.s_qkv[n]
        f = _rn32(Fraction(int(t["acc_qkv"][g, tok, n])) * f32(m) + f32(b.b_qkv[n]))
        name = ("a_q", "a_k", "a_v")[n // Cc]
        assert t["qkv"][g, tok, n] == _q_exact(f, b.q[name][0], b.q[name][1], bits)
        # attention output: o * (s_p*s_v) -> code
        n = rng.integers(Cc)
        f = _rn32(Fraction(int(t["acc_o"][g, tok, n])) * f32(np.float32(b.q["a_p"][0]) * np.float32(b.q["a_v"][0])))
        assert t["a_proj_in"][g, tok, n] == _q_exact(f, *b.q["a_proj_in"], bits)
        # projection epilogue + first residual: h = rn32(rn32(acc*m + bias) + shortcut), shortcut 0 on padding
        f = _rn32(Fraction(int(t["acc_proj"][g, tok, n])) * f32(np.float32(b.q["a_proj_in"][0]) * sh.s_proj[n]) + f32(b.b_proj[n]))
        assert t["h"][g, tok, n] == _rn32(f32(f) + f32(shortcut[g, tok, n]))
        # fc2 epilogue + residual
        f = _rn32(Fraction(int(t["acc_fc2"][g, tok, n])) * f32(np.float32(b.q["a_fc2_in"][0]) * sh.s_fc2[n]) + f32(b.b_fc2[n]))
        assert t["y_win"][g, tok, n] == np.float32(f + t["h"][g, tok, n])
        # fc1 epilogue: GELU evaluated by the pinned routine (itself pinned to erf above)
        n = rng.integers(4 * Cc)
        f = _rn32(Fraction(int(t["acc_fc1"][g, tok, n])) * f32(np.float32(b.q["a_fc1_in"][0]) * sh.s_fc1[n]) + f32(b.b_fc1[n]))
        assert t["a_fc2_in"][g, tok, n] == _q_exact(L.orc_gelu(float(f)), *b.q["a_fc2_in"], bits)
    # LN1 + quantizer against float64 numpy on the gathered windows: codes may differ by one
    # only where the float64 value sits within 1e-4 of a rounding boundary
    win, valid = O.gather_windows(spec, x, perm)
    for g in rng.integers(S, size=6):
        b = inp.branches[br_of_slot[g]]
        bits = spec.act_bits_high if br_of_slot[g] == 0 else spec.act_bits_low
        w64 = win[g].astype(np.float64)
        ln = (w64 - w64.mean(-1, keepdims=True)) / np.sqrt(w64.var(-1, keepdims=True) + spec.ln_eps) * b.ln1_gamma + b.ln1_beta
        ln *= valid[g][:, None]
        s_, z_ = b.q["a_qkv_in"]
        tq = ln / s_
        ref = np.clip(np.rint(tq) + z_, -(1 << (bits - 1)), (1 << (bits - 1)) - 1)
        near_tie = np.abs(tq - np.floor(tq) - 0.5) < 1e-4
        assert np.all((ref == t["a_qkv_in"][g]) | near_tie)
        assert np.all(t["a_qkv_in"][g][valid[g] == 0] == np.clip(z_, -(1 << (bits - 1)), (1 << (bits - 1)) - 1))
        # LN2 + quantizer from the h tap, same rule
        h64 = t["h"][g].astype(np.float64)
        ln = (h64 - h64.mean(-1, keepdims=True)) / np.sqrt(h64.var(-1, keepdims=True) + spec.ln_eps) * b.ln2_gamma + b.ln2_beta
        s_, z_ = b.q["a_fc1_in"]
        tq = ln / s_
        ref = np.clip(np.rint(tq) + z_, -(1 << (bits - 1)), (1 << (bits - 1)) - 1)
        assert np.all((ref == t["a_fc1_in"][g]) | (np.abs(tq - np.floor(tq) - 0.5) < 1e-4))
        # logits -> softmax -> P codes from the integer scores, natural-base float64 softmax
        d = O.make_desc(spec)
        msk = np.array([[L.orc_mask_pair(C.byref(d), int(perm.reshape(-1)[g]), i, j) for j in range(49)] for i in range(49)])
        lgt = t["acc_s"][g].astype(np.float64) * (b.q["a_q"][0] * b.q["a_k"][0] / np.sqrt(hd)) + sh.rel_pos_bias - 100.0 * msk
        e = np.exp(lgt - lgt.max(-1, keepdims=True))
        tq = e / e.sum(-1, keepdims=True) / b.q["a_p"][0]
        ref = np.clip(np.rint(tq) + b.q["a_p"][1], -(1 << (bits - 1)), (1 << (bits - 1)) - 1)
        assert np.all((ref == t["p"][g]) | (np.abs(tq - np.floor(tq) - 0.5) < 2e-3))


def test_softmax_rows_and_masked_codes():
    rng = np.random.default_rng(2)
    lg = (rng.standard_normal((64, 49)) * 3).astype(np.float32)
    lg[:, 40:] -= np.float32(100 * 1.4426950408889634)
    for row in lg:
        p = np.empty(49, dtype=np.float32)
        L.orc_softmax2(row.ctypes.data_as(O._FP), 49, p.ctypes.data_as(O._FP))
        nat = row.astype(np.float64) * np.log(2.0)               # base-2 logits -> natural logits
        ref = np.exp(nat - nat.max())
        ref /= ref.sum()
        assert abs(float(p.astype(np.float64).sum()) - 1.0) <= 1e-6
        assert np.max(np.abs(p - ref)) <= 5e-7
        assert np.all(p[40:] < 1e-30)
    # a softmax does not change when every logit moves by the same amount: on a grid of 1/16 the differences to the
    # row maximum are exact in binary32, so the result must be the same bits, also far outside the range of 2^x
    grid = np.round(rng.standard_normal((16, 49)) * 48).astype(np.float32) / np.float32(16)
    for row in grid:
        base = np.empty(49, dtype=np.float32)
        L.orc_softmax2(row.ctypes.data_as(O._FP), 49, base.ctypes.data_as(O._FP))
        for offset in (-1000.0, 200.0, 1000.0):
            moved, p = (row + np.float32(offset)).astype(np.float32), np.empty(49, dtype=np.float32)
            assert np.array_equal((moved - np.float32(offset)), row)
            L.orc_softmax2(moved.ctypes.data_as(O._FP), 49, p.ctypes.data_as(O._FP))
            assert np.array_equal(p, base)
    # inside a block: every masked pair carries the code of probability zero
    spec, inp, x = _setup(14, 21, 32, 1, 3, 24)
    perm = O.select_windows(O.score_windows(inp, x), 3)
    _, t = O.block_forward(inp, x, perm, 3, want_taps=("p",))
    d = O.make_desc(spec)
    for g in range(spec.nW):
        zp = inp.branches[0 if g < 3 else 1].q["a_p"][1]
        m = np.array([[L.orc_mask_pair(C.byref(d), int(perm[0, g]), i, j) for j in range(49)] for i in range(49)], dtype=bool)
        assert np.all(t["p"][g, 0][m] == zp)
    assert m.any()


def test_error_codes():
    spec, inp, x = _setup(14, 14, 32, 1, 0, 25)
    d, sh, br = O.make_desc(spec), O.make_shared(inp.shared), O.make_branches(inp.branches)
    y = np.zeros_like(x)
    bad = O.make_desc(spec)
    bad.act_bits_low = 9
    assert L.orc_block_forward(C.byref(bad), C.byref(sh), br, x.ctypes.data_as(O._FP), None, 1, y.ctypes.data_as(O._FP), None, 1) == -3
    bad = O.make_desc(spec)
    bad.heads = 5
    assert L.orc_block_forward(C.byref(bad), C.byref(sh), br, x.ctypes.data_as(O._FP), None, 1, y.ctypes.data_as(O._FP), None, 1) == -2
    assert L.orc_block_forward(C.byref(d), C.byref(sh), br, None, None, 1, y.ctypes.data_as(O._FP), None, 1) == -1
    assert L.orc_block_forward(C.byref(d), C.byref(sh), br, x.ctypes.data_as(O._FP), None, 99, y.ctypes.data_as(O._FP), None, 1) == -2


# ---------------------------------------------------------------- activation pruning (Sec. 3.4)
def test_pruned_windows_are_forwarded_and_the_rest_unchanged():
    """Pruning the lowest-score windows: their features pass through untouched; the other windows
    give exactly what they give without pruning when the block is not shifted (windows are
    independent), and selection puts the lowest scores in the pruned group."""
    spec, inp, x = _setup(28, 35, 64, 2, 0, 31, Bn=2)
    nW, kh, kl = spec.nW, 6, 8
    sc = O.score_windows(inp, x)
    perm3 = O.select_windows(sc, kh, k_low=kl)
    for b in range(2):
        order = np.lexsort((np.arange(nW), -sc[b]))
        assert np.array_equal(perm3[b], order)
    y3, _ = O.block_forward(inp, x, perm3, kh, k_low=kl)
    # same high group, every other window low: the un-pruned reference
    perm2 = perm3.copy()
    perm2[:, kh:] = np.sort(perm3[:, kh:], axis=1)
    y2, _ = O.block_forward(inp, x, perm2, kh)
    win3, _ = O.gather_windows(spec, y3, perm3)
    win2, _ = O.gather_windows(spec, y2, perm3)
    winx, _ = O.gather_windows(spec, x, perm3)
    win3, win2, winx = (a.reshape(2, nW, 49, 64) for a in (win3, win2, winx))
    assert np.array_equal(win3[:, kh + kl:], winx[:, kh + kl:])            # forwarded
    assert np.array_equal(win3[:, :kh + kl], win2[:, :kh + kl])            # computed as before
    assert not np.array_equal(win2[:, kh + kl:], winx[:, kh + kl:])
    # k_low = nW - k_high is the plain block; everything pruned is the identity
    ya, _ = O.block_forward(inp, x, perm2, kh, k_low=nW - kh)
    assert np.array_equal(ya, y2)
    yi, _ = O.block_forward(inp, x, perm2, 0, k_low=0)
    assert np.array_equal(yi, x)


# ---------------------------------------------------------------- layers between stages
def _ln64(v, g, b, eps):
    m = v.mean(axis=-1, keepdims=True)
    var = ((v - m) ** 2).mean(axis=-1, keepdims=True)
    return (v - m) / np.sqrt(var + eps) * g + b


def _merge_concat(x):
    """Swin's patch merging gather written with numpy slicing (zero padding to even sizes)."""
    B, H, W, Cc = x.shape
    xp = np.pad(x, ((0, 0), (0, H % 2), (0, W % 2), (0, 0)))
    return np.concatenate([xp[:, 0::2, 0::2], xp[:, 1::2, 0::2], xp[:, 0::2, 1::2], xp[:, 1::2, 1::2]], axis=-1)


def _patches(img, P):
    """Non-overlapping PxP patches flattened in (row, column, channel) order, zero padded."""
    B, H, W, Cc = img.shape
    ip = np.pad(img, ((0, 0), (0, -H % P), (0, -W % P), (0, 0)))
    Ho, Wo = ip.shape[1] // P, ip.shape[2] // P
    return ip.reshape(B, Ho, P, Wo, P, Cc).transpose(0, 1, 3, 2, 4, 5).reshape(B, Ho, Wo, P * P * Cc)


@pytest.mark.parametrize("H,W", [(8, 12), (9, 11)])
def test_patch_merging_against_numpy(H, W):
    sp = synth.DownSpec(1, 2, H, W, 8, 32)
    inp = synth.make_downsample_inputs(sp, 5)
    x = np.random.default_rng(3).standard_normal((2, H, W, 8)).astype(np.float32)
    out, codes, acc = O.downsample_forward(inp, x, want_taps=True, threads=2)
    cat = _merge_concat(x.astype(np.float64)).reshape(-1, sp.K)
    assert out.shape == (2, (H + 1) // 2, (W + 1) // 2, 32)
    ln = _ln64(cat, inp.ln_gamma.astype(np.float64), inp.ln_beta.astype(np.float64), sp.ln_eps)
    s, z = inp.a_in
    # codes decode to the float64 LayerNorm within half a step (+ float32 rounding) inside the clip range
    lo, hi = s * (-128 - z), s * (127 - z)
    inside = (ln > lo) & (ln < hi)
    deq = s * (codes.astype(np.float64) - z)
    assert np.max(np.abs(deq - ln)[inside]) <= 0.5 * s * (1 + 1e-4) + 1e-6
    # integer sums: int64 matmul with the zero point removed
    ref = (codes.astype(np.int64) - z) @ inp.w.astype(np.int64).T
    assert np.array_equal(acc.astype(np.int64), ref)
    # output: dequantized sums (no bias, no LayerNorm after the linear)
    f = acc.astype(np.float64) * (np.float32(s) * inp.s_w).astype(np.float64)
    assert np.max(np.abs(out.reshape(-1, 32) - f)) <= 1e-6 * max(1.0, np.abs(f).max())
    # and close to the float layer it approximates
    wf = inp.w.astype(np.float64) * inp.s_w.astype(np.float64)[:, None]
    flt = ln @ wf.T
    assert sqnr_db(flt, out.reshape(-1, 32)) >= 25.0           # 8-bit codes; the clip range cuts the largest LayerNorm outputs


@pytest.mark.parametrize("H,W", [(16, 24), (18, 21)])
def test_patch_embedding_against_numpy(H, W):
    sp = synth.DownSpec(0, 1, H, W, 3, 32, patch=4)
    inp = synth.make_downsample_inputs(sp, 6)
    img = synth.make_image(1, H, W, 9)
    out, codes, acc = O.downsample_forward(inp, img, want_taps=True, threads=2)
    pt = _patches(img, 4).reshape(-1, 48)
    s, z = inp.a_in
    want = np.array([[_q_exact(v, s, z, 8) for v in row] for row in pt], dtype=np.int64)
    assert np.array_equal(codes.astype(np.int64), want)        # gather order and quantizer, exactly
    ref = (want - z) @ inp.w.astype(np.int64).T
    assert np.array_equal(acc.astype(np.int64), ref)
    f = ref.astype(np.float64) * (np.float32(s) * inp.s_w).astype(np.float64) + inp.bias.astype(np.float64)
    ln = _ln64(f, inp.ln_gamma.astype(np.float64), inp.ln_beta.astype(np.float64), sp.ln_eps)
    assert np.max(np.abs(out.reshape(-1, 32) - ln)) <= 2e-5 * max(1.0, np.abs(ln).max())
