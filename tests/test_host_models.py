"""Cost model and ratio sampler (host-only helpers): the paper's printed values are the pins,
the plain Python version in oracle/ is the second opinion for the library's C functions."""
import os

import numpy as np
import pytest

from oracle import host_models as H
from paper_2507_19131_amd import binding as M

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_bops_tables.txt")


def _golden():
    rows, gm, c, samp = [], None, None, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = line.split()
        if p[0] == "gmacs":
            gm = [float(v) for v in p[1:]]
        elif p[0] == "c_gmacs":
            c = float(p[1])
        elif p[0] == "sampler":
            samp = [float(v) for v in p[1:]]
        else:
            rows.append((float(p[0]), float(p[1]), None if p[2] == "-" else float(p[2])))
    return rows, gm, c, samp


def test_bops_match_the_printed_tables():
    rows, gm, c, _ = _golden()
    total = sum(gm) + c                                     # 86.36 GMACs
    assert total == pytest.approx(86.36, abs=1e-9)
    base = None
    for bits, bops, speed in rows:
        for fn in (H.bops_tera, M.mixaq_bops_tera):
            got = fn(total, bits, 32.0)
            tol = 2e-3 if float(bits).is_integer() else 1.5e-2      # weighted rows print a rounded bit width
            assert got == pytest.approx(bops, rel=tol), (bits, got, bops)
        if bits == 4:
            base = bops
        if speed is not None:
            assert base / bops == pytest.approx(speed, abs=0.011)
    assert M.mixaq_bops_tera(total, 3.3, 32.0) == H.bops_tera(total, 3.3, 32.0)


def test_equivalent_act_bits_closed_forms():
    _, gm, c, _ = _golden()
    share = sum(gm) / (sum(gm) + c)
    for fn in (H.equivalent_act_bits, M.mixaq_equivalent_act_bits):
        assert fn(gm, c, [0.0] * 6, None, 4.0) == pytest.approx(4.0, abs=1e-12)
        for r in (0.1, 0.5, 0.8):                          # uniform ratio: base*(1 - r/2 * share)
            assert fn(gm, c, [r] * 6, None, 4.0) == pytest.approx(4.0 * (1 - r / 2 * share), rel=1e-12)
        # pure pruning (the SparseViT rule of the appendix): base*(1 - r*share)
        assert fn(gm, c, [0.0] * 6, [0.3] * 6, 4.0) == pytest.approx(4.0 * (1 - 0.3 * share), rel=1e-12)
        # pruning 30 % and compressing the rest of a pair
        assert fn(gm, c, [0.5] * 6, [0.3] * 6, 4.0) == pytest.approx(4.0 * (1 - 0.55 * share), rel=1e-12)
    assert H.equivalent_act_bits(gm, c, [0.5] * 6, None, 4.0) == pytest.approx(3.0347, abs=5e-5)
    rng = np.random.default_rng(0)
    for _ in range(20):
        r = list(rng.integers(0, 9, 6) / 10.0)
        assert M.mixaq_equivalent_act_bits(gm, c, r, None, 4.0) == pytest.approx(H.equivalent_act_bits(gm, c, r, None, 4.0), rel=1e-14)
    with pytest.raises(M.MixaqError):
        M.mixaq_equivalent_act_bits(gm, c, [0.9] * 6, [0.3] * 6, 4.0)


def test_sampler_invariants_and_agreement():
    _, _, _, (n, upper, s_min, s_max, cost_lo, cost_hi) = _golden()
    n = int(n)
    # the printed sum range follows from the relative-cost range: (1-cost)*n*2
    assert (1 - cost_hi) * n * 2 == pytest.approx(s_min) and (1 - cost_lo) * n * 2 == pytest.approx(s_max)
    rng = np.random.default_rng(3)
    sums = []
    for _ in range(300):
        u = rng.uniform(1e-12, 1.0, size=1 + n * 200000)      # high sums reject many Dirichlet draws
        got, used = M.mixaq_sample_ratios(n, s_min, s_max, upper, u)
        ref, used_ref = H.sample_ratios(n, s_min, s_max, upper, u[:used].tolist())
        assert got == ref and used == used_ref
        tenths = np.rint(np.array(got) * 10)
        assert np.allclose(np.array(got) * 10, tenths, atol=1e-9)              # multiples of 0.1
        assert tenths.min() >= 0 and tenths.max() <= round(upper * 10)           # bounded
        target = round(s_min * 10) + int(np.floor(u[0] * (round(s_max * 10) - round(s_min * 10) + 1)))
        assert tenths.sum() == target                                           # the sum is kept exactly
        assert (used - 1) % n == 0
        sums.append(tenths.sum())
    # the sum is uniform on [6, 42], not bell-shaped: all of the range shows up
    assert min(sums) <= 8 and max(sums) >= 40
    with pytest.raises(M.MixaqError) as e:
        M.mixaq_sample_ratios(n, s_min, s_max, upper, [0.5, 0.1])
    assert e.value.code == -4 and "random numbers" in str(e.value)
    with pytest.raises(M.MixaqError):
        M.mixaq_sample_ratios(2, 1.0, 3.0, 0.8, [0.5] * 100)                   # sum can exceed n*upper
