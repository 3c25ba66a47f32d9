"""TEST INFRASTRUCTURE ONLY -- plain Python versions of the two host-side formulas of the paper's
appendix, used to check the library's host helpers.

equivalent_act_bits: appendix "Calculation of Equivalent Activation Bits" (ratios_i = 1 - r_i/2 for
MixA-Q, 1 - r_i for pruning; weighted by the GMACs of each pair of blocks plus the constant part).
sample_ratios: Algorithm 1, "Uniform-Sum Compression Ratio Sampling", with the random numbers
passed in (reading: the Dirichlet is flat, alpha = 1, which the paper does not state).
"""
import math


def equivalent_act_bits(gmacs, c_gmacs, compress, prune, base_bits):
    prune = prune if prune is not None else [0.0] * len(gmacs)
    kept = sum((1.0 - p - r / 2.0) * g for g, r, p in zip(gmacs, compress, prune))
    return base_bits * (kept + c_gmacs) / (sum(gmacs) + c_gmacs)


def bops_tera(total_gmacs, act_bits, other_bits=32.0):
    return total_gmacs * 1e9 * act_bits * other_bits / 1e12


def sample_ratios(n, s_min, s_max, upper, uniforms):
    """Returns (ratios, number of uniforms used)."""
    it = iter(uniforms)
    used = 0
    lo, hi, cap = round(s_min * 10), round(s_max * 10), round(upper * 10)
    target = lo + int(math.floor(next(it) * (hi - lo + 1)))
    used += 1
    target = min(max(target, lo), hi)
    while True:
        draw = []
        for _ in range(n):
            draw.append(-math.log(next(it)))
            used += 1
        total = 0.0
        for v in draw:
            total += v
        scaled = [v / total * target for v in draw]
        if all(v <= cap for v in scaled):
            break
    whole = [int(math.floor(v)) for v in scaled]
    missing = target - sum(whole)
    by_remainder = sorted(range(n), key=lambda i: -(scaled[i] - whole[i]))     # stable: ties keep index order
    for i in by_remainder[:missing]:
        whole[i] += 1
    return [w / 10.0 for w in whole], used
