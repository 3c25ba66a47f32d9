// Host-only helpers around the block (no GPU work): the equivalent-activation-bit / BOPs cost
// model of the paper's appendix "Calculation of Equivalent Activation Bits", and the uniform-sum
// compression-ratio sampling of Algorithm 1 (appendix "Uniform-sum Compression Ratio Sampling").
#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/mixaq.h"

namespace mixaq { int fail(int code, const char* fmt, ...); }
using mixaq::fail;

extern "C" {

int mixaq_equivalent_act_bits(int32_t n_pairs, const double* gmacs, double c_gmacs, const double* compress_ratio,
                              const double* prune_ratio, double act_bits_base, double* act_bits_eq)
{
    if (!gmacs || !compress_ratio || !act_bits_eq) return fail(MIXAQ_E_NULL, "gmacs, compress_ratio or act_bits_eq is NULL");
    if (n_pairs < 1 || !(c_gmacs >= 0.0) || !(act_bits_base > 0.0)) return fail(MIXAQ_E_SHAPE, "need n_pairs >= 1, c_gmacs >= 0, act_bits_base > 0");
    double num = c_gmacs, den = c_gmacs;
    for (int i = 0; i < n_pairs; ++i) {
        const double r = compress_ratio[i], p = prune_ratio ? prune_ratio[i] : 0.0;
        if (!(r >= 0.0) || !(p >= 0.0) || r + p > 1.0 || !(gmacs[i] >= 0.0))
            return fail(MIXAQ_E_SHAPE, "pair %d: ratios must be >= 0 with compress + prune <= 1, gmacs >= 0", i);
        num += (1.0 - p - 0.5 * r) * gmacs[i];       // a pruned window saves all, a low-bit window half of its cost
        den += gmacs[i];
    }
    if (!(den > 0.0)) return fail(MIXAQ_E_SHAPE, "total GMACs must be positive");
    *act_bits_eq = act_bits_base * num / den;
    return MIXAQ_OK;
}

int mixaq_bops_tera(double total_gmacs, double act_bits, double other_operand_bits, double* bops_tera)
{
    if (!bops_tera) return fail(MIXAQ_E_NULL, "bops_tera is NULL");
    if (!(total_gmacs >= 0.0) || !(act_bits > 0.0) || !(other_operand_bits > 0.0))
        return fail(MIXAQ_E_SHAPE, "need total_gmacs >= 0 and positive bit widths");
    *bops_tera = total_gmacs * 1e9 * act_bits * other_operand_bits / 1e12;
    return MIXAQ_OK;
}

}  // extern "C"

// Uniform-sum sampling (Algorithm 1 of the appendix) as an apportionment problem: `seats` tenths are
// to be shared among n pairs in proportion to exponential weights (normalised exponentials are a flat
// Dirichlet draw).  A draw whose largest share exceeds the cap is thrown away.  The accepted shares are
// turned into whole seats by Hamilton's method: everyone gets the whole part of the share, and the seats
// still free go, one at a time, to the largest fractional part not yet served (first index on ties).
namespace {
struct Apportion {
    std::vector<double> weight, share;
    std::vector<long> seat;
    explicit Apportion(int n) : weight(n), share(n), seat(n) {}
    // returns false when a share exceeds the cap
    bool shares(long seats, long cap)
    {
        double total = 0.0;
        for (double w : weight) total += w;
        if (!(total > 0.0)) return false;
        for (size_t i = 0; i < weight.size(); ++i) {
            share[i] = weight[i] / total * (double)seats;
            if (share[i] > (double)cap) return false;
        }
        return true;
    }
    void hamilton(long seats)
    {
        const size_t n = share.size();
        std::vector<double> frac(n);
        long given = 0;
        for (size_t i = 0; i < n; ++i) {
            seat[i] = (long)std::floor(share[i]);
            frac[i] = share[i] - (double)seat[i];
            given += seat[i];
        }
        for (; given < seats; ++given) {
            size_t best = n;
            for (size_t i = 0; i < n; ++i)
                if (frac[i] >= 0.0 && (best == n || frac[i] > frac[best])) best = i;
            if (best == n) break;                            // every pair served once: cannot happen, the fractions sum to the free seats
            seat[best] += 1;
            frac[best] = -1.0;                               // served
        }
    }
};
}  // namespace

static int sample_ratios(int32_t n, double s_min, double s_max, double upper, const double* uniforms, size_t n_uniforms,
                         size_t* n_used, double* ratios);

// No C++ exception leaves the library: host containers that fail to allocate become an error code.
extern "C" int mixaq_sample_ratios(int32_t n, double s_min, double s_max, double upper, const double* uniforms, size_t n_uniforms,
                                   size_t* n_used, double* ratios)
{
    try {
        return sample_ratios(n, s_min, s_max, upper, uniforms, n_uniforms, n_used, ratios);
    } catch (const std::bad_alloc&) {
        return fail(MIXAQ_E_HIP, "out of host memory while sampling %d ratios", n);
    } catch (...) {
        return fail(MIXAQ_E_HIP, "unexpected C++ exception while sampling");
    }
}

static int sample_ratios(int32_t n, double s_min, double s_max, double upper, const double* uniforms, size_t n_uniforms,
                         size_t* n_used, double* ratios)
{
    if (!uniforms || !ratios) return fail(MIXAQ_E_NULL, "uniforms or ratios is NULL");
    if (n < 1 || !(s_min >= 0.0) || !(s_max >= s_min) || !(upper > 0.0) || upper > 1.0)
        return fail(MIXAQ_E_SHAPE, "need n >= 1, 0 <= s_min <= s_max, 0 < upper <= 1");
    const long lo = std::lround(s_min * 10.0), hi = std::lround(s_max * 10.0), cap = std::lround(upper * 10.0);
    if (hi > (long)n * cap) return fail(MIXAQ_E_SHAPE, "s_max exceeds n*upper: the bound could never be met");
    if (n_uniforms < 1) return fail(MIXAQ_E_WORKSPACE, "no random numbers supplied");
    size_t next = 0;
    const long seats = std::min(std::max(lo + (long)std::floor(uniforms[next++] * (double)(hi - lo + 1)), lo), hi);
    Apportion ap(n);
    bool accepted = false;
    while (!accepted) {
        if (n_uniforms - next < (size_t)n) {
            if (n_used) *n_used = next;
            return fail(MIXAQ_E_WORKSPACE, "ran out of random numbers after %zu (rejection sampling still running)", next);
        }
        for (int i = 0; i < n; ++i) {
            const double u = uniforms[next++];
            ap.weight[i] = -std::log(u > 0.0 ? u : 1e-300);
        }
        accepted = ap.shares(seats, cap);
    }
    ap.hamilton(seats);
    for (int i = 0; i < n; ++i) ratios[i] = (double)ap.seat[i] / 10.0;
    if (n_used) *n_used = next;
    return MIXAQ_OK;
}

