// Host-only helpers around the block (no GPU work): the equivalent-activation-bit / BOPs cost
// model of the paper's appendix "Calculation of Equivalent Activation Bits", and the uniform-sum
// compression-ratio sampling of Algorithm 1 (appendix "Uniform-sum Compression Ratio Sampling").
#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdint>
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

int mixaq_sample_ratios(int32_t n, double s_min, double s_max, double upper, const double* uniforms, size_t n_uniforms,
                        size_t* n_used, double* ratios)
{
    if (!uniforms || !ratios) return fail(MIXAQ_E_NULL, "uniforms or ratios is NULL");
    if (n < 1 || !(s_min >= 0.0) || !(s_max >= s_min) || !(upper > 0.0) || upper > 1.0)
        return fail(MIXAQ_E_SHAPE, "need n >= 1, 0 <= s_min <= s_max, 0 < upper <= 1");
    const long Smin = std::lround(s_min * 10.0), Smax = std::lround(s_max * 10.0), U = std::lround(upper * 10.0);
    if (Smax > (long)n * U) return fail(MIXAQ_E_SHAPE, "s_max exceeds n*upper: the bound could never be met");
    size_t pos = 0;
    if (n_uniforms < 1) return fail(MIXAQ_E_WORKSPACE, "no random numbers supplied");
    long S = Smin + (long)std::floor(uniforms[pos++] * (double)(Smax - Smin + 1));
    S = std::min(std::max(S, Smin), Smax);
    std::vector<double> r(n);
    for (;;) {                                           // rejection: every ratio at most the upper bound
        if (pos + (size_t)n > n_uniforms) {
            if (n_used) *n_used = pos;
            return fail(MIXAQ_E_WORKSPACE, "ran out of random numbers after %zu (rejection sampling still running)", pos);
        }
        double sum = 0.0;
        for (int i = 0; i < n; ++i) {                    // flat Dirichlet = normalised exponentials
            double u = uniforms[pos++];
            r[i] = -std::log(u > 0.0 ? u : 1e-300);
            sum += r[i];
        }
        bool ok = sum > 0.0;
        for (int i = 0; i < n && ok; ++i) { r[i] = r[i] / sum * (double)S; ok = r[i] <= (double)U; }
        if (ok) break;
    }
    std::vector<long> R(n);
    long acc = 0;
    for (int i = 0; i < n; ++i) { R[i] = (long)std::floor(r[i]); acc += R[i]; }
    long diff = S - acc;
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return (r[a] - (double)R[a]) > (r[b] - (double)R[b]); });
    for (long k = 0; k < diff && k < n; ++k) R[order[k]] += 1;   // largest remainder method
    for (int i = 0; i < n; ++i) ratios[i] = (double)R[i] / 10.0;
    if (n_used) *n_used = pos;
    return MIXAQ_OK;
}

}  // extern "C"
