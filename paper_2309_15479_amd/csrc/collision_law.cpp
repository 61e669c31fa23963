// Collision probabilities of E2LSH and FastLSH (Sec. 2.2, Eq. 2; Sec. 4.1, Eq. 9; Sec. 4.2),
// host code: the numbers a user needs to choose m and the bucket width.
//
// E2LSH: Eq. 2 integrates in closed form, with r = w / s,
//     p_w(s) = 2 Phi(r) - 1 - 2 / (sqrt(2 pi) r) * (1 - exp(-r^2 / 2)).
// FastLSH: the paper models the sampled squared distance s~^2 as N(mu~, sigma~^2) truncated to
// [0, inf) and reaches p(s, sigma) through the characteristic function of s~X and an inverse
// Fourier transform (Eq. 8, Eq. 9).  Given s~ the hash is an E2LSH hash of the sub-vector
// (Sec. 4.1), so the same number is the mixture E[p_w(s~)] over that truncated normal, which is
// what this file integrates: with u = s~,
//     p(s, sigma) = integral_0^inf p_w(u) * psi(u^2) * 2u du,
// psi the truncated normal density, by Gauss-Legendre panels over the part of [0, inf) where
// psi is not negligible.
#include <cmath>
#include <cstdint>

#include "lsh.h"

namespace {

const double kPi = 3.14159265358979323846;

double e2lsh_law(double s, double w) {
    if (!(s > 0.0)) return 1.0;  // identical projections always share a bucket
    const double r = w / s;
    return std::erf(r / std::sqrt(2.0)) - 2.0 / (std::sqrt(2.0 * kPi) * r) * (1.0 - std::exp(-0.5 * r * r));
}

// 1 - Phi(-mu/sigma) = Phi(mu/sigma): the mass the untruncated normal has on [0, inf)
double kept_mass(double mu, double sigma) { return 0.5 * std::erfc(-mu / (sigma * std::sqrt(2.0))); }

// 16-point Gauss-Legendre nodes and weights on [-1, 1] (positive half; the rule is symmetric)
const double kNode[8] = {0.0950125098376374401853193, 0.2816035507792589132304605, 0.4580167776572273863424194,
                         0.6178762444026437484466718, 0.7554044083550030338951012, 0.8656312023878317438804679,
                         0.9445750230732325760779884, 0.9894009349916499325961542};
const double kWeight[8] = {0.1894506104550684962853967, 0.1826034150449235888667637, 0.1691565193950025381893121,
                           0.1495959888165767320815017, 0.1246289712555338720524763, 0.0951585116824927848099251,
                           0.0622535239386478928628438, 0.0271524594117540948517806};

template <typename F>
double integrate_panels(F f, double lo, double hi, int panels) {
    const double h = (hi - lo) / panels;
    double total = 0.0;
    for (int p = 0; p < panels; ++p) {
        const double mid = lo + (p + 0.5) * h, half = 0.5 * h;
        double acc = 0.0;
        for (int i = 0; i < 8; ++i) acc += kWeight[i] * (f(mid - half * kNode[i]) + f(mid + half * kNode[i]));
        total += acc * half;
    }
    return total;
}

bool bad(double x) { return !(x > 0.0) || !std::isfinite(x); }

}  // namespace

extern "C" {

double lsh_equivalent_width(uint32_t n, uint32_t m, double w) {
    if (!n || !m) return 0.0;
    return w * std::sqrt((double)m / (double)n);
}

int lsh_e2lsh_collision_probability(double s, double w, double *p) {
    if (!p || !(s >= 0.0) || !std::isfinite(s) || bad(w)) return LSH_ERR_INVALID_ARG;
    *p = e2lsh_law(s, w);
    return LSH_OK;
}

int lsh_pair_statistics(const float *v, const float *u, uint32_t n, uint32_t m, double *mu_tilde,
                        double *sigma_tilde) {
    if (!v || !u || !n || !m || !mu_tilde || !sigma_tilde) return LSH_ERR_INVALID_ARG;
    double mean = 0.0;
    for (uint32_t i = 0; i < n; ++i) {
        const double d = (double)v[i] - (double)u[i];
        mean += d * d;
    }
    mean /= n;
    double var = 0.0;
    for (uint32_t i = 0; i < n; ++i) {
        const double d = (double)v[i] - (double)u[i];
        var += (d * d - mean) * (d * d - mean);
    }
    var /= n;
    *mu_tilde = m * mean;
    *sigma_tilde = std::sqrt(m * var);
    return LSH_OK;
}

int lsh_fastlsh_moment_factors(double mu_tilde, double sigma_tilde, double *epsilon, double *lambda) {
    if (!epsilon || !lambda || bad(mu_tilde) || !(sigma_tilde >= 0.0) || !std::isfinite(sigma_tilde))
        return LSH_ERR_INVALID_ARG;
    if (sigma_tilde == 0.0) {
        *epsilon = *lambda = 0.0;
        return LSH_OK;
    }
    const double ratio = sigma_tilde / mu_tilde;
    *epsilon = ratio * std::exp(-0.5 / (ratio * ratio)) / (std::sqrt(2.0 * kPi) * kept_mass(mu_tilde, sigma_tilde));
    *lambda = ratio * ratio + *epsilon;
    return LSH_OK;
}

int lsh_fastlsh_collision_probability(double mu_tilde, double sigma_tilde, double w, double *p) {
    if (!p || bad(mu_tilde) || bad(w) || !(sigma_tilde >= 0.0) || !std::isfinite(sigma_tilde))
        return LSH_ERR_INVALID_ARG;
    if (sigma_tilde < 1e-12 * mu_tilde) {  // no spread: s~ = sqrt(mu~)
        *p = e2lsh_law(std::sqrt(mu_tilde), w);
        return LSH_OK;
    }
    const double norm = 1.0 / (sigma_tilde * std::sqrt(2.0 * kPi) * kept_mass(mu_tilde, sigma_tilde));
    auto integrand = [&](double u) {
        const double z = (u * u - mu_tilde) / sigma_tilde;
        return e2lsh_law(u, w) * norm * std::exp(-0.5 * z * z) * 2.0 * u;
    };
    // psi is negligible (< 1e-40 of its peak) beyond 14 sigma~ from mu~
    const double y_lo = std::fmax(0.0, mu_tilde - 14.0 * sigma_tilde), y_hi = mu_tilde + 14.0 * sigma_tilde;
    *p = integrate_panels(integrand, std::sqrt(y_lo), std::sqrt(y_hi), 256);
    return LSH_OK;
}

int lsh_mips_collision_probability(double mu_tilde, double sigma_tilde, double delta, double w, double *p) {
    if (!(delta >= 0.0) || !std::isfinite(delta)) return LSH_ERR_INVALID_ARG;
    return lsh_fastlsh_collision_probability(mu_tilde + delta, sigma_tilde, w, p);
}

}  // extern "C"
