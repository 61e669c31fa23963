"""CPU oracle for the collision probability of FastLSH (Sec. 4.1-4.2 of the paper).

TEST INFRASTRUCTURE, not the product: a slow restatement of the paper's derivation with
scipy quadrature, in the paper's order and notation.  It shares nothing with the library's
own calculator (csrc/collision_law.cpp), which reaches the same number by another route.

Model (Sec. 4.1): the sampled squared distance s~^2 follows the normal N(mu~, sigma~^2),
mu~ = m*mu, sigma~^2 = m*sigma^2, truncated to [0, inf); mu and sigma^2 are the mean and the
variance of the n squared coordinate differences (v_i - u_i)^2.  Then

  characteristic function of s~X (second lemma of Sec. 4.1)
      phi(x) = exp(x^4 sigma~^2 / 8 - mu~ x^2 / 2) * erfc((x^2 sigma~^2 / 2 - mu~) / (sqrt(2) sigma~))
               / (2 (1 - Phi(-mu~ / sigma~)))
  density by the inverse Fourier transform (Eq. 8)
      f(t) = 1/(2 pi) * integral exp(-i t x) phi(x) dx
  collision probability (theorem of Sec. 4.1, Eq. 9)
      p(s, sigma) = integral_0^w f_|s~X|(t) (1 - t/w) dt,   f_|s~X| = 2 f on t >= 0
  moments (lemma of Sec. 4.2)
      E[(s~X)^2] = mu~ (1 + eps),  E[(s~X)^4] = 3 mu~^2 (1 + lambda),
      eps = sigma~ exp(-mu~^2 / (2 sigma~^2)) / (sqrt(2 pi) mu~ (1 - Phi(-mu~/sigma~))),
      lambda = sigma~^2 / mu~^2 + eps

and for E2LSH (Sec. 2.2, Eq. 2)  p(s) = integral_0^w (1/s) f_|X|(t/s) (1 - t/w) dt.
"""
import math

import numpy as np
from scipy import integrate, special


def pair_statistics(v, u, m):
    """(mu~, sigma~) of a vector pair for sample size m: m times the mean, sqrt(m) times the
    standard deviation of the squared coordinate differences (Sec. 4.1, first paragraph)."""
    d2 = (np.asarray(v, np.float64) - np.asarray(u, np.float64)) ** 2
    mu = d2.mean()
    var = ((d2 - mu) ** 2).mean()
    return m * mu, math.sqrt(m * var)


def e2lsh_collision_probability(s, w):
    """Eq. 2 by numerical quadrature (f_|X| is the half-normal density)."""
    def integrand(t):
        z = t / s
        return (1.0 / s) * 2.0 * math.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi) * (1.0 - t / w)
    val, _ = integrate.quad(integrand, 0.0, w, epsabs=1e-13, epsrel=1e-12, limit=400)
    return val


def char_fn(x, mu_t, sigma_t):
    """phi_{s~X}(x), real and even.  exp(a) * erfc(z) is evaluated as exp(a - z^2) * erfcx(z)
    for z > 0 (a - z^2 = -mu~^2 / (2 sigma~^2), a constant), which avoids inf * 0."""
    x = np.asarray(x, np.float64)
    norm = 2.0 * (1.0 - 0.5 * special.erfc(mu_t / (sigma_t * math.sqrt(2.0))))   # 2 (1 - Phi(-mu~/sigma~))
    a = x ** 4 * sigma_t ** 2 / 8.0 - mu_t * x ** 2 / 2.0
    z = (0.5 * x ** 2 * sigma_t ** 2 - mu_t) / (math.sqrt(2.0) * sigma_t)
    pos = z > 0
    out = np.empty_like(x)
    out[pos] = math.exp(-mu_t ** 2 / (2.0 * sigma_t ** 2)) * special.erfcx(z[pos])
    out[~pos] = np.exp(a[~pos]) * special.erfc(z[~pos])
    return out / norm


def pdf(t, mu_t, sigma_t):
    """f_{s~X}(t), Eq. 8: (1/pi) * integral_0^inf cos(t x) phi(x) dx (phi is even)."""
    # beyond x0 the erfc argument is positive and phi falls off like 1/x^2: split there and let
    # the Fourier-weighted rule take the tail
    x0 = math.sqrt(2.0 * mu_t) / sigma_t * 2.0 + 10.0 / math.sqrt(mu_t)
    head, _ = integrate.quad(lambda x: math.cos(t * x) * float(char_fn(np.array([x]), mu_t, sigma_t)[0]),
                             0.0, x0, epsabs=1e-13, epsrel=1e-12, limit=2000)
    if t == 0.0:
        tail, _ = integrate.quad(lambda x: float(char_fn(np.array([x]), mu_t, sigma_t)[0]), x0, np.inf,
                                 epsabs=1e-13, epsrel=1e-12, limit=2000)
    else:
        # integral_{x0}^inf cos(t x) phi(x) dx, x = x0 + y
        c, _ = integrate.quad(lambda y: float(char_fn(np.array([x0 + y]), mu_t, sigma_t)[0]), 0.0, np.inf,
                              weight="cos", wvar=t, epsabs=1e-13, limit=2000)
        s_, _ = integrate.quad(lambda y: float(char_fn(np.array([x0 + y]), mu_t, sigma_t)[0]), 0.0, np.inf,
                               weight="sin", wvar=t, epsabs=1e-13, limit=2000)
        tail = math.cos(t * x0) * c - math.sin(t * x0) * s_
    return (head + tail) / math.pi


def fastlsh_collision_probability(mu_t, sigma_t, w):
    """p(s, sigma), Eq. 9, with f_|s~X| from Eq. 8 (nested quadrature: slow)."""
    val, _ = integrate.quad(lambda t: 2.0 * pdf(t, mu_t, sigma_t) * (1.0 - t / w), 0.0, w,
                            epsabs=1e-10, epsrel=1e-9, limit=200)
    return val


def moment_factors(mu_t, sigma_t):
    """(eps, lambda) of the moment lemma of Sec. 4.2."""
    tail = 1.0 - 0.5 * special.erfc(mu_t / (sigma_t * math.sqrt(2.0)))       # 1 - Phi(-mu~/sigma~)
    eps = sigma_t * math.exp(-mu_t ** 2 / (2.0 * sigma_t ** 2)) / (math.sqrt(2.0 * math.pi) * mu_t * tail)
    return eps, sigma_t ** 2 / mu_t ** 2 + eps
