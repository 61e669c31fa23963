"""Pins of the collision-probability oracle (oracle/collision_law.py) against what the paper
prints and what the model fixes independently of the characteristic-function route."""
import math
import os

import numpy as np
import pytest
from scipy import integrate, stats

from oracle import collision_law as law


def _p_closed(s, w):
    """Eq. 2 integrated in closed form: 2 Phi(r) - 1 - 2/(sqrt(2 pi) r) (1 - exp(-r^2/2)), r = w/s."""
    r = w / s
    return 2 * stats.norm.cdf(r) - 1 - 2 / (math.sqrt(2 * math.pi) * r) * (1 - math.exp(-r * r / 2))


def test_epsilon_matches_the_pairs_the_paper_prints(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "epsilon_lambda_table.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 15
    for name, which, m, eps, lam in rows:
        eps, lam = float(eps), float(lam)
        ratio = math.sqrt(lam - eps)                       # sigma~ / mu~
        got_eps, got_lam = law.moment_factors(1.0, ratio)
        assert abs(got_eps - eps) < 4e-6, (name, which, m, got_eps, eps)
        assert abs(got_lam - lam) < 4e-6
        # the factors depend on the ratio only
        e2, l2 = law.moment_factors(37.5, 37.5 * ratio)
        assert abs(e2 - got_eps) < 1e-12 and abs(l2 - got_lam) < 1e-12


@pytest.mark.parametrize("mu_t,sigma_t", [(4.0, 1.0), (1.0, 1.4)])
def test_density_is_normalised_and_has_the_stated_moments(mu_t, sigma_t):
    eps, lam = law.moment_factors(mu_t, sigma_t)
    top = 14.0 * math.sqrt(mu_t + 3 * sigma_t)
    ts = np.linspace(0.0, top, 401)
    f = np.array([law.pdf(t, mu_t, sigma_t) for t in ts])
    assert (f > -1e-9).all()
    total = 2 * integrate.simpson(f, x=ts)
    second = 2 * integrate.simpson(f * ts ** 2, x=ts)
    fourth = 2 * integrate.simpson(f * ts ** 4, x=ts)
    assert abs(total - 1.0) < 1e-6
    assert abs(second - mu_t * (1 + eps)) < 1e-5 * mu_t
    assert abs(fourth - 3 * mu_t ** 2 * (1 + lam)) < 1e-4 * mu_t ** 2


def test_e2lsh_quadrature_against_closed_form(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "e2lsh_collision_law.txt"))
            if ln.strip() and not ln.startswith("#")]
    for w, s, p in rows:
        assert abs(law.e2lsh_collision_probability(float(s), float(w)) - float(p)) < 1e-9
        assert abs(law.e2lsh_collision_probability(float(s), float(w)) - _p_closed(float(s), float(w))) < 1e-10


def test_small_sigma_reduces_to_e2lsh_at_the_sampled_distance():
    # sigma~ -> 0: s~ is the constant sqrt(mu~), so p(s, sigma) -> p_w(sqrt(mu~))  (Sec. 4.2)
    for mu_t, w in [(4.0, 4.0), (1.0, 1.5), (30.0, 4.0)]:
        got = law.fastlsh_collision_probability(mu_t, 0.01 * mu_t, w)
        assert abs(got - _p_closed(math.sqrt(mu_t), w)) < 2e-5


@pytest.mark.parametrize("mu_t,sigma_t,w", [(4.0, 1.0, 4.0), (9.0, 6.0, 4.0), (1.0, 1.4, 1.5), (30.0, 12.0, 8.0)])
def test_collision_probability_is_the_mixture_of_eq2_over_the_truncated_normal(mu_t, sigma_t, w):
    # The model says s~^2 is truncated normal and, given s~, the hash is E2LSH on the
    # sub-vector: so p(s, sigma) must equal E[p_w(s~)], computed here without any
    # characteristic function, by quadrature and by simulation.
    got = law.fastlsh_collision_probability(mu_t, sigma_t, w)
    tn = stats.truncnorm(-mu_t / sigma_t, np.inf, loc=mu_t, scale=sigma_t)
    mix, _ = integrate.quad(lambda u: _p_closed(max(u, 1e-300), w) * tn.pdf(u * u) * 2 * u, 0.0,
                            math.sqrt(mu_t + 12 * sigma_t), epsabs=1e-12, epsrel=1e-11, limit=400)
    assert abs(got - mix) < 1e-7, (got, mix)
    rng = np.random.default_rng(7)
    y = tn.rvs(size=2_000_000, random_state=rng)
    d = np.sqrt(y) * rng.normal(size=y.size)
    mc = np.maximum(0.0, 1.0 - np.abs(d) / w)              # P[same bucket | projection difference d]
    assert abs(got - mc.mean()) < 5 * mc.std() / math.sqrt(y.size)


def test_pair_statistics():
    v = np.array([1.0, 2.0, 3.0, 4.0])
    u = np.array([0.0, 2.0, 5.0, 4.0])
    mu_t, sigma_t = law.pair_statistics(v, u, m=2)
    # squared differences 1, 0, 4, 0: mean 1.25, variance 2.6875
    assert mu_t == pytest.approx(2.5) and sigma_t == pytest.approx(math.sqrt(2 * 2.6875))
