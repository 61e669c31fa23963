"""Pins of the maximum-inner-product oracle (oracle/mips.py)."""
import math

import numpy as np

import oracle
from oracle import mips


def _setup(seed=3, n=24, N=300, k=32, m=8, w=2.0, L=4):
    rng = np.random.default_rng(seed)
    data = (rng.normal(size=(N, n)) * rng.uniform(0.2, 2.0, size=(N, 1))).astype(np.float32)
    queries = rng.normal(size=(20, n)).astype(np.float32)
    idx, coef, off = oracle.params_shared(n, k, m, w, seed, L)
    a0 = mips.extra_coefficients(k, seed)
    return data, queries, idx, coef, off, a0, w, L


def test_extra_coefficients_are_reproducible_standard_normals():
    a = mips.extra_coefficients(4000, 9)
    assert np.array_equal(a, mips.extra_coefficients(4000, 9)) and not np.array_equal(a[:100], mips.extra_coefficients(100, 10))
    assert abs(a.mean()) < 0.06 and abs(a.std() - 1.0) < 0.04
    # the same draw routine on table 1 gives the projection coefficients of the main oracle bit for bit;
    # table 3 is a separate one
    _, coef, _ = oracle.params(16, 200, 4, 1.0, 9)
    assert all(mips.standard_normal(9, 1, j, i) == coef[j, i] for j in range(200) for i in range(4))
    assert not np.array_equal(a[:200], coef[:, 0])


def test_transform_turns_inner_product_order_into_distance_order():
    # ||P~(v) - Q~(u)||^2 = kappa~^2 + 1 - 2 S(v).S(u)/||S(u)||: the nearest transformed vector is
    # the one with the largest inner product on the sampled coordinates (the appendix' identity)
    data, queries, idx, coef, off, a0, w, L = _setup()
    kappa2 = mips.kappa_squared(data, idx, L)
    P = mips.transformed_data(data, idx, L, kappa2)
    Q = mips.transformed_queries(queries, idx, L)
    g = idx.shape[0] // L
    for l in range(L):
        assert np.allclose((P[l] ** 2).sum(axis=1), kappa2[l], rtol=1e-12)          # all on one sphere
        assert np.allclose((Q[l] ** 2).sum(axis=1), 1.0, rtol=1e-12) and (Q[l][:, 0] == 0).all()
        sv = data.astype(np.float64)[:, idx[l * g].astype(np.int64)]
        su = queries.astype(np.float64)[:, idx[l * g].astype(np.int64)]
        ip = sv @ (su / np.linalg.norm(su, axis=1, keepdims=True)).T               # [N, Q]
        d2 = ((P[l][:, None, :] - Q[l][None, :, :]) ** 2).sum(axis=2)
        assert np.allclose(d2, kappa2[l] + 1.0 - 2.0 * ip, rtol=1e-10, atol=1e-10)
        assert (d2.argmin(axis=0) == ip.argmax(axis=0)).all()
    # kappa~ is attained
    assert all(np.isclose(P[l][:, 0].min(), 0.0, atol=1e-6) for l in range(L))


def test_hash_is_the_l2_hash_of_the_transformed_vectors():
    # independent route: build the (m + 1)-dimensional vectors and coefficient rows explicitly and
    # hash them with the E2LSH oracle (Eq. 1), table by table
    data, queries, idx, coef, off, a0, w, L = _setup()
    kappa2 = mips.kappa_squared(data, idx, L)
    val, ids, frac = mips.hash_data(data, idx, coef, a0, off, w, L, kappa2)
    qval, qids, _ = mips.hash_queries(queries, idx, coef, a0, off, w, L)
    P = mips.transformed_data(data, idx, L, kappa2)
    Q = mips.transformed_queries(queries, idx, L)
    g = idx.shape[0] // L
    for l in range(L):
        rows = np.concatenate([a0[l * g:(l + 1) * g, None], coef[l * g:(l + 1) * g]], axis=1).astype(np.float32)
        for vecs, got in ((P[l], ids), (Q[l], qids)):
            want = oracle.e2lsh(vecs.astype(np.float32), rows, off[l * g:(l + 1) * g], w, want=("ids", "frac"))
            near = (want["frac"] < 1e-5) | (want["frac"] > 1 - 1e-5)               # fp32 rounding of the inputs
            assert ((got[:, l * g:(l + 1) * g] == want["ids"]) | near).all()
    assert (ids == np.floor(val)).all() and (frac >= 0).all() and (frac < 1).all()


def test_collisions_grow_with_the_inner_product():
    # the point of the transform: a data vector with a larger inner product with the query
    # collides with it more often
    rng = np.random.default_rng(5)
    n, k, m, w, L = 32, 4096, 32, 2.0, 256            # m = n: all coordinates, 16 functions per table
    u = rng.normal(size=n)
    u /= np.linalg.norm(u)
    base = rng.normal(size=(6, n))
    base -= np.outer(base @ u, u)                        # orthogonal to u, then add a chosen component
    base /= np.linalg.norm(base, axis=1, keepdims=True)
    ips = np.array([0.9, 0.7, 0.5, 0.2, 0.0, -0.5])
    data = (np.sqrt(1 - ips ** 2)[:, None] * base + ips[:, None] * u).astype(np.float32)
    idx, coef, off = oracle.params_shared(n, k, m, w, 5, L)
    a0 = mips.extra_coefficients(k, 5)
    kappa2 = mips.kappa_squared(data, idx, L)
    _, ids, _ = mips.hash_data(data, idx, coef, a0, off, w, L, kappa2)
    _, qids, _ = mips.hash_queries(u[None].astype(np.float32), idx, coef, a0, off, w, L)
    rates = (ids == qids).mean(axis=1)
    assert all(a > b for a, b in zip(rates, rates[1:])), rates


def test_collision_probability_matches_simulation():
    # Monte Carlo of the appendix' model: I^2 ~ N(mu~ + delta, sigma~^2) truncated at 0, the
    # projection difference is I * X, the offset is uniform: collide iff both fall in one bucket
    rng = np.random.default_rng(11)
    mu_t, sigma_t, delta, w = 3.0, 1.5, 2.0, 4.0
    T = 2_000_000
    i2 = rng.normal(mu_t + delta, sigma_t, size=T)
    i2 = i2[i2 >= 0]
    d = np.abs(np.sqrt(i2) * rng.normal(size=i2.size))
    p_mc = np.where(d < w, 1.0 - d / w, 0.0).mean()          # P[same bucket | d] for a uniform offset
    p = mips.collision_probability(mu_t, sigma_t, delta, w)
    assert abs(p - p_mc) < 4 * math.sqrt(p_mc * (1 - p_mc) / i2.size) + 1e-4, (p, p_mc)
