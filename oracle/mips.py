"""CPU oracle for the maximum-inner-product extension of FastLSH (Appendix "Extension to
Maximum Inner Product Search").

TEST INFRASTRUCTURE, not the product.  numpy, fp64, the appendix' transformations written out:

  data     P~(v) = ( sqrt(kappa~^2 - ||S(v)||^2), S(v) ),   kappa~ = max_i ||S(v_i)||
  query    Q~(u) = ( 0, S(u) ) with ||S(u)|| = 1 (the query's sub-vector is normalised here)
  hash     the l2 hash (Eq. 1) of the transformed (m + 1)-dimensional vector:
           h_j(x) = floor((a_j^T x + b_j) / w),  a_j = (a0_j, a~_j)

The appendix speaks of "the sample operator S" and a constant kappa~: one sample S per table
(oracle.params_shared), kappa~_l per table l.  The extra coefficient a0_j ~ N(0,1) comes from
the repository's counter-based generator as table 3 (Box-Muller on the Philox block of
(table 3, function j, element 0), exactly as the coefficients of table 1).
"""
import math

import numpy as np

import oracle


def standard_normal(seed, table, j, i):
    """One N(0,1) draw of the generator's table `table` at (function j, element i), rounded to fp32."""
    r = oracle.philox4x64_10((i, j, table, 0), (seed, 0))
    u1 = (float(int(r[0]) >> 11) + 1.0) * 2.0 ** -53                     # (0, 1]
    u2 = float(int(r[1]) >> 11) * 2.0 ** -53                             # [0, 1)
    return np.float32(math.sqrt(-2.0 * math.log(u1)) * math.cos(6.283185307179586476925286766559 * u2))


def extra_coefficients(k, seed):
    """a0_j, j < k: fp32, table 3 of the generator."""
    return np.array([standard_normal(seed, 3, j, 0) for j in range(k)], np.float32)


def _sub(data, idx_table):
    return data.astype(np.float64)[:, idx_table.astype(np.int64)]          # [N, m]


def kappa_squared(data, idx, L):
    """kappa~_l^2 = max_i ||S_l(v_i)||^2 for every table l (idx rows are equal inside a table)."""
    g = idx.shape[0] // L
    return np.array([(_sub(data, idx[l * g]) ** 2).sum(axis=1).max() for l in range(L)])


def transformed_data(data, idx, L, kappa2):
    """P~_l(v) for every table: list of L arrays [N, m + 1]."""
    g = idx.shape[0] // L
    out = []
    for l in range(L):
        s = _sub(data, idx[l * g])
        first = np.sqrt(np.maximum(kappa2[l] - (s ** 2).sum(axis=1), 0.0))
        out.append(np.concatenate([first[:, None], s], axis=1))
    return out


def transformed_queries(queries, idx, L):
    """Q~_l(u) for every table: (0, S_l(u) / ||S_l(u)||); a zero sub-vector stays zero."""
    g = idx.shape[0] // L
    out = []
    for l in range(L):
        s = _sub(queries, idx[l * g])
        norm = np.sqrt((s ** 2).sum(axis=1))
        s = np.where(norm[:, None] > 0, s / np.where(norm > 0, norm, 1.0)[:, None], 0.0)
        out.append(np.concatenate([np.zeros((s.shape[0], 1)), s], axis=1))
    return out


def _hash(vectors_per_table, coef, a0, off, w):
    """Eq. 1 on the transformed vectors; returns (value (p + b) / w in fp64, ids, fractional part)."""
    L = len(vectors_per_table)
    k = coef.shape[0]
    g = k // L
    N = vectors_per_table[0].shape[0]
    val = np.empty((N, k))
    for j in range(k):
        a = np.concatenate([[np.float64(a0[j])], coef[j].astype(np.float64)])
        val[:, j] = (vectors_per_table[j // g] @ a + np.float64(off[j])) / np.float64(w)
    ids = np.floor(val)
    return val, ids.astype(np.int32), val - ids


def hash_data(data, idx, coef, a0, off, w, L, kappa2):
    return _hash(transformed_data(data, idx, L, kappa2), coef, a0, off, w)


def hash_queries(queries, idx, coef, a0, off, w, L):
    return _hash(transformed_queries(queries, idx, L), coef, a0, off, w)


def collision_probability(mu_t, sigma_t, delta, w):
    """Collision probability of a (data, query) pair under the transformed hash (last equation of
    the appendix): the squared distance of the transformed pair is s~^2 + delta with
    delta = kappa~^2 - ||S(v)||^2, so it follows N(mu~ + delta, sigma~^2) truncated at 0 and the
    law of Sec. 4.1 applies with the shifted mean."""
    from oracle import collision_law
    return collision_law.fastlsh_collision_probability(mu_t + delta, sigma_t, w)
