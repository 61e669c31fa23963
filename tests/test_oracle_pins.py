"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign or index, transposed
operand, wrong floor, wrong distribution of a table) fails at least one.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

import oracle

RNG = np.random.default_rng(12345)


# --------------------------------------------------------------------------
# Random number generator: published known answers + an independent library.
# --------------------------------------------------------------------------

def test_philox_known_answers(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "philox4x64_10_kat.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        out = oracle.philox4x64_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def _numpy_philox_block(ctr, key):
    # numpy's Philox advances its 256-bit counter before producing a block
    c = sum(int(x) << (64 * i) for i, x in enumerate(ctr))
    c = (c - 1) % (1 << 256)
    cc = np.array([(c >> (64 * i)) & (2 ** 64 - 1) for i in range(4)], dtype=np.uint64)
    bitgen = np.random.Philox(counter=cc, key=np.array(key, dtype=np.uint64))
    return bitgen.random_raw(4)


def test_philox_against_numpy():
    for _ in range(200):
        ctr = RNG.integers(0, 2 ** 64, size=4, dtype=np.uint64)
        key = RNG.integers(0, 2 ** 64, size=2, dtype=np.uint64)
        assert np.array_equal(oracle.philox4x64_10(ctr, key), _numpy_philox_block(ctr, key))


# --------------------------------------------------------------------------
# Sampling operator and floor: the paper's worked example (Sec. 3.1).
# --------------------------------------------------------------------------

def _read_example(golden_dir):
    vals = {}
    for ln in open(os.path.join(golden_dir, "sampling_example.txt")):
        if ln.startswith("#") or "=" not in ln:
            continue
        name, rhs = ln.split("=")
        vals[name.strip()] = [float(x) for x in rhs.split()]
    return vals


def test_sampling_example_from_paper(golden_dir):
    ex = _read_example(golden_dir)
    v = np.array([ex["v"]], np.float32)
    S = np.array([ex["S"]], np.uint32) - 1          # the paper counts coordinates from 1
    v_tilde = ex["S(v)"]
    # projecting with unit vector e_i picks out S(v)_i, in draw order, duplicate kept
    for i, want in enumerate(v_tilde):
        e = np.zeros((1, 3), np.float32)
        e[0, i] = 1.0
        got = oracle.fastlsh(v, S, e, None, None, want=("proj",))["proj"][0, 0]
        assert got == want
    # a~ = (1,1,1): p = 3+7+3 = 13; b = 0, w = 4 -> floor(3.25) = 3
    out = oracle.fastlsh(v, S, np.ones((1, 3), np.float32), np.zeros(1, np.float32), 4.0,
                         want=("proj", "ids", "frac", "abs_sum"))
    assert out["proj"][0, 0] == 13.0 and out["ids"][0, 0] == 3
    assert out["frac"][0, 0] == 0.25 and out["abs_sum"][0, 0] == 13.0
    # a~ = (1,-2,1): p = 3-14+3 = -8; b = 0.5, w = 4 -> floor(-1.875) = -2 (toward -inf)
    out = oracle.fastlsh(v, S, np.array([[1, -2, 1]], np.float32), np.array([0.5], np.float32),
                         4.0, want=("proj", "ids", "abs_sum"))
    assert out["proj"][0, 0] == -8.0 and out["ids"][0, 0] == -2
    assert out["abs_sum"][0, 0] == 20.0


# --------------------------------------------------------------------------
# Brute force in exact rational arithmetic on tiny inputs.
# --------------------------------------------------------------------------

def _exact_hash(v, S, a, b, w):
    p = sum(Fraction(float(a[i])) * Fraction(float(v[S[i]])) for i in range(len(S)))
    q = (p + Fraction(float(b))) / Fraction(float(w))
    return p, math.floor(q), q - math.floor(q)


@pytest.mark.parametrize("n,k,m,N,w", [(5, 3, 3, 7, 4.0), (8, 4, 4, 16, 0.75), (7, 2, 1, 5, 3.0)])
def test_bruteforce_exact_rational(n, k, m, N, w):
    data = RNG.normal(size=(N, n)).astype(np.float32) * 3
    S = RNG.integers(0, n, size=(k, m)).astype(np.uint32)      # duplicates allowed
    a = RNG.normal(size=(k, m)).astype(np.float32)
    b = (RNG.random(k) * w).astype(np.float32)
    out = oracle.fastlsh(data, S, a, b, w, want=("proj", "ids", "frac"))
    for r in range(N):
        for j in range(k):
            p, h, frac = _exact_hash(data[r], S[j], a[j], b[j], w)
            assert abs(out["proj"][r, j] - float(p)) <= 1e-13 * max(1.0, abs(float(p)))
            if 1e-9 < float(frac) < 1 - 1e-9:
                assert out["ids"][r, j] == h
            assert abs(out["frac"][r, j] - float(frac)) < 1e-9 or abs(abs(out["frac"][r, j] - float(frac)) - 1) < 1e-9


# --------------------------------------------------------------------------
# m = n: FastLSH is E2LSH (Eq. 5 with S = identity is Eq. 1); and the E2LSH
# oracle against the textbook dense product.
# --------------------------------------------------------------------------

def test_dense_reduction_against_matrix_product():
    N, n, k, w = 37, 19, 11, 2.5
    data = RNG.normal(size=(N, n)).astype(np.float32)
    a = RNG.normal(size=(k, n)).astype(np.float32)
    b = (RNG.random(k) * w).astype(np.float32)
    P = data.astype(np.float64) @ a.astype(np.float64).T              # [N,k]
    H = np.floor((P + b.astype(np.float64)[None, :]) / w).astype(np.int64)
    dense = oracle.e2lsh(data, a, b, w, want=("proj", "ids", "abs_sum"))
    ident = np.tile(np.arange(n, dtype=np.uint32), (k, 1))
    samp = oracle.fastlsh(data, ident, a, b, w, want=("proj", "ids", "abs_sum"))
    assert np.allclose(dense["proj"], P, rtol=0, atol=1e-12)
    assert np.array_equal(dense["proj"], samp["proj"])                 # same sum order
    assert np.array_equal(dense["ids"], H) and np.array_equal(samp["ids"], H)
    A1 = np.abs(data.astype(np.float64))[:, None, :] * np.abs(a.astype(np.float64))[None, :, :]
    assert np.allclose(dense["abs_sum"], A1.sum(-1), rtol=1e-13)
    assert np.array_equal(dense["abs_sum"], samp["abs_sum"])


def test_sampled_equals_dense_with_scattered_coefficients():
    # without replacement: scattering a~ into a dense vector (a[S[i]] = a~[i]) gives the
    # same projection; with duplicates the dense coefficient is the sum over occurrences
    N, n, k, m, w = 23, 40, 9, 12, 1.25
    data = RNG.normal(size=(N, n)).astype(np.float32)
    b = (RNG.random(k) * w).astype(np.float32)
    S = np.stack([RNG.permutation(n)[:m] for _ in range(k)]).astype(np.uint32)
    S[0, 3] = S[0, 1]                                                   # one duplicate
    a_t = RNG.normal(size=(k, m)).astype(np.float32)
    dense64 = np.zeros((k, n))
    for j in range(k):
        for i in range(m):
            dense64[j, S[j, i]] += float(a_t[j, i])
    P = data.astype(np.float64) @ dense64.T
    got = oracle.fastlsh(data, S, a_t, b, w, want=("proj", "ids"))
    assert np.allclose(got["proj"], P, rtol=0, atol=1e-12)
    H = np.floor((P + b.astype(np.float64)) / w)
    safe = np.abs((P + b) / w - np.round((P + b) / w)) > 1e-9
    assert np.array_equal(got["ids"][safe], H[safe].astype(np.int32))


# --------------------------------------------------------------------------
# Scaling fact (Sec. 4.2, the fact quoted from Datar et al.): hashing alpha*v
# with width alpha*w and offset alpha*b gives the same bucket; exact for
# alpha a power of two.
# --------------------------------------------------------------------------

@pytest.mark.parametrize("alpha", [2.0, 0.125, 1024.0])
def test_scaling_invariance(alpha):
    n, k, m, N, w = 64, 32, 16, 50, 4.0
    idx, coef, off = oracle.params(n, k, m, w, seed=7)
    data = RNG.normal(size=(N, n)).astype(np.float32) * 5
    h1 = oracle.fastlsh(data, idx, coef, off, w)["ids"]
    h2 = oracle.fastlsh(data * np.float32(alpha), idx, coef, off * np.float32(alpha), w * alpha)["ids"]
    assert np.array_equal(h1, h2)


# --------------------------------------------------------------------------
# Parameter tables: shapes, ranges, distributions.
# --------------------------------------------------------------------------

def test_tables_shapes_ranges_determinism():
    n, k, m, w = 128, 64, 32, 4.0
    idx, coef, off = oracle.params(n, k, m, w, seed=1)
    idx2, coef2, off2 = oracle.params(n, k, m, w, seed=1)
    assert np.array_equal(idx, idx2) and np.array_equal(coef, coef2) and np.array_equal(off, off2)
    idx3, coef3, _ = oracle.params(n, k, m, w, seed=2)
    assert not np.array_equal(idx, idx3) and not np.array_equal(coef, coef3)
    assert idx.min() >= 0 and idx.max() < n
    assert (off >= 0).all() and (off < w).all()
    for j in range(k):                          # without replacement: all distinct
        assert len(set(idx[j].tolist())) == m
    # functions are independent draws: no two functions share their sample list
    assert len({tuple(r) for r in idx.tolist()}) == k
    # a prefix property of the counter-based construction: fewer functions = first rows
    idx4, coef4, off4 = oracle.params(n, 16, m, w, seed=1)
    assert np.array_equal(idx4, idx[:16]) and np.array_equal(coef4, coef[:16]) and np.array_equal(off4, off[:16])


def test_m_equals_n_is_identity_sampling():
    for repl in (False, True):
        idx, coef, off = oracle.params(24, 5, 24, 2.0, seed=3, with_replacement=repl)
        assert np.array_equal(idx, np.tile(np.arange(24, dtype=np.uint32), (5, 1)))


def test_index_uniformity_both_modes():
    # "each entry has equal probability m/n of being chosen" (Sec. 3.1)
    n, k, m = 50, 4000, 10
    for repl in (False, True):
        idx, _, _ = oracle.params(n, k, m, 1.0, seed=11, with_replacement=repl)
        counts = np.bincount(idx.ravel(), minlength=n)
        chi2, pval = stats.chisquare(counts)
        assert pval > 1e-4, (repl, chi2, pval)
        # every draw position is uniform too (catches a shuffle that favours a position)
        for i in (0, m - 1):
            _, pv = stats.chisquare(np.bincount(idx[:, i], minlength=n))
            assert pv > 1e-4
    # with replacement: duplicate pairs per function ~ m(m-1)/(2n)
    idx, _, _ = oracle.params(n, k, m, 1.0, seed=11, with_replacement=True)
    dup_pairs = sum(sum(c * (c - 1) // 2 for c in np.bincount(r)) for r in idx)
    expect = k * m * (m - 1) / (2 * n)
    assert abs(dup_pairs - expect) < 5 * math.sqrt(expect)


def test_without_replacement_subsets_are_uniform():
    # n=4, m=2: the 12 ordered pairs must be equally likely
    idx, _, _ = oracle.params(4, 24000, 2, 1.0, seed=5)
    codes = idx[:, 0] * 4 + idx[:, 1]
    counts = np.bincount(codes, minlength=16)
    valid = [a * 4 + b for a in range(4) for b in range(4) if a != b]
    assert counts[[a * 4 + a for a in range(4)]].sum() == 0
    _, pval = stats.chisquare(counts[valid])
    assert pval > 1e-4


def test_coefficients_are_standard_normal_offsets_uniform():
    w = 3.0
    idx, coef, off = oracle.params(256, 4096, 16, w, seed=9)
    z = coef.ravel().astype(np.float64)
    assert stats.kstest(z, "norm").pvalue > 1e-4
    assert abs(z.mean()) < 5 / math.sqrt(z.size) and abs(z.var() - 1) < 5 * math.sqrt(2 / z.size)
    assert stats.kstest(off.astype(np.float64) / w, "uniform").pvalue > 1e-4
    # coefficients of different functions / samples are uncorrelated
    c = np.corrcoef(coef[:, 0], coef[:, 1])[0, 1]
    assert abs(c) < 5 / math.sqrt(coef.shape[0])
    # and independent of the sampled index
    c = np.corrcoef(coef.ravel(), idx.ravel().astype(np.float64))[0, 1]
    assert abs(c) < 5 / math.sqrt(z.size)


# --------------------------------------------------------------------------
# LSH property: collision probability (Sec. 2.2, Eq. 2) and its FastLSH form.
# --------------------------------------------------------------------------

def _p_closed(s, w):
    r = w / s
    return 2 * stats.norm.cdf(r) - 1 - 2 / (math.sqrt(2 * math.pi) * r) * (1 - math.exp(-r * r / 2))


def _read_law(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "e2lsh_collision_law.txt"))
            if ln.strip() and not ln.startswith("#")]
    return [(float(a), float(b), float(c)) for a, b, c in rows]


def test_closed_form_matches_quadrature_of_eq2(golden_dir):
    for w, s, p in _read_law(golden_dir):
        assert abs(_p_closed(s, w) - p) < 1e-9


def _pair_at_distance(n, s, rng):
    v = rng.normal(size=n)
    d = rng.normal(size=n)
    d *= s / np.linalg.norm(d)
    return np.stack([v, v + d]).astype(np.float32)


def test_e2lsh_collision_rate_follows_eq2_and_falls_with_distance(golden_dir):
    n, k = 32, 16384
    rng = np.random.default_rng(1)
    for w in (4.0, 1.5):
        idx, coef, off = oracle.params(n, k, n, w, seed=21)      # m = n: E2LSH
        rates = []
        for w_, s, p in [row for row in _read_law(golden_dir) if row[0] == w]:
            pair = _pair_at_distance(n, s, rng)
            s_true = np.linalg.norm(pair[0].astype(np.float64) - pair[1].astype(np.float64))
            ids = oracle.e2lsh(pair, coef, off, w)["ids"]
            rate = (ids[0] == ids[1]).mean()
            p_true = _p_closed(s_true, w)
            assert abs(p_true - p) < 1e-3                          # fp32 rounding of the pair
            assert abs(rate - p_true) < 4 * math.sqrt(p_true * (1 - p_true) / k), (w, s, rate, p_true)
            rates.append(rate)
        assert all(a > b for a, b in zip(rates, rates[1:])), rates


def test_fastlsh_collision_rate_conditional_law_and_monotone():
    # conditional on S_j, the FastLSH hash is E2LSH on the sub-vector (Sec. 4.1), so
    # P[collision] = mean_j p_w(s~_j), s~_j the distance between S_j(v) and S_j(u)
    n, k, m, w = 64, 16384, 16, 4.0
    rng = np.random.default_rng(2)
    direction = rng.normal(size=n)
    direction /= np.linalg.norm(direction)
    v = rng.normal(size=n)
    for repl in (False, True):
        idx, coef, off = oracle.params(n, k, m, w, seed=33, with_replacement=repl)
        rates = []
        for s in (1.0, 2.0, 4.0, 8.0, 16.0, 32.0):
            pair = np.stack([v, v + s * direction]).astype(np.float32)
            diff = pair[0].astype(np.float64) - pair[1].astype(np.float64)
            s_tilde = np.sqrt((diff[idx.astype(np.int64)] ** 2).sum(axis=1))       # [k]
            expect = np.mean([_p_closed(max(x, 1e-12), w) for x in s_tilde])
            ids = oracle.fastlsh(pair, idx, coef, off, w)["ids"]
            rate = (ids[0] == ids[1]).mean()
            assert abs(rate - expect) < 4 * math.sqrt(expect * (1 - expect) / k), (repl, s, rate, expect)
            rates.append(rate)
        assert all(a > b for a, b in zip(rates, rates[1:])), rates


# --------------------------------------------------------------------------
# One sample S per table (Sec. 3.1 read literally: one multiset S for the family).
# --------------------------------------------------------------------------

@pytest.mark.parametrize("repl", [False, True])
def test_shared_sample_tables_structure(repl):
    n, k, m, w, L = 50, 48, 7, 2.0, 6
    g = k // L
    idx_i, coef_i, off_i = oracle.params(n, k, m, w, seed=9, with_replacement=repl)
    idx_s, coef_s, off_s = oracle.params_shared(n, k, m, w, seed=9, L=L, with_replacement=repl)
    # a~ and b~ stay per function; S of table l is the S of its first function, for all g
    assert np.array_equal(coef_s.view(np.uint32), coef_i.view(np.uint32))
    assert np.array_equal(off_s.view(np.uint32), off_i.view(np.uint32))
    for l in range(L):
        for t in range(g):
            assert np.array_equal(idx_s[l * g + t], idx_i[l * g])
    # tables differ from one another (the draws of different tables are independent)
    assert len({tuple(idx_s[l * g]) for l in range(L)}) == L
    # L = k is the per-function case, L = 1 one sample for everything
    assert np.array_equal(oracle.params_shared(n, k, m, w, 9, L=k, with_replacement=repl)[0], idx_i)
    assert (oracle.params_shared(n, k, m, w, 9, L=1, with_replacement=repl)[0] == idx_i[0]).all()
    with pytest.raises(Exception):
        oracle.params_shared(n, k, m, w, 9, L=5)          # k % L != 0


def test_shared_sample_key_collision_law():
    # With one S per table the g functions of a table are independent E2LSH functions on the
    # same sub-vector, so a whole key collides with probability p_w(s~_l)^g given S_l, and the
    # rate over many tables is the mean of that: not the g-th power of the mean collision
    # rate, which is what per-function samples give.  A sparse difference vector makes the
    # two laws differ widely (s~ is 0 for most samples).
    n, m, w, g, L = 40, 4, 4.0, 4, 6000
    k = g * L
    v = np.random.default_rng(5).normal(size=n)
    diff = np.zeros(n)
    diff[:4] = 6.0                                       # only 4 of the 40 coordinates differ
    pair = np.stack([v, v + diff]).astype(np.float32)
    d64 = pair[0].astype(np.float64) - pair[1].astype(np.float64)

    def p_of(s_tilde):
        return 1.0 if s_tilde == 0 else _p_closed(s_tilde, w)

    idx, coef, off = oracle.params_shared(n, k, m, w, seed=77, L=L)
    ids = oracle.fastlsh(pair, idx, coef, off, w)["ids"].reshape(2, L, g)
    rate_shared = (ids[0] == ids[1]).all(axis=1).mean()
    s_tab = np.sqrt((d64[idx[::g].astype(np.int64)] ** 2).sum(axis=1))               # [L]
    expect_shared = np.mean([p_of(x) ** g for x in s_tab])
    assert abs(rate_shared - expect_shared) < 4 * math.sqrt(expect_shared * (1 - expect_shared) / L)

    idx, coef, off = oracle.params(n, k, m, w, seed=77)
    ids = oracle.fastlsh(pair, idx, coef, off, w)["ids"].reshape(2, L, g)
    rate_indep = (ids[0] == ids[1]).all(axis=1).mean()
    s_fn = np.sqrt((d64[idx.astype(np.int64)] ** 2).sum(axis=1)).reshape(L, g)
    expect_indep = np.mean([np.prod([p_of(x) for x in row]) for row in s_fn])
    assert abs(rate_indep - expect_indep) < 4 * math.sqrt(expect_indep * (1 - expect_indep) / L)
    # and the two readings are far apart here, so the test separates them
    assert rate_shared > rate_indep + 0.1


def test_fastlsh_tends_to_e2lsh_at_scaled_distance_for_large_m():
    # Corollary of Sec. 4.2: s~X -> N(0, m s^2 / n); so with the same w the FastLSH
    # collision rate approaches the E2LSH law at distance s*sqrt(m/n)
    n, k, m, w = 2048, 8192, 512, 4.0
    rng = np.random.default_rng(3)
    idx, coef, off = oracle.params(n, k, m, w, seed=44)
    for s in (4.0, 16.0):
        pair = _pair_at_distance(n, s, rng)
        ids = oracle.fastlsh(pair, idx, coef, off, w)["ids"]
        rate = (ids[0] == ids[1]).mean()
        p = _p_closed(s * math.sqrt(m / n), w)
        assert abs(rate - p) < 4 * math.sqrt(p * (1 - p) / k) + 0.01


def test_projection_difference_second_moment():
    # E[(a~^T S(v) - a~^T S(u))^2] = m s^2 / n over the draw of (S, a~)  (Sec. 4.1-4.2)
    n, k, m = 100, 20000, 10
    rng = np.random.default_rng(4)
    pair = _pair_at_distance(n, 3.0, rng)
    s2 = float(((pair[0].astype(np.float64) - pair[1]) ** 2).sum())
    for repl in (False, True):
        idx, coef, _ = oracle.params(n, k, m, 1.0, seed=55, with_replacement=repl)
        proj = oracle.fastlsh(pair, idx, coef, None, None, want=("proj",))["proj"]
        d = proj[0] - proj[1]
        assert abs(d.mean()) < 5 * math.sqrt(m * s2 / n / k)
        # fourth-moment-based standard error of the variance estimate, generous
        assert abs(d.var() - m * s2 / n) < 0.06 * m * s2 / n


# --------------------------------------------------------------------------
# Sign hashes and keys.
# --------------------------------------------------------------------------

def test_signs_reduce_to_plain_sign_random_projection_and_bit_order():
    N, n, k = 20, 24, 130                                              # 3 words, ragged last
    data = RNG.normal(size=(N, n)).astype(np.float32)
    idx, coef, _ = oracle.params(n, k, n, 1.0, seed=6)                  # m = n
    words, proj, npd = oracle.signs(data, idx, coef, want_proj=True, want_norm_prod=True)
    P = data.astype(np.float64) @ coef.astype(np.float64).T
    assert np.allclose(proj, P, atol=1e-12)
    bits = (P >= 0)
    padded = np.zeros((N, 192), bool)
    padded[:, :k] = bits
    expect = np.packbits(padded, axis=1, bitorder="little").view(np.uint64)
    assert np.array_equal(words, expect)
    want_npd = np.linalg.norm(coef.astype(np.float64), axis=1)[None, :] * \
        np.linalg.norm(data.astype(np.float64), axis=1)[:, None]
    assert np.allclose(npd, want_npd, rtol=1e-12)
    # p = 0 counts as non-negative
    z = np.zeros((1, n), np.float32)
    w0, _, _ = oracle.signs(z, idx, coef)
    assert int(w0[0, 0]) == 2 ** 64 - 1 and int(w0[0, 2]) == 3


def test_sign_collision_follows_angle_law():
    # conditional on S_j: P[equal bits] = 1 - angle(S_j(v), S_j(u)) / pi
    n, k, m = 64, 16384, 16
    rng = np.random.default_rng(8)
    idx, coef, _ = oracle.params(n, k, m, 1.0, seed=66)
    v = rng.normal(size=n)
    for mix in (0.2, 1.0, 3.0):
        u = v + mix * rng.normal(size=n)
        pair = np.stack([v, u]).astype(np.float32)
        words, _, _ = oracle.signs(pair, idx, coef)
        bits = np.unpackbits(words.view(np.uint8), axis=1, bitorder="little")[:, :k]
        rate = (bits[0] == bits[1]).mean()
        a = pair[0].astype(np.float64)[idx.astype(np.int64)]
        b = pair[1].astype(np.float64)[idx.astype(np.int64)]
        cosang = (a * b).sum(1) / (np.linalg.norm(a, axis=1) * np.linalg.norm(b, axis=1))
        expect = (1 - np.arccos(np.clip(cosang, -1, 1)) / math.pi).mean()
        assert abs(rate - expect) < 4 * math.sqrt(expect * (1 - expect) / k)


def test_keys_against_python_integers():
    N, k, L = 9, 24, 4
    ids = RNG.integers(-1000, 1000, size=(N, k)).astype(np.int32)
    keys = oracle.pack_keys(ids, L)
    M = 0x9E3779B97F4A7C15
    g = k // L
    for r in range(N):
        for l in range(L):
            acc = 0
            for t in range(g):
                acc += (int(ids[r, l * g + t]) % (1 << 32)) * pow(M, g - 1 - t, 1 << 64)
            assert int(keys[r, l]) == acc % (1 << 64)
    # g = 1: the key is the id itself as an unsigned 32-bit value
    keys1 = oracle.pack_keys(ids, k)
    assert np.array_equal(keys1, ids.astype(np.uint32).astype(np.uint64))
    with pytest.raises(ValueError):
        oracle.pack_keys(ids, 5)


def test_argument_errors():
    with pytest.raises(ValueError):
        oracle.params(8, 4, 9, 1.0, 1)           # m > n
    with pytest.raises(ValueError):
        oracle.params(8, 4, 4, 0.0, 1)           # w <= 0
    data = np.zeros((2, 4), np.float32)
    bad = np.full((1, 2), 4, np.uint32)          # index out of range
    with pytest.raises(ValueError):
        oracle.fastlsh(data, bad, np.ones((1, 2), np.float32), np.zeros(1, np.float32), 1.0)
    huge = np.full((1, 4), 3e38, np.float32)     # bucket id outside int32
    with pytest.raises(ValueError):
        oracle.fastlsh(huge, np.zeros((1, 1), np.uint32), np.full((1, 1), 3e38, np.float32),
                       np.zeros(1, np.float32), 1.0)
