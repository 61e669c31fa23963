"""Comparison rules between the GPU library's outputs and the CPU oracle's.

Bucket ids (integers decided by a floating-point value): identical, except where the
oracle's fp64 value (p + b)/w lies within BAND of an integer, i.e. the projection is within
1e-4*w of a bucket boundary; there either neighbouring id is accepted and the element is
counted as excluded.  Projections: |p_gpu - p_oracle| <= 1e-5 * sum_i |a_i v_i|.
Sign bits: identical unless |p_oracle| < 1e-4 * ||a|| * ||S(v)||.  Keys: bit-exact.
"""
import numpy as np

BAND = 1e-4          # in units of w
PROJ_RTOL = 1e-5     # relative to sum_i |a_i v_i|


def check_ids(gpu_ids, ora, label=""):
    """ora: dict with ids (i32) and frac (f64).  Returns the excluded fraction."""
    ids, frac = ora["ids"], ora["frac"]
    near = (frac < BAND) | (frac > 1.0 - BAND)
    diff = gpu_ids.astype(np.int64) - ids.astype(np.int64)
    bad_far = (diff != 0) & ~near
    assert not bad_far.any(), (f"{label}: {int(bad_far.sum())} bucket ids differ outside the boundary "
                               f"band; first at {np.argwhere(bad_far)[0].tolist()}, "
                               f"frac={frac[bad_far][0]}, diff={diff[bad_far][0]}")
    # inside the band only the bucket across the nearby boundary is acceptable
    lo = near & (frac < BAND)
    hi = near & (frac > 1.0 - BAND)
    assert np.isin(diff[lo], (0, -1)).all(), f"{label}: wrong id next to a lower boundary"
    assert np.isin(diff[hi], (0, 1)).all(), f"{label}: wrong id next to an upper boundary"
    return float(near.mean())


def check_proj(gpu_proj, ora, label=""):
    err = np.abs(gpu_proj.astype(np.float64) - ora["proj"])
    tol = PROJ_RTOL * ora["abs_sum"] + 1e-30
    worst = float((err / tol).max()) if err.size else 0.0
    assert worst <= 1.0, f"{label}: projection error {worst:.3f} x tolerance"
    # reported, not required: under cancellation no fp32 sum can be within 1e-5 of a projection near 0
    plain = float((err <= PROJ_RTOL * np.abs(ora["proj"])).mean()) if err.size else 1.0
    print(f"{label}: worst projection error {worst:.3f} x tolerance; within a plain relative "
          f"{PROJ_RTOL:g} of the value: {plain:.4f} of {err.size}")
    return worst


def check_signs(gpu_words, ora_words, proj, norm_prod, k, label=""):
    g = np.unpackbits(np.ascontiguousarray(gpu_words).view(np.uint8), axis=1, bitorder="little")
    o = np.unpackbits(np.ascontiguousarray(ora_words).view(np.uint8), axis=1, bitorder="little")
    assert not g[:, k:].any(), f"{label}: padding bits set"
    near = np.abs(proj) < BAND * norm_prod
    bad = (g[:, :k] != o[:, :k]) & ~near
    assert not bad.any(), f"{label}: {int(bad.sum())} sign bits differ away from zero"
    return float(near.mean())
