"""The error bounds behind the matrix-core kernels' bf16 split arithmetic, checked on the CPU
with torch's round-to-nearest bf16 conversion (no library code involved): the three-way split
of an fp32 number is exact, the six products of weight >= 2^-16 reproduce a dot product to
fp32 rounding level, and the three products of a two-way split stay inside half of the band
within which a sign bit is left open."""
import numpy as np
import torch


def _split(x, terms):
    """x (fp32 tensor) -> list of `terms` fp32 tensors holding bf16 values, by repeated rounding."""
    out, rest = [], x.clone()
    for _ in range(terms):
        t = rest.to(torch.bfloat16).to(torch.float32)
        out.append(t)
        rest = rest - t          # exact in fp32 (checked below through the final remainder)
    return out, rest


def _samples(seed, shape):
    g = torch.Generator().manual_seed(seed)
    mant = torch.randn(shape, generator=g, dtype=torch.float32)
    expo = torch.randint(-60, 60, shape, generator=g).to(torch.float32)
    return mant * torch.exp2(expo)


def test_three_way_split_is_exact():
    x = torch.cat([_samples(1, (200000,)), torch.tensor([0.0, 1.0, -1.0, 255.0, 1.0 + 2.0 ** -23, 3.0e38, 1e-30])])
    parts, rest = _split(x, 3)
    assert torch.all(rest == 0)
    total = parts[0].double() + parts[1].double() + parts[2].double()
    assert torch.all(total == x.double())
    # the sizes the bounds rely on: |x2| <= 2^-8 |x|, |x3| <= 2^-16 |x|
    ax = x.abs().double()
    assert torch.all(parts[1].abs().double() <= ax * 2.0 ** -8)
    assert torch.all(parts[2].abs().double() <= ax * 2.0 ** -16)


def test_six_products_reach_fp32_rounding_level():
    n, rows = 128, 4000
    a, v = _samples(2, (rows, n)), _samples(3, (rows, n))
    (a1, a2, a3), _ = _split(a, 3)
    (v1, v2, v3), _ = _split(v, 3)
    d = lambda t: t.double()
    exact = (d(a) * d(v)).sum(1)
    six = (d(a1) * d(v1) + d(a1) * d(v2) + d(a2) * d(v1) + d(a1) * d(v3) + d(a2) * d(v2) + d(a3) * d(v1)).sum(1)
    abs_sum = (d(a) * d(v)).abs().sum(1)
    worst = float(((six - exact).abs() / abs_sum).max())
    assert worst <= 2.0 ** -23 + 2.0 ** -31, worst          # a2 v3 + a3 v2 + a3 v3
    five = six - (d(a2) * d(v2)).sum(1)
    assert float(((five - exact).abs() / abs_sum).max()) > 2.0 ** -23   # the sixth product is needed for that


def test_three_products_of_two_way_splits_stay_inside_half_the_sign_band():
    n, rows = 128, 4000
    a, v = _samples(4, (rows, n)), _samples(5, (rows, n))
    (a1, a2), _ = _split(a, 2)
    (v1, v2), _ = _split(v, 2)
    d = lambda t: t.double()
    exact = (d(a) * d(v)).sum(1)
    three = (d(a1) * d(v1) + d(a1) * d(v2) + d(a2) * d(v1)).sum(1)
    abs_sum = (d(a) * d(v)).abs().sum(1)
    norm_prod = d(a).norm(dim=1) * d(v).norm(dim=1)
    err = (three - exact).abs()
    assert float((err / abs_sum).max()) <= 3.0 * 2.0 ** -16
    assert float((err / norm_prod).max()) <= 0.5e-4
    # so a sign taken from the three products can differ from the exact one only inside the band
    flipped = (three >= 0) != (exact >= 0)
    assert torch.all(exact.abs()[flipped] < 0.5e-4 * norm_prod[flipped])
