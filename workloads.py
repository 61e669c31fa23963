"""Seeded synthetic inputs shaped like the paper's workloads (Sec. 6, Table 1).

This module only draws input vectors.  It holds none of the hashing method's
arithmetic and is the one piece of code that both the CPU oracle's tests and
the GPU library's tests/benchmark use, so that both sides see the same bits.

The real datasets (Sift, Gist, Trevi, ...) are not available; each recipe below
is a stand-in with the same N x n shape and a comparable value range:

  tiny      N=10,000   n=128    i.i.d. N(0,1)
  sift      N=1,000,000 n=128   100-cluster Gaussian mixture, centres U[0,255),
                                std 20, rounded to integers, clipped to [0,255]
  gist      N=1,000,000 n=960   1,000-cluster mixture, centres U[0,1), std 0.05,
                                clipped to [0,1]
  highdim   N=200,000  n=4,096  i.i.d. N(0,1); the last 5% of rows are planted
                                near-duplicates: a random earlier row plus
                                N(0, variance 0.01) noise
  angular   N=500,000  n=16,384 N(0,1) rows scaled to unit l2 norm

Rows are generated in blocks with a torch.Generator seeded from the recipe's
seed, on whichever device is asked for (the CPU and GPU generators give
different, but each reproducible, streams).
"""
from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    n: int
    k: int
    m: tuple          # sampled-dimension settings to run (one or a sweep)
    w: float          # bucket width (unused by the sign hash)
    seed: int         # seed of the hash-function tables and of the data
    L: int = 0        # number of key groups (0: no key packing asked for)
    signs: bool = False
    planted: int = 0  # number of planted near-duplicate rows (at the end)
    extra: dict = field(default_factory=dict)


WORKLOADS = {
    "tiny": Workload("tiny", 10_000, 128, 64, (32,), 4.0, 1, L=8),
    "sift": Workload("sift", 1_000_000, 128, 512, (32,), 16.0, 2, L=32),
    "gist": Workload("gist", 1_000_000, 960, 1024, (128,), 1.0, 3, L=64),
    "highdim": Workload("highdim", 200_000, 4096, 2048, (64, 256, 1024), 8.0, 4, L=128,
                        planted=10_000),
    "angular": Workload("angular", 500_000, 16384, 4096, (512,), 1.0, 5, signs=True),
}

_BLOCK_BYTES = 1 << 30


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _blocks(N, n):
    rows = max(1, _BLOCK_BYTES // (4 * n))
    for r0 in range(0, N, rows):
        yield r0, min(N, r0 + rows)


def make_data(name, device="cpu", N=None):
    """Return (workload, data) with data a row-major fp32 tensor [N, n] on device.

    N overrides the recipe's row count (same generator stream, fewer rows of it;
    for "highdim" the planted fraction stays 5%)."""
    wl = WORKLOADS[name]
    N = wl.N if N is None else int(N)
    n = wl.n
    g = _gen(device, wl.seed)
    data = torch.empty((N, n), dtype=torch.float32, device=device)
    if name in ("tiny",):
        for r0, r1 in _blocks(N, n):
            data[r0:r1] = torch.randn((r1 - r0, n), generator=g, device=device)
    elif name in ("sift", "gist"):
        n_clusters, hi, std = (100, 255.0, 20.0) if name == "sift" else (1000, 1.0, 0.05)
        centres = torch.rand((n_clusters, n), generator=g, device=device) * hi
        for r0, r1 in _blocks(N, n):
            which = torch.randint(0, n_clusters, (r1 - r0,), generator=g, device=device)
            x = centres[which] + std * torch.randn((r1 - r0, n), generator=g, device=device)
            if name == "sift":
                x = torch.round(x)
            data[r0:r1] = torch.clamp(x, 0.0, hi)
    elif name == "highdim":
        planted = N // 20
        base_rows = N - planted
        for r0, r1 in _blocks(base_rows, n):
            data[r0:r1] = torch.randn((r1 - r0, n), generator=g, device=device)
        if planted:
            src = torch.randint(0, base_rows, (planted,), generator=g, device=device)
            for r0, r1 in _blocks(planted, n):
                noise = 0.1 * torch.randn((r1 - r0, n), generator=g, device=device)
                data[base_rows + r0:base_rows + r1] = data[src[r0:r1]] + noise
            wl = Workload(**{**wl.__dict__, "planted": planted,
                             "extra": {"planted_src": src.cpu()}})
    elif name == "angular":
        for r0, r1 in _blocks(N, n):
            x = torch.randn((r1 - r0, n), generator=g, device=device)
            data[r0:r1] = x / torch.linalg.vector_norm(x, dim=1, keepdim=True)
    else:
        raise KeyError(name)
    if N != wl.N:
        wl = Workload(**{**wl.__dict__, "N": N})
    return wl, data


def sample_rows(N, count, tile=64, seed=0):
    """A fixed pseudo-random set of row numbers for sampled parity checks: the
    first and last `tile` rows plus `count` rows drawn without replacement."""
    g = torch.Generator()
    g.manual_seed(seed)
    edge = torch.cat([torch.arange(0, min(tile, N)), torch.arange(max(0, N - tile), N)])
    if count >= N:
        return torch.arange(N)
    pick = torch.randperm(N, generator=g)[:count]
    return torch.unique(torch.cat([edge, pick]))
