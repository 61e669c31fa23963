"""GPU parity: every output of the HIP library, through the C ABI, against the CPU oracle on
the same seeded inputs.  Small shapes are compared element by element on all rows; the
full-size workloads on a fixed sample of rows (first/last tile plus random rows), in the
launch configuration the benchmark times."""
import os
import sys

import numpy as np
import pytest

import oracle
import workloads
from parity import BAND, check_ids, check_proj, check_signs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def lsh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_15479_amd as lib
    lib.load_library()           # raises if the HIP library is missing: no fallback
    return lib


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _tables(p):
    return p.indices(), p.coeffs(), p.offsets()


def _compare_all(lsh, p, data_gpu, rows, L=None, label="", dense=False, signs=True, dense_fp32=False, matrix=True):
    """Runs every entry point on data_gpu and checks the given rows against the oracle."""
    idx, coef, off = _tables(p)
    rows_t = torch.as_tensor(np.asarray(rows), device=data_gpu.device)
    sub = data_gpu[rows_t].cpu().numpy()
    stats = {}
    ora = oracle.fastlsh(sub, idx, coef, off, p.w, nthreads=THREADS,
                         want=("proj", "abs_sum", "ids", "frac"))
    ids_gpu = lsh.hash_fastlsh(p, data_gpu)
    proj_gpu = lsh.project_fastlsh(p, data_gpu)
    torch.cuda.synchronize()
    stats["proj_worst"] = check_proj(proj_gpu[rows_t].cpu().numpy(), ora, label + " fastlsh proj")
    stats["ids_excluded"] = check_ids(ids_gpu[rows_t].cpu().numpy(), ora, label + " fastlsh ids")
    if p.n == 128 and p.k % 32 == 0:
        # this shape runs as a dense product on the matrix cores by default (zeros at the
        # coordinates a function does not sample): the gathered fp32 kernels are checked as well
        p.set_dense_arithmetic(lsh.DENSE_FP32)
        ids_g = lsh.hash_fastlsh(p, data_gpu)
        proj_g = lsh.project_fastlsh(p, data_gpu)
        torch.cuda.synchronize()
        p.set_dense_arithmetic(lsh.DENSE_AUTO)
        stats["proj_worst_gathered"] = check_proj(proj_g[rows_t].cpu().numpy(), ora, label + " fastlsh proj (gathered)")
        check_ids(ids_g[rows_t].cpu().numpy(), ora, label + " fastlsh ids (gathered)")
    if p.n != 128 and p.n % 4 == 0 and p.m < p.n and matrix:
        # the same hashes as a dense product over all n coordinates on the matrix cores
        p.set_dense_arithmetic(lsh.DENSE_MATRIX)
        ids_m = lsh.hash_fastlsh(p, data_gpu)
        proj_m = lsh.project_fastlsh(p, data_gpu)
        torch.cuda.synchronize()
        p.set_dense_arithmetic(lsh.DENSE_AUTO)
        stats["proj_worst_matrix"] = check_proj(proj_m[rows_t].cpu().numpy(), ora, label + " fastlsh proj (matrix cores)")
        check_ids(ids_m[rows_t].cpu().numpy(), ora, label + " fastlsh ids (matrix cores)")
    if dense:
        assert p.m == p.n
        if dense_fp32:
            p.set_dense_arithmetic(lsh.DENSE_FP32)
        ora_d = oracle.e2lsh(sub, coef, off, p.w, nthreads=THREADS, want=("proj", "abs_sum", "ids", "frac"))
        ids_d = lsh.hash_e2lsh(p, data_gpu)
        proj_d = lsh.project_e2lsh(p, data_gpu)
        torch.cuda.synchronize()
        stats["dense_proj_worst"] = check_proj(proj_d[rows_t].cpu().numpy(), ora_d, label + " e2lsh proj")
        stats["dense_ids_excluded"] = check_ids(ids_d[rows_t].cpu().numpy(), ora_d, label + " e2lsh ids")
        p.set_dense_arithmetic(lsh.DENSE_AUTO)
    if signs:
        w_ora, pr, npd = oracle.signs(sub, idx, coef, nthreads=THREADS, want_proj=True, want_norm_prod=True)
        w_gpu = lsh.hash_signs(p, data_gpu)
        torch.cuda.synchronize()
        stats["signs_excluded"] = check_signs(w_gpu[rows_t].cpu().numpy().view(np.uint64), w_ora, pr, npd,
                                              p.k, label + " signs")
        if p.n == 128 and p.k % 64 == 0:
            # this shape's signs come from the matrix-core kernel by default: the gathered
            # fp32 kernel is checked as well
            p.set_dense_arithmetic(lsh.DENSE_FP32)
            w_gpu = lsh.hash_signs(p, data_gpu)
            torch.cuda.synchronize()
            p.set_dense_arithmetic(lsh.DENSE_AUTO)
            check_signs(w_gpu[rows_t].cpu().numpy().view(np.uint64), w_ora, pr, npd, p.k, label + " signs (gathered)")
    if L:
        keys = lsh.pack_keys(p, ids_gpu, L)
        torch.cuda.synchronize()
        ids_host = ids_gpu[rows_t].cpu().numpy()
        want = oracle.pack_keys(ids_host, L)
        assert np.array_equal(keys[rows_t].cpu().numpy().view(np.uint64), want), label + " keys"
        g = p.k // L
        if g & (g - 1) == 0 and g <= 64:
            # fused hashing + packing: the oracle's keys, except for keys that hold an id inside
            # the boundary band (the fused kernel may sum in another order than the ids kernel)
            fused = lsh.hash_fastlsh_keys(p, data_gpu, L)
            torch.cuda.synchronize()
            got = fused[rows_t].cpu().numpy().view(np.uint64)
            near = (ora["frac"] < BAND) | (ora["frac"] > 1.0 - BAND)
            key_near = near.reshape(len(rows_t), L, g).any(axis=2)
            bad = (got != oracle.pack_keys(ora["ids"], L)) & ~key_near
            assert not bad.any(), f"{label} fused keys: {int(bad.sum())} keys differ outside the boundary band"
            stats["fused_keys_excluded"] = float(key_near.mean())
    return stats


# ---------------------------------------------------------------------------------------
# the tiny workload: all rows, FastLSH and its E2LSH twin (m = n, same seed)
# ---------------------------------------------------------------------------------------

def test_tiny_all_rows(lsh):
    wl, data = workloads.make_data("tiny", "cuda")
    rows = np.arange(wl.N)
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed) as p:
        say("tiny fastlsh", _compare_all(lsh, p, data, rows, L=wl.L, label="tiny"))
    with lsh.LshParams(wl.n, wl.k, wl.n, wl.w, wl.seed) as p:
        say("tiny e2lsh", _compare_all(lsh, p, data, rows, L=wl.L, label="tiny-dense", dense=True))


# ---------------------------------------------------------------------------------------
# ragged and degenerate shapes, every tile variant of the sampled kernel
# ---------------------------------------------------------------------------------------

RAGGED = [
    # N, n, k, m, w, seed, with_replacement, L
    (1, 128, 64, 32, 4.0, 21, False, 8),
    (7, 100, 70, 30, 2.5, 22, True, 7),          # the paper's m = 30; k, n not multiples of anything
    (33, 37, 130, 37, 1.0, 23, False, 13),       # m = n (dense twin below), odd n
    (1003, 128, 512, 32, 16.0, 24, False, 32),   # several tiles and a ragged tail
    (257, 960, 1024, 128, 1.0, 25, False, 64),   # 32-vector tiles, streamed lists
    (41, 960, 100, 1, 0.75, 26, True, 0),        # m = 1, w not a power of two
    (29, 4096, 192, 64, 8.0, 27, False, 0),      # 8-vector tiles
    (13, 8000, 64, 100, 3.0, 28, True, 0),       # 4-vector tiles
    (9, 16384, 128, 512, 1.0, 29, False, 0),     # 2-vector tiles
    (40, 16384, 640, 96, 1.0, 33, False, 0),     # coordinate-range chunks, ragged functions
    (21, 5000, 1100, 40, 2.0, 34, True, 0),      # chunks, two workgroups along the functions
    (70, 2049, 512, 7, 2.0, 38, False, 0),       # nine ranges in sixteen stages, one function per lane, one-quad blocks, odd n
    (45, 2304, 1536, 100, 1.0, 39, True, 0),     # three functions per lane, nine ranges
    (33, 9004, 2048, 700, 4.0, 40, False, 64),   # 36 ranges in 40 stages, four functions per lane, keys
    (19, 3000, 1000, 33, 1.0, 41, True, 0),      # two functions per lane, one-quad blocks, k not a multiple of 64
    (5, 30000, 64, 40, 1.0, 30, False, 0),       # 1-vector tiles
    (3, 40384, 64, 33, 1.0, 32, True, 0),        # the largest dimension one LDS tile holds
    (300, 64, 2100, 16, 2.0, 31, False, 0),      # more functions than one workgroup holds
    (100, 256, 512, 64, 4.0, 35, False, 16),     # register lists of two chunks, two pieces per wave, whole tiles + tail
    (50, 128, 514, 20, 2.0, 36, True, 0),        # padded register lists, k not a multiple of 4
    (16, 128, 512, 32, 16.0, 37, False, 32),     # exactly one whole tile, no tail
]


@pytest.mark.parametrize("N,n,k,m,w,seed,repl,L", RAGGED)
def test_ragged_shapes(lsh, N, n, k, m, w, seed, repl, L):
    say(f"case N={N} n={n} k={k} m={m} w={w} seed={seed} repl={repl} L={L}")
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    data = torch.randn((N, n), generator=g, device="cuda") * 3.0
    with lsh.LshParams(n, k, m, w, seed, with_replacement=repl) as p:
        say(_compare_all(lsh, p, data, np.arange(N), L=L, label=f"ragged{seed}", dense=(m == n)))


# ---------------------------------------------------------------------------------------
# one sample per table: the matrix-core kernel and the shapes that fall back to the gather kernels
# ---------------------------------------------------------------------------------------

SHARED = [
    # N, n, k, m, w, seed, with_replacement, L
    (1000, 128, 64, 32, 4.0, 41, False, 8),      # tables of 8 functions: half-empty 16-function blocks
    (1003, 128, 512, 32, 16.0, 42, False, 32),   # the benchmark shape: two blocks per wave, ragged tail
    (77, 100, 72, 30, 2.5, 43, True, 6),         # tables of 12, duplicates in S, w not a power of two
    (300, 256, 512, 64, 4.0, 44, False, 16),     # tables of 32 (two blocks each), 16 MFMA steps, 64-vector tiles
    (50, 612, 64, 20, 2.0, 45, False, 4),        # 32-vector tiles
    (200, 64, 2048, 8, 1.0, 46, False, 128),     # several workgroups along the functions
    (1, 128, 16, 4, 1.0, 47, False, 1),          # one vector, one table
    (333, 128, 384, 32, 8.0, 51, False, 24),     # two blocks per wave with idle waves: whole-line stores
    (150, 128, 1024, 16, 2.0, 52, False, 32),    # tables of 32 = a wave's two blocks; two workgroups along the functions
    (40, 130, 64, 16, 1.0, 48, False, 8),        # n not a multiple of 4: gather kernels
    (90, 960, 128, 128, 1.0, 49, False, 8),      # 64 < m <= 128: 32 MFMA steps, 16-vector tiles (the GIST shape's geometry)
    (300, 256, 512, 100, 4.0, 53, True, 32),     # 32 steps with padded samples, 64-vector tiles
    (33, 1260, 64, 65, 2.0, 54, False, 4),       # the widest n the 32-step kernel takes
    (40, 1264, 64, 65, 2.0, 55, False, 4),       # one more: the kernel for large dimensions, five ranges in eight stages
    (40, 960, 128, 160, 1.0, 56, False, 8),      # m > 128: the same kernel, four ranges (the last one of 192 coordinates)
    (100, 4096, 256, 64, 8.0, 57, False, 16),    # 16 stages, tables of 16 = one block each, four blocks per wave with idle ones
    (37, 4100, 96, 40, 2.0, 58, True, 8),        # a seventeenth range of 4 coordinates in 24 stages, tables of 12, duplicates in S
    (50, 2048, 1024, 30, 4.0, 59, False, 64),    # eight blocks per wave
    (20, 4096, 4096, 64, 8.0, 60, False, 128),   # tables of 32 (two blocks each), four workgroups along the functions
    (33, 16384, 128, 512, 1.0, 61, False, 4),    # 64 stages
    (1, 4096, 64, 32, 4.0, 62, False, 4),        # one vector, one block per wave and idle blocks
    (17, 8192, 2048, 4, 8.0, 63, False, 128),    # four samples per table: most lists of a range are empty
    (45, 1264, 256, 200, 2.0, 64, True, 16),     # just above the whole-vector kernel's n: a fifth range of 240 coordinates, duplicates in S
    (40, 128, 60, 16, 1.0, 50, False, 10),       # tables of 6: gather kernels
    (60, 4096, 64, 48, 2.0, 67, False, 16),      # tables of 4: keys folded from one lane group of a block
    (61, 5000, 128, 80, 2.0, 68, True, 16),      # tables of 8: two lane groups
    (20, 40000, 64, 100, 2.0, 65, False, 4),     # 157 ranges in 160 stages, most of them without a turn
    (3, 262144, 512, 64, 4.0, 66, True, 2),      # 1024 stages (the table of turns takes 4 KB of LDS), tables of 256 functions
]


@pytest.mark.parametrize("N,n,k,m,w,seed,repl,L", SHARED)
def test_shared_sample_shapes(lsh, N, n, k, m, w, seed, repl, L):
    say(f"shared case N={N} n={n} k={k} m={m} w={w} seed={seed} repl={repl} L={L}")
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    data = torch.randn((N, n), generator=g, device="cuda") * 3.0
    with lsh.LshParams(n, k, m, w, seed, with_replacement=repl, shared_tables=L) as p:
        idx, coef, off = oracle.params_shared(n, k, m, w, seed, L, with_replacement=repl)
        assert np.array_equal(p.indices(), idx) and np.array_equal(p.coeffs().view(np.uint32), coef.view(np.uint32))
        say(_compare_all(lsh, p, data, np.arange(N), L=L, label=f"shared{seed}"))


@pytest.mark.parametrize("fp32_only", [False, True])
@pytest.mark.parametrize("N,n,k", [(130, 128, 128), (129, 100, 200), (1, 37, 5), (515, 36, 257), (64, 4096, 64),
                                   (300, 128, 192), (257, 128, 70), (400, 124, 256),
                                   # the bf16 x 3 kernel for n != 128: 256-vector x 256-function tiles in stages of
                                   # 16 coordinates; partial tiles both ways, n not a multiple of 16, k not of 4,
                                   # more function tiles than XCDs, a single vector, numbers of function tiles that
                                   # do and do not divide an XCD's workgroups, more vector tiles than XCDs
                                   (300, 960, 320), (131, 4096, 520), (257, 132, 260), (1000, 64, 2304), (1, 16, 4),
                                   (128, 20, 256), (640, 512, 1027), (3000, 64, 512), (2500, 48, 768)])
def test_dense_shapes(lsh, N, n, k, fp32_only):
    say(f"dense case N={N} n={n} k={k} fp32_only={fp32_only}")
    g = torch.Generator(device="cuda")
    g.manual_seed(N * 7 + n)
    # long rows: unit-variance data and w = 8 as in the high-dimensional workload (fp32 accumulation over
    # thousands of terms resolves a bucket boundary to about 1e-4 w only while sum |a_i v_i| / w stays in the hundreds)
    scale, w = (2.0, 1.5) if n < 512 else (1.0, 8.0)
    data = torch.randn((N, n), generator=g, device="cuda") * scale
    with lsh.LshParams(n, k, n, w, N + n + k) as p:
        say(_compare_all(lsh, p, data, np.arange(N), label=f"dense{N}x{n}x{k}", dense=True, signs=False,
                         dense_fp32=fp32_only))


@pytest.mark.parametrize("fp32_only", [False, True])
@pytest.mark.parametrize("N,k,w", [(1, 128, 2.0), (128, 128, 4.0), (127, 256, 1.5), (3000, 384, 2.0), (40000, 512, 0.5),
                                   (2049, 1152, 3.0), (65, 32, 1.0), (64, 96, 2.5), (1000, 288, 8.0), (333, 544, 1.0)])
def test_dense_n128_shapes(lsh, N, k, w, fp32_only):
    """n = 128 has kernels of its own, in both arithmetics (bf16 x 3 for k a multiple of 32, fp32
    MFMA with a lean variant for k a multiple of 128): single partial tile, exactly one full tile,
    several slices of functions, idle waves, more row tiles than workgroups, w a power of two or
    not.  The tolerances are the same for both."""
    say(f"dense n=128 case N={N} k={k} w={w} fp32_only={fp32_only}")
    g = torch.Generator(device="cuda")
    g.manual_seed(N * 3 + k)
    data = torch.randn((N, 128), generator=g, device="cuda") * 2.0
    with lsh.LshParams(128, k, 128, w, N + k) as p:
        say(_compare_all(lsh, p, data, np.arange(N) if N <= 4096 else workloads.sample_rows(N, 2048).numpy(),
                         label=f"dense128-{N}x{k}", dense=True, signs=False, dense_fp32=fp32_only))


@pytest.mark.parametrize("N,k,m,repl,seed", [(1, 64, 32, False, 61), (64, 128, 30, True, 62), (1000, 512, 32, False, 63),
                                             (333, 320, 128, False, 64), (4097, 1024, 8, True, 65)])
def test_signs_n128_matrix_core_kernel(lsh, N, k, m, repl, seed):
    """Sign hashes at n = 128 and k a multiple of 64 run on the matrix cores from the coefficients
    written out densely (sampling with replacement sums repeated coordinates): partial tiles,
    idle waves, several slices of functions, m = n.  Data with a heavy tail, so that the terms
    the two-way split leaves out matter if they are mishandled."""
    say(f"signs n=128 case N={N} k={k} m={m} repl={repl}")
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    data = torch.randn((N, 128), generator=g, device="cuda") * torch.exp(
        2.0 * torch.randn((N, 128), generator=g, device="cuda"))
    with lsh.LshParams(128, k, m, 4.0, seed, with_replacement=repl) as p:
        idx, coef, _ = _tables(p)
        w_ora, pr, npd = oracle.signs(data.cpu().numpy(), idx, coef, nthreads=THREADS, want_proj=True, want_norm_prod=True)
        w_gpu = lsh.hash_signs(p, data)
        torch.cuda.synchronize()
        excluded = check_signs(w_gpu.cpu().numpy().view(np.uint64), w_ora, pr, npd, k, "signs128")
        say(f"excluded {excluded:.2e}")
        assert excluded < 1e-3


@pytest.mark.parametrize("k,tiles,tail", [(512, 40, 17), (96, 2, 2), (320, 1, 0), (64, 0, 9), (1024, 300, 63)])
def test_dense_split_levels_by_tile(lsh, k, tiles, tail):
    """The bf16 split kernels skip the products of terms that are zero for a whole tile of 64
    vectors: byte-valued tiles (one term), tiles of 16-bit values (two terms), general tiles, and
    tiles that are byte-valued but for one element, in one batch and in an order that makes every
    workgroup meet several kinds; ids, projections and signs against the oracle."""
    g = torch.Generator(device="cuda")
    g.manual_seed(77 + k)
    N = 64 * tiles + tail
    data = torch.randn((N, 128), generator=g, device="cuda") * 40.0
    kind = torch.randint(0, 4, (tiles + 1,), generator=g, device="cuda")
    for t in range(tiles + 1):
        rows = slice(64 * t, min(N, 64 * (t + 1)))
        kd = int(kind[t])
        if kd == 0:
            data[rows] = torch.round(data[rows]).clamp(-255, 255)                  # 8 significant bits
        elif kd == 1:
            data[rows] = torch.round(data[rows] * 256.0).clamp(-65535, 65535) / 256.0  # 16 significant bits
        elif kd == 2:
            data[rows] = torch.round(data[rows]).clamp(-255, 255)
            data[rows.start + 5, 77] = 0.1234567                                  # one general element
    rows_all = np.arange(N) if N <= 4096 else workloads.sample_rows(N, 3000).numpy()
    with lsh.LshParams(128, k, 128, 16.0, 5) as p:
        say("levels dense", _compare_all(lsh, p, data, rows_all, label="levels-dense", dense=True, signs=True))
    with lsh.LshParams(128, k, 32, 16.0, 6) as p:
        say("levels signs", _compare_all(lsh, p, data, rows_all, label="levels-fast", signs=True))


@pytest.mark.parametrize("n", [128, 960])
def test_dense_split_products_error(lsh, n):
    """The bf16 x 3 product (both kernels: n = 128 and the general one) against the fp64 oracle on
    data with a wide range of magnitudes in one vector: the error stays at the level of fp32
    rounding (a few 2^-24 of sum |a_i v_i|), far inside the 1e-5 bound, and no worse than twice
    the fp32 MFMA path's."""
    N, k = 512, 256
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    data = torch.randn((N, n), generator=g, device="cuda") * torch.exp(
        6.0 * torch.randn((N, n), generator=g, device="cuda"))
    with lsh.LshParams(n, k, n, 4.0, 99) as p:
        _, coef, off = _tables(p)
        ora = oracle.e2lsh(data.cpu().numpy(), coef, off, p.w, nthreads=THREADS, want=("proj", "abs_sum"))
        split = lsh.project_e2lsh(p, data).cpu().numpy()
        p.set_dense_arithmetic(lsh.DENSE_FP32)
        plain = lsh.project_e2lsh(p, data).cpu().numpy()
    err_split = float((np.abs(split - ora["proj"]) / ora["abs_sum"]).max())
    err_plain = float((np.abs(plain - ora["proj"]) / ora["abs_sum"]).max())
    say(f"worst |error| / sum|a v|: bf16 x 3 {err_split:.3e}, fp32 MFMA {err_plain:.3e}")
    assert err_split < 2e-6 and err_split < 2.0 * err_plain + 2.0 ** -22


@pytest.mark.parametrize("N,n,k,m,seed", [(203, 128, 512, 32, 51),     # register lists, whole tiles + tail
                                          (4500, 128, 288, 128, 56),   # m = n, idle waves, many tiles
                                          (300, 128, 256, 32, 57),     # w not a power of two
                                          (19, 128, 64, 32, 52),       # one small workgroup
                                          (77, 960, 1024, 128, 53),    # streamed lists
                                          (45, 16384, 640, 96, 54),    # coordinate-range chunks
                                          (30, 4096, 192, 64, 55)])    # 8-vector tiles
def test_fused_key_group_sizes(lsh, N, n, k, m, seed):
    """Fused hashing + packing for every supported group size g = k / L (1 ... 64): the keys equal
    the oracle's packing of the oracle's ids wherever no id of the key lies in the boundary band."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    data = torch.randn((N, n), generator=g, device="cuda") * 3.0
    with lsh.LshParams(n, k, m, 2.5 if seed == 57 else 4.0, seed) as p:
        idx, coef, off = _tables(p)
        ora = oracle.fastlsh(data.cpu().numpy(), idx, coef, off, p.w, nthreads=THREADS, want=("ids", "frac"))
        near = (ora["frac"] < BAND) | (ora["frac"] > 1.0 - BAND)
        for gs in (1, 2, 4, 8, 16, 32, 64):
            if k % gs:
                continue
            L = k // gs
            key_near = near.reshape(N, L, gs).any(axis=2)
            assert key_near.mean() < 0.05
            # n = 128 with 4 ... 32 functions per table folds the keys in the matrix-core kernel by
            # default: the gathered kernel's fold is checked there too
            for mode in ((lsh.DENSE_AUTO, lsh.DENSE_FP32) if n == 128 else (lsh.DENSE_AUTO,)):
                say(f"fused keys N={N} n={n} k={k} m={m} g={gs} mode={mode}")
                p.set_dense_arithmetic(mode)
                fused = lsh.hash_fastlsh_keys(p, data, L)
                torch.cuda.synchronize()
                p.set_dense_arithmetic(lsh.DENSE_AUTO)
                got = fused.cpu().numpy().view(np.uint64)
                bad = (got != oracle.pack_keys(ora["ids"], L)) & ~key_near
                assert not bad.any(), f"g={gs} mode={mode}: {int(bad.sum())} keys differ outside the boundary band"


@pytest.mark.parametrize("k,L", [(64, 16), (64, 1), (512, 2), (1024, 2), (96, 8), (60, 60), (256, 32), (100, 5)])
def test_pack_keys_group_sizes(lsh, k, L):
    """Key packing is exact integer work: bit-exact against the oracle for every group size
    (16-byte quad path, generic path, one id per key), on ids that use the full int32 range."""
    N = 777
    g = torch.Generator(device="cuda")
    g.manual_seed(k * 131 + L)
    ids = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, k), generator=g, device="cuda", dtype=torch.int64).to(torch.int32)
    with lsh.LshParams(128, k, 8, 1.0, 5) as p:
        keys = lsh.pack_keys(p, ids, L)
        torch.cuda.synchronize()
        want = oracle.pack_keys(ids.cpu().numpy(), L)
        assert np.array_equal(keys.cpu().numpy().view(np.uint64), want)


@pytest.mark.parametrize("N,n,k,m,L,w,fp32,shared", [
    (1000, 128, 512, 32, 32, 16.0, False, 0),    # matrix-core kernel, tables of 16
    (333, 128, 256, 32, 64, 4.0, False, 0),      # tables of 4
    (333, 128, 256, 32, 32, 3.0, False, 0),      # tables of 8, w not a power of two
    (65, 128, 64, 16, 2, 4.0, False, 0),         # tables of 32
    (1, 128, 512, 32, 32, 16.0, False, 0),       # one vector
    (500, 128, 512, 32, 32, 16.0, True, 0),      # fp32 arithmetic: register-list kernel, two launches inside the call
    (300, 128, 96, 32, 48, 4.0, False, 0),       # tables of 2: two launches
    (257, 960, 1024, 128, 64, 1.0, False, 0),    # streamed lists, 16-vector tiles, tables of 16
    (90, 960, 256, 100, 64, 0.75, False, 0),     # tables of 4, w not a power of two
    (100, 4096, 2048, 64, 128, 8.0, False, 0),   # ranged kernel, tables of 16
    (37, 4100, 512, 40, 8, 2.0, False, 0),       # ranged kernel, tables of 64, ragged last range
    (50, 2048, 520, 30, 130, 4.0, False, 0),     # ranged kernel, k not a multiple of 64
    (200, 128, 512, 32, 32, 16.0, False, 32),    # one sample per table: two launches
    (70, 4096, 256, 64, 16, 8.0, False, 16),     # one sample per table at large n, tables of 16: one launch
    (45, 5000, 96, 50, 12, 3.0, False, 12),      # tables of 8, idle blocks, w not a power of two
    (30, 4096, 128, 64, 4, 8.0, False, 4),       # tables of 32 = two blocks: two launches
])
def test_ids_and_keys_in_one_call(lsh, N, n, k, m, L, w, fp32, shared):
    """lsh_hash_fastlsh_ids_keys: the ids are those of lsh_hash_fastlsh bit for bit, and the keys
    are the fold (Sec. 3.2) of exactly those ids, checked with the oracle's packing."""
    g = torch.Generator(device="cuda")
    g.manual_seed(N * 7 + n)
    scale = 40.0 if n == 128 else 1.0
    data = torch.randn((N, n), generator=g, device="cuda") * scale
    p = lsh.LshParams(n, k, m, w, 77, shared_tables=shared) if shared else lsh.LshParams(n, k, m, w, 77)
    with p:
        if fp32:
            p.set_dense_arithmetic(lsh.DENSE_FP32)
        want_ids = lsh.hash_fastlsh(p, data)
        # outputs pre-filled: every element must be written
        ids = torch.full((N, k), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        keys = torch.full((N, L), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
        lsh.hash_fastlsh_ids_keys(p, data, L, out_ids=ids, out_keys=keys)
        torch.cuda.synchronize()
        assert torch.equal(ids, want_ids)
        want_keys = oracle.pack_keys(ids.cpu().numpy(), L)
        assert np.array_equal(keys.cpu().numpy().view(np.uint64), want_keys)


def test_empty_input_and_errors(lsh):
    with lsh.LshParams(128, 64, 32, 4.0, 1) as p:
        data = torch.empty((0, 128), device="cuda")
        assert lsh.hash_fastlsh(p, data).shape == (0, 64)
        assert lsh.hash_signs(p, data).shape == (0, 1)
        x = torch.zeros((4, 128), device="cuda")
        with pytest.raises(lsh.LshError) as e:          # dense path needs m == n
            lsh.hash_e2lsh(p, x)
        assert e.value.status == -1
        ids = lsh.hash_fastlsh(p, x)
        with pytest.raises(lsh.LshError) as e:          # k % L != 0
            lsh.pack_keys(p, ids, 5)
        assert e.value.status == -1
        with pytest.raises(lsh.LshError) as e:          # k % L != 0 on the fused path too
            lsh.hash_fastlsh_keys(p, x, 5)
        assert e.value.status == -1
        with pytest.raises(lsh.LshError) as e:
            lsh.hash_fastlsh_ids_keys(p, x, 5)
        assert e.value.status == -1
        i0, k0 = lsh.hash_fastlsh_ids_keys(p, data, 8)
        assert i0.shape == (0, 64) and k0.shape == (0, 8)
    with lsh.LshParams(50000, 8, 4, 1.0, 1) as p:       # one vector does not fit in LDS
        with pytest.raises(lsh.LshError) as e:
            lsh.hash_fastlsh(p, torch.zeros((2, 50000), device="cuda"))
        assert e.value.status == -4
    with lsh.LshParams(96, 48, 8, 1.0, 1) as p:         # g = 48 / 4 = 12: fused keys unsupported
        with pytest.raises(lsh.LshError) as e:
            lsh.hash_fastlsh_keys(p, torch.zeros((2, 96), device="cuda"), 4)
        assert e.value.status == -4


def test_zero_vector_and_sign_of_zero(lsh):
    # v = 0: every projection is exactly 0, so h_j = floor(b_j / w) = 0 and every sign bit is 1
    with lsh.LshParams(128, 100, 32, 4.0, 3) as p:
        x = torch.zeros((3, 128), device="cuda")
        assert int(lsh.hash_fastlsh(p, x).abs().max()) == 0
        words = lsh.hash_signs(p, x).cpu().numpy().view(np.uint64)
        assert int(words[0, 0]) == 2 ** 64 - 1 and int(words[0, 1]) == 2 ** 36 - 1


def test_scaling_invariance_on_gpu(lsh):
    # (alpha v, alpha w, alpha b) gives the same ids (Sec. 4.2 fact); exact for alpha = 2^t,
    # which needs identical tables, so the seed is kept and only w scales: b = u*w scales too
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    data = torch.randn((500, 128), generator=g, device="cuda")
    with lsh.LshParams(128, 256, 32, 4.0, 9) as p1, lsh.LshParams(128, 256, 32, 32.0, 9) as p2:
        assert np.array_equal(p1.offsets() * np.float32(8), p2.offsets())
        h1 = lsh.hash_fastlsh(p1, data)
        h2 = lsh.hash_fastlsh(p2, data * 8.0)
        assert torch.equal(h1, h2)


# ---------------------------------------------------------------------------------------
# full-size workloads, sampled rows, benchmark launch configuration
# ---------------------------------------------------------------------------------------

def _sampled(N, count):
    return workloads.sample_rows(N, count).numpy()


def test_sift_full_size(lsh):
    wl, data = workloads.make_data("sift", "cuda")
    rows = _sampled(wl.N, 32768)
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed) as p:
        say("sift fastlsh", _compare_all(lsh, p, data, rows, L=wl.L, label="sift"))
    with lsh.LshParams(wl.n, wl.k, wl.n, wl.w, wl.seed) as p:
        say("sift e2lsh", _compare_all(lsh, p, data, rows, label="sift-dense", dense=True, signs=False))


def test_sift_full_size_shared_sample(lsh):
    wl, data = workloads.make_data("sift", "cuda")
    rows = _sampled(wl.N, 32768)
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed, shared_tables=wl.L) as p:
        say("sift shared-sample fastlsh", _compare_all(lsh, p, data, rows, L=wl.L, label="sift-shared"))


def test_gist_full_size_shared_sample(lsh):
    wl, data = workloads.make_data("gist", "cuda")
    rows = _sampled(wl.N, 8192)
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed, shared_tables=wl.L) as p:
        say("gist shared-sample fastlsh", _compare_all(lsh, p, data, rows, L=wl.L, label="gist-shared", signs=False))


def test_highdim_full_size_shared_sample(lsh):
    """The high-dimensional workload with one sample per table (L = 128 tables of 16 functions) at
    m = 64: the matrix-core kernel for large dimensions, in the launch configuration the benchmark times."""
    wl, data = workloads.make_data("highdim", "cuda")
    rows = _sampled(wl.N, 4096)
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed, shared_tables=wl.L) as p:
        say("highdim shared sample", _compare_all(lsh, p, data, rows, label="highdim-shared", signs=False))


def test_gist_full_size(lsh):
    wl, data = workloads.make_data("gist", "cuda")
    rows = _sampled(wl.N, 8192)
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed) as p:
        say("gist fastlsh", _compare_all(lsh, p, data, rows, L=wl.L, label="gist", signs=False))
    with lsh.LshParams(wl.n, wl.k, wl.n, wl.w, wl.seed) as p:
        say("gist e2lsh", _compare_all(lsh, p, data, rows, label="gist-dense", dense=True, signs=False))


def test_highdim_full_size(lsh):
    wl, data = workloads.make_data("highdim", "cuda")
    rows = _sampled(wl.N, 4096)
    # planted near-duplicates and their sources: collision counts must separate them from random pairs
    src = wl.extra["planted_src"].numpy()
    planted_rows = np.arange(wl.N - wl.planted, wl.N)
    for m in wl.m:
        with lsh.LshParams(wl.n, wl.k, m, wl.w, wl.seed) as p:
            say(f"highdim m={m}", _compare_all(lsh, p, data, rows, label=f"highdim-m{m}", signs=False))
            ids = lsh.hash_fastlsh(p, data)
            a = ids[torch.as_tensor(planted_rows[:256], device="cuda")]
            b = ids[torch.as_tensor(src[:256], device="cuda")]
            c = ids[torch.as_tensor(src[1:257], device="cuda")]
            near = (a == b).float().mean().item()
            far = (a == c).float().mean().item()
            say(f"  collision rate planted {near:.3f} random {far:.3f}")
            assert near > far + 0.2
    with lsh.LshParams(wl.n, wl.k, wl.n, wl.w, wl.seed) as p:
        say("highdim e2lsh", _compare_all(lsh, p, data, rows[:512], label="highdim-dense", dense=True, signs=False))


def test_angular_full_size(lsh):
    wl, data = workloads.make_data("angular", "cuda")
    rows = _sampled(wl.N, 4096)
    idxs = torch.as_tensor(rows, device="cuda")
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed) as p:
        idx, coef, _ = _tables(p)
        sub = data[idxs].cpu().numpy()
        w_ora, pr, npd = oracle.signs(sub, idx, coef, nthreads=THREADS, want_proj=True, want_norm_prod=True)
        w_gpu = lsh.hash_signs(p, data)
        torch.cuda.synchronize()
        ex = check_signs(w_gpu[idxs].cpu().numpy().view(np.uint64), w_ora, pr, npd, p.k, "angular")
        say("angular signs excluded fraction", ex)


def test_bucket_ids_saturate_outside_int32(lsh):
    """Projections beyond +-2^31 buckets come out as INT32_MAX / INT32_MIN on every path (the
    conversion saturates); the oracle's fp64 value says which elements those are."""
    N, n, k, L = 300, 128, 128, 8
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    data = torch.randn((N, n), generator=g, device="cuda") * 3.0e10
    data[::7] *= 1e-9                                   # some vectors stay in range
    host = data.cpu().numpy()
    lo, hi = -2 ** 31, 2 ** 31 - 1
    for m, shared in ((32, 0), (32, L), (n, 0)):
        with lsh.LshParams(n, k, m, 1.0, 5, shared_tables=shared) as p:
            idx, coef, off = _tables(p)
            terms = host.astype(np.float64)[:, idx.astype(np.int64)] * coef.astype(np.float64)[None]
            val, abs_sum = terms.sum(axis=2) + off, np.abs(terms).sum(axis=2)
            want = np.clip(np.floor(val), lo, hi)
            sure = (np.abs(val) > 2.0 ** 31 * 1.001) | (np.abs(val) < 2.0 ** 31 * 0.999)
            calls = [lsh.hash_fastlsh] + ([lsh.hash_e2lsh] if m == n else [])
            for call in calls:
                got = call(p, data).cpu().numpy().astype(np.float64)
                big = np.abs(val) > 2.0 ** 31 * 1.001
                assert big.any() and (~big).any()
                assert np.array_equal(got[big], want[big]), f"{call.__name__} m={m} shared={shared}: saturation"
                inside = sure & ~big          # in range: the id within the projection tolerance (w = 1)
                assert (np.abs(got[inside] - want[inside]) <= 1.0 + 1e-5 * abs_sum[inside]).all()
