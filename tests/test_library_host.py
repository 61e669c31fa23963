"""Host-side checks of liblsh that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments, and draws tables bit-identical to the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2309_15479_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    header = open(os.path.join(ROOT, "include", "lsh.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(lsh_[a-z0-9_]+)\s*\(", header)))
    assert declared == sorted(binding.EXPORTS)
    lib = binding.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings():
    assert binding.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert binding.status_string(code) not in ("ok", "unknown status")
    assert binding.status_string(-99) == "unknown status"


@pytest.mark.parametrize("args", [
    (0, 4, 1, 1.0), (8, 0, 4, 1.0), (8, 4, 0, 1.0), (8, 4, 9, 1.0), (8, 4, 4, 0.0), (8, 4, 4, -1.0),
    (8, 4, 4, float("nan")), (8, 4, 4, float("inf")),
])
def test_create_rejects_bad_arguments(args):
    n, k, m, w = args
    with pytest.raises(binding.LshError) as e:
        binding.LshParams(n, k, m, w, 1)
    assert e.value.status == -1


def test_null_and_flag_arguments():
    lib = binding.load_library()
    assert lib.lsh_params_create(8, 4, 4, 1.0, 1, None) == -1
    h = ctypes.c_void_p()
    assert lib.lsh_params_create_ex(8, 4, 4, 1.0, 1, 7, ctypes.byref(h)) == -1
    assert lib.lsh_params_get_indices(None, None) == -1
    assert lib.lsh_hash_fastlsh(None, None, 1, None, None) == -1
    assert lib.lsh_hash_fastlsh(None, None, 0, None, None) == -1   # no params object
    lib.lsh_params_destroy(None)          # no-op
    assert lib.lsh_params_set_dense_arithmetic(None, 0) == -1


def test_dense_arithmetic_modes():
    with binding.LshParams(128, 64, 32, 4.0, 1) as p:
        p.set_dense_arithmetic(binding.DENSE_FP32)
        p.set_dense_arithmetic(binding.DENSE_AUTO)
        p.set_dense_arithmetic(binding.DENSE_MATRIX)     # n == 128: nothing more to build
        p.set_dense_arithmetic(binding.DENSE_AUTO)
        with pytest.raises(binding.LshError) as e:
            p.set_dense_arithmetic(3)
        assert e.value.status == -1
    with binding.LshParams(961, 64, 100, 4.0, 1) as p:   # n not a multiple of 4: no matrix-core kernel
        with pytest.raises(binding.LshError) as e:
            p.set_dense_arithmetic(binding.DENSE_MATRIX)
        assert e.value.status == -4
    with binding.LshParams(960, 64, 100, 4.0, 1) as p:   # builds device tables: needs a device
        try:
            p.set_dense_arithmetic(binding.DENSE_MATRIX)
        except binding.LshError as e:
            assert e.status == -5


CASES = [
    (128, 64, 32, 4.0, 1, False), (128, 64, 128, 4.0, 1, False),         # tiny + its E2LSH twin
    (128, 512, 32, 16.0, 2, False), (960, 1024, 128, 1.0, 3, False),
    (4096, 2048, 64, 8.0, 4, False), (4096, 2048, 1024, 8.0, 4, False),
    (16384, 4096, 512, 1.0, 5, False),
    (100, 70, 30, 2.5, 11, True), (100, 70, 30, 2.5, 11, False), (7, 3, 1, 0.3, 12, True),
    (37, 130, 37, 1.0, 13, True),
]


@pytest.mark.parametrize("n,k,m,w,seed,repl", CASES)
def test_tables_bit_identical_to_oracle(n, k, m, w, seed, repl):
    with binding.LshParams(n, k, m, w, seed, with_replacement=repl) as p:
        idx, coef, off = oracle.params(n, k, m, w, seed, with_replacement=repl)
        assert np.array_equal(p.indices(), idx)
        assert np.array_equal(p.coeffs().view(np.uint32), coef.view(np.uint32))
        assert np.array_equal(p.offsets().view(np.uint32), off.view(np.uint32))
        s = p.shape()
        assert (s["n"], s["k"], s["m"], s["flags"], s["seed"]) == (n, k, m, int(repl), seed)
        assert s["w"] == np.float32(w)


@pytest.mark.parametrize("n,k,m,w,seed,repl,L", [
    (128, 512, 32, 16.0, 2, False, 32), (128, 64, 32, 4.0, 1, False, 8), (100, 72, 30, 2.5, 11, True, 6),
    (960, 1024, 128, 1.0, 3, False, 64), (64, 60, 64, 1.0, 4, False, 5), (50, 48, 7, 2.0, 9, False, 48),
])
def test_shared_sample_tables_bit_identical_to_oracle(n, k, m, w, seed, repl, L):
    with binding.LshParams(n, k, m, w, seed, with_replacement=repl, shared_tables=L) as p:
        idx, coef, off = oracle.params_shared(n, k, m, w, seed, L, with_replacement=repl)
        assert np.array_equal(p.indices(), idx)
        assert np.array_equal(p.coeffs().view(np.uint32), coef.view(np.uint32))
        assert np.array_equal(p.offsets().view(np.uint32), off.view(np.uint32))
        assert p.shared_tables() == L
        # a0 of the maximum-inner-product transform (appendix): the generator's table 3
        from oracle import mips
        assert np.array_equal(p.mips_coeffs().view(np.uint32), mips.extra_coefficients(k, seed).view(np.uint32))
    with binding.LshParams(n, k, m, w, seed, with_replacement=repl) as p:
        assert p.shared_tables() == 0
        with pytest.raises(binding.LshError):
            p.mips_coeffs()


def test_shared_sample_rejects_bad_table_count():
    with pytest.raises(binding.LshError) as e:
        binding.LshParams(128, 64, 32, 4.0, 1, shared_tables=7)
    assert e.value.status == -1


def _pass_groups(k, group):
    """Functions served by one pass of an LDS read, as the header documents them."""
    quads = {32: [list(range(8)), list(range(8, 16))],
             16: [[0, 3, 5, 6], [1, 2, 4, 7], [8, 11, 13, 14], [9, 10, 12, 15]]}[group]
    out = []
    for w0 in range(0, k, 64):
        for qs in quads:
            fn = [w0 + 4 * q + t for q in qs for t in range(4) if w0 + 4 * q + t < k]
            if fn:
                out.append(np.array(fn))
    return out


@pytest.mark.parametrize("n,k,m,repl", [(128, 512, 32, False), (100, 70, 30, True), (960, 200, 128, False),
                                        (1024, 520, 30, False)])
def test_gather_schedule_is_a_padded_permutation(n, k, m, repl):
    """The kernel may visit a function's samples in any order (a projection is a sum); the
    schedule must hold every canonical sample exactly once plus padding, and its modelled
    cost must be what its own entries imply."""
    with binding.LshParams(n, k, m, 1.0, 77, with_replacement=repl) as p:
        order, group, classes, passes = p.schedule()
        idx = p.indices()
        steps = order.shape[1]
        assert steps % 32 == 0 and m <= steps < m + 32
        pad = (order & 0x80000000) != 0
        copy_b = ~pad & ((order & 0x40000000) != 0)      # sample read from the class-rotated tile copy
        pos = np.where(pad, 0, order & 0x3fffffff).astype(np.int64)
        assert (pad.sum(axis=1) == steps - m).all()
        for j in range(k):
            assert sorted(pos[j][~pad[j]].tolist()) == list(range(m))
        assert ((order[pad] & 0x7fffffff) < classes).all()
        # recompute the modelled cost: per pass group and step, the most popular class
        coord = np.take_along_axis(idx, pos, axis=1).astype(np.int64)
        rotated = (coord + coord // classes) % classes
        cls = np.where(pad, order & 0x7fffffff, np.where(copy_b, rotated, coord % classes))
        groups = _pass_groups(k, group)
        total = 0
        for fn in groups:
            block = cls[fn]                                  # [lanes, steps]
            for i in range(steps):
                total += np.bincount(block[:, i], minlength=classes).max()
        assert total == passes
        assert passes >= len(groups) * steps
        # far better than visiting samples in draw order
        naive = 0
        for fn in groups:
            block = idx[fn] % classes
            for i in range(m):
                naive += np.bincount(block[:, i], minlength=classes).max()
        if m >= 30 and k >= group:
            assert passes / (len(groups) * steps) < 0.75 * naive / (len(groups) * m)
        if copy_b.any():    # two tile copies: every sample has two classes to choose from
            assert passes / (len(groups) * steps) < 1.05


@pytest.mark.parametrize("n,k,m,repl", [(16384, 520, 40, False), (30000, 512, 33, True), (4096, 600, 256, False)])
def test_windowed_gather_schedule_is_a_padded_permutation(n, k, m, repl):
    """Large n: the samples are visited range by range (a sample of range r in one of the
    stages r - 6 .. r of the tile), all functions of a workgroup in lockstep.  Every canonical
    sample must still appear exactly once and the functions of a workgroup must have rows of
    equal length; that every entry's range is in the ring when it is read is checked by
    walking the device tables (test_list_tables_walked_on_the_host)."""
    with binding.LshParams(n, k, m, 1.0, 78, with_replacement=repl) as p:
        order, group, classes, passes = p.schedule()
        unused = order == 0xFFFFFFFF
        pad = ~unused & ((order & 0x80000000) != 0)
        real = ~unused & ~pad
        assert group == 16 and classes == 16
        used_len = (~unused).sum(axis=1)
        assert len(set(used_len.tolist())) == 1                # k <= 2048: one workgroup
        assert (used_len % 4 == 0).all()                       # lists are stored as quads of entries
        for j in range(k):
            row = order[j][real[j]]
            assert sorted(row.tolist()) == list(range(m))
            assert not unused[j][:used_len[j]].any()           # the unused part is a tail
        assert ((order[pad] & 0x7fffffff) < classes).all()
        assert passes >= (~unused).sum() / group
        assert p.check_lists() < 1e-12


@pytest.mark.parametrize("n,k,m,entries,lds", [(4096, 2048, 64, 1.15, 1.25), (4096, 2048, 256, 1.05, 1.15),
                                               (16384, 4096, 512, 1.10, 1.10)])
def test_windowed_gather_schedule_needs_little_padding(n, k, m, entries, lds):
    """The shapes of the high-dimensional workloads: entries visited per sample, and modelled
    LDS passes per conflict-free pass, stay within the bounds the kernel's timing relies on
    (with one fixed stage per 1024-coordinate range they were 1.63 / 1.28 / 1.47 entries per
    sample)."""
    with binding.LshParams(n, k, m, 8.0, 4) as p:
        order, group, classes, passes = p.schedule()
        used = int((order != 0xFFFFFFFF).sum())
        assert used / (k * m) <= entries
        assert passes / (used / group) <= lds


@pytest.mark.parametrize("n,k,m,w,seed,repl,L", [
    (4096, 2048, 64, 8.0, 4, False, 0),      # ranged gather kernel, four functions per lane
    (4096, 520, 256, 8.0, 5, True, 0),       # k not a multiple of 64, duplicates in S
    (4100, 512, 40, 2.0, 6, False, 0),       # seventeen ranges in 24 stages, the last of four coordinates
    (16384, 1024, 96, 1.0, 7, False, 0),     # 64 ranges
    (2049, 512, 7, 2.0, 38, False, 0),       # one function per lane, one-quad blocks, odd n
    (2304, 1536, 100, 1.0, 39, True, 0),     # three functions per lane
    (9004, 2048, 700, 4.0, 40, False, 0),    # 36 ranges in 40 stages
    (3000, 1000, 33, 1.0, 41, True, 0),      # two functions per lane, k not a multiple of 64
    (16384, 4096, 512, 1.0, 5, False, 0),    # two workgroups along the functions
    (4096, 2048, 64, 8.0, 4, False, 128),    # one sample per table: 16 stages, some of them without a turn of the list ring
    (4096, 2048, 256, 8.0, 4, False, 128),   # several turns per stage
    (4096, 1024, 1024, 8.0, 4, False, 32),   # tables of 32 functions (two blocks), eight blocks per wave
    (4100, 96, 40, 2.0, 58, True, 8),        # tables of 12, idle blocks, a seventeenth range of four coordinates in 24 stages
    (8192, 2048, 4, 8.0, 63, False, 128),    # nearly empty lists
    (1264, 64, 65, 2.0, 55, False, 4),       # five ranges in eight stages, four blocks per wave (turns of eight steps per block)
    (16384, 128, 512, 1.0, 61, False, 4),    # 64 stages
    (2048, 1024, 30, 4.0, 59, False, 64),    # one ring of ranges holds the whole vector
    (40000, 64, 100, 2.0, 65, False, 4),     # 157 ranges in 160 stages
    (1000000, 16, 8, 2.0, 3, False, 1),      # 3912 stages: the table of turns nearly fills what LDS the ring leaves
    (1100000, 16, 8, 2.0, 3, False, 1),      # one more ring and it no longer fits: the object falls back to the gather kernel
])
def test_list_tables_walked_on_the_host(n, k, m, w, seed, repl, L):
    """The list tables of the kernels that work by coordinate ranges, built as for the device and
    walked on the host the way the kernels walk them, give the projections of Eq. 5 taken
    straight from the canonical tables (lsh_params_check_lists; no GPU involved)."""
    with binding.LshParams(n, k, m, w, seed, with_replacement=repl, shared_tables=L) as p:
        for vector_seed in (1, 2):
            assert p.check_lists(vector_seed) < 1e-14


@pytest.mark.parametrize("n,k,m,L,steps_max", [(4096, 2048, 64, 128, 18), (4096, 2048, 256, 128, 66),
                                               (4096, 2048, 1024, 128, 260), (16384, 4096, 512, 256, 141)])
def test_shared_sample_schedule_needs_little_padding(n, k, m, L, steps_max):
    """One sample per table on the high-dimensional shapes: the stages of a tile give every table
    the same number of MFMA steps of four samples, and dealing the samples by their last possible
    stage keeps that number within a few percent of m / 4 (12 % at m = 64, where a turn of the
    list ring is two steps per block; one fixed stage per 1024-coordinate range needed 32, 96,
    320 steps on the first three shapes)."""
    with binding.LshParams(n, k, m, 8.0, 4, shared_tables=L) as p:
        stages, steps = p.shared_schedule()
        assert stages == (n + 255) // 256 and stages % 8 == 0
        assert m <= 4 * steps <= 4 * steps_max
    with binding.LshParams(n, k, m, 8.0, 4) as p:   # per-function samples: the gather kernel
        with pytest.raises(binding.LshError) as e:
            p.shared_schedule()
        assert e.value.status == -4


def test_list_check_needs_a_ranged_kernel():
    with binding.LshParams(128, 64, 32, 4.0, 1) as p:   # whole vectors in LDS, lists in registers
        with pytest.raises(binding.LshError) as e:
            p.check_lists()
        assert e.value.status == -4
