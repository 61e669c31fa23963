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
