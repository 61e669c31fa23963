"""CPU fp64 oracle for l2 LSH hash evaluation -- TEST INFRASTRUCTURE ONLY.

A thin ctypes wrapper over ``fastlsh_oracle.c`` (plain C, fp64), which restates
the paper's definitions: the E2LSH hash (Sec. 2.2, Eq. 1), the sampling
operator and the FastLSH hash (Sec. 3.1, Eq. 5), the compound code (Sec. 3.2).
Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library never does, and this package imports nothing of
the GPU library.

Parity status: arithmetic pinned (see tests/test_oracle_pins.py); parameter
tables "parity unpinned" by the paper (it names no random number generator).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastlsh_oracle.c")
_LIB = os.path.join(_HERE, "libfastlsh_oracle.so")

OK, ERR_ARG, ERR_ALLOC, ERR_RANGE = 0, -1, -2, -3


def build(force=False):
    """Compile the C oracle with gcc (a second or so)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u32, u64, f32, i32 = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float, ctypes.c_int
        p = ctypes.c_void_p
        lib.oracle_philox4x64_10.argtypes = [p, p, p]
        lib.oracle_philox4x64_10.restype = None
        lib.oracle_params.argtypes = [u32, u32, u32, f32, u64, u32, p, p, p]
        lib.oracle_params_shared.argtypes = [u32, u32, u32, f32, u64, u32, u32, p, p, p]
        lib.oracle_fastlsh.argtypes = [p, u64, u32, u32, u32, p, p, p, f32, p, p, p, p, i32]
        lib.oracle_e2lsh.argtypes = [p, u64, u32, u32, p, p, f32, p, p, p, p, i32]
        lib.oracle_signs.argtypes = [p, u64, u32, u32, u32, p, p, p, p, p, i32]
        lib.oracle_pack_keys.argtypes = [p, u64, u32, u32, p]
        lib.oracle_max_threads.argtypes = []
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(status, what):
    if status != OK:
        raise ValueError(f"oracle {what}: status {status}")


def max_threads():
    return int(_load().oracle_max_threads())


def philox4x64_10(counter, key):
    """One Philox4x64-10 block: counter (4 x u64), key (2 x u64) -> 4 x u64."""
    c = _c(counter, np.uint64)
    k = _c(key, np.uint64)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, np.uint64)
    _load().oracle_philox4x64_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def params(n, k, m, w, seed, with_replacement=False):
    """Tables of the k hash functions: (idx u32 [k,m], coef f32 [k,m], off f32 [k])."""
    idx = np.empty((k, m), np.uint32)
    coef = np.empty((k, m), np.float32)
    off = np.empty(k, np.float32)
    _check(_load().oracle_params(n, k, m, w, seed, int(bool(with_replacement)),
                                 _ptr(idx), _ptr(coef), _ptr(off)), "params")
    return idx, coef, off


def params_shared(n, k, m, w, seed, L, with_replacement=False):
    """The same tables with one sample S per table of k/L functions (the table's first
    function's S); coefficients and offsets stay per function."""
    idx = np.empty((k, m), np.uint32)
    coef = np.empty((k, m), np.float32)
    off = np.empty(k, np.float32)
    _check(_load().oracle_params_shared(n, k, m, w, seed, int(bool(with_replacement)), L,
                                        _ptr(idx), _ptr(coef), _ptr(off)), "params_shared")
    return idx, coef, off


def fastlsh(data, idx, coef, off, w, nthreads=1, want=("ids",)):
    """FastLSH (Eq. 5) on row-major fp32 data [N,n]; returns a dict of the
    requested arrays among proj (f64), abs_sum (f64), ids (i32), frac (f64)."""
    data = _c(data, np.float32)
    idx = _c(idx, np.uint32)
    coef = _c(coef, np.float32)
    N, n = data.shape
    k, m = idx.shape
    assert coef.shape == (k, m)
    off_c = None if off is None else _c(off, np.float32)
    out = {name: np.empty((N, k), np.int32 if name == "ids" else np.float64) for name in want}
    _check(_load().oracle_fastlsh(_ptr(data), N, n, k, m, _ptr(idx), _ptr(coef), _ptr(off_c),
                                  float(w) if w is not None else 0.0,
                                  _ptr(out.get("proj")), _ptr(out.get("abs_sum")),
                                  _ptr(out.get("ids")), _ptr(out.get("frac")), nthreads),
           "fastlsh")
    return out


def e2lsh(data, a, off, w, nthreads=1, want=("ids",)):
    """E2LSH (Eq. 1) with dense coefficient matrix a [k,n]."""
    data = _c(data, np.float32)
    a = _c(a, np.float32)
    N, n = data.shape
    k = a.shape[0]
    assert a.shape == (k, n)
    off_c = None if off is None else _c(off, np.float32)
    out = {name: np.empty((N, k), np.int32 if name == "ids" else np.float64) for name in want}
    _check(_load().oracle_e2lsh(_ptr(data), N, n, k, _ptr(a), _ptr(off_c),
                                float(w) if w is not None else 0.0,
                                _ptr(out.get("proj")), _ptr(out.get("abs_sum")),
                                _ptr(out.get("ids")), _ptr(out.get("frac")), nthreads), "e2lsh")
    return out


def signs(data, idx, coef, nthreads=1, want_proj=False, want_norm_prod=False):
    """Packed sign hashes; returns (words u64 [N, ceil(k/64)], proj|None, norm_prod|None)."""
    data = _c(data, np.float32)
    idx = _c(idx, np.uint32)
    coef = _c(coef, np.float32)
    N, n = data.shape
    k, m = idx.shape
    words = np.empty((N, (k + 63) // 64), np.uint64)
    proj = np.empty((N, k), np.float64) if want_proj else None
    npd = np.empty((N, k), np.float64) if want_norm_prod else None
    _check(_load().oracle_signs(_ptr(data), N, n, k, m, _ptr(idx), _ptr(coef), _ptr(words),
                                _ptr(proj), _ptr(npd), nthreads), "signs")
    return words, proj, npd


def pack_keys(ids, L):
    """64-bit keys of the L groups of k/L consecutive bucket ids (Sec. 3.2)."""
    ids = _c(ids, np.int32)
    N, k = ids.shape
    keys = np.empty((N, L), np.uint64)
    _check(_load().oracle_pack_keys(_ptr(ids), N, k, L, _ptr(keys)), "pack_keys")
    return keys
