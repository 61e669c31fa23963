"""ctypes binding of liblsh.so; names and arguments mirror include/lsh.h.

PyTorch is used for device memory and streams only: tensors are passed as raw device
pointers, the current torch stream as the hipStream_t.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblsh.so")
_lib = None

LSH_OK = 0
SAMPLE_WITHOUT_REPLACEMENT = 0
SAMPLE_WITH_REPLACEMENT = 1
DENSE_AUTO = 0
DENSE_FP32 = 1
DENSE_MATRIX = 2

EXPORTS = [
    "lsh_params_create", "lsh_params_create_ex", "lsh_params_create_shared", "lsh_params_destroy",
    "lsh_params_get_indices", "lsh_params_get_coeffs", "lsh_params_get_offsets", "lsh_params_get_shape",
    "lsh_params_get_tables", "lsh_params_get_mips_coeffs", "lsh_params_get_schedule", "lsh_params_check_lists",
    "lsh_params_get_shared_schedule",
    "lsh_params_set_dense_arithmetic",
    "lsh_hash_fastlsh",
    "lsh_hash_e2lsh", "lsh_hash_signs", "lsh_pack_keys", "lsh_hash_fastlsh_keys", "lsh_hash_fastlsh_ids_keys",
    "lsh_project_fastlsh", "lsh_project_e2lsh", "lsh_time_launches", "lsh_status_string",
    "lsh_e2lsh_collision_probability", "lsh_pair_statistics", "lsh_fastlsh_collision_probability",
    "lsh_fastlsh_moment_factors", "lsh_equivalent_width", "lsh_mips_collision_probability",
    "lsh_mips_kappa", "lsh_hash_mips_data", "lsh_hash_mips_query", "lsh_project_mips_data",
    "lsh_project_mips_query",
    "lsh_index_build", "lsh_index_destroy", "lsh_index_tables", "lsh_index_probe",
    "lsh_index_candidate_offsets", "lsh_index_candidate_offsets_static", "lsh_index_candidates", "lsh_index_nearest", "lsh_index_best_inner_product",
]


class LshError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def library_path():
    return _LIB_PATH


def load_library():
    """Loads liblsh.so (built by paper_2309_15479_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2309_15479_amd.build` "
            "(there is no fallback implementation)")
    try:
        import torch  # noqa: F401  -- so that liblsh binds to the HIP runtime torch already loaded
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    u32, u64, f32, p, i = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int
    lib.lsh_params_create.argtypes = [u32, u32, u32, f32, u64, ctypes.POINTER(p)]
    lib.lsh_params_create_ex.argtypes = [u32, u32, u32, f32, u64, u32, ctypes.POINTER(p)]
    lib.lsh_params_create_shared.argtypes = [u32, u32, u32, f32, u64, u32, u32, ctypes.POINTER(p)]
    lib.lsh_params_get_tables.argtypes = [p, p]
    lib.lsh_params_set_dense_arithmetic.argtypes = [p, i]
    lib.lsh_params_destroy.argtypes = [p]
    lib.lsh_params_destroy.restype = None
    for name in ("lsh_params_get_indices", "lsh_params_get_coeffs", "lsh_params_get_offsets",
                 "lsh_params_get_mips_coeffs"):
        getattr(lib, name).argtypes = [p, p]
    lib.lsh_params_get_shape.argtypes = [p, p, p, p, p, p, p]
    lib.lsh_params_get_schedule.argtypes = [p, p, p, p, p, p]
    for name in ("lsh_hash_fastlsh", "lsh_hash_e2lsh", "lsh_hash_signs", "lsh_project_fastlsh",
                 "lsh_project_e2lsh"):
        getattr(lib, name).argtypes = [p, p, u64, p, p]
    for name in ("lsh_hash_mips_query", "lsh_project_mips_query"):
        getattr(lib, name).argtypes = [p, p, u64, p, p]
    for name in ("lsh_hash_mips_data", "lsh_project_mips_data"):
        getattr(lib, name).argtypes = [p, p, u64, p, p, p]
    lib.lsh_mips_kappa.argtypes = [p, p, u64, i, p, p]
    lib.lsh_pack_keys.argtypes = [p, p, u64, u32, p, p]
    lib.lsh_hash_fastlsh_keys.argtypes = [p, p, u64, u32, p, p]
    lib.lsh_hash_fastlsh_ids_keys.argtypes = [p, p, u64, u32, p, p, p]
    lib.lsh_time_launches.argtypes = [p, i, p, u64, u32, p, p, i, ctypes.POINTER(f32)]
    f64 = ctypes.c_double
    lib.lsh_e2lsh_collision_probability.argtypes = [f64, f64, p]
    lib.lsh_pair_statistics.argtypes = [p, p, u32, u32, p, p]
    lib.lsh_fastlsh_collision_probability.argtypes = [f64, f64, f64, p]
    lib.lsh_fastlsh_moment_factors.argtypes = [f64, f64, p, p]
    lib.lsh_equivalent_width.argtypes = [u32, u32, f64]
    lib.lsh_equivalent_width.restype = f64
    lib.lsh_mips_collision_probability.argtypes = [f64, f64, f64, f64, p]
    lib.lsh_index_build.argtypes = [p, u64, u32, p, ctypes.POINTER(p)]
    lib.lsh_index_destroy.argtypes = [p]
    lib.lsh_index_destroy.restype = None
    lib.lsh_index_tables.argtypes = [p, p, p, p, p]
    lib.lsh_index_probe.argtypes = [p, p, u64, p, p, p]
    lib.lsh_index_candidate_offsets.argtypes = [p, u64, p, p]
    lib.lsh_index_candidate_offsets_static.argtypes = [p, u64, p, p]
    lib.lsh_index_candidates.argtypes = [p, p, p, p, u64, p, p]
    lib.lsh_index_nearest.argtypes = [p, p, p, u32, p, p, u64, u32, p, p, p]
    lib.lsh_index_best_inner_product.argtypes = [p, p, p, u32, p, p, u64, u32, p, p, p]
    lib.lsh_status_string.argtypes = [i]
    lib.lsh_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status):
    return load_library().lsh_status_string(int(status)).decode()


def _check(status, what):
    if status != LSH_OK:
        raise LshError(status, what)


class LshParams:
    """Owns one lsh_params_t (the k hash functions and their device tables)."""

    def __init__(self, n, k, m, w, seed, with_replacement=False, shared_tables=0):
        """shared_tables = L > 0: the k/L functions of each table share one sample S."""
        lib = load_library()
        handle = ctypes.c_void_p()
        flags = SAMPLE_WITH_REPLACEMENT if with_replacement else SAMPLE_WITHOUT_REPLACEMENT
        _check(lib.lsh_params_create_shared(n, k, m, w, seed, flags, shared_tables, ctypes.byref(handle)),
               "lsh_params_create_shared")
        self._h = handle
        self.n, self.k, self.m, self.w, self.seed = int(n), int(k), int(m), float(w), int(seed)

    def close(self):
        if getattr(self, "_h", None):
            load_library().lsh_params_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: module globals may already be gone
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    @property
    def handle(self):
        if not self._h:
            raise ValueError("params object is closed")
        return self._h

    def indices(self):
        out = np.empty((self.k, self.m), np.uint32)
        _check(load_library().lsh_params_get_indices(self.handle, out.ctypes.data), "get_indices")
        return out

    def coeffs(self):
        out = np.empty((self.k, self.m), np.float32)
        _check(load_library().lsh_params_get_coeffs(self.handle, out.ctypes.data), "get_coeffs")
        return out

    def offsets(self):
        out = np.empty(self.k, np.float32)
        _check(load_library().lsh_params_get_offsets(self.handle, out.ctypes.data), "get_offsets")
        return out

    def set_dense_arithmetic(self, mode):
        """DENSE_AUTO: bf16 x 3 matrix-core product where the shape allows; DENSE_FP32: fp32 MFMA;
        DENSE_MATRIX: as DENSE_AUTO, and FastLSH ids / projections with m < n as a dense product too."""
        _check(load_library().lsh_params_set_dense_arithmetic(self.handle, int(mode)), "set_dense_arithmetic")

    def mips_coeffs(self):
        """a0 [k] of the maximum-inner-product transform (objects with shared_tables > 0)."""
        out = np.empty(self.k, np.float32)
        _check(load_library().lsh_params_get_mips_coeffs(self.handle, out.ctypes.data), "get_mips_coeffs")
        return out

    def schedule(self):
        """(order u32 [k, steps], group, classes, modelled_passes) of the sampled kernel."""
        steps, group, classes = (ctypes.c_uint32() for _ in range(3))
        passes = ctypes.c_uint64()
        lib = load_library()
        _check(lib.lsh_params_get_schedule(self.handle, None, ctypes.addressof(steps), ctypes.addressof(group),
                                           ctypes.addressof(classes), ctypes.addressof(passes)), "get_schedule")
        order = np.empty((self.k, steps.value), np.uint32)
        _check(lib.lsh_params_get_schedule(self.handle, order.ctypes.data, None, None, None, None), "get_schedule")
        return order, group.value, classes.value, passes.value

    def check_lists(self, seed=1):
        """Largest relative deviation of the kernel-side list tables, walked on the host as the
        ranged kernels walk them, from the projections of the canonical tables."""
        worst = ctypes.c_double()
        lib = load_library()
        lib.lsh_params_check_lists.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
        _check(lib.lsh_params_check_lists(self.handle, seed, ctypes.addressof(worst)), "lsh_params_check_lists")
        return worst.value

    def shared_schedule(self):
        """(stages per tile, MFMA steps of four samples per block of 16 functions and tile) of the
        one-sample-per-table kernel that works by coordinate ranges."""
        stages, steps = ctypes.c_uint32(), ctypes.c_uint32()
        lib = load_library()
        lib.lsh_params_get_shared_schedule.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _check(lib.lsh_params_get_shared_schedule(self.handle, ctypes.addressof(stages), ctypes.addressof(steps)),
               "lsh_params_get_shared_schedule")
        return stages.value, steps.value

    def shared_tables(self):
        L = ctypes.c_uint32()
        _check(load_library().lsh_params_get_tables(self.handle, ctypes.addressof(L)), "get_tables")
        return L.value

    def shape(self):
        n, k, m, fl = (ctypes.c_uint32() for _ in range(4))
        w, seed = ctypes.c_float(), ctypes.c_uint64()
        _check(load_library().lsh_params_get_shape(self.handle, *(ctypes.addressof(x) for x in
                                                                  (n, k, m, fl, w, seed))), "get_shape")
        return dict(n=n.value, k=k.value, m=m.value, flags=fl.value, w=w.value, seed=seed.value)


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_in(t, dtype, cols):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()
            and t.dim() == 2 and t.shape[1] == cols):
        raise ValueError(f"expected a contiguous CUDA tensor [N,{cols}] of {dtype}")
    return t


def _out(data, N, cols, dtype, out):
    import torch
    if out is None:
        return torch.empty((N, cols), dtype=dtype, device=data.device)
    _dev_in(out, dtype, cols)
    if out.shape[0] != N:
        raise ValueError("output has the wrong number of rows")
    return out


def _hash_call(name, params, data, cols, dtype, out, stream):
    import torch
    _dev_in(data, torch.float32, params.n)
    N = data.shape[0]
    out = _out(data, N, cols, dtype, out)
    fn = getattr(load_library(), name)
    _check(fn(params.handle, data.data_ptr(), N, out.data_ptr(), _stream(stream)), name)
    return out


def hash_fastlsh(params, data, out=None, stream=None):
    import torch
    return _hash_call("lsh_hash_fastlsh", params, data, params.k, torch.int32, out, stream)


def hash_e2lsh(params, data, out=None, stream=None):
    import torch
    return _hash_call("lsh_hash_e2lsh", params, data, params.k, torch.int32, out, stream)


def hash_signs(params, data, out=None, stream=None):
    """Packed sign bits as int64 words [N, ceil(k/64)] (bit patterns of the uint64 words)."""
    import torch
    return _hash_call("lsh_hash_signs", params, data, (params.k + 63) // 64, torch.int64, out, stream)


def project_fastlsh(params, data, out=None, stream=None):
    import torch
    return _hash_call("lsh_project_fastlsh", params, data, params.k, torch.float32, out, stream)


def project_e2lsh(params, data, out=None, stream=None):
    import torch
    return _hash_call("lsh_project_e2lsh", params, data, params.k, torch.float32, out, stream)


def mips_kappa(params, data, out=None, accumulate=False, stream=None):
    """kappa~_l^2 = max_i ||S_l(v_i)||^2, float32 [L]; accumulate=True only raises what `out` holds."""
    import torch
    _dev_in(data, torch.float32, params.n)
    L = params.shared_tables()
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs the array to raise")
        out = torch.empty(L, dtype=torch.float32, device=data.device)
    if not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == L):
        raise ValueError(f"expected a contiguous CUDA float32 tensor of {L} elements")
    _check(load_library().lsh_mips_kappa(params.handle, data.data_ptr(), data.shape[0], int(bool(accumulate)),
                                         out.data_ptr(), _stream(stream)), "lsh_mips_kappa")
    return out


def _mips_data_call(name, params, data, kappa2, dtype, out, stream):
    import torch
    _dev_in(data, torch.float32, params.n)
    if not (kappa2.is_cuda and kappa2.dtype == torch.float32 and kappa2.is_contiguous()
            and kappa2.numel() == params.shared_tables()):
        raise ValueError("kappa2: expected the float32 CUDA tensor [L] of mips_kappa")
    N = data.shape[0]
    out = _out(data, N, params.k, dtype, out)
    _check(getattr(load_library(), name)(params.handle, data.data_ptr(), N, kappa2.data_ptr(), out.data_ptr(),
                                         _stream(stream)), name)
    return out


def hash_mips_data(params, data, kappa2, out=None, stream=None):
    import torch
    return _mips_data_call("lsh_hash_mips_data", params, data, kappa2, torch.int32, out, stream)


def project_mips_data(params, data, kappa2, out=None, stream=None):
    import torch
    return _mips_data_call("lsh_project_mips_data", params, data, kappa2, torch.float32, out, stream)


def hash_mips_query(params, queries, out=None, stream=None):
    import torch
    return _hash_call("lsh_hash_mips_query", params, queries, params.k, torch.int32, out, stream)


def project_mips_query(params, queries, out=None, stream=None):
    import torch
    return _hash_call("lsh_project_mips_query", params, queries, params.k, torch.float32, out, stream)


def pack_keys(params, buckets, L, out=None, stream=None):
    """64-bit keys as int64 [N, L] (bit patterns of the uint64 keys)."""
    import torch
    _dev_in(buckets, torch.int32, params.k)
    N = buckets.shape[0]
    out = _out(buckets, N, L, torch.int64, out)
    _check(load_library().lsh_pack_keys(params.handle, buckets.data_ptr(), N, L, out.data_ptr(),
                                        _stream(stream)), "lsh_pack_keys")
    return out


def hash_fastlsh_keys(params, data, L, out=None, stream=None):
    import torch
    _dev_in(data, torch.float32, params.n)
    N = data.shape[0]
    out = _out(data, N, L, torch.int64, out)
    _check(load_library().lsh_hash_fastlsh_keys(params.handle, data.data_ptr(), N, L, out.data_ptr(),
                                                _stream(stream)), "lsh_hash_fastlsh_keys")
    return out


def hash_fastlsh_ids_keys(params, data, L, out_ids=None, out_keys=None, stream=None):
    """Bucket ids [N, k] (int32) and compound keys [N, L] (uint64 bit patterns in int64) in one call."""
    import torch
    _dev_in(data, torch.float32, params.n)
    N = data.shape[0]
    out_ids = _out(data, N, params.k, torch.int32, out_ids)
    out_keys = _out(data, N, L, torch.int64, out_keys)
    _check(load_library().lsh_hash_fastlsh_ids_keys(params.handle, data.data_ptr(), N, L, out_ids.data_ptr(),
                                                    out_keys.data_ptr(), _stream(stream)), "lsh_hash_fastlsh_ids_keys")
    return out_ids, out_keys


_WHICH = {"fastlsh": 0, "e2lsh": 1, "signs": 2, "pack_keys": 3, "fastlsh_keys": 4}


class LshIndex:
    """Owns one lsh_index_t: L hash tables built from the keys [N, L] of the indexed vectors."""

    def __init__(self, keys, stream=None):
        import torch
        assert keys.is_cuda and keys.dtype == torch.int64 and keys.dim() == 2 and keys.is_contiguous()
        handle = ctypes.c_void_p()
        _check(load_library().lsh_index_build(keys.data_ptr(), keys.shape[0], keys.shape[1], _stream(stream),
                                              ctypes.byref(handle)), "lsh_index_build")
        self._h = handle
        self.N, self.L, self.device = int(keys.shape[0]), int(keys.shape[1]), keys.device

    @property
    def handle(self):
        if not getattr(self, "_h", None):
            raise ValueError("LshIndex is closed")
        return self._h

    def close(self):
        if getattr(self, "_h", None):
            load_library().lsh_index_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def probe(self, qkeys, stream=None):
        """Bucket of every (query, table): (start [Q, L], count [Q, L]) int32 tensors (uint32 bits)."""
        import torch
        assert qkeys.is_cuda and qkeys.dtype == torch.int64 and qkeys.is_contiguous() and qkeys.shape[1] == self.L
        Q = qkeys.shape[0]
        start = torch.empty((Q, self.L), dtype=torch.int32, device=qkeys.device)
        count = torch.empty((Q, self.L), dtype=torch.int32, device=qkeys.device)
        _check(load_library().lsh_index_probe(self.handle, qkeys.data_ptr(), Q, start.data_ptr(), count.data_ptr(),
                                              _stream(stream)), "lsh_index_probe")
        return start, count

    def candidates(self, start, count, stream=None):
        """(offsets [Q*L + 1] int64, ids [total] int32): the bucket of item q*L + l is
        ids[offsets[item] : offsets[item + 1]]."""
        import torch
        items = start.numel()
        offsets = candidate_offsets(count, stream=stream)
        total = int(offsets[-1].item())
        ids = torch.empty(total, dtype=torch.int32, device=start.device)
        if total:
            _check(load_library().lsh_index_candidates(self.handle, start.data_ptr(), count.data_ptr(),
                                                       offsets.data_ptr(), start.shape[0], ids.data_ptr(),
                                                       _stream(stream)), "lsh_index_candidates")
        return offsets, ids

    def best_inner_product(self, data, queries, start, count, max_candidates=0, stream=None):
        """Candidate with the largest inner product: (best id [Q] int32 with -1 for none, inner
        product [Q] float32, -inf for none)."""
        return self._best("lsh_index_best_inner_product", data, queries, start, count, max_candidates, stream)

    def nearest(self, data, queries, start, count, max_candidates=0, stream=None):
        """Nearest candidate: (best id [Q] int32 with -1 for none, squared distance [Q] float32).
        max_candidates = 0: every candidate (exact version); else only the first max_candidates
        of each query's combined list (the paper's approximate version uses 3 * L)."""
        return self._best("lsh_index_nearest", data, queries, start, count, max_candidates, stream)

    def _best(self, name, data, queries, start, count, max_candidates, stream):
        import torch
        assert data.is_cuda and data.dtype == torch.float32 and data.is_contiguous() and data.shape[0] == self.N
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        Q, n = queries.shape
        assert data.shape[1] == n and start.shape == (Q, self.L)
        best = torch.empty(Q, dtype=torch.int32, device=data.device)
        dist = torch.empty(Q, dtype=torch.float32, device=data.device)
        _check(getattr(load_library(), name)(self.handle, data.data_ptr(), queries.data_ptr(), n,
                                             start.data_ptr(), count.data_ptr(), Q, max_candidates,
                                             best.data_ptr(), dist.data_ptr(), _stream(stream)), name)
        return best, dist


def candidate_offsets(count, out=None, static_scratch=False, stream=None):
    """Exclusive prefix sum of the bucket sizes: int64 [items + 1], the last entry the total.
    static_scratch=True takes the entry point that allocates nothing and does not wait."""
    import torch
    assert count.is_cuda and count.dtype == torch.int32 and count.is_contiguous()
    items = count.numel()
    if out is None:
        out = torch.empty(items + 1, dtype=torch.int64, device=count.device)
    assert out.is_cuda and out.dtype == torch.int64 and out.is_contiguous() and out.numel() == items + 1
    name = "lsh_index_candidate_offsets_static" if static_scratch else "lsh_index_candidate_offsets"
    _check(getattr(load_library(), name)(count.data_ptr(), items, out.data_ptr(), _stream(stream)), name)
    return out


def e2lsh_collision_probability(s, w):
    out = ctypes.c_double()
    _check(load_library().lsh_e2lsh_collision_probability(s, w, ctypes.addressof(out)),
           "lsh_e2lsh_collision_probability")
    return out.value


def pair_statistics(v, u, m):
    """(mu~, sigma~) of a pair of host float32 vectors for sample size m."""
    v = np.ascontiguousarray(v, np.float32)
    u = np.ascontiguousarray(u, np.float32)
    assert v.shape == u.shape and v.ndim == 1
    mu, sigma = ctypes.c_double(), ctypes.c_double()
    _check(load_library().lsh_pair_statistics(v.ctypes.data, u.ctypes.data, v.size, m, ctypes.addressof(mu),
                                              ctypes.addressof(sigma)), "lsh_pair_statistics")
    return mu.value, sigma.value


def fastlsh_collision_probability(mu_tilde, sigma_tilde, w):
    out = ctypes.c_double()
    _check(load_library().lsh_fastlsh_collision_probability(mu_tilde, sigma_tilde, w, ctypes.addressof(out)),
           "lsh_fastlsh_collision_probability")
    return out.value


def mips_collision_probability(mu_tilde, sigma_tilde, delta, w):
    out = ctypes.c_double()
    _check(load_library().lsh_mips_collision_probability(mu_tilde, sigma_tilde, delta, w, ctypes.addressof(out)),
           "lsh_mips_collision_probability")
    return out.value


def fastlsh_moment_factors(mu_tilde, sigma_tilde):
    eps, lam = ctypes.c_double(), ctypes.c_double()
    _check(load_library().lsh_fastlsh_moment_factors(mu_tilde, sigma_tilde, ctypes.addressof(eps),
                                                     ctypes.addressof(lam)), "lsh_fastlsh_moment_factors")
    return eps.value, lam.value


def equivalent_width(n, m, w):
    return load_library().lsh_equivalent_width(n, m, w)


def time_launches(params, which, d_in, d_out, L=0, reps=10, stream=None):
    """Mean milliseconds per launch of one hash call, by HIP events on the launch stream."""
    ms = ctypes.c_float()
    _check(load_library().lsh_time_launches(params.handle, _WHICH[which], d_in.data_ptr(), d_in.shape[0],
                                            L, d_out.data_ptr(), _stream(stream), reps, ctypes.byref(ms)),
           "lsh_time_launches")
    return float(ms.value)
