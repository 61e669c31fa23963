#!/usr/bin/env python3
"""Benchmark of the LSH hash-evaluation hot path on one MI355X.

Headline workload: the high-dimensional configuration (N = 200,000 vectors, n = 4,096, k = 2,048
functions, w = 8; i.i.d. N(0,1) rows plus 5 % planted near-duplicates).  One step = one pass of the
whole path over that batch, inputs and outputs resident in HBM:

    FastLSH bucket ids at m = 64, m = 256 and m = 1024 sampled coordinates  ->  dense E2LSH
    bucket ids (m = n, same seed)

`value` is hashes per second over the whole step (4 * N * k hash evaluations per step).  Per-kernel
times come from HIP events recorded on the launch stream inside the timed region.  Outside the
timed region the other paper-shaped workloads (tiny, SIFT-shaped, GIST-shaped, angular) are timed
call by call and reported in `configs`, each with its rooflines, and sampled rows of every output
are compared with the CPU oracle (mismatch counts, boundary-excluded fraction, fraction of
projections within a plain relative 1e-5).  Prints ONE JSON line.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3    # dense fp32 matrix peak
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16 matrix peak
# fp32 multiply-adds on the vector ALU without packed instructions (this library is compiled
# without them): 256 CUs x 64 lanes per clock x 2.4 GHz = 39.3 T FMA/s = 78.6 TFLOP/s
VALU_FMA_PEAK_T = 256 * 64 * 2.4e9 / 1e12
VALU_UNPACKED_PEAK_TFLOPS = 2.0 * VALU_FMA_PEAK_T

BAND = 1e-4        # ids may differ where the oracle's (p + b)/w is within BAND of an integer
PROJ_RTOL = 1e-5   # projections: |dp| <= PROJ_RTOL * sum_i |a_i v_i|  (pass/fail rule of the tests)

CSRC = os.path.join(ROOT, "paper_2309_15479_amd", "csrc")

# HBM bytes per launch from rocprofv3's FETCH_SIZE and WRITE_SIZE counters (two runs, each scaled
# by what the same counter reads for a 1 GiB device copy: factors 1.0000 and 1.0000), per kernel
# and workload: name -> (fetch bytes, write bytes, summary under profiles/, {source file: sha256
# prefix of the kernel source the counters were taken on}).  An entry is reported only while its
# source files still hash to the recorded values; otherwise `traffic` is null.  (FETCH_SIZE counts
# 64 bytes per read request and these kernels fetch 128-byte lines: a lower bound, see the summary.)
_KIB = 1024
_RANGED = {"ranged_kernel.hip": "27e4edf7a84e975a", "sampled_common.h": "9d6a9ea08ffad892", "schedule.cpp": "e034f03d037e1a15"}
_STREAMED = {"sampled_kernel.hip": "bea9b29ed7d9a478", "sampled_common.h": "9d6a9ea08ffad892"}
_SUMMARY = "profiles/hbm_traffic_all_workloads.md"
MEASURED_TRAFFIC = {
    "highdim/fastlsh/m64": (1770052 * _KIB, 1600000 * _KIB, _SUMMARY, _RANGED),
    "highdim/fastlsh/m256": (2217169 * _KIB, 1600000 * _KIB, _SUMMARY, _RANGED),
    "highdim/fastlsh/m1024": (4057910 * _KIB, 1600000 * _KIB, _SUMMARY, _RANGED),
    "highdim/e2lsh": (6674183 * _KIB, 2180306 * _KIB, _SUMMARY, {"dense_split_wide_kernel.hip": "f5c3c396883fe4bb"}),
    "sift/fastlsh/m32": (250604 * _KIB, 2000000 * _KIB, _SUMMARY, _STREAMED),
    "gist/fastlsh/m128": (2371799 * _KIB, 4000000 * _KIB, _SUMMARY, _STREAMED),
    "gist/e2lsh": (3704539 * _KIB, 5497154 * _KIB, _SUMMARY, {"dense_split_wide_kernel.hip": "f5c3c396883fe4bb"}),
    "angular/signs/m512": (58290677 * _KIB, 250024 * _KIB, _SUMMARY, _RANGED),
}


def source_hash(name):
    with open(os.path.join(CSRC, name), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def traffic_of(key):
    """HBM bytes per launch from the counters (a number), or None when there is no figure for the
    kernel as it stands."""
    entry = MEASURED_TRAFFIC.get(key)
    if not entry:
        return None
    fetch, write, summary, sources = entry
    if any(source_hash(f) != h for f, h in sources.items()):
        return None
    return fetch + write


def with_traffic(roofline, key):
    """Attaches the measured HBM traffic of `key` (bytes per launch, and where it comes from)."""
    roofline["traffic"] = traffic_of(key)
    detail = traffic_detail(key)
    if detail:
        roofline["traffic_detail"] = detail
    return roofline


def traffic_detail(key):
    entry = MEASURED_TRAFFIC.get(key)
    if not entry or traffic_of(key) is None:
        return None
    return {"fetch_bytes": entry[0], "write_bytes": entry[1], "from": entry[2]}


class Timer:
    """HIP-event timing of back-to-back launches on torch's current stream (the stream the binding
    hands to the library)."""

    def __init__(self, torch):
        self.torch = torch

    def run(self, fn, reps):
        e0, e1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        self.torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def settle(self, fn, busy_ms=150.0):
        """Untimed launches for about busy_ms of GPU time: the clocks ramp up over the first
        ~100 ms of load, whatever --warmup says."""
        ms = self.run(fn, 2)
        self.run(fn, max(1, min(400, int(busy_ms / max(ms, 1e-3)))))
        return ms

    def measure(self, fn, budget_ms=250.0, lo=5, hi=100):
        ms = self.settle(fn)
        return self.run(fn, max(lo, min(hi, int(budget_ms / max(ms, 1e-3)))))


def padding_ratio(p):
    """Entries the gather kernel visits per function sample (1.0 = no padding entries)."""
    import numpy as np
    try:
        order, group, classes, passes = p.schedule()
    except Exception:
        return None
    used = int((order != np.uint32(0xFFFFFFFF)).sum())
    return {"entries_per_sample": used / float(p.k * p.m),
            "lds_passes_per_conflict_free_pass": passes / (used / float(group))}


def hbm_roofline(bytes_per_launch, ms, traffic=None):
    a = bytes_per_launch / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
            "traffic": traffic}


def gather_roofline(N, n, k, m, out_bytes_per_vector, ms, traffic=None):
    """Sampled projection.  Per vector it moves 4n bytes in + the outputs and does k*m multiply-adds,
    each of which takes a vector-ALU lane slot (no packed fp32 here) and 4 bytes of LDS.  The
    roofline that binds is the one with the longer ideal time; the other is reported beside it."""
    hbm = hbm_roofline(N * (4 * n + out_bytes_per_vector), ms, traffic)
    fma = N * k * m / (ms * 1e-3) / 1e12
    alu = {"bound": "alu", "achieved": 2.0 * fma, "peak": VALU_UNPACKED_PEAK_TFLOPS, "unit": "TFLOP/s",
           "frac": fma / VALU_FMA_PEAK_T, "traffic": traffic, "gather_fma_per_s": fma * 1e12}
    t_hbm = (4 * n + out_bytes_per_vector) / (HBM_PEAK_GBS * 1e9)
    t_alu = k * m / (VALU_FMA_PEAK_T * 1e12)
    if t_alu >= t_hbm:
        alu["hbm"] = {k_: hbm[k_] for k_ in ("achieved", "peak", "unit", "frac")}
        return alu
    hbm["on_chip"] = {k_: alu[k_] for k_ in ("bound", "achieved", "peak", "unit", "frac")}
    return hbm


def dense_roofline(N, n, k, ms, arithmetic, traffic=None):
    tf = 2.0 * N * n * k / (ms * 1e-3) / 1e12
    if arithmetic == "fp32":
        return {"bound": "mfma", "achieved": tf, "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_FP32_PEAK_TFLOPS, "traffic": traffic, "arithmetic": "fp32 MFMA"}
    products = arithmetic["products"]
    return {"bound": "mfma", "achieved": products * tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": products * tf / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
            "arithmetic": f"bf16 x 3 exact splits, fp32 accumulation, {products} of 6 MFMA products per coordinate",
            "fp32_equivalent_tflops": tf}


def shared_roofline(N, n, k, m, ms):
    """One sample per table: the gathered coordinates of a table meet its functions on the fp32
    matrix cores (2 k m flops per vector); the roofline that binds is the one with the longer
    ideal time."""
    hbm = hbm_roofline(N * (4 * n + 4 * k), ms)
    tf = 2.0 * N * k * m / (ms * 1e-3) / 1e12
    mfma = {"bound": "mfma", "achieved": tf, "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": tf / MFMA_FP32_PEAK_TFLOPS, "traffic": None}
    first, second = (hbm, mfma) if hbm["frac"] >= mfma["frac"] else (mfma, hbm)
    first = dict(first)
    first["other"] = second
    return first


def parity_ids(torch, oracle, threads, host_rows, got_ids, got_proj, tables, w, dense):
    """Sampled rows against the oracle: ids outside the boundary band must agree; reports the
    excluded fraction and how many projections meet a plain relative 1e-5."""
    import numpy as np
    want = ("proj", "abs_sum", "ids", "frac")
    if dense:
        ora = oracle.e2lsh(host_rows, tables[1], tables[2], w, nthreads=threads, want=want)
    else:
        ora = oracle.fastlsh(host_rows, tables[0], tables[1], tables[2], w, nthreads=threads, want=want)
    near = (ora["frac"] < BAND) | (ora["frac"] > 1.0 - BAND)
    diff = got_ids.astype(np.int64) - ora["ids"].astype(np.int64)
    err = np.abs(got_proj.astype(np.float64) - ora["proj"])
    return {"rows_checked": int(host_rows.shape[0]),
            "ids_checked": int(diff.size),
            "id_mismatches_outside_band": int(((diff != 0) & ~near).sum()),
            "id_mismatches_inside_band": int(((diff != 0) & near).sum()),
            "boundary_excluded_fraction": float(near.mean()),
            "projection_worst_error_over_tolerance": float((err / (PROJ_RTOL * ora["abs_sum"] + 1e-30)).max()),
            "projections_within_plain_relative_1e-5": float((err <= PROJ_RTOL * np.abs(ora["proj"])).mean())}


def parity_signs(oracle, threads, host_rows, got_words, tables, k):
    import numpy as np
    words, proj, norm_prod = oracle.signs(host_rows, tables[0], tables[1], nthreads=threads, want_proj=True,
                                          want_norm_prod=True)
    g = np.unpackbits(np.ascontiguousarray(got_words).view(np.uint8), axis=1, bitorder="little")[:, :k]
    o = np.unpackbits(np.ascontiguousarray(words).view(np.uint8), axis=1, bitorder="little")[:, :k]
    near = np.abs(proj) < BAND * norm_prod
    return {"rows_checked": int(host_rows.shape[0]), "bits_checked": int(g.size),
            "bit_mismatches_outside_band": int(((g != o) & ~near).sum()),
            "bit_mismatches_inside_band": int(((g != o) & near).sum()),
            "band_excluded_fraction": float(near.mean())}


class Bench:
    def __init__(self, args):
        import torch
        import paper_2309_15479_amd as lsh
        import workloads
        self.torch, self.lsh, self.workloads, self.args = torch, lsh, workloads, args
        assert torch.cuda.is_available(), "bench.py needs a GPU"
        lsh.load_library()
        self.dev = "cuda:0"
        self.timer = Timer(torch)
        self.oracle = None
        if not args.no_parity or not args.no_cpu_baseline:
            import oracle
            self.oracle = oracle
            self.threads = oracle.max_threads()

    def rows(self, wl, count):
        rows = self.workloads.sample_rows(wl.N, count, tile=16, seed=wl.seed)
        if wl.planted:
            rows = self.torch.unique(self.torch.cat([rows, self.torch.arange(wl.N - 8, wl.N)]))
        return rows.to(self.dev)

    def check_ids(self, p, wl, data, out, dense, count=96):
        if self.args.no_parity:
            return None
        lsh, torch = self.lsh, self.torch
        rows = self.rows(wl, count)
        sub = data[rows].contiguous()
        proj = (lsh.project_e2lsh if dense else lsh.project_fastlsh)(p, sub)
        torch.cuda.synchronize()
        tables = (p.indices(), p.coeffs(), p.offsets())
        return parity_ids(torch, self.oracle, self.threads, sub.cpu().numpy(), out[rows].cpu().numpy(),
                          proj.cpu().numpy(), tables, wl.w, dense)

    def fastlsh_entry(self, wl, data, m, out):
        """Times FastLSH ids at m sampled coordinates (the gathered sampled-projection kernel; at
        n = 128 the default matrix-core route is timed beside it)."""
        lsh = self.lsh
        N, n, k = wl.N, wl.n, wl.k
        entry = {"workload": wl.name, "call": "lsh_hash_fastlsh", "N": N, "n": n, "k": k, "m": m, "w": wl.w}
        with lsh.LshParams(n, k, m, wl.w, wl.seed) as p:
            default_ms = self.timer.measure(lambda: lsh.hash_fastlsh(p, data, out=out))
            routed_dense = n == 128 and k % 32 == 0
            if routed_dense:
                # the default at n = 128 is a dense product over the zero-filled coefficients on the
                # bf16 matrix cores; the figure for the sampled-projection kernel is the gathered one
                p.set_dense_arithmetic(lsh.DENSE_FP32)
                ms = self.timer.measure(lambda: lsh.hash_fastlsh(p, data, out=out))
                entry["matrix_core_route_ms"] = default_ms
                entry["matrix_core_route_hbm_frac"] = N * (4 * n + 4 * k) / (default_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
            else:
                ms = default_ms
            entry["parity"] = self.check_ids(p, wl, data, out, dense=False)
            if routed_dense:
                p.set_dense_arithmetic(lsh.DENSE_AUTO)
            entry["schedule"] = padding_ratio(p)
        entry.update({"ms": ms, "hashes_per_s": N * k / (ms * 1e-3), "vectors_per_s": N / (ms * 1e-3),
                      "dtype": "f32",
                      "roofline": with_traffic(gather_roofline(N, n, k, m, 4 * k, ms), f"{wl.name}/fastlsh/m{m}")})
        return entry

    def e2lsh_entry(self, wl, data, out):
        lsh = self.lsh
        N, n, k = wl.N, wl.n, wl.k
        entry = {"workload": wl.name, "call": "lsh_hash_e2lsh", "N": N, "n": n, "k": k, "m": n, "w": wl.w}
        with lsh.LshParams(n, k, n, wl.w, wl.seed) as p:
            ms = self.timer.measure(lambda: lsh.hash_e2lsh(p, data, out=out))
            entry["parity"] = self.check_ids(p, wl, data, out, dense=True, count=48 if n > 1024 else 96)
            split = (n == 128 and k % 32 == 0) or (n != 128 and n % 4 == 0)
            if split:
                # bf16 x 3 products; at n = 128 half of the six products are skipped by tile on byte-valued data
                integer_data = n == 128 and bool((data[:4096] == data[:4096].round()).all().item())
                arithmetic = {"products": 3 if integer_data else 6}
                p.set_dense_arithmetic(lsh.DENSE_FP32)
                fp32_ms = self.timer.measure(lambda: lsh.hash_e2lsh(p, data, out=out))
                p.set_dense_arithmetic(lsh.DENSE_AUTO)
                entry["fp32_mfma_route"] = {"ms": fp32_ms, "roofline": dense_roofline(N, n, k, fp32_ms, "fp32")}
                entry["speedup_over_fp32_mfma"] = fp32_ms / ms
                if integer_data:
                    full = data + self.torch.rand_like(data)
                    full_ms = self.timer.measure(lambda: lsh.hash_e2lsh(p, full, out=out))
                    del full
                    entry["full_significand_data"] = {
                        "ms": full_ms, "roofline": dense_roofline(N, n, k, full_ms, {"products": 6}),
                        "hbm_frac": N * (4 * n + 4 * k) / (full_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
            else:
                arithmetic = "fp32"
        entry.update({"ms": ms, "hashes_per_s": N * k / (ms * 1e-3), "vectors_per_s": N / (ms * 1e-3),
                      "dtype": "f32" if arithmetic == "fp32" else "bf16x3+f32acc",
                      "roofline": with_traffic(dense_roofline(N, n, k, ms, arithmetic), f"{wl.name}/e2lsh")})
        entry["roofline"]["hbm_frac"] = N * (4 * n + 4 * k) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        return entry

    def config(self, name):
        """All calls of one paper-shaped workload, each timed back to back after a clock-settling
        warm-up; returns the list of entries."""
        torch, lsh = self.torch, self.lsh
        wl, data = self.workloads.make_data(name, self.dev)
        N, n, k = wl.N, wl.n, wl.k
        entries = []
        if wl.signs:
            words = torch.empty((N, (k + 63) // 64), dtype=torch.int64, device=self.dev)
            m = wl.m[0]
            with lsh.LshParams(n, k, m, wl.w, wl.seed) as p:
                ms = self.timer.measure(lambda: lsh.hash_signs(p, data, out=words), budget_ms=400.0, lo=3)
                entry = {"workload": name, "call": "lsh_hash_signs", "N": N, "n": n, "k": k, "m": m,
                         "ms": ms, "hashes_per_s": N * k / (ms * 1e-3), "vectors_per_s": N / (ms * 1e-3),
                         "dtype": "f32", "schedule": padding_ratio(p),
                         "roofline": with_traffic(gather_roofline(N, n, k, m, 8 * ((k + 63) // 64), ms),
                                                  f"{name}/signs/m{m}")}
                if not self.args.no_parity:
                    import numpy as np
                    rows = self.rows(wl, 48)
                    entry["parity"] = parity_signs(self.oracle, self.threads, data[rows].cpu().numpy(),
                                                   words[rows].cpu().numpy().view(np.uint64),
                                                   (p.indices(), p.coeffs()), k)
            entries.append(entry)
            return entries
        out = torch.empty((N, k), dtype=torch.int32, device=self.dev)
        for m in wl.m:
            entries.append(self.fastlsh_entry(wl, data, m, out))
        dense = self.e2lsh_entry(wl, data, out)
        for e in entries:
            e["speedup_over_e2lsh"] = dense["ms"] / e["ms"]
            e["operation_count_ratio_n_over_m"] = n / e["m"]
        entries.append(dense)
        if wl.L and name in ("sift", "gist"):
            keys = torch.empty((N, wl.L), dtype=torch.int64, device=self.dev)
            with lsh.LshParams(n, k, wl.m[0], wl.w, wl.seed) as p:
                lsh.hash_fastlsh(p, data, out=out)
                ms = self.timer.measure(lambda: lsh.pack_keys(p, out, wl.L, out=keys))
                entries.append({"workload": name, "call": "lsh_pack_keys", "N": N, "k": k, "L": wl.L, "ms": ms,
                                "dtype": "u64",
                                "roofline": with_traffic(hbm_roofline(N * (4 * k + 8 * wl.L), ms), f"{name}/pack_keys")})
                if not self.args.no_parity:
                    import numpy as np
                    rows = self.rows(wl, 96)
                    want = self.oracle.pack_keys(out[rows].cpu().numpy(), wl.L)
                    entries[-1]["parity"] = {"keys_checked": int(want.size), "key_mismatches": int(
                        (keys[rows].cpu().numpy().view(np.uint64) != want).sum())}
                ms = self.timer.measure(lambda: lsh.hash_fastlsh_keys(p, data, wl.L, out=keys))
                entries.append({"workload": name, "call": "lsh_hash_fastlsh_keys", "N": N, "n": n, "k": k,
                                "m": wl.m[0], "L": wl.L, "ms": ms, "dtype": "f32",
                                # at n = 128 this call runs on the matrix cores (dense product with zeros)
                                "roofline": hbm_roofline(N * (4 * n + 8 * wl.L), ms) if n == 128 else
                                gather_roofline(N, n, k, wl.m[0], 8 * wl.L, ms)})
                # ids and keys in one call (one launch on these shapes), against the two launches
                ids2 = torch.empty_like(out)
                ms = self.timer.measure(lambda: lsh.hash_fastlsh_ids_keys(p, data, wl.L, out_ids=ids2, out_keys=keys))
                two = entries[0]["matrix_core_route_ms"] if "matrix_core_route_ms" in entries[0] else entries[0]["ms"]
                entry = {"workload": name, "call": "lsh_hash_fastlsh_ids_keys", "N": N, "n": n, "k": k, "m": wl.m[0],
                         "L": wl.L, "ms": ms, "dtype": "f32", "two_launches_ms": two + entries[-2]["ms"],
                         "roofline": hbm_roofline(N * (4 * n + 4 * k + 8 * wl.L), ms) if n == 128 else
                         gather_roofline(N, n, k, wl.m[0], 4 * k + 8 * wl.L, ms)}
                if not self.args.no_parity:
                    import numpy as np
                    lsh.hash_fastlsh(p, data, out=out)
                    rows = self.rows(wl, 96)
                    entry["parity"] = {
                        "ids_differing_from_lsh_hash_fastlsh": int((ids2 != out).sum().item()),
                        "keys_checked": int(rows.numel() * wl.L),
                        "key_mismatches": int((keys[rows].cpu().numpy().view(np.uint64) !=
                                               self.oracle.pack_keys(ids2[rows].cpu().numpy(), wl.L)).sum())}
                entries.append(entry)
                del ids2
                entries.extend(self.index_entries(wl, data, p, keys))
            del keys
        if name == "tiny":
            entries.append(self.graph_entry(wl, data))
        del out, data
        torch.cuda.empty_cache()
        return entries

    def index_entries(self, wl, data, p, keys):
        """Sec. 3.2 beyond the hash: the L tables built from the keys of the whole batch, the bucket
        lookup of 4096 queries (perturbed copies of indexed vectors) and the exact evaluation of
        their candidates; a few queries are checked against the definition written out in numpy."""
        import numpy as np
        torch, lsh = self.torch, self.lsh
        N, n, L, Q = wl.N, wl.n, wl.L, 4096
        lsh.hash_fastlsh_keys(p, data, L, out=keys)
        torch.cuda.synchronize()
        lsh.LshIndex(keys).close()  # first build: one-time set-up
        builds = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ix = lsh.LshIndex(keys)
            e1.record()
            torch.cuda.synchronize()
            builds.append(e0.elapsed_time(e1))
            ix.close()
        g = torch.Generator(device=self.dev)
        g.manual_seed(wl.seed + 100)
        rows = torch.randint(0, N, (Q,), generator=g, device=self.dev)
        scale = float(data[:1024].std().item())
        queries = (data[rows] + 0.01 * scale * torch.randn((Q, n), generator=g, device=self.dev)).contiguous()
        qkeys = lsh.hash_fastlsh_keys(p, queries, L)
        out = []
        with lsh.LshIndex(keys) as ix:
            probe_ms = self.timer.measure(lambda: ix.probe(qkeys))
            start, count = ix.probe(qkeys)
            nearest_ms = self.timer.measure(lambda: ix.nearest(data, queries, start, count))
            best, dist2 = ix.nearest(data, queries, start, count)
            torch.cuda.synchronize()
            candidates = int(count.to(torch.int64).sum().item())
            found_source = float((best.to(torch.int64) == rows).float().mean().item())
            parity = None
            if not self.args.no_parity:
                # the definition, for 6 queries: table l's bucket = ids (ascending) whose key equals the query's
                off, cand = ix.candidates(start[:6].contiguous(), count[:6].contiguous())
                off, cand = off.cpu().numpy(), cand.cpu().numpy()
                hk, hq = keys.cpu().numpy(), qkeys[:6].cpu().numpy()
                hd, hqv = data, queries[:6].cpu().numpy().astype(np.float64)
                bad_buckets = bad_nearest = 0
                for q in range(6):
                    mine = []
                    for l in range(L):
                        want = np.nonzero(hk[:, l] == hq[q, l])[0]
                        got = cand[off[q * L + l]:off[q * L + l + 1]]
                        bad_buckets += int(not np.array_equal(want, got))
                        mine.extend(want.tolist())
                    uniq = sorted(set(mine))
                    if uniq:
                        d = ((hd[torch.as_tensor(uniq, device=self.dev)].cpu().numpy().astype(np.float64) - hqv[q]) ** 2).sum(1)
                        j = int(np.argmin(d))
                        got_id = int(best[q].item())
                        ok = got_id == uniq[j] or (got_id in uniq and d[uniq.index(got_id)] <= d[j] * (1 + 1e-5))
                        bad_nearest += int(not ok)
                    else:
                        bad_nearest += int(int(best[q].item()) != -1)
                parity = {"queries_checked": 6, "buckets_checked": 6 * L, "bucket_mismatches": bad_buckets,
                          "nearest_mismatches": bad_nearest}
        build_ms = sum(builds) / len(builds)
        base = {"workload": wl.name, "N": N, "L": L, "dtype": "u64"}
        out.append(dict(base, call="lsh_index_build", ms=build_ms, pairs_per_s=N * L / (build_ms * 1e-3),
                        # 8 passes of 8 bits over <key, id> pairs: per pass the keys are read for the histogram (8 B)
                        # and the pairs are read and written (12 + 12 B)
                        roofline=hbm_roofline(N * L * 8 * 32, build_ms)))
        out.append(dict(base, call="lsh_index_probe", queries=Q, ms=probe_ms, parity=parity))
        out.append(dict(base, call="lsh_index_nearest", queries=Q, ms=nearest_ms, candidates=candidates,
                        dtype="f32", queries_whose_source_vector_is_returned=found_source,
                        roofline=hbm_roofline(candidates * 4 * n, nearest_ms)))
        return out

    def graph_entry(self, wl, data):
        """The launch-bound shape as it should be run: the step's four launches captured once in a
        HIP graph and replayed (the hash calls allocate nothing and never synchronise)."""
        torch, lsh = self.torch, self.lsh
        N, n, k, L = wl.N, wl.n, wl.k, wl.L
        ids = torch.empty((N, k), dtype=torch.int32, device=self.dev)
        dense = torch.empty_like(ids)
        keys = torch.empty((N, L), dtype=torch.int64, device=self.dev)
        words = torch.empty((N, (k + 63) // 64), dtype=torch.int64, device=self.dev)
        with lsh.LshParams(n, k, wl.m[0], wl.w, wl.seed) as pf, lsh.LshParams(n, k, n, wl.w, wl.seed) as pd:
            def step():
                lsh.hash_fastlsh(pf, data, out=ids)
                lsh.pack_keys(pf, ids, L, out=keys)
                lsh.hash_e2lsh(pd, data, out=dense)
                lsh.hash_signs(pf, data, out=words)
            step()  # eager once: raises the kernels' LDS limits
            torch.cuda.synchronize()
            eager_ms = self.timer.measure(step)
            want = ids.clone()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    step()
            ids.zero_()
            graph_ms = self.timer.measure(graph.replay)
            torch.cuda.synchronize()
            same = bool(torch.equal(ids, want))
        bytes_per_step = N * (3 * 4 * n + 4 * k + 4 * k + 8 * L + 4 * k + 8 * ((k + 63) // 64))
        return {"workload": wl.name, "call": "fastlsh ids + pack_keys + e2lsh ids + signs as one HIP graph", "N": N,
                "n": n, "k": k, "ms": graph_ms, "eager_ms": eager_ms, "dtype": "f32",
                "replay_equals_eager": same, "roofline": hbm_roofline(bytes_per_step, graph_ms)}

    def cpu_baseline(self, wl, data, params, budget_s=14.0):
        """The oracle as it stands on a bounded sample of the headline batch: all four legs of the
        step, once with every host thread and once single-threaded."""
        oracle = self.oracle
        tabs = [(p.indices(), p.coeffs(), p.offsets()) for p in params]

        def run(rows, threads):
            t0 = time.perf_counter()
            for (idx, coef, off), p in zip(tabs, params):
                if p.m == p.n:
                    oracle.e2lsh(rows, coef, off, wl.w, nthreads=threads)
                else:
                    oracle.fastlsh(rows, idx, coef, off, wl.w, nthreads=threads)
            return time.perf_counter() - t0

        out = {}
        for label, threads, budget in (("all_threads", self.threads, budget_s), ("single_thread", 1, budget_s / 2)):
            pilot_rows = 64 * threads
            t_pilot = run(data[:pilot_rows].cpu().numpy(), threads)
            count = int(max(pilot_rows, min(data.shape[0], pilot_rows * budget / max(t_pilot, 1e-6))))
            t = run(data[:count].cpu().numpy(), threads)
            out[label] = {"hashes_per_s": len(params) * count * wl.k / t, "rows": count, "seconds": t,
                          "threads": threads}
        a = out["all_threads"]
        return {"value": a["hashes_per_s"], "unit": "hashes/s", "cores": a["threads"], "kind": "oracle",
                "sample": f"first {a['rows']} rows of the headline batch, all four legs of the step "
                          f"(FastLSH m=64/256/1024 + E2LSH), {a['seconds']:.1f} s",
                "single_thread": {"value": out["single_thread"]["hashes_per_s"], "unit": "hashes/s",
                                  "sample": f"first {out['single_thread']['rows']} rows, "
                                            f"{out['single_thread']['seconds']:.1f} s"}}

    def headline(self):
        torch, lsh, args = self.torch, self.lsh, self.args
        wl, data = self.workloads.make_data("highdim", self.dev)
        N, n, k = wl.N, wl.n, wl.k
        params = [lsh.LshParams(n, k, m, wl.w, wl.seed) for m in wl.m] + [lsh.LshParams(n, k, n, wl.w, wl.seed)]
        legs = [f"fastlsh_m{m}" for m in wl.m] + ["e2lsh"]
        out = torch.empty((N, k), dtype=torch.int32, device=self.dev)

        def step(events=None):
            for p in params:
                if events is not None:
                    e = torch.cuda.Event(enable_timing=True)
                    e.record()      # torch's current stream = the stream the library launches on
                    events.append(e)
                (lsh.hash_e2lsh if p.m == p.n else lsh.hash_fastlsh)(p, data, out=out)
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                events.append(e)

        self.timer.settle(step)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        all_events = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ev = []
            step(ev)
            all_events.append(ev)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ms = {leg: sum(ev[i].elapsed_time(ev[i + 1]) for ev in all_events) / args.steps for i, leg in enumerate(legs)}

        entries = []
        for leg, p in zip(legs, params):
            dense = p.m == p.n
            (lsh.hash_e2lsh if dense else lsh.hash_fastlsh)(p, data, out=out)
            e = {"workload": "highdim", "call": "lsh_hash_e2lsh" if dense else "lsh_hash_fastlsh", "N": N, "n": n,
                 "k": k, "m": p.m, "w": wl.w, "ms": ms[leg], "hashes_per_s": N * k / (ms[leg] * 1e-3),
                 "vectors_per_s": N / (ms[leg] * 1e-3), "dtype": "f32", "timed": "inside the step",
                 "parity": self.check_ids(p, wl, data, out, dense, count=48 if dense else 96)}
            if dense:
                e["dtype"] = "bf16x3+f32acc"
                e["roofline"] = with_traffic(dense_roofline(N, n, k, ms[leg], {"products": 6}), "highdim/e2lsh")
                e["roofline"]["hbm_frac"] = N * (4 * n + 4 * k) / (ms[leg] * 1e-3) / 1e9 / HBM_PEAK_GBS
                # the same launch on the fp32 matrix cores, timed outside the step
                p.set_dense_arithmetic(lsh.DENSE_FP32)
                fp32_ms = self.timer.measure(lambda: lsh.hash_e2lsh(p, data, out=out))
                p.set_dense_arithmetic(lsh.DENSE_AUTO)
                e["fp32_mfma_route"] = {"ms": fp32_ms, "roofline": dense_roofline(N, n, k, fp32_ms, "fp32")}
                e["speedup_over_fp32_mfma"] = fp32_ms / ms[leg]
            else:
                e["schedule"] = padding_ratio(p)
                e["roofline"] = with_traffic(gather_roofline(N, n, k, p.m, 4 * k, ms[leg]), f"highdim/fastlsh/m{p.m}")
                e["speedup_over_e2lsh"] = ms["e2lsh"] / ms[leg]
                e["operation_count_ratio_n_over_m"] = n / p.m
                if p.m * 8 >= n:
                    # dense enough for the matrix cores to compete: the same call with the sampled
                    # coefficients written out over all n coordinates (LSH_DENSE_MATRIX), timed
                    # outside the step
                    p.set_dense_arithmetic(lsh.DENSE_MATRIX)
                    mat_ms = self.timer.measure(lambda: lsh.hash_fastlsh(p, data, out=out))
                    mat_parity = self.check_ids(p, wl, data, out, False, count=48)
                    p.set_dense_arithmetic(lsh.DENSE_AUTO)
                    e["matrix_core_route"] = {"ms": mat_ms, "parity": mat_parity,
                                              "roofline": dense_roofline(N, n, k, mat_ms, {"products": 6})}
            entries.append(e)
        # the variant with one sample S per table (Sec. 3.1 read literally), timed outside the step
        L = wl.L or 128
        for m in wl.m:
            with lsh.LshParams(n, k, m, wl.w, wl.seed, shared_tables=L) as p:
                sms = self.timer.measure(lambda: lsh.hash_fastlsh(p, data, out=out))
                entries.append({"workload": "highdim", "call": "lsh_hash_fastlsh", "variant": "one sample per table",
                                "L": L, "N": N, "n": n, "k": k, "m": m, "w": wl.w, "ms": sms,
                                "hashes_per_s": N * k / (sms * 1e-3), "vectors_per_s": N / (sms * 1e-3),
                                "dtype": "f32", "timed": "outside the step",
                                "parity": self.check_ids(p, wl, data, out, dense=False),
                                "schedule": {"mfma_steps_per_block_and_tile": p.shared_schedule()[1],
                                             "sample_slots_per_sample": 4.0 * p.shared_schedule()[1] / m},
                                "roofline": shared_roofline(N, n, k, m, sms),
                                "speedup_over_per_function_samples": ms[f"fastlsh_m{m}"] / sms})
        dominant = max(legs, key=lambda leg: ms[leg])
        dom = entries[legs.index(dominant)]
        result = {"elapsed": elapsed, "ms": ms, "entries": entries, "dominant": dominant, "roofline": dom["roofline"],
                  "N": N, "k": k, "n": n, "wl": wl}
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = self.cpu_baseline(wl, data, params)
        for p in params:
            p.close()
        del out, data
        torch.cuda.empty_cache()
        return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3,
                    help="untimed steps after a time-based warm-up of about 150 ms of launches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle comparison of sampled rows")
    ap.add_argument("--only", default="", help="comma-separated subset of: highdim,tiny,sift,gist,angular")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known HBM traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU only (rows shard trivially, but no "
                 "multi-GPU path exists); use --gpus 1")
    only = [s for s in args.only.split(",") if s] or ["highdim", "tiny", "sift", "gist", "angular"]

    b = Bench(args)
    torch = b.torch
    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=b.dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    configs = []
    head = b.headline() if "highdim" in only else None
    if head:
        configs.extend(head["entries"])
    for name in ("tiny", "sift", "gist", "angular"):
        if name in only:
            configs.extend(b.config(name))

    if head is None:
        print(json.dumps({"configs": configs}))
        return
    N, k, n = head["N"], head["k"], head["n"]
    hashes_per_step = 4.0 * N * k
    out = {
        "metric": "hashes/sec (N*k per sec), FastLSH vs E2LSH, 1 GPU",
        "value": hashes_per_step * args.steps / head["elapsed"],
        "unit": "hashes/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["elapsed"] / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 (sampled projections); bf16x3+f32acc (dense product: exact three-way bf16 splits, fp32 accumulation)",
        "data": "synthetic",
        "config": {"workload": "high-dimensional: N=200000 n=4096 k=2048 w=8, i.i.d. N(0,1) rows + 5% planted "
                               "near-duplicates; FastLSH at m=64, 256, 1024 and dense E2LSH (m=n)",
                   "step": "fastlsh ids m=64 + fastlsh ids m=256 + fastlsh ids m=1024 + dense e2lsh ids",
                   "hashes_per_step": hashes_per_step,
                   "warmup_note": "about 150 ms of untimed steps precede the --warmup steps (clock ramp)"},
        "vectors_per_s": 4.0 * N * args.steps / head["elapsed"],
        "kernel_ms": head["ms"],
        "fastlsh_speedup_over_e2lsh": {leg: head["ms"]["e2lsh"] / v for leg, v in head["ms"].items() if leg != "e2lsh"},
        "dominant_kernel": head["dominant"],
        "roofline": head["roofline"],
        "configs": configs,
        "paper_context": "the paper reports up to ~80x faster hash evaluation than E2LSH at n=4096, m=30 on a "
                         "6-core laptop CPU (Sec. 6, Experiment 1); other hardware, not a target",
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
