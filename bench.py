#!/usr/bin/env python3
"""Benchmark of the LSH hash-evaluation hot path on one MI355X.

One step = one pass of the whole path over the SIFT-shaped batch (N = 1,000,000 vectors,
n = 128, k = 512 functions, m = 32 sampled coordinates, w = 16), inputs resident in HBM:

    FastLSH bucket ids  ->  key packing (L = 32 keys of 16 ids)  ->  dense E2LSH bucket ids
    (m = n, same seed)  ->  sign hashes

Prints ONE JSON line.  `value` is hashes per second over the whole step: a step evaluates
3*N*k hash functions (N*k FastLSH, N*k E2LSH, N*k sign hashes).  Per-kernel times come
from HIP events recorded on the launch stream inside the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # dense fp32 matrix peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix peak
# fp32 vector peak with packed instructions: 256 CUs x 128 FMA lanes/clk x 2 flop x 2.4 GHz.
# This library is compiled without packed fp32 operations; a plain 64-lane v_fma_f32 occupies a
# SIMD for four cycles, i.e. 64 lanes/clk/CU, half of that peak.
VALU_FP32_PEAK_TFLOPS = 157.3
VALU_FP32_UNPACKED_TFLOPS = 78.6

# HBM bytes per launch on this workload from rocprofv3's FETCH_SIZE and WRITE_SIZE counters
# (two runs, each scaled by what the same counter reads for a 1 GiB device copy: 2 KiB and
# 1 KiB per count), taken on the kernels as they stand; the summary and its commands are in
# profiles/sift_step_hbm_traffic.md.  Set an entry to None when its kernel changes.
MEASURED_TRAFFIC_BYTES = {
    "fastlsh": 252146 * 2048 + 2000010 * 1024,    # 0.516 GB read + 2.048 GB written (matrix-core kernel)
    "fastlsh_gathered": 250604 * 2048 + 2000000 * 1024,  # 0.513 GB read + 2.048 GB written (gathered fp32 kernel)
    "pack_keys": 1000042 * 2048 + 250000 * 1024,  # 2.048 GB + 0.256 GB
    "e2lsh": 252330 * 2048 + 2000016 * 1024,      # 0.517 GB + 2.048 GB (the same kernel on the E2LSH matrix)
    "e2lsh_fp32": 251082 * 2048 + 2020697 * 1024,  # 0.514 GB + 2.069 GB (fp32 MFMA kernel)
    "signs": 251162 * 2048 + 62500 * 1024,        # 0.514 GB + 0.064 GB (matrix-core kernel)
    "signs_gathered": 250574 * 2048 + 62500 * 1024,  # 0.513 GB + 0.064 GB (gathered fp32 kernel)
    "fastlsh_shared_sample": 250411 * 2048 + 2000000 * 1024,  # 0.513 GB + 2.048 GB
}


def cpu_baseline(wl, data, p_fast, p_dense, budget_s=12.0):
    """Times the CPU oracle (all host threads) on a bounded sample of rows of the same batch."""
    import numpy as np
    import oracle
    threads = oracle.max_threads()
    tabs_f = (p_fast.indices(), p_fast.coeffs(), p_fast.offsets())
    tabs_d = (p_dense.coeffs(), p_dense.offsets())

    def run(rows):
        t0 = time.perf_counter()
        ids = oracle.fastlsh(rows, *tabs_f, wl.w, nthreads=threads)["ids"]
        oracle.pack_keys(ids, wl.L)
        oracle.e2lsh(rows, *tabs_d, wl.w, nthreads=threads)
        oracle.signs(rows, tabs_f[0], tabs_f[1], nthreads=threads)
        return time.perf_counter() - t0

    pilot = data[:2048].cpu().numpy()
    t_pilot = run(pilot)
    count = int(max(2048, min(data.shape[0], 2048 * budget_s / max(t_pilot, 1e-6))))
    rows = data[:count].cpu().numpy()
    t = run(rows)
    return {"value": 3.0 * count * wl.k / t, "unit": "hashes/s", "cores": threads, "kind": "oracle",
            "sample": f"first {count} rows of the same batch, all four stages, {t:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    # the GPU's clocks ramp up over the first ~100 ms of load: warm up for about that long
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known HBM traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU only (rows shard trivially, but no "
                 "multi-GPU path exists); use --gpus 1")

    import torch
    import paper_2309_15479_amd as lsh
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    lsh.load_library()
    dev = "cuda:0"
    wl, data = workloads.make_data("sift", dev)
    N, n, k, m, L = wl.N, wl.n, wl.k, wl.m[0], wl.L
    p_fast = lsh.LshParams(n, k, m, wl.w, wl.seed)
    p_dense = lsh.LshParams(n, k, n, wl.w, wl.seed)
    ids_f = torch.empty((N, k), dtype=torch.int32, device=dev)
    ids_d = torch.empty((N, k), dtype=torch.int32, device=dev)
    keys = torch.empty((N, L), dtype=torch.int64, device=dev)
    words = torch.empty((N, (k + 63) // 64), dtype=torch.int64, device=dev)

    stages = ["fastlsh", "pack_keys", "e2lsh", "signs"]

    def step(events=None):
        def mark():
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()          # on torch's current stream = the stream the library launches on
                events.append(e)
        mark()
        lsh.hash_fastlsh(p_fast, data, out=ids_f)
        mark()
        lsh.pack_keys(p_fast, ids_f, L, out=keys)
        mark()
        lsh.hash_e2lsh(p_dense, data, out=ids_d)
        mark()
        lsh.hash_signs(p_fast, data, out=words)
        mark()

    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

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

    ms = {s: 0.0 for s in stages}
    for ev in all_events:
        for i, s in enumerate(stages):
            ms[s] += ev[i].elapsed_time(ev[i + 1])
    ms = {s: v / args.steps for s, v in ms.items()}

    def hbm(stage, bytes_per_launch):
        a = bytes_per_launch / (ms[stage] * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": a / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES[stage]}

    rooflines = {
        # algorithmic bytes per vector: 4n read + 4k written (ids) / 8 per 64 functions (signs)
        "fastlsh": hbm("fastlsh", N * (4 * n + 4 * k)),
        "pack_keys": hbm("pack_keys", N * (4 * k + 8 * L)),
    }
    # The dense product runs as bf16 MFMA products of exact three-way splits (fp32 accuracy).  On
    # this integer-valued batch the second and third terms of the data are zero and their
    # products are skipped: 3 of the 6 remain, 6 n k bf16 flop per vector, and the launch is
    # bound by the 4n + 4k bytes per vector it moves.
    tf = 2.0 * N * n * k / (ms["e2lsh"] * 1e-3) / 1e12
    gbs = N * (4 * n + 4 * k) / (ms["e2lsh"] * 1e-3) / 1e9
    rooflines["e2lsh"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": gbs / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES["e2lsh"],
                          "arithmetic": "bf16 x 3 splits, fp32 accumulation; 3 of 6 MFMA products (zero terms skipped)",
                          "mfma_tflops": 3.0 * tf, "mfma_frac_of_bf16_peak": 3.0 * tf / MFMA_BF16_PEAK_TFLOPS,
                          "fp32_equivalent_tflops": tf,
                          "fp32_equivalent_frac_of_fp32_mfma_peak": tf / MFMA_FP32_PEAK_TFLOPS}
    # Sign hashes at n = 128 run on the same matrix-core kernel from the coefficients written out
    # densely, with two-way splits and three products (two on this integer-valued batch: 4 n k
    # bf16 flop per vector): only the sign is needed, and it is compared outside 1e-4 |a| |S(v)|
    # of zero.
    tf = 2.0 * N * n * k / (ms["signs"] * 1e-3) / 1e12
    gbs = N * (4 * n + 8 * ((k + 63) // 64)) / (ms["signs"] * 1e-3) / 1e9
    rooflines["signs"] = {"bound": "mfma", "achieved": 2.0 * tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "frac": 2.0 * tf / MFMA_BF16_PEAK_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES["signs"],
                          "arithmetic": "bf16 x 2 splits of the densely written coefficients; 2 of 3 MFMA products (zero terms skipped)",
                          "hbm_gbs": gbs, "hbm_frac": gbs / HBM_PEAK_GBS}
    # FastLSH ids at n = 128 run on the same matrix-core kernel as the dense product, over the
    # coefficients written out densely (zeros at the coordinates a function does not sample)
    tf = 2.0 * N * n * k / (ms["fastlsh"] * 1e-3) / 1e12
    rooflines["fastlsh"]["arithmetic"] = rooflines["e2lsh"]["arithmetic"]
    rooflines["fastlsh"]["mfma_tflops"] = 3.0 * tf
    rooflines["fastlsh"]["mfma_frac_of_bf16_peak"] = 3.0 * tf / MFMA_BF16_PEAK_TFLOPS
    dominant = max(stages, key=lambda s: ms[s])

    # Outside the timed step: the same FastLSH shape with one sample per table (L = 32 tables
    # of 16 functions), which runs on the matrix cores; reported beside the step's kernels.
    p_shared = lsh.LshParams(n, k, m, wl.w, wl.seed, shared_tables=L)
    for _ in range(args.warmup):
        lsh.hash_fastlsh(p_shared, data, out=ids_f)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        lsh.hash_fastlsh(p_shared, data, out=ids_f)
    e1.record()
    torch.cuda.synchronize()
    ms_shared = e0.elapsed_time(e1) / args.steps
    a = N * (4 * n + 4 * k) / (ms_shared * 1e-3) / 1e9
    shared_sample = {"ms": ms_shared, "bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": a / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES["fastlsh_shared_sample"],
                     "mfma_tflops": 2.0 * N * k * m / (ms_shared * 1e-3) / 1e12,
                     "hashes_per_s": N * k / (ms_shared * 1e-3)}

    # and the dense product on the fp32 matrix cores (the library's other dense arithmetic)
    p_dense.set_dense_arithmetic(lsh.DENSE_FP32)
    for _ in range(args.warmup):
        lsh.hash_e2lsh(p_dense, data, out=ids_d)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        lsh.hash_e2lsh(p_dense, data, out=ids_d)
    e1.record()
    torch.cuda.synchronize()
    p_dense.set_dense_arithmetic(lsh.DENSE_AUTO)
    ms_fp32 = e0.elapsed_time(e1) / args.steps
    tf32 = 2.0 * N * n * k / (ms_fp32 * 1e-3) / 1e12
    e2lsh_fp32 = {"ms": ms_fp32, "bound": "mfma", "achieved": tf32, "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                  "frac": tf32 / MFMA_FP32_PEAK_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES["e2lsh_fp32"]}
    # and the FastLSH ids and sign hashes by the gathered fp32 kernels (the sampled projection
    # as the paper writes it: m multiply-adds per function)
    p_fast.set_dense_arithmetic(lsh.DENSE_FP32)
    gathered_ms = {}
    for name, fn in (("ids", lambda: lsh.hash_fastlsh(p_fast, data, out=ids_f)),
                     ("signs", lambda: lsh.hash_signs(p_fast, data, out=words))):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        gathered_ms[name] = e0.elapsed_time(e1) / args.steps
    p_fast.set_dense_arithmetic(lsh.DENSE_AUTO)
    ms_ig = gathered_ms["ids"]
    gbs_ig = N * (4 * n + 4 * k) / (ms_ig * 1e-3) / 1e9
    alu_ig = 2.0 * N * k * m / (ms_ig * 1e-3) / 1e12
    fastlsh_gathered = {"ms": ms_ig, "bound": "hbm", "achieved": gbs_ig, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs_ig / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES["fastlsh_gathered"],
                        "alu_tflops": alu_ig, "alu_frac_of_unpacked_fp32_issue_rate": alu_ig / VALU_FP32_UNPACKED_TFLOPS}
    ms_sg = gathered_ms["signs"]
    gbs_sg = N * (4 * n + 8 * ((k + 63) // 64)) / (ms_sg * 1e-3) / 1e9
    alu_sg = 2.0 * N * k * m / (ms_sg * 1e-3) / 1e12
    signs_gathered = {"ms": ms_sg, "bound": "alu", "achieved": alu_sg, "peak": VALU_FP32_UNPACKED_TFLOPS,
                      "unit": "TFLOP/s", "frac": alu_sg / VALU_FP32_UNPACKED_TFLOPS,
                      "traffic": MEASURED_TRAFFIC_BYTES["signs_gathered"], "hbm_gbs": gbs_sg}

    # The matrix-core kernels skip, tile by tile, the products of split terms that are zero: the
    # SIFT-shaped batch is integer-valued (one bf16 term per coordinate), so its tiles take 3 of
    # the 6 products (signs: 2 of 3).  The same launches on a batch with full fp32 significands:
    data_full = data + torch.rand_like(data)
    timings_full = {}
    for name, fn in (("e2lsh_ms", lambda: lsh.hash_e2lsh(p_dense, data_full, out=ids_d)),
                     ("fastlsh_ms", lambda: lsh.hash_fastlsh(p_fast, data_full, out=ids_f)),
                     ("signs_ms", lambda: lsh.hash_signs(p_fast, data_full, out=words))):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        timings_full[name] = e0.elapsed_time(e1) / args.steps
    del data_full

    hashes_per_step = 3.0 * N * k
    out = {
        "metric": "hashes/sec (N*k per sec), FastLSH vs E2LSH, 1 GPU",
        "value": hashes_per_step * args.steps / elapsed,
        "unit": "hashes/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16x3+f32acc",
        "data": "synthetic",
        "config": {"workload": "sift-shaped: N=1000000 n=128 k=512 m=32 w=16 L=32, 100-cluster mixture in [0,255]",
                   "step": "fastlsh ids + key packing + dense e2lsh ids (m=n) + sign hashes",
                   "hashes_per_step": hashes_per_step,
                   "dense_arithmetic": "bf16 x 3 exact splits on the bf16 matrix cores, fp32 accumulation"},
        "vectors_per_s": N * args.steps / elapsed,
        "kernel_ms": ms,
        "fastlsh_hashes_per_s": N * k / (ms["fastlsh"] * 1e-3),
        "e2lsh_hashes_per_s": N * k / (ms["e2lsh"] * 1e-3),
        "fastlsh_speedup_over_e2lsh": ms["e2lsh"] / ms["fastlsh"],
        "dominant_kernel": dominant,
        "roofline": rooflines[dominant],
        "rooflines": rooflines,
        "fastlsh_shared_sample_per_table": shared_sample,
        "e2lsh_fp32_mfma": e2lsh_fp32,
        "signs_gathered_fp32": signs_gathered,
        # the same four stages with LSH_DENSE_FP32 (gathered fp32 kernels, fp32 MFMA), from the
        # legs timed above one kernel at a time: the step if no bf16 product were used
        "fp32_arithmetic_step": {
            "ms": ms_ig + ms["pack_keys"] + ms_fp32 + ms_sg,
            "hashes_per_s": hashes_per_step / ((ms_ig + ms["pack_keys"] + ms_fp32 + ms_sg) * 1e-3)},
        "precision": "every output meets the same bar as the fp32 kernels against the fp64 oracle "
                     "(projections within 1e-5 * sum|a_i v_i|, ids identical outside 1e-4 of a boundary, sign "
                     "bits identical outside 1e-4 |a||S(v)| of zero); the bf16 terms are exact splits of the fp32 operands",
        "fastlsh_gathered_fp32": fastlsh_gathered,
        "matrix_core_kernels_on_full_significand_data": timings_full,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, data, p_fast, p_dense)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
