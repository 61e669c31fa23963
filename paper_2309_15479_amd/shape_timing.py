"""Kernel times of the hash calls on the paper-shaped workloads, one line per call.

    python -m paper_2309_15479_amd.shape_timing [tiny|sift|gist|highdim|angular ...]

Each call is timed with HIP events around back-to-back launches on the current stream
(lsh_time_launches), inputs and outputs resident in HBM, after enough untimed launches for
the GPU's clocks to settle (they ramp up over the first ~100 ms of load).  Printed per call: milliseconds per
launch, the algorithmic HBM rate (4n bytes read + ids / keys / sign words written per
vector), gather-FMAs per second for the sampled calls and flop/s for the dense call.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def settle(launch, busy_ms=150.0):
    """Untimed launches for about busy_ms of GPU time."""
    ms = launch(2)
    launch(max(1, min(200, int(busy_ms / max(ms, 1e-3)))))


def main(names):
    import torch
    import workloads
    import paper_2309_15479_amd as lsh

    lsh.load_library()
    for name in names:
        wl, data = workloads.make_data(name, "cuda")
        N, n, k = wl.N, wl.n, wl.k
        for m in wl.m:
            with lsh.LshParams(n, k, m, wl.w, wl.seed) as p:
                order, group, classes, passes = p.schedule()
                used = int((order != 0xFFFFFFFF).sum())
                conflict = passes / (used / group)
                if wl.signs:
                    out = torch.empty((N, (k + 63) // 64), dtype=torch.int64, device="cuda")
                    which, out_bytes = "signs", 8 * ((k + 63) // 64)
                else:
                    out = torch.empty((N, k), dtype=torch.int32, device="cuda")
                    which, out_bytes = "fastlsh", 4 * k
                settle(lambda reps: lsh.time_launches(p, which, data, out, reps=reps))
                ms = lsh.time_launches(p, which, data, out, reps=10)
                print(f"{name} n={n} k={k} m={m} {which}: {ms:.3f} ms  "
                      f"{N * (4 * n + out_bytes) / ms / 1e6:.0f} GB/s algorithmic  "
                      f"{N * k * m / ms / 1e9:.2f} T gather-FMA/s  "
                      f"(schedule: {conflict:.3f} x conflict-free)", flush=True)
                if wl.L and not wl.signs:
                    keys = torch.empty((N, wl.L), dtype=torch.int64, device="cuda")
                    settle(lambda reps: lsh.time_launches(p, "pack_keys", out, keys, L=wl.L, reps=reps))
                    ms = lsh.time_launches(p, "pack_keys", out, keys, L=wl.L, reps=10)
                    print(f"{name} pack_keys L={wl.L}: {ms:.3f} ms  "
                          f"{N * (4 * k + 8 * wl.L) / ms / 1e6:.0f} GB/s algorithmic", flush=True)
                    g = k // wl.L
                    if g & (g - 1) == 0 and g <= 64:
                        settle(lambda reps: lsh.time_launches(p, "fastlsh_keys", data, keys, L=wl.L, reps=reps))
                        ms = lsh.time_launches(p, "fastlsh_keys", data, keys, L=wl.L, reps=10)
                        print(f"{name} m={m} fastlsh_keys L={wl.L}: {ms:.3f} ms  "
                              f"{N * (4 * n + 8 * wl.L) / ms / 1e6:.0f} GB/s algorithmic", flush=True)
                del out
            if wl.L and not wl.signs:
                # one sample per table (matrix-core kernel where the shape allows)
                with lsh.LshParams(n, k, m, wl.w, wl.seed, shared_tables=wl.L) as p:
                    out = torch.empty((N, k), dtype=torch.int32, device="cuda")
                    settle(lambda reps: lsh.time_launches(p, "fastlsh", data, out, reps=reps))
                    ms = lsh.time_launches(p, "fastlsh", data, out, reps=10)
                    print(f"{name} n={n} k={k} m={m} fastlsh, one sample per table (L={wl.L}): {ms:.3f} ms  "
                          f"{N * (4 * n + 4 * k) / ms / 1e6:.0f} GB/s algorithmic  "
                          f"{2 * N * k * m / ms / 1e9:.1f} TFLOP/s", flush=True)
                    # maximum-inner-product transform (appendix): kappa~ pass, data hash, query hash
                    try:
                        kap = lsh.mips_kappa(p, data)
                    except lsh.LshError:
                        kap = None           # shape outside the matrix-core kernel
                    if kap is not None:
                        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                        for _ in range(3):
                            lsh.mips_kappa(p, data, out=kap)
                            lsh.hash_mips_data(p, data, kap, out=out)
                            lsh.hash_mips_query(p, data, out=out)
                        reps = 10
                        ev[0].record()
                        for _ in range(reps):
                            lsh.mips_kappa(p, data, out=kap)
                        ev[1].record()
                        for _ in range(reps):
                            lsh.hash_mips_data(p, data, kap, out=out)
                        ev[2].record()
                        for _ in range(reps):
                            lsh.hash_mips_query(p, data, out=out)
                        ev[3].record()
                        torch.cuda.synchronize()
                        t = [ev[i].elapsed_time(ev[i + 1]) / reps for i in range(3)]
                        print(f"{name} n={n} k={k} m={m} maximum inner product: kappa {t[0]:.3f} ms "
                              f"({N * 4 * n / t[0] / 1e6:.0f} GB/s), data hash {t[1]:.3f} ms "
                              f"({N * (4 * n + 4 * k) / t[1] / 1e6:.0f} GB/s), query hash {t[2]:.3f} ms", flush=True)
                    del out
        if wl.L and not wl.signs:
            # index: build the L tables from the keys, probe 4096 of the vectors as queries
            import time
            with lsh.LshParams(n, k, wl.m[0], wl.w, wl.seed) as p:
                keys = lsh.hash_fastlsh_keys(p, data, wl.L)
            torch.cuda.synchronize()
            lsh.LshIndex(keys).close()                       # warm-up (first launches, allocator)
            t0 = time.perf_counter()
            ix = lsh.LshIndex(keys)                          # waits for the sorts
            build_ms = (time.perf_counter() - t0) * 1e3
            qkeys = keys[:4096].contiguous()
            queries = data[:4096].contiguous()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            start, count = ix.probe(qkeys)
            ix.nearest(data, queries, start, count)
            torch.cuda.synchronize()
            ev[0].record()
            start, count = ix.probe(qkeys)
            ev[1].record()
            best, dist = ix.nearest(data, queries, start, count)
            ev[2].record()
            torch.cuda.synchronize()
            cands = int(count.to(torch.int64).sum().item())
            print(f"{name} index L={wl.L}: build {build_ms:.1f} ms ({N * wl.L / build_ms / 1e3:.0f} M pairs/s)  "
                  f"probe of 4096 queries {ev[0].elapsed_time(ev[1]):.3f} ms  exact nearest over {cands} candidates "
                  f"{ev[1].elapsed_time(ev[2]):.3f} ms", flush=True)
            ix.close()
            del keys, qkeys, queries
        if not wl.signs:
            with lsh.LshParams(n, k, n, wl.w, wl.seed) as p:
                out = torch.empty((N, k), dtype=torch.int32, device="cuda")
                settle(lambda reps: lsh.time_launches(p, "e2lsh", data, out, reps=reps))
                ms = lsh.time_launches(p, "e2lsh", data, out, reps=5)
                print(f"{name} n={n} k={k} e2lsh (dense): {ms:.3f} ms  "
                      f"{2 * N * n * k / ms / 1e9:.1f} TFLOP/s", flush=True)
                del out
        del data
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main(sys.argv[1:] or ["tiny", "sift", "gist", "highdim", "angular"])
