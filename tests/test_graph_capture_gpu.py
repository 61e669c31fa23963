"""The hash calls allocate nothing, synchronise nothing and record no memset, so a step can be
captured in a HIP graph (after one eager call per kernel, which raises the kernels' LDS limits)
and replayed: every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_step_replays_from_a_graph():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_15479_amd as lsh
    lsh.load_library()
    wl, data = workloads.make_data("tiny", "cuda")
    N, n, k, m, L = wl.N, wl.n, wl.k, wl.m[0], wl.L
    with lsh.LshParams(n, k, m, wl.w, wl.seed) as pf, lsh.LshParams(n, k, n, wl.w, wl.seed) as pd, \
            lsh.LshParams(n, k, m, wl.w, wl.seed, shared_tables=L) as ps:
        outs = dict(ids=torch.empty((N, k), dtype=torch.int32, device="cuda"),
                    keys=torch.empty((N, L), dtype=torch.int64, device="cuda"),
                    dense=torch.empty((N, k), dtype=torch.int32, device="cuda"),
                    words=torch.empty((N, (k + 63) // 64), dtype=torch.int64, device="cuda"),
                    shared=torch.empty((N, k), dtype=torch.int32, device="cuda"),
                    kappa=torch.empty(L, dtype=torch.float32, device="cuda"),
                    mips=torch.empty((N, k), dtype=torch.int32, device="cuda"))

        def step():
            lsh.hash_fastlsh(pf, data, out=outs["ids"])
            lsh.pack_keys(pf, outs["ids"], L, out=outs["keys"])
            lsh.hash_e2lsh(pd, data, out=outs["dense"])
            lsh.hash_signs(pf, data, out=outs["words"])
            lsh.hash_fastlsh(ps, data, out=outs["shared"])
            lsh.mips_kappa(ps, data, out=outs["kappa"])
            lsh.hash_mips_data(ps, data, outs["kappa"], out=outs["mips"])

        step()                                   # eager: also the one-time attribute calls
        torch.cuda.synchronize()
        want = {name: t.clone() for name, t in outs.items()}
        side = torch.cuda.Stream()               # default priority
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        for replay in range(3):
            for t in outs.values():
                t.zero_()
            other = torch.randn(1 << 20, device="cuda").sum()      # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name, t in outs.items():
                assert torch.equal(t, want[name]), f"replay {replay}: {name} differs from the eager result"
            assert torch.isfinite(other)
