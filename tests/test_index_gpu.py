"""GPU parity of the LSH index (build, probe, candidates, exact nearest) against the dictionary
oracle: integer work, compared bit for bit."""
import sys

import numpy as np
import pytest

import oracle
import workloads
from oracle import index as oindex

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lsh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_15479_amd as lib
    lib.load_library()
    return lib


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _check_against_oracle(lsh, keys_np, qkeys_np, label):
    keys = torch.as_tensor(keys_np.view(np.int64), device="cuda")
    qkeys = torch.as_tensor(qkeys_np.view(np.int64), device="cuda")
    N, L = keys_np.shape
    tables = oindex.build(keys_np)
    want = oindex.probe(tables, qkeys_np)
    with lsh.LshIndex(keys) as ix:
        start, count = ix.probe(qkeys)
        offsets, ids = ix.candidates(start, count)
        torch.cuda.synchronize()
        start_h, count_h = start.cpu().numpy().view(np.uint32), count.cpu().numpy().view(np.uint32)
        off_h, ids_h = offsets.cpu().numpy(), ids.cpu().numpy().view(np.uint32)
        assert off_h[0] == 0 and (np.diff(off_h) == count_h.reshape(-1)).all(), label
        for q in range(qkeys_np.shape[0]):
            for l in range(L):
                item = q * L + l
                got = ids_h[off_h[item]:off_h[item + 1]].tolist()
                assert got == want[q][l], f"{label}: bucket of query {q} in table {l}"
            combined = ids_h[off_h[q * L]:off_h[(q + 1) * L]].tolist()
            assert combined == oindex.candidates(want[q])
    return want


@pytest.mark.parametrize("N,L,Q,spread,seed", [(1, 1, 3, 2, 1), (1000, 4, 50, 37, 2), (5000, 7, 64, 10 ** 12, 3),
                                               (4097, 32, 20, 300, 4), (300, 3, 10, 1, 5)])
def test_index_on_synthetic_keys(lsh, N, L, Q, spread, seed):
    """Few distinct keys (long buckets), many (mostly empty lookups), one key for everything;
    queries are a mix of indexed keys and unseen ones, with keys using all 64 bits."""
    say(f"index case N={N} L={L} Q={Q} spread={spread}")
    rng = np.random.default_rng(seed)
    base = rng.integers(0, 2 ** 63, size=L, dtype=np.uint64) * np.uint64(2) + np.uint64(1)
    keys = (rng.integers(0, spread, size=(N, L)).astype(np.uint64) * base)
    qkeys = np.vstack([keys[rng.integers(0, N, size=Q // 2)],
                       rng.integers(0, spread + 3, size=(Q - Q // 2, L)).astype(np.uint64) * base])
    _check_against_oracle(lsh, keys, qkeys, f"synthetic{seed}")


def test_index_end_to_end_with_fastlsh_keys_and_exact_nearest(lsh):
    """Hash -> keys -> index -> probe -> exact nearest on planted near neighbours, every stage on
    the GPU, against the oracle's dictionaries and fp64 distances."""
    rng = np.random.default_rng(11)
    n, N, k, m, w, L, Q = 64, 20000, 128, 16, 8.0, 16, 48
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    data = torch.randn((N, n), generator=g, device="cuda") * 3.0
    src = rng.integers(0, N, size=Q)
    noise = torch.randn((Q, n), generator=g, device="cuda") * 0.05
    queries = (data[torch.as_tensor(src, device="cuda")] + noise).contiguous()
    queries[-4:] = torch.randn((4, n), generator=g, device="cuda") * 50.0      # far from everything
    with lsh.LshParams(n, k, m, w, 3) as p:
        keys = lsh.hash_fastlsh_keys(p, data, L)
        qkeys = lsh.hash_fastlsh_keys(p, queries, L)
        torch.cuda.synchronize()
    want = _check_against_oracle(lsh, keys.cpu().numpy().view(np.uint64), qkeys.cpu().numpy().view(np.uint64), "e2e")
    data_h, queries_h = data.cpu().numpy(), queries.cpu().numpy()
    with lsh.LshIndex(keys) as ix:
        start, count = ix.probe(qkeys)
        best, dist = ix.nearest(data, queries, start, count)
        torch.cuda.synchronize()
    best_h, dist_h = best.cpu().numpy(), dist.cpu().numpy()
    found = 0
    for q in range(Q):
        cand = oindex.candidates(want[q])
        expect = oindex.nearest(data_h, queries_h[q], cand)
        if expect < 0:
            assert best_h[q] == -1 and np.isinf(dist_h[q])
            continue
        d2 = ((data_h[expect].astype(np.float64) - queries_h[q].astype(np.float64)) ** 2).sum()
        assert abs(dist_h[q] - d2) <= 1e-5 * d2 + 1e-12
        if best_h[q] != expect:      # only a near-tie in fp32 may pick another candidate
            other = ((data_h[best_h[q]].astype(np.float64) - queries_h[q].astype(np.float64)) ** 2).sum()
            assert best_h[q] in cand and abs(other - d2) <= 1e-5 * d2
        found += int(best_h[q] == src[q])
    say(f"planted neighbours found: {found} of {Q - 4}")
    assert found >= (Q - 4) * 0.8
    # the same candidates ranked by inner product (maximum inner product search), all and first 5
    with lsh.LshIndex(keys) as ix:
        start, count = ix.probe(qkeys)
        for limit in (0, 5):
            bip, ip = ix.best_inner_product(data, queries, start, count, max_candidates=limit)
            torch.cuda.synchronize()
            bip_h, ip_h = bip.cpu().numpy(), ip.cpu().numpy()
            for q in range(Q):
                cand = oindex.candidates(want[q])
                expect = oindex.best_inner_product(data_h, queries_h[q], cand, max_candidates=limit)
                if expect < 0:
                    assert bip_h[q] == -1 and np.isneginf(ip_h[q])
                    continue
                scale = float(np.abs(data_h[expect].astype(np.float64) * queries_h[q].astype(np.float64)).sum())
                e_ip = float((data_h[expect].astype(np.float64) * queries_h[q].astype(np.float64)).sum())
                assert abs(ip_h[q] - e_ip) <= 1e-5 * scale + 1e-12
                if bip_h[q] != expect:   # only a near-tie in fp32 may pick another candidate
                    o_ip = float((data_h[bip_h[q]].astype(np.float64) * queries_h[q].astype(np.float64)).sum())
                    assert bip_h[q] in (cand[:limit] if limit else cand) and abs(o_ip - e_ip) <= 1e-5 * scale
    # approximate version: only the first 3 candidates of the combined list
    with lsh.LshIndex(keys) as ix:
        start, count = ix.probe(qkeys)
        best3, dist3 = ix.nearest(data, queries, start, count, max_candidates=3)
        torch.cuda.synchronize()
    best3_h = best3.cpu().numpy()
    for q in range(Q):
        cand = oindex.candidates(want[q])
        expect = oindex.nearest(data_h, queries_h[q], cand, max_candidates=3)
        if best3_h[q] != expect:
            d_e = ((data_h[expect].astype(np.float64) - queries_h[q].astype(np.float64)) ** 2).sum()
            d_g = ((data_h[best3_h[q]].astype(np.float64) - queries_h[q].astype(np.float64)) ** 2).sum()
            assert best3_h[q] in cand[:3] and abs(d_g - d_e) <= 1e-5 * d_e


def test_index_sift_shape_build_and_probe(lsh):
    """The benchmark shape: 1e6 vectors, 32 tables; sampled queries against the oracle built on
    the same keys (dictionary of the queried keys only, to keep the CPU side short)."""
    wl, data = workloads.make_data("sift", "cuda")
    with lsh.LshParams(wl.n, wl.k, wl.m[0], wl.w, wl.seed) as p:
        keys = lsh.hash_fastlsh_keys(p, data, wl.L)
        torch.cuda.synchronize()
    rows = np.random.default_rng(5).integers(0, wl.N, size=64)
    qkeys = keys[torch.as_tensor(rows, device="cuda")].contiguous()
    with lsh.LshIndex(keys) as ix:
        start, count = ix.probe(qkeys)
        offsets, ids = ix.candidates(start, count)
        torch.cuda.synchronize()
    keys_h = keys.cpu().numpy().view(np.uint64)
    off_h, ids_h = offsets.cpu().numpy(), ids.cpu().numpy().view(np.uint32)
    for qi, row in enumerate(rows):
        for l in range(wl.L):
            expect = np.nonzero(keys_h[:, l] == keys_h[row, l])[0]
            got = ids_h[off_h[qi * wl.L + l]:off_h[qi * wl.L + l + 1]]
            assert np.array_equal(got, expect.astype(np.uint32))
            assert row in got


def test_index_errors(lsh):
    lib = lsh.load_library()
    import ctypes
    h = ctypes.c_void_p()
    assert lib.lsh_index_build(None, 10, 2, None, ctypes.byref(h)) == -1
    keys = torch.zeros((4, 2), dtype=torch.int64, device="cuda")
    assert lib.lsh_index_build(keys.data_ptr(), 0, 2, None, ctypes.byref(h)) == -1
    with lsh.LshIndex(keys) as ix:
        assert lib.lsh_index_probe(ix.handle, None, 3, None, None, None) == -1
        assert lib.lsh_index_probe(ix.handle, None, 0, None, None, None) == 0
        start, count = ix.probe(torch.zeros((0, 2), dtype=torch.int64, device="cuda"))
        assert start.shape == (0, 2)
