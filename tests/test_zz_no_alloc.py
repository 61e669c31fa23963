"""The offsets scan that allocates nothing (lsh_index_candidate_offsets_static) against the
allocating entry point: same outputs bit for bit, on two calls in a row that share the
library's static scratch array, the second with a smaller input."""
import ctypes
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lsh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_15479_amd as lib
    lib.load_library()
    return lib


def _counts(items, seed, hi):
    rng = np.random.default_rng(seed)
    c = rng.integers(0, hi, size=items, dtype=np.uint32)
    if items > 10:
        c[rng.integers(0, items, size=3)] = np.uint32(0xFFFFFFF0)   # sums need 64 bits
    return c


def test_static_scratch_offsets_match_the_allocating_call(lsh):
    # spans several 2048-count blocks with a ragged tail, then a smaller input that reuses the
    # scratch words the first call left behind, then the smallest and the empty case
    for items, seed, hi in ((3 * 2048 * 37 + 1234, 1, 1000), (2048 + 17, 2, 50), (5, 3, 7), (0, 4, 2)):
        print(f"offsets scan: items={items}", flush=True)
        sys.stdout.flush()
        counts_h = _counts(items, seed, hi)
        counts = torch.as_tensor(counts_h.view(np.int32), device="cuda")
        if items == 0:
            counts = torch.zeros(1, dtype=torch.int32, device="cuda")[:0]   # a valid pointer, no elements
        want = lsh.candidate_offsets(counts)
        out = torch.full((items + 1,), -1, dtype=torch.int64, device="cuda")
        got = lsh.candidate_offsets(counts, out=out, static_scratch=True)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"items={items}"
        expect = np.concatenate([[0], np.cumsum(counts_h.astype(np.uint64))]).astype(np.uint64)
        assert np.array_equal(got.cpu().numpy().view(np.uint64), expect), f"items={items}"


def test_static_scratch_limit_and_arguments(lsh):
    lib = lsh.load_library()
    buf = torch.zeros(8, dtype=torch.int64, device="cuda")
    cnt = torch.zeros(8, dtype=torch.int32, device="cuda")
    assert lib.lsh_index_candidate_offsets_static(cnt.data_ptr(), (1 << 22) + 1, buf.data_ptr(), None) == -4
    assert lib.lsh_index_candidate_offsets_static(None, 4, buf.data_ptr(), None) == -1
    assert lib.lsh_index_candidate_offsets_static(cnt.data_ptr(), 4, None, None) == -1


def test_static_scratch_at_the_limit(lsh):
    items = 1 << 22
    counts_h = _counts(items, 9, 3)
    counts = torch.as_tensor(counts_h.view(np.int32), device="cuda")
    got = lsh.candidate_offsets(counts, static_scratch=True)
    want = lsh.candidate_offsets(counts)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    assert int(got[-1].item()) == int(counts_h.astype(np.uint64).sum())
