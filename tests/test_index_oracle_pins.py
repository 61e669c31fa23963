"""Pins of the index oracle (oracle/index.py): a hand-checked example and the invariants of a
hash table."""
import numpy as np

import oracle
from oracle import index as oindex


def test_hand_example():
    # 5 vectors, 2 tables
    keys = np.array([[7, 1], [9, 1], [7, 2], [7, 1], [8, 3]], np.uint64)
    tables = oindex.build(keys)
    assert tables[0] == {7: [0, 2, 3], 9: [1], 8: [4]}
    assert tables[1] == {1: [0, 1, 3], 2: [2], 3: [4]}
    buckets = oindex.probe(tables, np.array([[7, 3], [5, 1]], np.uint64))
    assert buckets[0] == [[0, 2, 3], [4]]
    assert buckets[1] == [[], [0, 1, 3]]
    assert oindex.candidates(buckets[0]) == [0, 2, 3, 4]


def test_every_id_is_in_exactly_one_bucket_per_table_and_buckets_share_their_key():
    rng = np.random.default_rng(1)
    keys = rng.integers(0, 40, size=(300, 4)).astype(np.uint64)
    tables = oindex.build(keys)
    for l, table in enumerate(tables):
        ids = sorted(i for bucket in table.values() for i in bucket)
        assert ids == list(range(300))
        for key, bucket in table.items():
            assert bucket == sorted(bucket)
            assert all(int(keys[i, l]) == key for i in bucket)
    # a data vector used as query finds itself in every table
    buckets = oindex.probe(tables, keys[17:18])
    assert all(17 in b for b in buckets[0])


def test_near_duplicates_are_found_through_real_hashes():
    # end to end with the hash oracle: a planted near neighbour shares most buckets with its
    # source, a random vector few; exact processing returns the planted neighbour
    rng = np.random.default_rng(2)
    n, N, k, m, w, L = 32, 400, 64, 16, 4.0, 8
    data = rng.normal(size=(N, n)).astype(np.float32) * 3
    query = (data[123] + 0.05 * rng.normal(size=n)).astype(np.float32)
    idx, coef, off = oracle.params(n, k, m, w, seed=5)
    ids = oracle.fastlsh(np.vstack([data, query[None]]), idx, coef, off, w)["ids"]
    keys = oracle.pack_keys(ids, L)
    tables = oindex.build(keys[:N])
    buckets = oindex.probe(tables, keys[N:])[0]
    cand = oindex.candidates(buckets)
    assert cand.count(123) >= L // 2
    assert oindex.nearest(data, query, cand) == 123


def test_best_inner_product_is_the_brute_force_argmax():
    import numpy as np
    from oracle import index as ix
    rng = np.random.default_rng(3)
    data = rng.normal(size=(50, 7)).astype(np.float32)
    q = rng.normal(size=7).astype(np.float32)
    cand = [4, 9, 9, 30, 2, 41, 4]
    ips = data.astype(np.float64) @ q.astype(np.float64)
    assert ix.best_inner_product(data, q, cand) == max(set(cand), key=lambda i: ips[i])
    assert ix.best_inner_product(data, q, cand, max_candidates=3) == max({4, 9}, key=lambda i: ips[i])
    assert ix.best_inner_product(data, q, []) == -1
    # ties go to the smaller id; and it is NOT the nearest vector in general
    data[9] = data[4]
    assert ix.best_inner_product(data, q, [9, 4]) == 4
    far = np.array([[10.0, 0.0], [0.9, 0.0]], np.float32)
    u = np.array([1.0, 0.0], np.float32)
    assert ix.best_inner_product(far, u, [0, 1]) == 0 and ix.nearest(far, u, [0, 1]) == 1
