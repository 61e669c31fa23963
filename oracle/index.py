"""CPU oracle for the LSH index of Sec. 3.2: L hash tables of <key, id> pairs, and the lookup
of a query's L buckets.

TEST INFRASTRUCTURE, not the product.  Plain Python dictionaries, one per table:

  build:  table l maps the key H_l(v) to the ids of all vectors v with that key (Sec. 3.2,
          "adding the 2-tuple <H(v), id of v> into the corresponding bucket"), ids ascending.
  probe:  for a query with keys H_1(u), ..., H_L(u): the bucket of each table, and their
          concatenation in table order (the "combined set of candidates"; the same id may
          come from several tables).
  exact processing of the candidates (Sec. 3.2, last paragraph): every distinct candidate is
          evaluated and the nearest one returned.
"""
import numpy as np


def build(keys):
    """keys: uint64 [N][L].  Returns a list of L dicts key -> list of ids (ascending)."""
    keys = np.asarray(keys, np.uint64)
    N, L = keys.shape
    tables = []
    for l in range(L):
        table = {}
        for i in range(N):
            table.setdefault(int(keys[i, l]), []).append(i)
        tables.append(table)
    return tables


def probe(tables, qkeys):
    """qkeys: uint64 [Q][L].  Returns buckets[q][l] = list of ids whose key in table l equals
    the query's."""
    qkeys = np.asarray(qkeys, np.uint64)
    return [[tables[l].get(int(qkeys[q, l]), []) for l in range(len(tables))] for q in range(qkeys.shape[0])]


def candidates(buckets_of_query):
    """The combined candidates of one query: its L buckets one after the other."""
    return [i for bucket in buckets_of_query for i in bucket]


def nearest(data, query, cand, max_candidates=0):
    """Processing of the candidates: the distinct candidate nearest to the query in l2 (ties:
    the smaller id), or -1 when there is none.  Distances in fp64.  max_candidates = 0: all of
    them (the exact version); otherwise only the first max_candidates entries of the combined
    list (the approximate version evaluates no more than 3L points)."""
    if max_candidates:
        cand = cand[:max_candidates]
    best, best_d = -1, np.inf
    for i in sorted(set(cand)):
        d = float(((data[i].astype(np.float64) - query.astype(np.float64)) ** 2).sum())
        if d < best_d:
            best, best_d = i, d
    return best


def best_inner_product(data, query, cand, max_candidates=0):
    """Processing of the candidates for maximum inner product search (the appendix on maximum
    inner product search ranks the transformed vectors by distance, which is the order of the
    inner products v . u): the distinct candidate with the largest inner product with the query
    (ties: the smaller id), or -1 when there is none.  fp64."""
    if max_candidates:
        cand = cand[:max_candidates]
    best, best_ip = -1, -np.inf
    for i in sorted(set(cand)):
        ip = float((data[i].astype(np.float64) * query.astype(np.float64)).sum())
        if ip > best_ip:
            best, best_ip = i, ip
    return best
