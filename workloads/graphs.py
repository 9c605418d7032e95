"""Seeded random graph generators (undirected, simple, no self-loops) returning a CSR pattern.

Self-written; no dataset and no third-party generator is used. The adjacency pattern that
comes out is the paper's binary matrix A (Section 3.1): rowptr[N+1], colidx[nnz] with the
columns of every row in ascending order and A symmetric.
"""
from __future__ import annotations

import numpy as np


def _pattern_from_edges(n: int, src: np.ndarray, dst: np.ndarray):
    """Symmetrise an edge list, drop duplicates and self-loops, build the CSR pattern."""
    keep = src != dst
    src, dst = src[keep], dst[keep]
    a = np.concatenate([src, dst]).astype(np.int64)
    b = np.concatenate([dst, src]).astype(np.int64)
    key = np.unique(a * n + b)                 # sorted => rows ascending, columns ascending
    rows = (key // n).astype(np.int64)
    cols = (key % n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr).astype(np.int32)
    return rowptr, cols


def erdos_renyi(n: int, avg_degree: float, rng: np.random.Generator):
    """G(n, p) with p = avg_degree / (n - 1)."""
    total = n * (n - 1) // 2
    p = avg_degree / (n - 1)
    m = int(rng.binomial(total, p))
    # draw m distinct unordered pairs: oversample linear pair ids, dedupe, trim
    ids = np.unique(rng.integers(0, total, size=int(m * 1.2) + 16))
    while ids.size < m:
        ids = np.unique(np.concatenate([ids, rng.integers(0, total, size=m)]))
    ids = rng.permutation(ids)[:m]
    # decode pair id -> (i, j), i < j, rows enumerated i = 0..n-2 with n-1-i entries each
    i = (n - 2 - np.floor(np.sqrt(-8.0 * ids + 4.0 * n * (n - 1) - 7) / 2.0 - 0.5)).astype(np.int64)
    j = (ids + i + 1 - n * (n - 1) // 2 + (n - i) * ((n - i) - 1) // 2).astype(np.int64)
    return _pattern_from_edges(n, i, j)


def preferential_attachment(n: int, m_cycle, rng: np.random.Generator):
    """Barabasi-Albert style growth: node v attaches to m distinct earlier nodes chosen with
    probability proportional to degree; m cycles through `m_cycle` (e.g. (3,) or (3, 4))."""
    m_cycle = tuple(int(x) for x in m_cycle)
    m0 = max(m_cycle) + 1
    src, dst = [], []
    # seed clique on m0 nodes
    for a in range(m0):
        for b in range(a + 1, m0):
            src.append(a)
            dst.append(b)
    cap = 2 * (len(src) + sum(m_cycle) * ((n - m0) // len(m_cycle) + 1))
    ends = np.empty(cap, dtype=np.int64)       # every edge endpoint once: degree-proportional urn
    k = 0
    for a, b in zip(src, dst):
        ends[k] = a
        ends[k + 1] = b
        k += 2
    draws_per_node = 4 * max(m_cycle)
    u = rng.random((n, draws_per_node))
    e_src = np.empty(cap // 2, dtype=np.int64)
    e_dst = np.empty(cap // 2, dtype=np.int64)
    ne = len(src)
    e_src[:ne] = src
    e_dst[:ne] = dst
    for v in range(m0, n):
        m = m_cycle[(v - m0) % len(m_cycle)]
        chosen = []
        for t in range(draws_per_node):
            c = int(ends[int(u[v, t] * k)])
            if c not in chosen:
                chosen.append(c)
                if len(chosen) == m:
                    break
        c = 0
        while len(chosen) < m:                  # practically unreachable; keeps the degree exact
            if c not in chosen:
                chosen.append(c)
            c += 1
        for c in chosen:
            e_src[ne] = v
            e_dst[ne] = c
            ne += 1
            ends[k] = v
            ends[k + 1] = c
            k += 2
    return _pattern_from_edges(n, e_src[:ne], e_dst[:ne])


def make_graph(kind: str, n: int, param, rng: np.random.Generator):
    if kind == "er":
        return erdos_renyi(n, float(param[0]), rng)
    if kind == "pa":
        return preferential_attachment(n, param, rng)
    raise ValueError(f"unknown graph family {kind!r}")
