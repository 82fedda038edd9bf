"""Small helpers for tests: CSR from edge lists, random small graphs, exact brute-force
enumerations (fractions) of the sampling process.  Nothing here is used by the product."""
from fractions import Fraction
from functools import lru_cache
from itertools import combinations

import numpy as np


def csr_from_edges(n, edges):
    """edges: iterable of (src, dst), kept in the given order within each row."""
    rows = [[] for _ in range(n)]
    for s, d in edges:
        rows[s].append(d)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    for v in range(n):
        rowptr[v + 1] = rowptr[v] + len(rows[v])
    col = np.array([d for r in rows for d in r], dtype=np.int32)
    return rowptr, col


def parse_edges(tokens):
    return [tuple(int(x) for x in t.split(">")) for t in tokens]


def random_graph(rng, n, max_deg, allow_self=True):
    edges = []
    for v in range(n):
        d = int(rng.integers(0, max_deg + 1))
        cand = [u for u in range(n) if allow_self or u != v]
        d = min(d, len(cand))
        for u in rng.choice(cand, size=d, replace=False):
            edges.append((v, int(u)))
    return csr_from_edges(n, edges)


def adjacency(rowptr, col):
    return [list(map(int, col[rowptr[v]:rowptr[v + 1]])) for v in range(len(rowptr) - 1)]


def brute_expected_tree(adj, fanouts):
    """Exhaustive enumeration of uniform without-replacement neighbour sampling.

    Returns (size, occ): size[v] = expected number of nodes (with multiplicity) in the sampled
    tree rooted at v, the root included; occ[v][i] = expected number of times node i appears in
    that tree.  Every min(deg, l)-subset of every adjacency list is enumerated explicitly.
    """
    n, K = len(adj), len(fanouts)

    @lru_cache(maxsize=None)
    def below(v, k):
        """(expected #nodes, expected occurrence vector) strictly below v, v sitting at hop k."""
        zero = (Fraction(0), tuple([Fraction(0)] * n))
        if k == K or not adj[v]:
            return zero
        m = min(len(adj[v]), fanouts[k])
        tot, occ, cnt = Fraction(0), [Fraction(0)] * n, 0
        for subset in combinations(range(len(adj[v])), m):
            cnt += 1
            for j in subset:
                u = adj[v][j]
                s_u, o_u = below(u, k + 1)
                tot += 1 + s_u
                occ[u] += 1
                for i in range(n):
                    occ[i] += o_u[i]
        return tot / cnt, tuple(o / cnt for o in occ)

    size, occ = [], []
    for v in range(n):
        s, o = below(v, 0)
        o = list(o)
        o[v] += 1
        size.append(1 + s)
        occ.append(o)
    return size, occ
