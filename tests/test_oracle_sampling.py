"""Pins for the oracle's sampler, reindex and gather (CPU only).

What fixes the oracle here, other than itself:
  * Philox4x32-10: the published known-answer vectors (tests/golden/philox4x32_10_kat.txt).
  * rand_below: Python big-integer arithmetic on the pinned generator's output.
  * selection: the law it must follow -- every size-l subset equally likely (chi-square over many
    seeds), true neighbours only, no position twice, everything taken when deg <= fanout -- and an
    independently structured Python re-derivation (sets, rescans) on small graphs.
  * gather: numpy fancy indexing / memcpy.
"""
import math
from itertools import combinations

import numpy as np
import pytest

import oracle
from conftest import read_golden
from helpers import adjacency, random_graph


# ------------------------------------------------------------------------------------------------
def test_philox_known_answers():
    rows = 0
    with open(__import__("os").path.join(__import__("conftest").GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            out = oracle.philox4x32_10(w[0:4], w[4:6])
            assert [int(x) for x in out] == w[6:10]
            rows += 1
    assert rows == 3


def test_rand_below_is_high_half_of_product():
    rng = np.random.default_rng(1)
    for _ in range(200):
        seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        node, hop, slot = int(rng.integers(0, 2 ** 31)), int(rng.integers(1, 9)), int(rng.integers(0, 4096))
        bound = int(rng.integers(1, 2 ** 62))
        x = oracle.philox4x32_10([node, hop, slot, 0], [seed & 0xFFFFFFFF, seed >> 32])
        r64 = (int(x[1]) << 32) | int(x[0])
        assert oracle.rand_below(seed, node, hop, slot, bound) == (r64 * bound) >> 64
    assert oracle.rand_below(123, 4, 1, 0, 1) == 0          # a bound of 1 leaves one outcome


def test_counter_words_are_not_interchangeable():
    # node / hop / slot each move the stream: a swapped or dropped counter word would collide
    base = oracle.rand_below(99, 5, 2, 3, 2 ** 40)
    assert len({base, oracle.rand_below(99, 2, 5, 3, 2 ** 40), oracle.rand_below(99, 5, 3, 2, 2 ** 40),
                oracle.rand_below(99, 3, 2, 5, 2 ** 40), oracle.rand_below(98, 5, 2, 3, 2 ** 40)}) == 5


# ------------------------------------------------------------------------------------------------
def py_positions(seed, node, hop, deg, fanout):
    """Floyd's selection with a Python set, structured independently of the oracle."""
    if deg <= fanout:
        return list(range(deg))
    chosen, order = set(), []
    for s, j in enumerate(range(deg - fanout, deg)):
        t = oracle.rand_below(seed, node, hop, s, j + 1)
        pick = j if t in chosen else t
        assert pick not in chosen
        chosen.add(pick)
        order.append(pick)
    return order


def test_positions_match_independent_floyd_and_invariants():
    rng = np.random.default_rng(2)
    for _ in range(400):
        deg = int(rng.integers(0, 200))
        fanout = int(rng.integers(1, 80))
        seed = int(rng.integers(0, 2 ** 62))
        node, hop = int(rng.integers(0, 10 ** 6)), int(rng.integers(1, 5))
        pos = oracle.sample_positions(seed, node, hop, deg, fanout).tolist()
        assert len(pos) == min(deg, fanout)
        assert len(set(pos)) == len(pos)
        assert all(0 <= p < deg for p in pos)
        if deg <= fanout:
            assert pos == list(range(deg))
        assert pos == py_positions(seed, node, hop, deg, fanout)


@pytest.mark.parametrize("deg,fanout", [(5, 3), (7, 2), (6, 5), (4, 1)])
def test_selection_is_uniform_over_subsets(deg, fanout):
    n_trials = 40000
    counts = {c: 0 for c in combinations(range(deg), fanout)}
    first_slot = np.zeros(deg, dtype=np.int64)
    for s in range(n_trials):
        pos = oracle.sample_positions(1000 + s, 17, 1, deg, fanout)
        counts[tuple(sorted(pos.tolist()))] += 1
        first_slot[pos[0]] += 1
    exp = n_trials / len(counts)
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    dof = len(counts) - 1
    # chi-square upper bound at ~5 sigma (Wilson-Hilferty would be tighter; this is ample)
    assert chi2 < dof + 5 * math.sqrt(2 * dof) + 10, (chi2, dof)
    # each position is included with probability fanout/deg
    incl = np.zeros(deg)
    for c, k in counts.items():
        for p in c:
            incl[p] += k
    assert np.allclose(incl / n_trials, fanout / deg, atol=5 * math.sqrt(0.25 / n_trials))


def test_uniform_also_across_nodes_hops_with_fixed_seed():
    # the stream must decorrelate over node and hop too, not only over the seed
    deg, fanout = 6, 2
    counts = {c: 0 for c in combinations(range(deg), fanout)}
    n = 0
    for node in range(3000):
        for hop in (1, 2, 3):
            counts[tuple(sorted(oracle.sample_positions(7, node, hop, deg, fanout).tolist()))] += 1
            n += 1
    exp = n / len(counts)
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    dof = len(counts) - 1
    assert chi2 < dof + 5 * math.sqrt(2 * dof) + 10


# ------------------------------------------------------------------------------------------------
def py_multi_hop(adj, seeds, fanouts, rng_seed, cumulative=False):
    """Multi-hop sampling + relabel written differently from the oracle: per-hop lists, dedup by
    rescanning lists with `in` / index(), no hash map carried between the steps."""
    n_id = []
    for s in seeds:
        if s not in n_id:
            n_id.append(s)
    frontiers = [list(n_id)]
    edges = []          # (hop, target_global, nbr_global)
    for k, l in enumerate(fanouts, start=1):
        hop_nbrs = []
        for v in (list(n_id) if cumulative else frontiers[-1]):
            for p in py_positions(rng_seed, v, k, len(adj[v]), l):
                hop_nbrs.append((v, adj[v][p]))
        nxt = []
        for _, g in hop_nbrs:
            if g not in nxt:
                nxt.append(g)
        for g in nxt:           # first appearance order within the hop == order of nxt
            if g not in n_id:
                n_id.append(g)
        edges += [(k, v, g) for v, g in hop_nbrs]
        frontiers.append(nxt)
    return n_id, frontiers, edges


@pytest.mark.parametrize("trial", range(12))
def test_multi_hop_matches_independent_python(trial):
    rng = np.random.default_rng(100 + trial)
    n = int(rng.integers(5, 40))
    rowptr, col = random_graph(rng, n, max_deg=int(rng.integers(1, 9)))
    adj = adjacency(rowptr, col)
    K = int(rng.integers(1, 4))
    fanouts = [int(rng.integers(1, 6)) for _ in range(K)]
    seeds = rng.integers(0, n, size=int(rng.integers(1, 10))).astype(np.int32)   # repeats likely
    rs = int(rng.integers(0, 2 ** 62))
    o = oracle.sample(rowptr, col, seeds, fanouts, rs)
    n_id, frontiers, edges = py_multi_hop(adj, seeds.tolist(), fanouts, rs)
    assert o["n_id"].tolist() == n_id
    assert o["frontier"].tolist() == [g for f in frontiers for g in f]
    assert o["frontier_off"].tolist() == np.cumsum([0] + [len(f) for f in frontiers]).tolist()
    assert o["nbr_global"].tolist() == [g for _, _, g in edges]
    assert [n_id[i] for i in o["row_local"]] == [v for _, v, _ in edges]
    assert [n_id[i] for i in o["col_local"]] == [g for _, _, g in edges]
    per_hop = [sum(1 for e in edges if e[0] == k) for k in range(1, K + 1)]
    assert o["edge_off"].tolist() == np.cumsum([0] + per_hop).tolist()


@pytest.mark.parametrize("trial", range(8))
def test_cumulative_mode_matches_independent_python(trial):
    # every node sampled so far is expanded again in each hop (nested blocks)
    rng = np.random.default_rng(700 + trial)
    n = int(rng.integers(5, 40))
    rowptr, col = random_graph(rng, n, max_deg=int(rng.integers(1, 9)))
    adj = adjacency(rowptr, col)
    fanouts = [int(rng.integers(1, 5)) for _ in range(int(rng.integers(1, 4)))]
    seeds = rng.integers(0, n, size=int(rng.integers(1, 8))).astype(np.int32)
    rs = int(rng.integers(0, 2 ** 62))
    o = oracle.sample(rowptr, col, seeds, fanouts, rs, cumulative=True)
    n_id, frontiers, edges = py_multi_hop(adj, seeds.tolist(), fanouts, rs, cumulative=True)
    assert o["n_id"].tolist() == n_id
    assert o["frontier"].tolist() == [g for f in frontiers for g in f]
    assert o["nbr_global"].tolist() == [g for _, _, g in edges]
    assert [n_id[i] for i in o["row_local"]] == [v for _, v, _ in edges]
    assert [n_id[i] for i in o["col_local"]] == [g for _, _, g in edges]
    # hop k expands exactly the first node_off[k] local ids, in order, each with its full segment
    deg = np.diff(rowptr)
    for k in range(1, len(fanouts) + 1):
        expanded = o["n_id"][:o["node_off"][k]]
        m = np.minimum(deg[expanded], fanouts[k - 1])
        rows = o["row_local"][o["edge_off"][k - 1]:o["edge_off"][k]]
        assert np.array_equal(rows, np.repeat(np.arange(len(expanded)), m))
    # with one hop the two modes coincide
    a = oracle.sample(rowptr, col, seeds, fanouts[:1], rs, cumulative=True)
    b = oracle.sample(rowptr, col, seeds, fanouts[:1], rs)
    assert all(np.array_equal(a[k], b[k]) for k in a)


def check_sample_invariants(rowptr, col, seeds, fanouts, o):
    adj_sets = None
    n_id = o["n_id"]
    K = len(fanouts)
    assert len(set(n_id.tolist())) == len(n_id)                       # no duplicates
    uniq_seeds = list(dict.fromkeys(seeds.tolist()))
    assert n_id[:len(uniq_seeds)].tolist() == uniq_seeds              # seeds first, in order
    assert o["node_off"][1] == len(uniq_seeds)
    assert np.array_equal(n_id[o["col_local"]], o["nbr_global"])
    fo, eo = o["frontier_off"], o["edge_off"]
    for k in range(1, K + 1):
        F_prev = o["frontier"][fo[k - 1]:fo[k]]
        F_k = o["frontier"][fo[k]:fo[k + 1]]
        tgt = n_id[o["row_local"][eo[k - 1]:eo[k]]]
        nbr = o["nbr_global"][eo[k - 1]:eo[k]]
        deg = (rowptr[F_prev.astype(np.int64) + 1] - rowptr[F_prev]).astype(np.int64)
        m = np.minimum(deg, fanouts[k - 1])
        assert np.array_equal(tgt, np.repeat(F_prev, m))              # segment sizes and order
        assert len(set(F_k.tolist())) == len(F_k)
        assert set(F_k.tolist()) == set(nbr.tolist())
        start = 0
        for v, mv, d in zip(F_prev.tolist(), m.tolist(), deg.tolist()):
            seg = nbr[start:start + mv].tolist()
            row = col[rowptr[v]:rowptr[v + 1]].tolist()
            if d <= fanouts[k - 1]:
                assert seg == row                                      # everything taken, CSR order
            else:
                assert all(g in row for g in seg)                      # true neighbours
                assert len(set(seg)) == len(seg)                       # rows hold distinct ids here
            start += mv
    assert o["node_off"][K + 1] == len(n_id)
    return adj_sets


def test_invariants_on_tiny_workload(tiny_graph):
    w, rowptr, col = tiny_graph
    for b in range(4):
        seeds = w.seeds(b)
        o = oracle.sample(rowptr, col, seeds, w.fanouts, w.rng_seed(b))
        check_sample_invariants(rowptr, col, seeds, w.fanouts, o)
        assert o["edge_off"][-1] > 200


def test_sample_hop_and_reindex_compose_to_sample(tiny_graph):
    w, rowptr, col = tiny_graph
    seeds = w.seeds(7)
    rs = w.rng_seed(7)
    o = oracle.sample(rowptr, col, seeds, w.fanouts, rs)
    n_id, local0, F = oracle.reindex(np.zeros(0, np.int32), seeds)
    assert np.array_equal(F, n_id)
    rows, cols = [], []
    for k, l in enumerate(w.fanouts, start=1):
        nbr, off = oracle.sample_hop(rowptr, col, F, l, rs, k)
        lut = {g: i for i, g in enumerate(n_id.tolist())}
        rows.append(np.repeat(np.array([lut[g] for g in F.tolist()], dtype=np.int32), np.diff(off)))
        n_id, local, F = oracle.reindex(n_id, nbr)
        cols.append(local)
    assert np.array_equal(n_id, o["n_id"])
    assert np.array_equal(np.concatenate(rows), o["row_local"])
    assert np.array_equal(np.concatenate(cols), o["col_local"])


def test_reindex_rejects_repeated_known_ids_and_handles_empty():
    with pytest.raises(ValueError):
        oracle.reindex(np.array([3, 3], np.int32), np.array([1], np.int32))
    n_id, local, F = oracle.reindex(np.array([5, 2], np.int32), np.zeros(0, np.int32))
    assert n_id.tolist() == [5, 2] and len(local) == 0 and len(F) == 0
    n_id, local, F = oracle.reindex(np.array([5, 2], np.int32), np.array([2, 9, 2, 5, 9, 1], np.int32))
    assert n_id.tolist() == [5, 2, 9, 1]
    assert local.tolist() == [1, 2, 1, 0, 2, 3]
    assert F.tolist() == [2, 9, 5, 1]


def test_degenerate_inputs():
    rowptr = np.array([0, 0, 2, 2], dtype=np.int64)          # node 0 and 2 are sinks
    col = np.array([0, 2], dtype=np.int32)
    o = oracle.sample(rowptr, col, np.array([0, 0, 2], np.int32), [3, 3], 5)
    assert o["n_id"].tolist() == [0, 2] and o["edge_off"].tolist() == [0, 0, 0]
    o = oracle.sample(rowptr, col, np.array([1], np.int32), [1, 4], 5)
    assert o["edge_off"][1] == 1 and o["edge_off"][2] == 1     # hop 2 expands a sink
    o = oracle.sample(rowptr, col, np.zeros(0, np.int32), [2], 5)
    assert len(o["n_id"]) == 0 and o["edge_off"].tolist() == [0, 0]
    with pytest.raises(ValueError):
        oracle.sample(rowptr, col, np.array([3], np.int32), [2], 5)


# ------------------------------------------------------------------------------------------------
def test_gather_is_plain_row_indexing():
    rng = np.random.default_rng(3)
    for dtype, dim in ((np.float32, 64), (np.float16, 128), (np.float32, 301), (np.float16, 7)):
        table = rng.standard_normal((500, dim)).astype(dtype)
        ids = rng.integers(0, 500, size=1200).astype(np.int32)       # repeats, any order
        out = oracle.gather(table, ids)
        assert out.tobytes() == table[ids].tobytes()
        ident = oracle.gather(table, np.arange(500, dtype=np.int32))
        assert ident.tobytes() == table.tobytes()
    assert oracle.gather(table, np.zeros(0, np.int32)).shape == (0, dim)
    with pytest.raises(ValueError):
        oracle.gather(table, np.array([500], np.int32))
