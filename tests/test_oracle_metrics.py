"""Pins for the oracle's PSGS, feature-access-probability and placement functions (CPU only).

What fixes them, other than themselves:
  * the paper's two worked examples (tests/golden/psgs_example.txt, fap_example.txt);
  * closed forms on regular graphs, stars and chains;
  * exhaustive enumeration of every sampling outcome with exact fractions on small graphs;
  * explicit dense matrix products A_1 .. A_k with numpy;
  * Monte-Carlo runs of the (separately pinned) sampler on an out-tree;
  * the identity  sum_i P[i] = sum_s p0[s] Q[s]  (accesses per request == expected sample size).
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from conftest import read_golden
from helpers import adjacency, brute_expected_tree, csr_from_edges, parse_edges, random_graph


def frac(tok):
    return Fraction(tok)


# ------------------------------------------------------------------------------------------------
def test_psgs_worked_example_from_paper():
    g = read_golden("psgs_example.txt")
    n = int(g["nodes"][0])
    rowptr, col = csr_from_edges(n, parse_edges(g["edges"]))
    fanouts = [int(x) for x in g["fanouts"]]
    v = int(g["node"][0])
    q = oracle.psgs_forward(rowptr, col, fanouts, v)
    assert [Fraction(x).limit_denominator(1000) for x in q] == [frac(t) for t in g["q"]]
    Q = oracle.psgs(rowptr, col, fanouts)
    assert Fraction(Q[v]).limit_denominator(1000) == frac(g["Q"][0])
    # the fanouts the sentence announces (2 then 1) do not give the printed numbers
    assert oracle.psgs(rowptr, col, [2, 1])[v] == 4.0


def test_fap_worked_example_from_paper():
    g = read_golden("fap_example.txt")
    n = int(g["nodes"][0])
    fanouts = [int(x) for x in g["fanouts"]]
    v = int(g["node"][0])
    rowptr, col = csr_from_edges(n, parse_edges(g["edges"]))
    P, layers = oracle.access_prob(rowptr, col, fanouts, layers=True)
    assert [Fraction(x).limit_denominator(1000) for x in layers[:, v]] == [frac(t) for t in g["p"]]
    assert Fraction(P[v]).limit_denominator(1000) == frac(g["P"][0])
    rowptr, col = csr_from_edges(n, parse_edges(g["selfloop_edges"]))
    _, layers = oracle.access_prob(rowptr, col, fanouts, layers=True)
    assert [Fraction(x).limit_denominator(1000) for x in layers[:, v]] == [frac(t) for t in g["selfloop_p"]]


# ------------------------------------------------------------------------------------------------
def circulant(n, d):
    return csr_from_edges(n, [(v, (v + j) % n) for v in range(n) for j in range(1, d + 1)])


@pytest.mark.parametrize("d,fanouts", [(4, [2, 3]), (3, [5, 1, 2]), (6, [6, 6]), (5, [1])])
def test_regular_graph_closed_forms(d, fanouts):
    n = 23
    rowptr, col = circulant(n, d)
    want, prod = 1.0, 1.0
    for l in fanouts:
        prod *= min(d, l)
        want += prod
    assert np.allclose(oracle.psgs(rowptr, col, fanouts), want, rtol=1e-14)
    assert np.allclose(oracle.access_prob(rowptr, col, fanouts), want / n, rtol=1e-13)


def test_star_and_chain_closed_forms():
    n = 9                                               # centre 0, leaves 1..9
    out_star = csr_from_edges(n + 1, [(0, i) for i in range(1, n + 1)])
    Q = oracle.psgs(*out_star, [4, 3])
    assert Q[0] == 1 + 4 and np.all(Q[1:] == 1)
    sym = csr_from_edges(n + 1, [(0, i) for i in range(1, n + 1)] + [(i, 0) for i in range(1, n + 1)])
    l = [4, 3, 2]
    m = [min(n, x) for x in l]
    Q = oracle.psgs(*sym, l)
    assert np.isclose(Q[0], 1 + m[0] + m[0] * 1 + m[0] * 1 * m[2])        # centre->leaves->centre->leaves
    assert np.allclose(Q[1:], 1 + 1 + m[1] + m[1] * 1)                    # leaf->centre->leaves->centre
    chain = csr_from_edges(6, [(i, i + 1) for i in range(5)])
    Q = oracle.psgs(*chain, [3, 3, 3])
    assert Q.tolist() == [4, 4, 4, 3, 2, 1]
    P = oracle.access_prob(*chain, [3, 3, 3])
    assert np.allclose(P * 6, [1, 2, 3, 4, 4, 4])


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("trial", range(8))
def test_exhaustive_enumeration_matches(trial):
    rng = np.random.default_rng(500 + trial)
    n = int(rng.integers(3, 8))
    rowptr, col = random_graph(rng, n, max_deg=min(5, n))
    fanouts = [int(rng.integers(1, 4)) for _ in range(int(rng.integers(1, 4)))]
    size, occ = brute_expected_tree(adjacency(rowptr, col), fanouts)
    Q = oracle.psgs(rowptr, col, fanouts)
    assert np.allclose(Q, [float(s) for s in size], rtol=1e-13)
    for v in range(n):                                   # printed order of the definition
        assert np.isclose(oracle.psgs_forward(rowptr, col, fanouts, v).sum(), float(size[v]), rtol=1e-13)
    p0 = rng.random(n)
    p0 /= p0.sum()
    for seed_dist in (None, p0):
        w = np.full(n, 1.0 / n) if seed_dist is None else seed_dist
        want = [sum(w[s] * float(occ[s][i]) for s in range(n)) for i in range(n)]
        assert np.allclose(oracle.access_prob(rowptr, col, fanouts, p0=seed_dist), want, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("trial", range(4))
def test_dense_matrix_products(trial):
    rng = np.random.default_rng(600 + trial)
    n = 40
    rowptr, col = random_graph(rng, n, max_deg=12)
    fanouts = [5, 3, 7][:int(rng.integers(1, 4))]
    deg = np.diff(rowptr)
    A = []
    for l in fanouts:
        M = np.zeros((n, n))
        for v in range(n):
            for u in col[rowptr[v]:rowptr[v + 1]]:
                M[v, u] += min(deg[v], l) / deg[v]
        A.append(M)
    delta = np.eye(n)
    Q = np.ones(n)
    p0 = np.full(n, 1.0 / n)
    P = p0.copy()
    for k, l in enumerate(fanouts):
        Q += delta @ np.minimum(deg, l)                  # q_k = sum_j delta_{k-1}(i,j) min(deg j, l_k)
        delta = delta @ A[k]
        P += p0 @ delta                                  # p_k = sum_j p0[j] delta_k(j,i)
    assert np.allclose(oracle.psgs(rowptr, col, fanouts), Q, rtol=1e-12)
    assert np.allclose(oracle.access_prob(rowptr, col, fanouts), P, rtol=1e-12)


def test_forward_and_backward_orders_agree_on_tiny_workload(tiny_graph):
    w, rowptr, col = tiny_graph
    for fanouts in (w.fanouts, [15, 10, 5]):
        Q = oracle.psgs(rowptr, col, fanouts)
        for v in np.random.default_rng(4).integers(0, w.n, size=25):
            assert np.isclose(oracle.psgs_forward(rowptr, col, fanouts, int(v)).sum(), Q[v], rtol=1e-12)


def test_access_counts_sum_to_expected_sample_size(tiny_graph):
    w, rowptr, col = tiny_graph
    rng = np.random.default_rng(5)
    p0 = rng.random(w.n) ** 3
    p0 /= p0.sum()
    for fanouts in (w.fanouts, [15, 10, 5], [1]):
        Q = oracle.psgs(rowptr, col, fanouts)
        assert np.isclose(oracle.access_prob(rowptr, col, fanouts).sum(), Q.mean(), rtol=1e-12)
        assert np.isclose(oracle.access_prob(rowptr, col, fanouts, p0=p0).sum(), (p0 * Q).sum(), rtol=1e-12)
        # plain 1/deg weights (the other way to read "weighted adjacency") lose this identity:
        # their PSGS still counts min(deg, l) per node but the FAP mass stays 1 per hop
        P1 = oracle.access_prob(rowptr, col, fanouts, weight_mode=1)
        assert P1.sum() <= len(fanouts) + 1 + 1e-9
        if fanouts != [1]:
            assert not np.isclose(P1.sum(), Q.mean(), rtol=1e-3)


def test_monte_carlo_on_an_out_tree():
    # every node has one parent, so sampled nodes never coincide and the number of sampled nodes
    # equals the tree-expansion size whose mean is Q
    rng = np.random.default_rng(6)
    edges, nxt, level = [], 1, [0]
    for depth in range(3):
        new = []
        for v in level:
            for _ in range(int(rng.integers(0, 7))):
                edges.append((v, nxt))
                new.append(nxt)
                nxt += 1
        level = new
    rowptr, col = csr_from_edges(nxt, edges)
    fanouts = [3, 2, 4]
    Q = oracle.psgs(rowptr, col, fanouts)
    P = oracle.access_prob(rowptr, col, fanouts, p0=np.eye(nxt)[0])
    trials = 4000
    sizes = np.zeros(trials)
    hits = np.zeros(nxt)
    for t in range(trials):
        o = oracle.sample(rowptr, col, np.array([0], np.int32), fanouts, 31337 + t)
        sizes[t] = len(o["n_id"])
        assert len(o["n_id"]) == 1 + o["edge_off"][-1]
        hits[o["n_id"]] += 1
    assert abs(sizes.mean() - Q[0]) < 5 * sizes.std() / np.sqrt(trials) + 1e-9
    se = np.sqrt(np.maximum(P * (1 - P), 1e-12) / trials)
    assert np.all(np.abs(hits / trials - P) < 5 * se + 1e-9)


def test_general_graph_unique_count_is_bounded_by_psgs(tiny_graph):
    w, rowptr, col = tiny_graph
    Q = oracle.psgs(rowptr, col, w.fanouts)
    tot_u = tot_q = tot_e = 0.0
    for b in range(30):
        seeds = w.seeds(b)
        o = oracle.sample(rowptr, col, seeds, w.fanouts, w.rng_seed(b))
        uniq_seeds = np.unique(seeds)
        tot_u += len(o["n_id"])
        tot_e += len(uniq_seeds) + o["edge_off"][-1]
        tot_q += Q[uniq_seeds].sum()
    assert tot_u <= tot_e
    # dedup between hops only removes work, so edges stay at or below the PSGS total; and on
    # this sparse workload they stay close to it
    assert tot_e <= tot_q * 1.02
    assert tot_e >= 0.8 * tot_q


# ------------------------------------------------------------------------------------------------
def test_placement_properties():
    rng = np.random.default_rng(7)
    prob = rng.random(1000).astype(np.float32)
    prob[rng.integers(0, 1000, 300)] = np.float32(0.25)               # many ties
    for n_hot in (0, 1, 137, 1000, 1500):
        rank, loc = oracle.place(prob, n_hot)
        assert sorted(rank.tolist()) == list(range(1000))
        key = [(-float(prob[i]), int(i)) for i in rank]
        assert key == sorted(key)                                      # desc prob, ties by id
        h = min(n_hot, 1000)
        hot_ids = rank[:h]
        assert np.array_equal(loc[hot_ids], np.arange(h))
        cold_ids = np.sort(rank[h:])
        assert np.array_equal(~loc[cold_ids], np.arange(1000 - h))
        if 0 < h < 1000:
            assert prob[hot_ids].min() >= prob[cold_ids].max()
