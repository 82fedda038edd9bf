"""CPU-side checks of the product's host logic (no GPU, no compute calls):
  * libqv.so loads and exports every symbol include/qv.h declares;
  * the a-priori bound arithmetic;
  * the rule the sampling kernel uses to run Floyd's selection for all slots of a node at once
    (pairwise-duplicate test + dependency on one earlier slot), emulated lane by lane in Python
    and compared with the sequential oracle, for one round of up to 64 slots and for the
    64-slots-at-a-time scheme used above a fanout of 64;
  * the way the sampling kernel deals a frontier over its groups of lanes (every round gives each
    group the same number of consecutive entries, what is left divided by the groups, at most 8),
    emulated index by index: every entry is taken exactly once, whatever the sizes;
  * how the blocked gather of the access probabilities cuts a long row into work items (emulated from the
    cut points): the items tile the row, stay inside one block of sources and hold at most 256 edges.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2305_10863_amd as qv
    if not os.path.exists(qv.LIB_PATH):
        pytest.skip("libqv.so not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(qv.LIB_PATH)
    names = declared_symbols()
    assert len(names) >= 18
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(qv.EXPORTS) == names


def test_bounds_arithmetic_without_gpu():
    import paper_2305_10863_amd as qv
    if not os.path.exists(qv.LIB_PATH):
        pytest.skip("libqv.so not built")
    assert qv.qv_sample_bounds(1024, [15, 10, 5], 111_000_000) == (1024 * (1 + 15 + 150 + 750), 1024 * (15 + 150 + 750),
                                                                  1024 * (1 + 15 + 150 + 750))
    assert qv.qv_sample_bounds(64, [10, 5], 100) == (100, 64 * 10 + 100 * 5, 64 + 100 + 100)
    assert qv.qv_sample_bounds(64, [10, 5], 100) == oracle.sample_bounds(64, [10, 5], 100)
    with pytest.raises(qv.QvError):
        qv.qv_sample_bounds(8, [0], 100)
    with pytest.raises(qv.QvError):
        qv.qv_sample_bounds(8, [2] * 9, 100)


# ------------------------------------------------------------------------------------------------
def resolve_round(t, base, first_slot, n_active, pre):
    """Lane-by-lane emulation of one round: lanes 0..n_active-1 hold draws t[.]; `pre[i]` says the
    draw already equals a pick of an earlier round.  Returns the picks of this round."""
    dup = list(pre)
    for r in range(n_active - 1):
        for sub in range(n_active):
            if r < sub and t[r] == t[sub]:
                dup[sub] = True
    dep = [-1] * n_active
    for sub in range(n_active):
        s = first_slot + sub
        if not dup[sub] and t[sub] >= base:
            r = t[sub] - base
            if first_slot <= r < s:
                dep[sub] = r - first_slot
    known = [dup[i] or dep[i] < 0 for i in range(n_active)]
    coll = [dup[i] for i in range(n_active)]
    rounds = 0
    while not all(known):
        snap_k, snap_c = list(known), list(coll)        # all lanes shuffle before any lane updates
        for i in range(n_active):
            if not known[i] and snap_k[dep[i]]:
                coll[i], known[i] = snap_c[dep[i]], True
        rounds += 1
        assert rounds <= n_active
    return [base + first_slot + i if coll[i] else t[i] for i in range(n_active)]


def parallel_positions(seed, node, hop, deg, fanout):
    if deg <= fanout:
        return list(range(deg))
    base = deg - fanout
    picks = []
    for c0 in range(0, fanout, 64):
        n_active = min(64, fanout - c0)
        t = [oracle.rand_below(seed, node, hop, c0 + i, base + c0 + i + 1) for i in range(n_active)]
        pre = [t[i] in picks for i in range(n_active)]
        picks += resolve_round(t, base, c0, n_active, pre)
    return picks


def test_all_slots_at_once_rule_equals_sequential_floyd():
    rng = np.random.default_rng(11)
    cases = []
    for _ in range(1500):
        fanout = int(rng.integers(1, 65))
        deg = fanout + int(rng.integers(1, 4 if rng.random() < 0.5 else 200))     # many tight cases
        cases.append((deg, fanout))
    for _ in range(150):
        fanout = int(rng.integers(65, 400))
        deg = fanout + int(rng.integers(1, 6 if rng.random() < 0.6 else 3000))
        cases.append((deg, fanout))
    chains = 0
    for i, (deg, fanout) in enumerate(cases):
        seed, node, hop = 900 + i, int(rng.integers(0, 10 ** 6)), int(rng.integers(1, 4))
        want = oracle.sample_positions(seed, node, hop, deg, fanout).tolist()
        got = parallel_positions(seed, node, hop, deg, fanout)
        assert got == want, (deg, fanout, seed)
        chains += sum(1 for s, p in enumerate(want) if p == deg - fanout + s)
    assert chains > 500            # the collision path was exercised, not just the easy one


def test_sampling_rounds_cover_every_frontier_entry_once():
    # k_sample: group g of n_groups takes, in a round that starts at `done`, the S entries from
    # done + g * S on, with S = min(8, ceil(left / n_groups)); lane `sub` of the group loads entry sub < S
    rng = np.random.default_rng(5)
    cases = [(0, 16), (1, 16), (7, 1), (1024, 8 * 16), (1024, 64 * 16), (32_391, 64 * 32), (12_345, 60 * 16), (100_000, 8)]
    cases += [(int(rng.integers(0, 50_000)), int(rng.integers(1, 3000))) for _ in range(30)]
    for F, n_groups in cases:
        taken = np.zeros(F, dtype=np.int32)
        done, rounds = 0, 0
        while done < F:
            left = F - done
            S = 8 if left >= n_groups * 8 else -(-left // n_groups)
            assert 1 <= S <= 8
            g = np.arange(n_groups)[:, None]
            f = done + g * S + np.arange(S)[None, :]
            np.add.at(taken, f[f < F], 1)
            done += n_groups * S
            rounds += 1
        assert (taken == 1).all(), (F, n_groups)
        # no round leaves more than one entry per group unused: the last one is spread over the whole grid
        assert rounds <= -(-F // (n_groups * 8)) + 1 if F else rounds == 0


def test_long_row_work_items_tile_the_row():
    # the in-edge CSR's long rows: cut points where the (ascending) sources pass from one block of 2^L ids to
    # the next, then items of at most 256 edges, listed block by block
    rng = np.random.default_rng(6)
    L, n = 6, 5000
    blocks = -(-n // (1 << L))
    rows = [np.sort(rng.integers(0, n, 9000)),                       # parallel edges allowed
            np.sort(rng.choice(n, size=4321, replace=False)), np.sort(rng.choice(n, size=300, replace=False))]
    starts = np.concatenate([[0], np.cumsum([len(r) for r in rows])])
    col = np.concatenate(rows)
    items = []                                                       # (block, row, first, count)
    for b in range(blocks):
        for k, r in enumerate(rows):
            e0 = starts[k] + np.searchsorted(r, b << L, side="left")
            e1 = starts[k] + np.searchsorted(r, (b + 1) << L, side="left")
            e = e0
            while e < e1:
                items.append((b, k, e, min(256, e1 - e)))
                e += 256
    for k in range(len(rows)):
        mine = sorted((first, cnt) for b, kk, first, cnt in items if kk == k)
        assert mine[0][0] == starts[k] and mine[-1][0] + mine[-1][1] == starts[k + 1]
        assert all(a[0] + a[1] == b2[0] for a, b2 in zip(mine, mine[1:]))
    for b, k, first, cnt in items:
        assert 1 <= cnt <= 256
        assert (col[first:first + cnt] >> L == b).all()
    assert [it[0] for it in items] == sorted(it[0] for it in items)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only and says so instead of starting."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
