"""CPU-side checks of the product's host logic (no GPU, no compute calls):
  * libqv.so loads and exports every symbol include/qv.h declares;
  * the a-priori bound arithmetic;
  * the rule the sampling kernel uses to run Floyd's selection for all slots of a node at once
    (pairwise-duplicate test + dependency on one earlier slot), emulated lane by lane in Python
    and compared with the sequential oracle, for one round of up to 64 slots and for the
    64-slots-at-a-time scheme used above a fanout of 64.
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


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only and says so instead of starting."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
