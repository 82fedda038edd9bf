"""The synthetic input generators: determinism, structure, and the shapes the workloads name."""
import numpy as np

import qvgen


def rows_sorted_and_distinct(rowptr, col):
    d = np.diff(col.astype(np.int64))
    starts = rowptr[1:-1]
    starts = starts[(starts > 0) & (starts < len(col))]
    inner = np.ones(len(col) - 1, dtype=bool)
    inner[starts - 1] = False                       # pairs that straddle two rows
    return bool(np.all(d[inner] > 0))


def test_tiny_workload_shape(tiny_graph):
    w, rowptr, col = tiny_graph
    deg = np.diff(rowptr)
    assert len(rowptr) == 10_001 and abs(len(col) - 200_000) < 200
    assert deg.min() == 1 and deg.max() == 2_000
    assert col.min() >= 0 and col.max() < w.n
    assert rows_sorted_and_distinct(rowptr, col)
    assert rowptr.dtype == np.int32 and col.dtype == np.int32


def test_thread_count_does_not_change_the_graph(monkeypatch):
    w = qvgen.workload("co_purchase", scale=0.01)
    a = w.graph()
    monkeypatch.setattr(qvgen, "n_threads", lambda: 1)
    b = w.graph()
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_symmetrised_graph_is_symmetric():
    w = qvgen.workload("co_purchase", scale=0.005)
    rowptr, col = w.graph()
    assert rows_sorted_and_distinct(rowptr, col)
    src = np.repeat(np.arange(w.n), np.diff(rowptr))
    fwd = set(zip(src.tolist(), col.tolist()))
    assert all((b, a) in fwd for a, b in list(fwd)[:20000])
    assert abs(len(col) / w.n - 50) < 10


def test_citation_shape_has_in_degree_skew_and_int64_rowptr():
    w = qvgen.workload("citation", scale=0.002)
    rowptr, col = w.graph()
    assert rowptr.dtype == np.int64
    assert rows_sorted_and_distinct(rowptr, col)
    assert abs(len(col) / w.n - 14.4) < 1.0
    indeg = np.bincount(col, minlength=w.n)
    assert indeg.max() > 200 * indeg.mean()            # heavy head
    assert np.diff(rowptr).max() <= 4096


def test_features_host_rows_and_f16_rounding():
    full = qvgen.features_host(11, 300, 64, np.float32)
    ids = np.array([5, 299, 0, 5], dtype=np.int32)
    assert qvgen.feature_rows_host(11, ids, 64, np.float32).tobytes() == full[ids].tobytes()
    assert qvgen.features_host(11, 100, 64, np.float32, row_begin=200).tobytes() == full[200:].tobytes()
    assert abs(full.mean()) < 0.02 and abs(full.std() - 1) < 0.02
    half = qvgen.features_host(11, 300, 64, np.float16)
    assert half.tobytes() == full.astype(np.float16).tobytes()      # numpy rounds to nearest even


def test_seed_batches_and_popularity():
    n = 5000
    s0 = qvgen.seeds(3, n, 0, 256)
    assert np.array_equal(s0, qvgen.seeds(3, n, 0, 256)) and not np.array_equal(s0, qvgen.seeds(3, n, 1, 256))
    assert s0.min() >= 0 and s0.max() < n
    p0 = qvgen.seed_popularity(3, n)
    assert np.isclose(p0.sum(), 1.0) and p0.min() > 0
    drawn = np.concatenate([qvgen.seeds(3, n, b, 512, mode=1) for b in range(200)])
    top = np.argsort(-p0)[:50]
    emp = np.isin(drawn, top).mean()
    assert abs(emp - p0[top].sum()) < 0.02
    assert qvgen.batch_rng_seed(3, 0) != qvgen.batch_rng_seed(3, 1)
