"""ctypes binding of the CPU oracle (oracle/qv_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's cpu_baseline
leg.  The product package never imports this module and shares no code with it.

All functions take and return numpy arrays.  `rowptr` may be int32 or int64 (widened here);
`col`, ids and fanouts are int32.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qv_oracle.cpp")
_SO = os.path.join(_HERE, "libqv_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with g++ (single-threaded, no HIP headers)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-Wall",
                               "-o", _SO, _SRC])
    return _SO


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def lib():
    global _lib
    if _lib is None:
        # QV_ORACLE_LIB: load this build of the oracle instead (tests/test_oracle_mutations.py points
        # it at deliberately broken builds to check that the pins notice)
        override = os.environ.get("QV_ORACLE_LIB")
        if override:
            _lib = C.CDLL(override)
        else:
            build()
            _lib = C.CDLL(_SO)
        _lib.o_rand_below.restype = C.c_uint64
        _lib.o_rand_below.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.o_sample_positions.restype = C.c_int64
        _lib.o_sample_hop.restype = C.c_int64
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().o_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def rand_below(seed, node, hop, slot, bound):
    return int(lib().o_rand_below(seed, node, hop, slot, bound))


def sample_positions(seed, node, hop, deg, fanout):
    out = np.zeros(max(1, min(deg, fanout)), dtype=np.int64)
    m = lib().o_sample_positions(C.c_uint64(seed), C.c_int32(node), C.c_int32(hop),
                                 C.c_int64(deg), C.c_int32(fanout), _p(out, C.c_int64))
    return out[:m]


def sample_hop(rowptr, col, frontier, fanout, seed, hop):
    """-> (nbr int32[total], off int64[F+1])"""
    rowptr, col, frontier = _i64(rowptr), _i32(col), _i32(frontier)
    n = len(rowptr) - 1
    F = len(frontier)
    off = np.zeros(F + 1, dtype=np.int64)
    nbr = np.zeros(max(1, F * fanout), dtype=np.int32)
    tot = lib().o_sample_hop(C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                             _p(frontier, C.c_int32), C.c_int64(F), C.c_int32(fanout),
                             C.c_uint64(seed), C.c_int32(hop), _p(nbr, C.c_int32),
                             _p(off, C.c_int64))
    if tot < 0:
        raise ValueError("frontier id out of range")
    return nbr[:tot].copy(), off


def reindex(known, nbr):
    """-> (n_id, local, frontier)"""
    known, nbr = _i32(known), _i32(nbr)
    n_id = np.zeros(max(1, len(known) + len(nbr)), dtype=np.int32)
    local = np.zeros(max(1, len(nbr)), dtype=np.int32)
    front = np.zeros(max(1, len(nbr)), dtype=np.int32)
    n1, n2 = C.c_int64(0), C.c_int64(0)
    rc = lib().o_reindex(_p(known, C.c_int32), C.c_int64(len(known)), _p(nbr, C.c_int32),
                         C.c_int64(len(nbr)), _p(n_id, C.c_int32), C.byref(n1),
                         _p(local, C.c_int32), _p(front, C.c_int32), C.byref(n2))
    if rc != 0:
        raise ValueError("known ids are not distinct")
    return n_id[:n1.value].copy(), local[:len(nbr)].copy(), front[:n2.value].copy()


def sample_bounds(n_seeds, fanouts, n_nodes, cumulative=False):
    """A-priori output sizes: (nodes, edges, frontier entries)."""
    f, nodes, edges, front = n_seeds, n_seeds, 0, n_seeds
    for l in fanouts:
        e = f * int(l)
        edges += e
        front += min(e, n_nodes)
        nodes = min(nodes + e, n_nodes)
        f = nodes if cumulative else min(e, n_nodes)
    return min(nodes, n_nodes), edges, front


def sample(rowptr, col, seeds, fanouts, rng_seed, cumulative=False):
    """Multi-hop sampling + reindex.  Returns a dict of numpy arrays."""
    rowptr, col, seeds, fanouts = _i64(rowptr), _i32(col), _i32(seeds), _i32(fanouts)
    n = len(rowptr) - 1
    K = len(fanouts)
    nb, eb, fb = sample_bounds(len(seeds), fanouts, n, cumulative)
    n_id = np.zeros(max(1, nb), dtype=np.int32)
    row = np.zeros(max(1, eb), dtype=np.int32)
    cl = np.zeros(max(1, eb), dtype=np.int32)
    ng = np.zeros(max(1, eb), dtype=np.int32)
    fr = np.zeros(max(1, fb), dtype=np.int32)
    node_off = np.zeros(K + 2, dtype=np.int64)
    edge_off = np.zeros(K + 1, dtype=np.int64)
    fr_off = np.zeros(K + 2, dtype=np.int64)
    rc = lib().o_sample(C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                        _p(seeds, C.c_int32), C.c_int64(len(seeds)), _p(fanouts, C.c_int32),
                        C.c_int32(K), C.c_uint64(rng_seed), C.c_int32(1 if cumulative else 0), _p(n_id, C.c_int32),
                        _p(row, C.c_int32), _p(cl, C.c_int32), _p(ng, C.c_int32),
                        _p(fr, C.c_int32), _p(node_off, C.c_int64), _p(edge_off, C.c_int64),
                        _p(fr_off, C.c_int64))
    if rc != 0:
        raise ValueError("seed id out of range")
    E, U, Fn = edge_off[K], node_off[K + 1], fr_off[K + 1]
    return dict(n_id=n_id[:U].copy(), row_local=row[:E].copy(), col_local=cl[:E].copy(),
                nbr_global=ng[:E].copy(), frontier=fr[:Fn].copy(), node_off=node_off,
                edge_off=edge_off, frontier_off=fr_off)


def gather(table, ids):
    """table: 2-D C-contiguous array of any dtype; -> table[ids] copied row by row."""
    table = np.ascontiguousarray(table)
    ids = _i32(ids)
    row_bytes = table.strides[0]
    out = np.empty((len(ids),) + table.shape[1:], dtype=table.dtype)
    rc = lib().o_gather(table.ctypes.data_as(C.POINTER(C.c_uint8)), C.c_int64(table.shape[0]),
                        C.c_int64(row_bytes), _p(ids, C.c_int32), C.c_int64(len(ids)),
                        out.ctypes.data_as(C.POINTER(C.c_uint8)))
    if rc != 0:
        raise ValueError("row id out of range")
    return out


def psgs(rowptr, col, fanouts, weight_mode=0):
    rowptr, col, fanouts = _i64(rowptr), _i32(col), _i32(fanouts)
    n = len(rowptr) - 1
    Q = np.zeros(n, dtype=np.float64)
    lib().o_psgs(C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32), _p(fanouts, C.c_int32),
                 C.c_int32(len(fanouts)), C.c_int32(weight_mode), _p(Q, C.c_double))
    return Q


def psgs_forward(rowptr, col, fanouts, start, weight_mode=0):
    """q_0..q_K of one start node, evaluated in the printed order of the definition."""
    rowptr, col, fanouts = _i64(rowptr), _i32(col), _i32(fanouts)
    n = len(rowptr) - 1
    q = np.zeros(len(fanouts) + 1, dtype=np.float64)
    lib().o_psgs_forward(C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                         _p(fanouts, C.c_int32), C.c_int32(len(fanouts)), C.c_int32(weight_mode),
                         C.c_int64(start), _p(q, C.c_double))
    return q


def access_prob(rowptr, col, fanouts, p0=None, weight_mode=0, layers=False):
    rowptr, col, fanouts = _i64(rowptr), _i32(col), _i32(fanouts)
    n = len(rowptr) - 1
    P = np.zeros(n, dtype=np.float64)
    p0a = None if p0 is None else np.ascontiguousarray(p0, dtype=np.float64)
    lay = np.zeros((len(fanouts) + 1, n), dtype=np.float64) if layers else None
    lib().o_access_prob(C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                        _p(fanouts, C.c_int32), C.c_int32(len(fanouts)),
                        _p(p0a, C.c_double) if p0a is not None else None,
                        C.c_int32(weight_mode), _p(P, C.c_double),
                        _p(lay, C.c_double) if lay is not None else None)
    return (P, lay) if layers else P


def place(prob, n_hot):
    """-> (rank int32[n], loc int32[n])"""
    prob = np.ascontiguousarray(prob, dtype=np.float32)
    n = len(prob)
    rank = np.zeros(n, dtype=np.int32)
    loc = np.zeros(n, dtype=np.int32)
    lib().o_place(_p(prob, C.c_float), C.c_int64(n), C.c_int64(n_hot), _p(rank, C.c_int32),
                  _p(loc, C.c_int32))
    return rank, loc
