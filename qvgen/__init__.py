"""Seeded synthetic inputs shared by the oracle's tests and the GPU library's tests.

Pure data: power-law CSR graphs, feature tables, seed batches.  No sampler, no metric, no Philox
lives here.  The five named workloads stand in for the public graphs the paper measures on
(Section 6, datasets table): their node / edge / feature shapes, with synthetic structure.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.cpp")
_SO = os.path.join(_HERE, "libqvgen.so")
_DEV_SRC = os.path.join(_HERE, "gen_dev.hip")
_DEV_SO = os.path.join(_HERE, "libqvgen_dev.so")
_lib = None
_dev = None

MASTER_SEED = 2305108630


def n_threads():
    return max(1, min(16, os.cpu_count() or 1))


def build(force=False, device=True):
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread", "-Wall",
                               "-o", _SO, _SRC])
    if device and (force or not os.path.exists(_DEV_SO)
                   or os.path.getmtime(_DEV_SO) < os.path.getmtime(_DEV_SRC)):
        subprocess.check_call(["hipcc", "-O3", "--offload-arch=gfx950", "-shared", "-fPIC",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-o", _DEV_SO, _DEV_SRC])
    return _SO


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build(device=False)
        _lib = C.CDLL(_SO)
        _lib.qg_hash.restype = C.c_uint64
        _lib.qg_hash.argtypes = [C.c_uint64] * 4
        _lib.qg_perm.restype = C.c_uint64
        _lib.qg_perm.argtypes = [C.c_uint64] * 3
        _lib.qg_calibrate_degree_scale.restype = C.c_double
        _lib.qg_calibrate_degree_scale.argtypes = [C.c_int64, C.c_double, C.c_int64, C.c_int64, C.c_double]
        _lib.qg_graph_rowptr.restype = C.c_int64
        _lib.qg_graph_rowptr.argtypes = [C.c_int64, C.c_double, C.c_double, C.c_int64, C.c_int64,
                                         C.c_uint64, C.c_int, C.c_void_p]
        _lib.qg_graph_col.restype = None
        _lib.qg_graph_col.argtypes = [C.c_int64, C.c_void_p, C.c_int, C.c_double, C.c_double,
                                      C.c_uint64, C.c_int, C.c_void_p]
        _lib.qg_symmetrise.restype = C.c_int64
        _lib.qg_symmetrise.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        _lib.qg_features.restype = None
        _lib.qg_features.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]
        _lib.qg_feature_rows.restype = None
        _lib.qg_feature_rows.argtypes = [C.c_uint64, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]
        _lib.qg_seeds.restype = None
        _lib.qg_seeds.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_void_p]
        _lib.qg_seed_popularity.restype = None
        _lib.qg_seed_popularity.argtypes = [C.c_uint64, C.c_int64, C.c_int, C.c_void_p]
        _lib.qg_batch_rng_seed.restype = C.c_uint64
        _lib.qg_batch_rng_seed.argtypes = [C.c_uint64, C.c_int64]
    return _lib


def dev():
    """Device-side feature generator (fills HBM directly); needs a GPU."""
    global _dev
    if _dev is None:
        if not os.path.exists(_DEV_SO):
            raise RuntimeError("qvgen device library not built: run __graft_entry__.build()")
        _dev = C.CDLL(_DEV_SO)
        _dev.qg_features_device.restype = C.c_int
        _dev.qg_features_device.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                            C.c_void_p, C.c_void_p]
        _dev.qg_copy_device.restype = C.c_int
        _dev.qg_copy_device.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    return _dev


# ---------------------------------------------------------------------------------------------
# graphs
# ---------------------------------------------------------------------------------------------
def power_law_graph(n, edge_target, deg_s, dmin, dmax, seed, endpoint_mode=0, ep_s=0.0, ep_q=1.0,
                    symmetrise=False, rowptr_dtype=np.int64):
    """CSR (rowptr, col int32).  Degrees follow d(r) = clamp(floor(C r^-s), dmin, dmax) over a
    seeded permutation of the nodes, with C calibrated so that the edge count meets the target;
    endpoints are distinct within a row and sorted."""
    L = lib()
    T = n_threads()
    dmax = min(dmax, n)
    c = L.qg_calibrate_degree_scale(n, deg_s, dmin, dmax, float(edge_target))
    rowptr = np.zeros(n + 1, dtype=np.int64)
    E = L.qg_graph_rowptr(n, c, deg_s, dmin, dmax, seed, T, rowptr.ctypes.data)
    col = np.empty(E, dtype=np.int32)
    L.qg_graph_col(n, rowptr.ctypes.data, endpoint_mode, ep_s, ep_q, seed, T, col.ctypes.data)
    if symmetrise:
        new_rowptr = np.zeros(n + 1, dtype=np.int64)
        E2 = L.qg_symmetrise(n, rowptr.ctypes.data, col.ctypes.data, new_rowptr.ctypes.data, None, T)
        new_col = np.empty(E2, dtype=np.int32)
        L.qg_symmetrise(n, rowptr.ctypes.data, col.ctypes.data, new_rowptr.ctypes.data,
                        new_col.ctypes.data, T)
        rowptr, col = new_rowptr, new_col
    if rowptr_dtype == np.int32:
        assert rowptr[-1] < 2 ** 31
        rowptr = rowptr.astype(np.int32)
    return rowptr, col


def features_host(seed, n_rows, dim, dtype, row_begin=0):
    dtype = np.dtype(dtype)
    out = np.empty((n_rows, dim), dtype=dtype)
    lib().qg_features(seed, row_begin, row_begin + n_rows, dim, dtype.itemsize, n_threads(), out.ctypes.data)
    return out


def feature_rows_host(seed, ids, dim, dtype):
    dtype = np.dtype(dtype)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty((len(ids), dim), dtype=dtype)
    lib().qg_feature_rows(seed, ids.ctypes.data, len(ids), dim, dtype.itemsize, n_threads(), out.ctypes.data)
    return out


def features_device(seed, n_rows, dim, torch_dtype, device="cuda:0"):
    """Fill an (n_rows, dim) table directly in HBM; bit-identical to features_host."""
    import torch
    out = torch.empty((n_rows, dim), dtype=torch_dtype, device=device)
    rc = dev().qg_features_device(seed, 0, n_rows, dim, out.element_size(), out.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("qg_features_device failed: hip error %d" % rc)
    return out


def copy_device(src, dst):
    """Plain device copy kernel of src.nbytes bytes (counter calibration yardstick)."""
    import torch
    n = src.numel() * src.element_size()
    rc = dev().qg_copy_device(src.data_ptr(), dst.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("qg_copy_device failed: hip error %d" % rc)
    return n


def seeds(seed, n_nodes, batch, n_seeds, mode=0):
    out = np.empty(n_seeds, dtype=np.int32)
    lib().qg_seeds(seed, n_nodes, batch, n_seeds, mode, out.ctypes.data)
    return out


def seed_popularity(seed, n_nodes):
    p0 = np.empty(n_nodes, dtype=np.float64)
    lib().qg_seed_popularity(seed, n_nodes, n_threads(), p0.ctypes.data)
    return p0


def batch_rng_seed(seed, batch):
    return int(lib().qg_batch_rng_seed(seed, batch))


# ---------------------------------------------------------------------------------------------
# the five workloads
# ---------------------------------------------------------------------------------------------
class Workload:
    def __init__(self, name, cfg, n, edge_target, deg_s, dmin, dmax, dim, feat_dtype, fanouts,
                 batch, endpoint_mode=0, ep_s=0.0, ep_q=1.0, symmetrise=False,
                 rowptr_dtype=np.int32, seed_mode=0, hbm_budget=None, batch_sweep=None):
        self.name, self.cfg, self.n, self.edge_target = name, cfg, n, edge_target
        self.deg_s, self.dmin, self.dmax = deg_s, dmin, dmax
        self.dim, self.feat_dtype, self.fanouts, self.batch = dim, np.dtype(feat_dtype), list(fanouts), batch
        self.endpoint_mode, self.ep_s, self.ep_q, self.symmetrise = endpoint_mode, ep_s, ep_q, symmetrise
        self.rowptr_dtype, self.seed_mode, self.hbm_budget = rowptr_dtype, seed_mode, hbm_budget
        self.batch_sweep = batch_sweep
        self.seed = MASTER_SEED + cfg

    def graph(self):
        return power_law_graph(self.n, self.edge_target, self.deg_s, self.dmin, self.dmax, self.seed,
                               self.endpoint_mode, self.ep_s, self.ep_q, self.symmetrise,
                               self.rowptr_dtype)

    def seeds(self, batch_index, n_seeds=None):
        return seeds(self.seed, self.n, batch_index, n_seeds or self.batch, self.seed_mode)

    def rng_seed(self, batch_index):
        return batch_rng_seed(self.seed, batch_index)

    @property
    def row_bytes(self):
        return self.dim * self.feat_dtype.itemsize


def workload(name, scale=1.0):
    """The named workloads.  `scale` < 1 shrinks node and edge counts together (for CPU tests of
    the recipe); 1.0 is the size the workload is defined at."""
    def S(x):
        return max(16, int(round(x * scale)))
    if name == "tiny":             # 10k nodes, ~200k edges, Zipf(1.1) degrees in [1, 2000]
        return Workload(name, 1, S(10_000), S(200_000), 1.1, 1, 2_000, 64, np.float32, [10, 5], 64)
    if name == "dense_social":     # Reddit-like shape: mean degree ~492, degrees capped at 20k
        return Workload(name, 2, S(232_965), S(114_600_000), 0.9, 1, 20_000, 602, np.float32,
                        [25, 10], 1_000)
    if name == "co_purchase":      # ogbn-products-like shape: symmetrised power law, mean ~50
        return Workload(name, 3, S(2_449_029), S(123_700_000 // 2), 1.2, 1, 100_000, 100, np.float32,
                        [15, 10, 5], 4_096, symmetrise=True, batch_sweep=[1, 8, 64, 512, 4_096])
    if name == "citation":         # ogbn-papers100M-like shape: int64 rowptr, in-degree skew
        return Workload(name, 4, S(111_000_000), S(1_600_000_000), 0.5, 1, 4_096, 128, np.float16,
                        [15, 10, 5], 1_024, endpoint_mode=1, ep_s=1.3, ep_q=250.0,
                        rowptr_dtype=np.int64)
    if name == "tiered":           # graph of co_purchase, 4 KiB rows, 2 GiB HBM feature budget
        w = Workload(name, 5, S(2_449_029), S(123_700_000 // 2), 1.2, 1, 100_000, 1_024, np.float32,
                     [15, 10, 5], 512, symmetrise=True, seed_mode=1,
                     hbm_budget=int(2 * 2 ** 30 * scale))
        w.seed = MASTER_SEED + 3   # same graph as co_purchase
        return w
    raise KeyError(name)


WORKLOADS = ["tiny", "dense_social", "co_purchase", "citation", "tiered"]
