"""Python binding of libqv.so: argument marshalling only.

PyTorch supplies device memory (tensors) and streams; every step of the path runs in the HIP
kernels behind the C ABI declared in include/qv.h.  There is no CPU fallback: if the library is
missing or the GPU is absent, calls raise.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqv.so")
_lib = None

QV_OK, QV_EINVAL, QV_ENOMEM, QV_EHIP, QV_ECAPACITY, QV_ERANGE = 0, -1, -2, -3, -4, -5
QV_MAX_HOPS, QV_MAX_FANOUT, QV_MAX_BATCHES = 8, 1024, 256
QV_STEP_LANES, QV_MAX_STEP_BATCHES = 4, 4 * 256
QV_NOALLOC_MAX_FRONTIER = 1 << 20
QV_SAMPLE_CUMULATIVE, QV_FEAT_OWN_COPY = 1, 1
QV_DEDUP_AUTO, QV_DEDUP_TABLE, QV_DEDUP_PARTITIONED = 0, 1, 2

EXPORTS = [
    "qv_ctx_create", "qv_ctx_destroy", "qv_last_error", "qv_ctx_sync", "qv_ctx_reserve", "qv_ctx_set_epoch", "qv_ctx_set_table_budget", "qv_ctx_set_dedup", "qv_ctx_set_fap_direction", "qv_ctx_set_fap_block", "qv_csr_fap_items",
    "qv_sample_bounds", "qv_csr_create", "qv_csr_destroy", "qv_csr_transpose", "qv_csr_rowptr", "qv_csr_col", "qv_sample_hop", "qv_sample_hop_noalloc", "qv_sample", "qv_sample_many",
    "qv_reindex", "qv_feat_create", "qv_feat_destroy", "qv_feat_hot_rows", "qv_feat_loc", "qv_feat_row_stride",
    "qv_gather", "qv_gather_many", "qv_step_many", "qv_psgs", "qv_psgs_batch_sum", "qv_access_prob", "qv_place_rank",
]


class QvError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("qv status %d: %s" % (status, message))
        self.status = status


class _SampleOut(C.Structure):
    _fields_ = [("n_id", C.c_void_p), ("n_id_cap", C.c_int64),
                ("row_local", C.c_void_p), ("col_local", C.c_void_p), ("nbr_global", C.c_void_p),
                ("edge_cap", C.c_int64),
                ("frontier", C.c_void_p), ("frontier_cap", C.c_int64),
                ("node_off", C.c_void_p), ("edge_off", C.c_void_p), ("frontier_off", C.c_void_p)]


def lib():
    """Load libqv.so (built in-tree by paper_2305_10863_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libqv.so is not built: run `python -c 'import __graft_entry__ as g; "
                               "g.build()'` (hipcc, gfx950). There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, u64 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64
        L.qv_ctx_create.argtypes = [C.c_int, vp, C.POINTER(vp)]
        L.qv_ctx_destroy.argtypes = [vp]
        L.qv_ctx_destroy.restype = None
        L.qv_last_error.argtypes = [vp]
        L.qv_last_error.restype = C.c_char_p
        L.qv_ctx_sync.argtypes = [vp]
        L.qv_ctx_reserve.argtypes = [vp, i64, C.POINTER(i32), i32, i64, C.c_uint32, i32]
        L.qv_ctx_set_epoch.argtypes = [vp, C.c_uint32]
        L.qv_ctx_set_table_budget.argtypes = [vp, i64]
        L.qv_ctx_set_dedup.argtypes = [vp, i32, i32]
        L.qv_ctx_set_fap_direction.argtypes = [vp, i32]
        L.qv_ctx_set_fap_block.argtypes = [vp, i32]
        L.qv_sample_bounds.argtypes = [i64, C.POINTER(i32), i32, i64, C.c_uint32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
        L.qv_csr_create.argtypes = [vp, i64, i64, vp, i32, vp, i32, C.POINTER(vp)]
        L.qv_csr_destroy.argtypes = [vp]
        L.qv_csr_destroy.restype = None
        L.qv_csr_transpose.argtypes = [vp, vp, C.POINTER(vp)]
        L.qv_csr_rowptr.argtypes = [vp]
        L.qv_csr_rowptr.restype = vp
        L.qv_csr_col.argtypes = [vp]
        L.qv_csr_col.restype = vp
        L.qv_csr_fap_items.argtypes = [vp, C.POINTER(vp), C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]
        L.qv_csr_fap_items.restype = vp
        L.qv_sample_hop.argtypes = [vp, vp, vp, i64, i32, u64, i32, vp, i64, vp]
        L.qv_sample_hop_noalloc.argtypes = [vp, vp, vp, i64, i32, u64, i32, vp, i64, vp]
        L.qv_sample.argtypes = [vp, vp, vp, i64, C.POINTER(i32), i32, u64, C.c_uint32, C.POINTER(_SampleOut)]
        L.qv_sample_many.argtypes = [vp, vp, i32, C.POINTER(vp), C.POINTER(i64), C.POINTER(i32), i32,
                                     C.POINTER(u64), C.c_uint32, C.POINTER(_SampleOut)]
        L.qv_gather_many.argtypes = [vp, vp, i32, C.POINTER(vp), C.POINTER(i64), C.POINTER(vp), C.POINTER(vp), i64]
        L.qv_step_many.argtypes = [vp, vp, vp, i32, C.POINTER(vp), C.POINTER(i64), C.POINTER(i32), i32, C.POINTER(u64),
                                   C.c_uint32, C.POINTER(_SampleOut), C.POINTER(vp), C.POINTER(i64), i64]
        L.qv_reindex.argtypes = [vp, vp, i64, vp, i64, i64, vp, i64, vp, vp, vp, vp]
        L.qv_feat_create.argtypes = [vp, vp, i32, i64, i32, i32, i64, vp, i32, C.POINTER(vp)]
        L.qv_feat_destroy.argtypes = [vp]
        L.qv_feat_destroy.restype = None
        L.qv_feat_hot_rows.argtypes = [vp]
        L.qv_feat_hot_rows.restype = i64
        L.qv_feat_loc.argtypes = [vp]
        L.qv_feat_loc.restype = vp
        L.qv_feat_row_stride.argtypes = [vp]
        L.qv_feat_row_stride.restype = i64
        L.qv_gather.argtypes = [vp, vp, vp, i64, vp, vp, i64]
        L.qv_psgs.argtypes = [vp, vp, C.POINTER(i32), i32, vp]
        L.qv_psgs_batch_sum.argtypes = [vp, vp, i64, vp, i64, vp]
        L.qv_access_prob.argtypes = [vp, vp, vp, C.POINTER(i32), i32, vp, vp]
        L.qv_place_rank.argtypes = [vp, vp, i64, vp]
        _lib = L
    return _lib


def _fan(fanouts):
    arr = (C.c_int32 * len(fanouts))(*[int(x) for x in fanouts])
    return arr, len(fanouts)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev_i32(t, name):
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError("%s must be a contiguous int32 CUDA tensor" % name)
    return t


class Context:
    """One qv_ctx: a GPU, a stream, a scratch arena.  One batch in flight per context."""

    def __init__(self, device=0, stream=None):
        self.device = torch.device("cuda", device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        rc = lib().qv_ctx_create(device, C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if rc != QV_OK:
            raise QvError(rc, lib().qv_last_error(None).decode())
        self.h = h

    def check(self, rc):
        if rc != QV_OK:
            raise QvError(rc, lib().qv_last_error(self.h).decode())

    def sync(self):
        """Wait for the stream and raise on a deferred device-side error."""
        self.check(lib().qv_ctx_sync(self.h))

    def set_table_budget(self, n_bytes):
        """0 forces the hashed dedup table; see qv_ctx_set_table_budget."""
        self.check(lib().qv_ctx_set_table_budget(self.h, n_bytes))

    def set_dedup(self, form, partitions_log2=-1):
        """form: 0 auto, 1 tables, 2 partitioned; see qv_ctx_set_dedup."""
        self.check(lib().qv_ctx_set_dedup(self.h, form, partitions_log2))

    def set_fap_direction(self, direction):
        """0 choose per sweep (default), 1 gather only, 2 scatter only; see qv_ctx_set_fap_direction."""
        self.check(lib().qv_ctx_set_fap_direction(self.h, direction))

    def set_fap_block(self, nodes_log2):
        """Block size (log2 of node ids) of the long rows' work items that later transposes build; see qv_ctx_set_fap_block."""
        self.check(lib().qv_ctx_set_fap_block(self.h, nodes_log2))

    def reserve(self, n_seeds, fanouts, n_nodes, cumulative=False, n_batches=8):
        arr, k = _fan(fanouts)
        self.check(lib().qv_ctx_reserve(self.h, n_seeds, arr, k, n_nodes, 1 if cumulative else 0, n_batches))

    def close(self):
        if getattr(self, "h", None):
            lib().qv_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Graph:
    """qv_csr over two tensors (kept alive here): CUDA tensors, or pinned CPU tensors for a graph
    that is read zero-copy over the host link."""

    def __init__(self, ctx, rowptr, col, validate=True):
        for t, name in ((rowptr, "rowptr"), (col, "col")):
            if not t.is_contiguous() or not (t.is_cuda or t.is_pinned()):
                raise TypeError("%s must be a contiguous CUDA tensor or a pinned CPU tensor" % name)
        if rowptr.dtype not in (torch.int32, torch.int64) or col.dtype != torch.int32:
            raise TypeError("rowptr must be int32/int64 and col int32")
        self.ctx, self.rowptr, self.col, self._rowptr_dtype = ctx, rowptr, col, rowptr.dtype
        self.n_nodes, self.n_edges = rowptr.numel() - 1, col.numel()
        h = C.c_void_p()
        ctx.check(lib().qv_csr_create(ctx.h, self.n_nodes, self.n_edges, _ptr(rowptr),
                                      32 if rowptr.dtype == torch.int32 else 64, _ptr(col),
                                      1 if validate else 0, C.byref(h)))
        self.h = h

    def transpose(self):
        """The in-edge CSR as a Graph whose arrays the library owns (qv_csr_transpose)."""
        h = C.c_void_p()
        self.ctx.check(lib().qv_csr_transpose(self.ctx.h, self.h, C.byref(h)))
        t = Graph.__new__(Graph)
        t.ctx, t.rowptr, t.col, t.h = self.ctx, None, None, h
        t.n_nodes, t.n_edges, t._rowptr_dtype = self.n_nodes, self.n_edges, self._rowptr_dtype
        return t

    def fap_items(self):
        """(long_rows, items[n_items, 4] as int32 words: first lo, first hi, k, count; block_log2) as CUDA tensors
        (copies), or None; see qv_csr_fap_items."""
        rows_p, n_long, n_items, log2 = C.c_void_p(), C.c_int32(), C.c_int64(), C.c_int32()
        items_p = lib().qv_csr_fap_items(self.h, C.byref(rows_p), C.byref(n_long), C.byref(n_items), C.byref(log2))
        if not items_p:
            return None
        out = []
        for ptr, shape in ((rows_p.value, (n_long.value,)), (items_p, (n_items.value, 4))):
            view = type("_DevView", (), {"__cuda_array_interface__": {
                "shape": shape, "typestr": "<i4", "data": (ptr, False), "version": 2, "strides": None}})()
            out.append(torch.as_tensor(view, device=self.ctx.device).clone())
        return out[0], out[1], log2.value

    def arrays(self):
        """(rowptr, col) as CUDA tensors; for a transposed graph, copies of the library's arrays."""
        if self.rowptr is not None:
            return self.rowptr, self.col
        out = []
        for ptr, n, dt, ts in ((lib().qv_csr_rowptr(self.h), self.n_nodes + 1, self._rowptr_dtype,
                                "<i4" if self._rowptr_dtype == torch.int32 else "<i8"),
                               (lib().qv_csr_col(self.h), self.n_edges, torch.int32, "<i4")):
            if n == 0 or not ptr:
                out.append(torch.empty(0, dtype=dt, device=self.ctx.device))
                continue
            view = type("_DevView", (), {"__cuda_array_interface__": {
                "shape": (n,), "typestr": ts, "data": (ptr, False), "version": 2, "strides": None}})()
            out.append(torch.as_tensor(view, device=self.ctx.device).clone())
        return tuple(out)

    def close(self):
        if getattr(self, "h", None):
            lib().qv_csr_destroy(self.h)
            self.h = None

    def __del__(self):
        try:                    # at interpreter exit the module's globals may be gone already
            self.close()
        except Exception:
            pass


class Features:
    """qv_feat.  `table` is a 2-D torch tensor (CUDA or CPU) of fp16/fp32 (or any 2/4-byte type)."""

    def __init__(self, ctx, table, hbm_budget_bytes=-1, rank=None, own_copy=False):
        if table.dim() != 2 or not table.is_contiguous() or table.element_size() not in (2, 4):
            raise TypeError("table must be a contiguous 2-D tensor of 2- or 4-byte elements")
        self.ctx, self.dtype = ctx, table.dtype
        self.n_rows, self.dim = table.shape
        self.row_bytes = self.dim * table.element_size()
        h = C.c_void_p()
        ctx.check(lib().qv_feat_create(ctx.h, _ptr(table), 1 if table.is_cuda else 0, self.n_rows, self.dim,
                                       table.element_size(), hbm_budget_bytes,
                                       None if rank is None else _ptr(_dev_i32(rank, "rank")),
                                       1 if own_copy else 0, C.byref(h)))
        self.h = h
        self.n_hot = lib().qv_feat_hot_rows(h)
        self.row_stride = lib().qv_feat_row_stride(h)          # bytes; also a good output stride
        # a borrowed device table must stay alive as long as the handle
        self._keep = table if (table.is_cuda and self.n_hot == self.n_rows) else None

    def loc(self):
        """Copy of the lookup table (int32[n_rows]: >= 0 HBM row, < 0 ~host row), or None when every
        row is in HBM in id order."""
        ptr = lib().qv_feat_loc(self.h)
        if not ptr:
            return None
        view = type("_DevView", (), {"__cuda_array_interface__": {
            "shape": (self.n_rows,), "typestr": "<i4", "data": (ptr, False), "version": 2, "strides": None}})()
        return torch.as_tensor(view, device=self.ctx.device).clone()

    def empty_rows(self, n, device):
        """An (n, dim) output tensor whose rows start at the tier's (line-aligned) stride."""
        esz = self.row_bytes // self.dim
        padded = torch.empty((max(n, 1), self.row_stride // esz), dtype=self.dtype, device=device)
        return padded[:, :self.dim]

    def close(self):
        if getattr(self, "h", None):
            lib().qv_feat_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def qv_sample_bounds(n_seeds, fanouts, n_nodes, cumulative=False):
    arr, k = _fan(fanouts)
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    rc = lib().qv_sample_bounds(n_seeds, arr, k, n_nodes, 1 if cumulative else 0, C.byref(a), C.byref(b), C.byref(c))
    if rc != QV_OK:
        raise QvError(rc, lib().qv_last_error(None).decode())
    return a.value, b.value, c.value


class SampleBuffers:
    """Caller-side output arrays of qv_sample, sized to the a-priori bounds (or given caps)."""

    def __init__(self, ctx, n_seeds, fanouts, n_nodes, caps=None, want_frontier=True, want_nbr_global=True,
                 cumulative=False):
        nb, eb, fb = qv_sample_bounds(n_seeds, fanouts, n_nodes, cumulative)
        if caps is not None:
            nb, eb, fb = caps
        dev, K = ctx.device, len(fanouts)
        e = lambda n, dt=torch.int32: torch.empty(max(int(n), 1), dtype=dt, device=dev)
        self.n_id, self.row_local, self.col_local = e(nb), e(eb), e(eb)
        self.nbr_global = e(eb) if want_nbr_global else None
        self.frontier = e(fb) if want_frontier else None
        self.caps = (int(nb), int(eb), int(fb))
        self.node_off = torch.zeros(K + 2, dtype=torch.int64, device=dev)
        self.edge_off = torch.zeros(K + 1, dtype=torch.int64, device=dev)
        self.frontier_off = torch.zeros(K + 2, dtype=torch.int64, device=dev)
        self.n_hops = K

    def struct(self):
        return _SampleOut(self.n_id.data_ptr(), self.caps[0], self.row_local.data_ptr(),
                          self.col_local.data_ptr(),
                          None if self.nbr_global is None else self.nbr_global.data_ptr(), self.caps[1],
                          None if self.frontier is None else self.frontier.data_ptr(), self.caps[2],
                          self.node_off.data_ptr(), self.edge_off.data_ptr(), self.frontier_off.data_ptr())

    def to_host(self):
        """Synchronising copy of the results, trimmed to their true lengths (numpy arrays)."""
        node_off = self.node_off.cpu().numpy()
        edge_off = self.edge_off.cpu().numpy()
        fr_off = self.frontier_off.cpu().numpy()
        U, E, Fn = int(node_off[-1]), int(edge_off[-1]), int(fr_off[-1])
        U, E, Fn = min(U, self.caps[0]), min(E, self.caps[1]), min(Fn, self.caps[2])
        out = dict(n_id=self.n_id[:U].cpu().numpy(), row_local=self.row_local[:E].cpu().numpy(),
                   col_local=self.col_local[:E].cpu().numpy(), node_off=node_off, edge_off=edge_off,
                   frontier_off=fr_off)
        if self.nbr_global is not None:
            out["nbr_global"] = self.nbr_global[:E].cpu().numpy()
        if self.frontier is not None:
            out["frontier"] = self.frontier[:Fn].cpu().numpy()
        return out


def qv_sample(ctx, graph, seeds, fanouts, rng_seed, out=None, cumulative=False):
    """Multi-hop sampling + reindex of one batch; asynchronous.  Returns the SampleBuffers.
    cumulative=True: every hop expands all nodes sampled so far (nested blocks)."""
    _dev_i32(seeds, "seeds")
    if out is None:
        out = SampleBuffers(ctx, seeds.numel(), fanouts, graph.n_nodes, cumulative=cumulative)
    arr, k = _fan(fanouts)
    st = out.struct()
    ctx.check(lib().qv_sample(ctx.h, graph.h, _ptr(seeds), seeds.numel(), arr, k, C.c_uint64(rng_seed),
                              1 if cumulative else 0, C.byref(st)))
    return out


class ManyPlan:
    """Pre-marshalled argument arrays for qv_sample_many + qv_gather_many over fixed buffers, so
    that a serving loop only swaps seed pointers and rng seeds."""

    def __init__(self, ctx, graph, feat, bufs, rows, fanouts, cumulative=False):
        n = len(bufs)
        self.ctx, self.graph, self.feat, self.bufs, self.rows, self.n = ctx, graph, feat, bufs, rows, n
        self.flags = 1 if cumulative else 0
        self.fan, self.k = _fan(fanouts)
        self.seed_ptrs = (C.c_void_p * n)()
        self.n_seeds = (C.c_int64 * n)()
        self.rng = (C.c_uint64 * n)()
        self.outs = (_SampleOut * n)(*[b.struct() for b in bufs])
        if feat is not None:
            K = bufs[0].n_hops
            self.ids = (C.c_void_p * n)(*[b.n_id.data_ptr() for b in bufs])
            self.n_ids = (C.c_int64 * n)(*[b.caps[0] for b in bufs])
            self.n_dev = (C.c_void_p * n)(*[b.node_off.data_ptr() + 8 * (K + 1) for b in bufs])
            self.out_ptrs = (C.c_void_p * n)(*[r.data_ptr() for r in rows])
            self.stride = rows[0].stride(0) * rows[0].element_size()

    def refresh_outputs(self):
        """Call after swapping a buffer's offset tensors."""
        K = self.bufs[0].n_hops
        for i, b in enumerate(self.bufs):
            self.outs[i] = b.struct()
            if self.feat is not None:
                self.n_dev[i] = b.node_off.data_ptr() + 8 * (K + 1)

    def run(self, seeds, rng_seeds, n_batches=None):
        n = len(seeds) if n_batches is None else n_batches
        for i in range(n):
            self.seed_ptrs[i] = seeds[i].data_ptr()
            self.n_seeds[i] = seeds[i].numel()
            self.rng[i] = rng_seeds[i]
        L, c = lib(), self.ctx
        c.check(L.qv_sample_many(c.h, self.graph.h, n, self.seed_ptrs, self.n_seeds, self.fan, self.k, self.rng,
                                 self.flags, self.outs))
        if self.feat is not None:
            c.check(L.qv_gather_many(c.h, self.feat.h, n, self.ids, self.n_ids, self.n_dev, self.out_ptrs, self.stride))

    def step(self, seeds, rng_seeds, n_batches=None):
        """The same through qv_step_many (up to QV_MAX_STEP_BATCHES batches; groups beyond the first run on the
        context's own streams); rows are gathered up to each batch's `n_ids` entry."""
        n = len(seeds) if n_batches is None else n_batches
        for i in range(n):
            self.seed_ptrs[i] = seeds[i].data_ptr()
            self.n_seeds[i] = seeds[i].numel()
            self.rng[i] = rng_seeds[i]
        c = self.ctx
        c.check(lib().qv_step_many(c.h, self.graph.h, self.feat.h, n, self.seed_ptrs, self.n_seeds, self.fan, self.k, self.rng,
                                   self.flags, self.outs, self.out_ptrs, self.n_ids, self.stride))


def qv_sample_many(ctx, graph, seeds_list, fanouts, rng_seeds, outs=None, cumulative=False):
    """Several independent batches through one set of launches.  Returns the SampleBuffers list."""
    n = len(seeds_list)
    for s in seeds_list:
        _dev_i32(s, "seeds")
    if outs is None:
        outs = [SampleBuffers(ctx, s.numel(), fanouts, graph.n_nodes, cumulative=cumulative) for s in seeds_list]
    plan = ManyPlan(ctx, graph, None, outs, None, fanouts, cumulative=cumulative)
    plan.run(seeds_list, rng_seeds, n)
    return outs


def qv_gather_many(ctx, feat, ids_list, n_ids_dev_list=None, outs=None):
    n = len(ids_list)
    if outs is None:
        outs = [feat.empty_rows(t.numel(), ctx.device) for t in ids_list]
    ids = (C.c_void_p * n)(*[_dev_i32(t, "ids").data_ptr() for t in ids_list])
    cnt = (C.c_int64 * n)(*[t.numel() for t in ids_list])
    ndev = None
    if n_ids_dev_list is not None:
        ndev = (C.c_void_p * n)(*[None if t is None else t.data_ptr() for t in n_ids_dev_list])
    optr = (C.c_void_p * n)(*[o.data_ptr() for o in outs])
    ctx.check(lib().qv_gather_many(ctx.h, feat.h, n, ids, cnt, ndev, optr, outs[0].stride(0) * outs[0].element_size()))
    return outs


def qv_sample_hop(ctx, graph, frontier, fanout, rng_seed, hop, nbr_cap=None, out=None, noalloc=False):
    """One hop.  Returns (nbr int32[cap], off int64[F+1]) device tensors; off[-1] = count.
    `out` = (nbr, off) tensors to write into; noalloc=True calls qv_sample_hop_noalloc (the
    library's fixed scratch, no device allocation inside the call)."""
    _dev_i32(frontier, "frontier")
    F = frontier.numel()
    cap = F * fanout if nbr_cap is None else nbr_cap
    if out is None:
        nbr = torch.empty(max(cap, 1), dtype=torch.int32, device=ctx.device)
        off = torch.zeros(F + 1, dtype=torch.int64, device=ctx.device)
    else:
        nbr, off = out
    fn = lib().qv_sample_hop_noalloc if noalloc else lib().qv_sample_hop
    ctx.check(fn(ctx.h, graph.h, _ptr(frontier), F, fanout, C.c_uint64(rng_seed), hop, _ptr(nbr), cap, _ptr(off)))
    return nbr, off


def qv_reindex(ctx, known, nbr, n_nodes=0, n_id_cap=None):
    """Dedup + relabel.  Returns (n_id, n_id_len, local, frontier, frontier_len) device tensors."""
    _dev_i32(known, "known")
    _dev_i32(nbr, "nbr")
    cap = known.numel() + nbr.numel() if n_id_cap is None else n_id_cap
    dev = ctx.device
    n_id = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    local = torch.empty(max(nbr.numel(), 1), dtype=torch.int32, device=dev)
    front = torch.empty(max(nbr.numel(), 1), dtype=torch.int32, device=dev)
    lens = torch.zeros(2, dtype=torch.int64, device=dev)
    ctx.check(lib().qv_reindex(ctx.h, _ptr(known), known.numel(), _ptr(nbr), nbr.numel(), n_nodes, _ptr(n_id), cap,
                               C.c_void_p(lens.data_ptr()), _ptr(local), _ptr(front),
                               C.c_void_p(lens.data_ptr() + 8)))
    return n_id, lens[0:1], local, front, lens[1:2]


def qv_gather(ctx, feat, ids, n_ids_dev=None, out=None, n_ids=None):
    """out[r] = table[ids[r]].  `n_ids_dev` (int64 device scalar tensor) clamps the row count on
    the device, so a gather can be enqueued straight after qv_sample."""
    _dev_i32(ids, "ids")
    n = ids.numel() if n_ids is None else n_ids
    if out is None:
        out = feat.empty_rows(n, ctx.device)
    ctx.check(lib().qv_gather(ctx.h, feat.h, _ptr(ids), n, _ptr(n_ids_dev), _ptr(out), out.stride(0) * out.element_size()))
    return out


def qv_psgs(ctx, graph, fanouts, out=None):
    if out is None:
        out = torch.empty(max(graph.n_nodes, 1), dtype=torch.float32, device=ctx.device)
    arr, k = _fan(fanouts)
    ctx.check(lib().qv_psgs(ctx.h, graph.h, arr, k, _ptr(out)))
    return out[:graph.n_nodes]


def qv_psgs_batch_sum(ctx, psgs, seeds):
    out = torch.zeros(1, dtype=torch.float64, device=ctx.device)
    ctx.check(lib().qv_psgs_batch_sum(ctx.h, _ptr(psgs), psgs.numel(), _ptr(_dev_i32(seeds, "seeds")), seeds.numel(), _ptr(out)))
    return out


def qv_access_prob(ctx, graph, fanouts, p0=None, out=None, graph_in=None):
    """graph_in: Graph of the in-edges (the transpose; the graph itself if it is symmetric) for the
    atomic-free gather sweeps, or None for scatter sweeps."""
    if p0 is not None and (p0.dtype != torch.float32 or not p0.is_cuda or p0.numel() != graph.n_nodes):
        raise TypeError("p0 must be a float32 CUDA tensor with one entry per node")
    if out is None:
        out = torch.empty(max(graph.n_nodes, 1), dtype=torch.float32, device=ctx.device)
    arr, k = _fan(fanouts)
    ctx.check(lib().qv_access_prob(ctx.h, graph.h, None if graph_in is None else graph_in.h, arr, k, _ptr(p0), _ptr(out)))
    return out[:graph.n_nodes]


def qv_place_rank(ctx, prob):
    if prob.dtype != torch.float32 or not prob.is_cuda:
        raise TypeError("prob must be a float32 CUDA tensor")
    rank = torch.empty(max(prob.numel(), 1), dtype=torch.int32, device=ctx.device)
    ctx.check(lib().qv_place_rank(ctx.h, _ptr(prob), prob.numel(), _ptr(rank)))
    return rank[:prob.numel()]
