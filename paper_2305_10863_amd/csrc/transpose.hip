// In-edge CSR of a graph, built on the device: the form the gather sweeps of the feature access
// probability read (Section 5.1: p_k[i] sums over the edges that END at i).
//
//   1. src[e]  = the row that edge e belongs to               (one group of lanes per row)
//   2. stable radix sort of the pairs (col[e], src[e]) by col  (rocPRIM; least-significant-digit
//      passes keep equal keys in edge order, so every in-row lists its sources in ascending order)
//   3. rowptr_t[v] = first sorted position whose key is >= v   (boundary detection, no atomics)
//
//   4. the rows longer than kLongRow are listed; the positions at which the sources of every block of
//      2^18 node ids begin in each are found by binary search (step 2 left the sources ascending);
//      the parts so cut off are cut again into work items of at most 256 edges, listed block by
//      block (the blocked gather of qv_access_prob)
//
// The result is owned by the handle and freed by qv_csr_destroy.
#include <cstring>
#include <string.h>

#include <rocprim/rocprim.hpp>

#include "qv_internal.hpp"

using namespace qv;

namespace {

template <int G, typename RP>
__global__ void __launch_bounds__(256) k_edge_sources(const RP* __restrict__ rowptr, int64_t n, int32_t* __restrict__ src) {
    const int sub = threadIdx.x % G;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / G;
    const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / G;
    for (int64_t v = group; v < n; v += n_groups) {
        const int64_t rs = (int64_t)rowptr[v], re = (int64_t)rowptr[v + 1];
        for (int64_t e = rs + sub; e < re; e += G) src[e] = (int32_t)v;
    }
}

// keys: the sorted destination ids.  Position e (0..n_edges) closes every row between the key
// before it and its own key; position n_edges closes the rows after the last key.
template <typename RP>
__global__ void k_rowptr_from_sorted(const int32_t* __restrict__ keys, int64_t n_edges, int64_t n, RP* __restrict__ rowptr_t) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = tid; e <= n_edges; e += stride) {
        const int64_t prev = e > 0 ? (int64_t)keys[e - 1] : -1;
        const int64_t cur = e < n_edges ? (int64_t)keys[e] : n;
        for (int64_t v = prev + 1; v <= cur; ++v) rowptr_t[v] = (RP)e;
    }
}

template <typename RP>
qv_status transpose(qv_ctx* ctx, const qv_csr* g, void* rowptr_t, int32_t* col_t, int32_t* src, int32_t* keys_sorted,
                    void* temp, size_t temp_bytes) {
    const int64_t n = g->n_nodes, E = g->n_edges;
    const RP* rp = (const RP*)g->rowptr;
    if (E > 0) {
        const int blocks = grid_for(n * 16, 256, ctx->n_cu * 32);
        hipLaunchKernelGGL((k_edge_sources<16, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, n, src);
        QV_LAUNCH_CHECK(ctx, "k_edge_sources");
        unsigned end_bit = 1;
        while (end_bit < 31 && ((int64_t)1 << end_bit) < n) ++end_bit;
        hipError_t e = rocprim::radix_sort_pairs(temp, temp_bytes, g->col, keys_sorted, (const int32_t*)src, col_t, (size_t)E,
                                                 0u, end_bit, ctx->stream);
        if (e != hipSuccess) return fail(ctx, QV_EHIP, "qv_csr_transpose: sort failed: %s", hipGetErrorString(e));
    }
    const int blocks = grid_for(E + 1, 256 * 4, ctx->n_cu * 16);
    hipLaunchKernelGGL((k_rowptr_from_sorted<RP>), dim3(blocks), dim3(256), 0, ctx->stream, (const int32_t*)keys_sorted, E, n,
                       (RP*)rowptr_t);
    QV_LAUNCH_CHECK(ctx, "k_rowptr_from_sorted");
    return QV_OK;
}

// --- work items of the long rows --------------------------------------------------------------
constexpr int kFapBlockLog2 = 18;                   // 2^18 sources = 2 MB of fp64 values: half of one XCD's L2
constexpr size_t kFapAnnexMaxBytes = (size_t)1 << 30;

// counts[0] += rows longer than kLongRow, counts[1] += their edges
template <typename RP>
__global__ void __launch_bounds__(256) k_long_count(const RP* __restrict__ rowptr_t, int64_t n, unsigned long long* counts) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    unsigned long long rows = 0, edges = 0;
    for (int64_t i = tid; i < n; i += stride) {
        const int64_t len = (int64_t)rowptr_t[i + 1] - (int64_t)rowptr_t[i];
        if (len > kLongRow) { ++rows; edges += (unsigned long long)len; }
    }
#pragma unroll
    for (int o = kWave / 2; o >= 1; o >>= 1) {
        rows += __shfl_xor(rows, o);
        edges += __shfl_xor(edges, o);
    }
    if (threadIdx.x % kWave == 0 && rows) {
        atomicAdd(&counts[0], rows);
        atomicAdd(&counts[1], edges);
    }
}

// long_rows[0 .. n_long): the rows longer than kLongRow, in the order their threads get here
template <typename RP>
__global__ void __launch_bounds__(256) k_long_list(const RP* __restrict__ rowptr_t, int64_t n, unsigned long long* cursor,
                                                   int32_t* __restrict__ long_rows, int32_t n_long) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) {
        if ((int64_t)rowptr_t[i + 1] - (int64_t)rowptr_t[i] > kLongRow) {
            const unsigned long long k = atomicAdd(cursor, 1ull);
            if (k < (unsigned long long)n_long) long_rows[k] = (int32_t)i;
        }
    }
}

// Piece q = b * n_long + k is the part of long row k whose sources lie in block b.
// cuts[q] = first edge of long row k whose source is >= b << log2  (b = 0 .. blocks)
template <typename RP>
__global__ void __launch_bounds__(256) k_long_cuts(const RP* __restrict__ rowptr_t, const int32_t* __restrict__ col_t,
                                                   const int32_t* __restrict__ long_rows, int32_t n_long, int32_t blocks,
                                                   int log2, int64_t* __restrict__ cuts) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t total = (int64_t)(blocks + 1) * n_long;
    for (int64_t q = tid; q < total; q += stride) {
        const int64_t b = q / n_long;
        const int64_t i = long_rows[q - b * n_long];
        int64_t lo = (int64_t)rowptr_t[i], hi = (int64_t)rowptr_t[i + 1];
        const int64_t first = b << log2;
        while (lo < hi) {
            const int64_t mid = lo + (hi - lo) / 2;
            if ((int64_t)col_t[mid] < first) lo = mid + 1; else hi = mid;
        }
        cuts[q] = lo;
    }
}

// items a piece is cut into: runs of at most kFapItemEdges edges
__global__ void __launch_bounds__(256) k_item_counts(const int64_t* __restrict__ cuts, int32_t n_long, int64_t pieces,
                                                     uint32_t* __restrict__ count) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = tid; q < pieces; q += stride)
        count[q] = (uint32_t)((cuts[q + n_long] - cuts[q] + kFapItemEdges - 1) / kFapItemEdges);
}

// offset[q]: items of the pieces before q (an exclusive scan of count)
__global__ void __launch_bounds__(256) k_item_fill(const int64_t* __restrict__ cuts, int32_t n_long, int64_t pieces,
                                                   const uint32_t* __restrict__ offset, FapItem* __restrict__ items) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = tid; q < pieces; q += stride) {
        const int64_t e1 = cuts[q + n_long];
        int64_t e = cuts[q];
        const int32_t k = (int32_t)(q % n_long);
        for (uint32_t at = offset[q]; e < e1; e += kFapItemEdges, ++at) {
            const int64_t left = e1 - e;
            items[at] = FapItem{e, k, (int32_t)(left < kFapItemEdges ? left : kFapItemEdges)};
        }
    }
}

// device allocations of build_fap_items: freed on every way out unless handed over
struct AnnexBuffers {
    unsigned long long* counts = nullptr;
    int32_t* long_rows = nullptr;
    int64_t* cuts = nullptr;
    uint32_t *count = nullptr, *offset = nullptr;
    void* temp = nullptr;
    FapItem* items = nullptr;
    ~AnnexBuffers() {
        for (void* p : {(void*)counts, (void*)long_rows, (void*)cuts, (void*)count, (void*)offset, temp, (void*)items})
            if (p) (void)hipFree(p);
    }
};

// Fills t's long_rows / long_items.  Not having them only costs speed, so running out of memory here
// is not an error; a failing launch or copy is.
template <typename RP>
qv_status build_fap_items(qv_ctx* ctx, qv_csr* t) {
    const int64_t n = t->n_nodes;
    int log2 = ctx->fap_block_log2 ? ctx->fap_block_log2 : kFapBlockLog2;
    if (t->n_edges <= kLongRow || n <= ((int64_t)1 << log2)) return QV_OK;
    const RP* rp = (const RP*)t->rowptr;
    AnnexBuffers d;
    auto alloc = [](void** p, size_t bytes) {
        if (hipMalloc(p, bytes) == hipSuccess) return true;
        (void)hipGetLastError();
        *p = nullptr;
        return false;
    };
    if (!alloc((void**)&d.counts, 2 * sizeof(unsigned long long))) return QV_OK;
    unsigned long long h_counts[2] = {0, 0};
    const int blocks_n = grid_for(n, 256 * 4, ctx->n_cu * 16);
    QV_HIP(ctx, hipMemsetAsync(d.counts, 0, sizeof(h_counts), ctx->stream));
    hipLaunchKernelGGL((k_long_count<RP>), dim3(blocks_n), dim3(256), 0, ctx->stream, rp, n, d.counts);
    QV_LAUNCH_CHECK(ctx, "k_long_count");
    QV_HIP(ctx, hipMemcpyAsync(h_counts, d.counts, sizeof(h_counts), hipMemcpyDeviceToHost, ctx->stream));
    QV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (h_counts[0] == 0 || h_counts[0] > 0x7FFFFFFFull) return QV_OK;
    const int32_t n_long = (int32_t)h_counts[0];
    const int64_t long_edges = (int64_t)h_counts[1];
    // the items and, while they are made, 16 bytes per piece must fit the limit: larger blocks otherwise
    int64_t blocks = (n + ((int64_t)1 << log2) - 1) >> log2;
    auto too_big = [&](int64_t nb) {
        const size_t pieces = (size_t)nb * (size_t)n_long;
        return pieces * 16 > kFapAnnexMaxBytes ||
               (pieces + (size_t)(long_edges / kFapItemEdges)) * sizeof(FapItem) > kFapAnnexMaxBytes;
    };
    while (blocks >= 2 && too_big(blocks)) {
        ++log2;
        blocks = (n + ((int64_t)1 << log2) - 1) >> log2;
    }
    if (blocks < 2) return QV_OK;
    const int64_t pieces = blocks * n_long;
    size_t temp_bytes = 0;
    if (rocprim::exclusive_scan((void*)nullptr, temp_bytes, (const uint32_t*)nullptr, (uint32_t*)nullptr, 0u, (size_t)pieces,
                                rocprim::plus<uint32_t>(), ctx->stream) != hipSuccess)
        return fail(ctx, QV_EHIP, "qv_csr_transpose: scan sizing failed");
    if (!alloc((void**)&d.long_rows, (size_t)n_long * 4) || !alloc((void**)&d.cuts, (size_t)(pieces + n_long) * sizeof(int64_t)) ||
        !alloc((void**)&d.count, (size_t)pieces * 4) || !alloc((void**)&d.offset, (size_t)pieces * 4) ||
        !alloc(&d.temp, temp_bytes ? temp_bytes : 16))
        return QV_OK;
    QV_HIP(ctx, hipMemsetAsync(d.counts, 0, sizeof(h_counts), ctx->stream));
    hipLaunchKernelGGL((k_long_list<RP>), dim3(blocks_n), dim3(256), 0, ctx->stream, rp, n, d.counts, d.long_rows, n_long);
    QV_LAUNCH_CHECK(ctx, "k_long_list");
    const int blocks_p = grid_for(pieces + n_long, 256, ctx->n_cu * 32);
    hipLaunchKernelGGL((k_long_cuts<RP>), dim3(blocks_p), dim3(256), 0, ctx->stream, rp, t->col, (const int32_t*)d.long_rows, n_long,
                       (int32_t)blocks, log2, d.cuts);
    QV_LAUNCH_CHECK(ctx, "k_long_cuts");
    hipLaunchKernelGGL(k_item_counts, dim3(blocks_p), dim3(256), 0, ctx->stream, (const int64_t*)d.cuts, n_long, pieces, d.count);
    QV_LAUNCH_CHECK(ctx, "k_item_counts");
    QV_HIP(ctx, rocprim::exclusive_scan(d.temp, temp_bytes, (const uint32_t*)d.count, d.offset, 0u, (size_t)pieces,
                                        rocprim::plus<uint32_t>(), ctx->stream));
    uint32_t h_last[2] = {0, 0};                        // items before the last piece, items of the last piece
    QV_HIP(ctx, hipMemcpyAsync(&h_last[0], d.offset + (pieces - 1), 4, hipMemcpyDeviceToHost, ctx->stream));
    QV_HIP(ctx, hipMemcpyAsync(&h_last[1], d.count + (pieces - 1), 4, hipMemcpyDeviceToHost, ctx->stream));
    QV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const int64_t n_items = (int64_t)h_last[0] + (int64_t)h_last[1];
    if (n_items == 0 || !alloc((void**)&d.items, (size_t)n_items * sizeof(FapItem))) return QV_OK;
    hipLaunchKernelGGL(k_item_fill, dim3(blocks_p), dim3(256), 0, ctx->stream, (const int64_t*)d.cuts, n_long, pieces,
                       (const uint32_t*)d.offset, d.items);
    QV_LAUNCH_CHECK(ctx, "k_item_fill");
    QV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    t->long_rows = d.long_rows; d.long_rows = nullptr;
    t->long_items = d.items; d.items = nullptr;
    t->n_items = n_items;
    t->n_long = n_long;
    t->long_blocks = (int32_t)blocks;
    t->long_block_log2 = log2;
    t->long_edges = long_edges;
    return QV_OK;
}

}  // namespace

extern "C" {

qv_status qv_csr_transpose(qv_ctx* ctx, const qv_csr* csr, qv_csr** out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_csr_transpose: ctx is NULL");
    if (!csr || !out) return fail(ctx, QV_EINVAL, "qv_csr_transpose: null argument");
    *out = nullptr;
    const int64_t n = csr->n_nodes, E = csr->n_edges;
    const size_t rp_bytes = (size_t)(n + 1) * (csr->rowptr_bits / 8);
    size_t temp_bytes = 0;
    if (E > 0) {
        hipError_t e = rocprim::radix_sort_pairs((void*)nullptr, temp_bytes, (const int32_t*)nullptr, (int32_t*)nullptr,
                                                 (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)E, 0u, 31u, ctx->stream);
        if (e != hipSuccess) return fail(ctx, QV_EHIP, "qv_csr_transpose: sort sizing failed: %s", hipGetErrorString(e));
    }
    void* rowptr_t = nullptr;
    int32_t *col_t = nullptr, *src = nullptr, *keys_sorted = nullptr;
    void* temp = nullptr;
    auto release = [&](bool all) {
        if (src) (void)hipFree(src);
        if (keys_sorted) (void)hipFree(keys_sorted);
        if (temp) (void)hipFree(temp);
        if (all) {
            if (rowptr_t) (void)hipFree(rowptr_t);
            if (col_t) (void)hipFree(col_t);
        }
    };
    hipError_t a = hipMalloc(&rowptr_t, rp_bytes);
    if (a == hipSuccess && E > 0) a = hipMalloc((void**)&col_t, (size_t)E * 4);
    if (a == hipSuccess && E > 0) a = hipMalloc((void**)&src, (size_t)E * 4);
    if (a == hipSuccess && E > 0) a = hipMalloc((void**)&keys_sorted, (size_t)E * 4);
    if (a == hipSuccess && temp_bytes > 0) a = hipMalloc(&temp, temp_bytes);
    if (a != hipSuccess) {
        (void)hipGetLastError();
        release(true);
        return fail(ctx, a == hipErrorOutOfMemory ? QV_ENOMEM : QV_EHIP,
                    "qv_csr_transpose: device allocation failed (%s); needs about %lld bytes", hipGetErrorString(a),
                    (long long)(rp_bytes + (size_t)E * 12 + temp_bytes));
    }
    qv_status rc = csr->rowptr_bits == 32 ? transpose<int32_t>(ctx, csr, rowptr_t, col_t, src, keys_sorted, temp, temp_bytes)
                                          : transpose<int64_t>(ctx, csr, rowptr_t, col_t, src, keys_sorted, temp, temp_bytes);
    const qv_status sync_rc = qv_ctx_sync(ctx);          // the temporaries are released below
    if (rc == QV_OK) rc = sync_rc;
    release(rc != QV_OK);
    if (rc != QV_OK) return rc;
    qv_csr* t = new (std::nothrow) qv_csr{ctx, ctx->device, n, E, rowptr_t, csr->rowptr_bits, col_t, rowptr_t, col_t};
    if (!t) {
        (void)hipFree(rowptr_t);
        if (col_t) (void)hipFree(col_t);
        return fail(ctx, QV_ENOMEM, "qv_csr_transpose: out of host memory");
    }
    rc = csr->rowptr_bits == 32 ? build_fap_items<int32_t>(ctx, t) : build_fap_items<int64_t>(ctx, t);
    if (rc != QV_OK) {
        qv_csr_destroy(t);
        return rc;
    }
    *out = t;
    return QV_OK;
}

}  // extern "C"
