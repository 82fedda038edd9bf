// In-edge CSR of a graph, built on the device: the form the gather sweeps of the feature access
// probability read (Section 5.1: p_k[i] sums over the edges that END at i).
//
//   1. src[e]  = the row that edge e belongs to               (one group of lanes per row)
//   2. stable radix sort of the pairs (col[e], src[e]) by col  (rocPRIM; least-significant-digit
//      passes keep equal keys in edge order, so every in-row lists its sources in ascending order)
//   3. rowptr_t[v] = first sorted position whose key is >= v   (boundary detection, no atomics)
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
    *out = t;
    return QV_OK;
}

}  // extern "C"
