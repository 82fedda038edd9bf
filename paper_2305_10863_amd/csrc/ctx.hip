// Context, scratch arena, deferred status, CSR handle and its validation kernel.
#include "qv_internal.hpp"
#include <cstring>
#include <new>

namespace qv {

static thread_local std::string g_error;

void set_global_error(const char* msg) { g_error = msg; }

qv_status fail(qv_ctx* ctx, qv_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    else g_error = buf;
    return code;
}

qv_status arena_begin(qv_ctx* ctx, size_t total_bytes) {
    ctx->arena_used = 0;
    if (total_bytes <= ctx->arena_bytes) return QV_OK;
    // earlier calls may still be reading the old arena
    QV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->arena) QV_HIP(ctx, hipFree(ctx->arena));
    ctx->arena = nullptr;
    ctx->arena_bytes = 0;
    size_t want = align_up(total_bytes + total_bytes / 8, 1 << 20);
    QV_HIP(ctx, hipMalloc((void**)&ctx->arena, want));
    ctx->arena_bytes = want;
    return QV_OK;
}

void* arena_take(qv_ctx* ctx, size_t bytes) {
    size_t at = align_up(ctx->arena_used);
    if (at + bytes > ctx->arena_bytes) return nullptr;   // callers size the arena first
    ctx->arena_used = at + bytes;
    return ctx->arena + at;
}

// ---- CSR validation -----------------------------------------------------------------------
template <typename RP>
__global__ void k_validate_csr(int64_t n, int64_t n_edges, const RP* __restrict__ rowptr,
                               const int32_t* __restrict__ col, int32_t* status) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t v = tid; v < n; v += stride) {
        int64_t a = (int64_t)rowptr[v], b = (int64_t)rowptr[v + 1];
        if (b < a || b - a >= (int64_t)0x7FFFFFFF) bad = true;
    }
    if (tid == 0 && ((int64_t)rowptr[0] != 0 || (int64_t)rowptr[n] != n_edges)) bad = true;
    for (int64_t e = tid; e < n_edges; e += stride) {
        int32_t c = col[e];
        if (c < 0 || (int64_t)c >= n) bad = true;
    }
    if (bad) atomicOr(status, kStatInval);
}

}  // namespace qv

using namespace qv;

extern "C" {

qv_status qv_ctx_create(int device, void* hip_stream, qv_ctx** out) {
    if (!out) return fail(nullptr, QV_EINVAL, "qv_ctx_create: out is NULL");
    *out = nullptr;
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess || device < 0 || device >= n_dev)
        return fail(nullptr, QV_EHIP, "qv_ctx_create: no GPU %d (%s, %d visible)", device,
                    hipGetErrorString(e), n_dev);
    qv_ctx* ctx = new (std::nothrow) qv_ctx();
    if (!ctx) return fail(nullptr, QV_ENOMEM, "qv_ctx_create: out of host memory");
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    hipDeviceProp_t prop;
    if ((e = hipSetDevice(device)) != hipSuccess ||
        (e = hipGetDeviceProperties(&prop, device)) != hipSuccess ||
        (e = hipMalloc((void**)&ctx->d_status, 256)) != hipSuccess ||
        (e = hipHostMalloc((void**)&ctx->h_status, 256, hipHostMallocDefault)) != hipSuccess ||
        (e = hipMemsetAsync(ctx->d_status, 0, 256, ctx->stream)) != hipSuccess) {
        (void)hipGetLastError();
        qv_status rc = fail(nullptr, QV_EHIP, "qv_ctx_create: %s", hipGetErrorString(e));
        qv_ctx_destroy(ctx);
        return rc;
    }
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    qv_status rc = static_scratch_bind(ctx);
    if (rc != QV_OK) {
        set_global_error(ctx->err.c_str());
        qv_ctx_destroy(ctx);
        return rc;
    }
    *out = ctx;
    return QV_OK;
}

void qv_ctx_destroy(qv_ctx* ctx) {
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);
    for (int g = 0; g < QV_STEP_LANES - 1; ++g) {
        if (ctx->lanes[g]) qv_ctx_destroy(ctx->lanes[g]);
        if (ctx->lane_done[g]) (void)hipEventDestroy(ctx->lane_done[g]);
    }
    if (ctx->step_fork) (void)hipEventDestroy(ctx->step_fork);
    if (ctx->arena) (void)hipFree(ctx->arena);
    if (ctx->table_keyw) (void)hipFree(ctx->table_keyw);
    if (ctx->table_slots) (void)hipFree(ctx->table_slots);
    if (ctx->d_status) (void)hipFree(ctx->d_status);
    if (ctx->h_status) (void)hipHostFree(ctx->h_status);
    if (ctx->args_ring) (void)hipHostFree(ctx->args_ring);
    for (int i = 0; i < kArgsRing; ++i)
        if (ctx->args_ev_live[i]) (void)hipEventDestroy(ctx->args_ev[i]);
    if (ctx->owns_stream && ctx->stream) (void)hipStreamDestroy(ctx->stream);
    delete ctx;
}

const char* qv_last_error(const qv_ctx* ctx) { return ctx ? ctx->err.c_str() : g_error.c_str(); }

qv_status qv_ctx_sync(qv_ctx* ctx) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_sync: ctx is NULL");
    QV_HIP(ctx, hipMemcpyAsync(ctx->h_status, ctx->d_status, sizeof(int32_t), hipMemcpyDeviceToHost,
                               ctx->stream));
    QV_HIP(ctx, hipStreamSynchronize(ctx->stream));
    int32_t s = ctx->h_status[0];
    // the groups of qv_step_many that ran on the context's own streams (their work was joined into
    // ctx->stream when it was enqueued, so it is complete by now) report here as well
    for (int g = 0; g < QV_STEP_LANES - 1; ++g) {
        qv_ctx* lane = ctx->lanes[g];
        if (!lane) continue;
        QV_HIP(ctx, hipMemcpyAsync(lane->h_status, lane->d_status, sizeof(int32_t), hipMemcpyDeviceToHost, lane->stream));
        QV_HIP(ctx, hipStreamSynchronize(lane->stream));
        if (lane->h_status[0] != 0) {
            s |= lane->h_status[0];
            QV_HIP(ctx, hipMemsetAsync(lane->d_status, 0, sizeof(int32_t), lane->stream));
        }
    }
    if (s == 0) return QV_OK;
    if (ctx->h_status[0] != 0) QV_HIP(ctx, hipMemsetAsync(ctx->d_status, 0, sizeof(int32_t), ctx->stream));
    if (s & kStatInval) return fail(ctx, QV_EINVAL, "device check failed: malformed input (e.g. repeated known ids)");
    if (s & kStatRange) return fail(ctx, QV_ERANGE, "device check failed: an id was outside [0, n)");
    return fail(ctx, QV_ECAPACITY, "device check failed: an output array was too small; results are truncated");
}

// ---- qv_step_many ---------------------------------------------------------------------------
static qv_status step_lane(qv_ctx* ctx, int g, qv_ctx** out) {
    if (!ctx->lanes[g]) {
        hipStream_t s = nullptr;
        QV_HIP(ctx, hipSetDevice(ctx->device));
        QV_HIP(ctx, hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        qv_ctx* lane = nullptr;
        const qv_status rc = qv_ctx_create(ctx->device, (void*)s, &lane);
        if (rc != QV_OK) {
            (void)hipStreamDestroy(s);
            return fail(ctx, rc, "qv_step_many: internal context: %s", qv_last_error(nullptr));
        }
        lane->owns_stream = true;
        ctx->lanes[g] = lane;
    }
    if (!ctx->lane_done[g]) QV_HIP(ctx, hipEventCreateWithFlags(&ctx->lane_done[g], hipEventDisableTiming));
    qv_ctx* lane = ctx->lanes[g];
    lane->direct_budget_bytes = ctx->direct_budget_bytes;      // the caller's settings apply to every group
    lane->dedup_form = ctx->dedup_form;
    lane->part_log2 = ctx->part_log2;
    *out = lane;
    return QV_OK;
}

qv_status qv_step_many(qv_ctx* ctx, const qv_csr* csr, const qv_feat* feat, int32_t n_batches,
                       const int32_t* const* seeds, const int64_t* n_seeds, const int32_t* fanouts,
                       int32_t n_hops, const uint64_t* rng_seeds, uint32_t flags,
                       const qv_sample_out* outs, void* const* rows_out, const int64_t* rows_cap,
                       int64_t out_row_stride_bytes) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_step_many: ctx is NULL");
    if (!csr || !feat || !seeds || !n_seeds || !rng_seeds || !outs || !rows_out || !rows_cap)
        return fail(ctx, QV_EINVAL, "qv_step_many: null argument");
    if (n_batches < 1 || n_batches > QV_MAX_STEP_BATCHES)
        return fail(ctx, QV_EINVAL, "qv_step_many: n_batches %d outside [1, %d]", n_batches, QV_MAX_STEP_BATCHES);
    if (n_hops < 1 || n_hops > QV_MAX_HOPS) return fail(ctx, QV_EINVAL, "qv_step_many: n_hops %d outside [1, %d]", n_hops, QV_MAX_HOPS);
    const int groups = (n_batches + kMaxBatch - 1) / kMaxBatch;
    const int per = (n_batches + groups - 1) / groups;
    qv_ctx* target[QV_STEP_LANES] = {ctx};
    for (int g = 1; g < groups; ++g) {
        const qv_status rc = step_lane(ctx, g - 1, &target[g]);
        if (rc != QV_OK) return rc;
    }
    if (groups > 1) {
        if (!ctx->step_fork) QV_HIP(ctx, hipEventCreateWithFlags(&ctx->step_fork, hipEventDisableTiming));
        QV_HIP(ctx, hipEventRecord(ctx->step_fork, ctx->stream));
        for (int g = 1; g < groups; ++g) QV_HIP(ctx, hipStreamWaitEvent(target[g]->stream, ctx->step_fork, 0));
    }
    // Sampling of every group first, then the gathers.  What the groups gain from each other is that their
    // latency-bound sampling kernels run side by side; a group's sampling beside another's gather gains
    // nothing (both are limited by the memory system: a chain in which group g+1 sampled while group g
    // gathered took as long as the parts one after the other).
    qv_status rc = QV_OK;
    const int32_t* ids[kMaxBatch];
    int64_t n_ids[kMaxBatch];
    const int64_t* n_ids_dev[kMaxBatch];
    for (int pass = 0; pass < 2 && rc == QV_OK; ++pass) {
        for (int g = 0; g < groups && rc == QV_OK; ++g) {
            const int b0 = g * per, nb = (b0 + per <= n_batches ? per : n_batches - b0);
            if (nb <= 0) continue;
            if (pass == 0) {
                rc = qv_sample_many(target[g], csr, nb, seeds + b0, n_seeds + b0, fanouts, n_hops, rng_seeds + b0, flags, outs + b0);
            } else {
                for (int i = 0; i < nb; ++i) {
                    const qv_sample_out& o = outs[b0 + i];
                    ids[i] = o.n_id;
                    n_ids[i] = rows_cap[b0 + i] < o.n_id_cap ? rows_cap[b0 + i] : o.n_id_cap;
                    n_ids_dev[i] = o.node_off + (n_hops + 1);
                }
                rc = qv_gather_many(target[g], feat, nb, ids, n_ids, n_ids_dev, rows_out + b0, out_row_stride_bytes);
            }
            if (rc != QV_OK && target[g] != ctx) ctx->err = target[g]->err;
        }
    }
    // the join happens whatever was enqueued: the caller's stream must not run ahead of the internal ones
    for (int g = 1; g < groups; ++g) {
        QV_HIP(ctx, hipEventRecord(ctx->lane_done[g - 1], target[g]->stream));
        QV_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->lane_done[g - 1], 0));
    }
    return rc;
}

qv_status qv_ctx_set_epoch(qv_ctx* ctx, uint32_t epoch) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_set_epoch: ctx is NULL");
    if (epoch < ctx->epoch) return fail(ctx, QV_EINVAL, "qv_ctx_set_epoch: the epoch counter only moves forward");
    ctx->epoch = epoch > kEpochLimit ? kEpochLimit : epoch;
    return QV_OK;
}

qv_status qv_ctx_set_table_budget(qv_ctx* ctx, int64_t bytes) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_set_table_budget: ctx is NULL");
    if (bytes < 0) return fail(ctx, QV_EINVAL, "qv_ctx_set_table_budget: negative budget");
    ctx->direct_budget_bytes = bytes;
    return QV_OK;
}

qv_status qv_ctx_set_dedup(qv_ctx* ctx, int32_t form, int32_t partitions_log2) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_set_dedup: ctx is NULL");
    if (form < QV_DEDUP_AUTO || form > QV_DEDUP_PARTITIONED) return fail(ctx, QV_EINVAL, "qv_ctx_set_dedup: unknown form %d", form);
    if (partitions_log2 < -1 || partitions_log2 > 8) return fail(ctx, QV_EINVAL, "qv_ctx_set_dedup: partitions_log2 %d outside [-1, 8]", partitions_log2);
    ctx->dedup_form = form;
    ctx->part_log2 = partitions_log2;
    return QV_OK;
}

qv_status qv_ctx_set_fap_direction(qv_ctx* ctx, int32_t direction) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_set_fap_direction: ctx is NULL");
    if (direction < 0 || direction > 2) return fail(ctx, QV_EINVAL, "qv_ctx_set_fap_direction: 0 (choose), 1 (gather) or 2 (scatter)");
    ctx->fap_direction = direction;
    return QV_OK;
}

qv_status qv_ctx_set_fap_block(qv_ctx* ctx, int32_t nodes_log2) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_set_fap_block: ctx is NULL");
    if (nodes_log2 != 0 && (nodes_log2 < 6 || nodes_log2 > 30))
        return fail(ctx, QV_EINVAL, "qv_ctx_set_fap_block: nodes_log2 %d is neither 0 (default) nor in [6, 30]", nodes_log2);
    ctx->fap_block_log2 = nodes_log2;
    return QV_OK;
}

qv_status qv_sample_bounds(int64_t n_seeds, const int32_t* fanouts, int32_t n_hops, int64_t n_nodes, uint32_t flags,
                           int64_t* max_nodes, int64_t* max_edges, int64_t* max_frontier) {
    if (n_seeds < 0 || n_hops < 1 || n_hops > QV_MAX_HOPS || !fanouts || n_nodes < 0)
        return fail(nullptr, QV_EINVAL, "qv_sample_bounds: bad arguments");
    const bool cumulative = (flags & QV_SAMPLE_CUMULATIVE) != 0;
    int64_t f = n_seeds, nodes = n_seeds < n_nodes ? n_seeds : n_nodes, edges = 0, front = n_seeds;
    for (int k = 0; k < n_hops; ++k) {
        if (fanouts[k] < 1 || fanouts[k] > QV_MAX_FANOUT)
            return fail(nullptr, QV_EINVAL, "qv_sample_bounds: fanout %d outside [1, %d]", fanouts[k], QV_MAX_FANOUT);
        int64_t e = f * (int64_t)fanouts[k];
        if (e >= ((int64_t)1 << 31)) return fail(nullptr, QV_EINVAL, "qv_sample_bounds: a hop may exceed 2^31 edges");
        edges += e;
        front += e < n_nodes ? e : n_nodes;
        nodes = nodes + e < n_nodes ? nodes + e : n_nodes;
        f = cumulative ? nodes : (e < n_nodes ? e : n_nodes);
    }
    if (max_nodes) *max_nodes = nodes;
    if (max_edges) *max_edges = edges;
    if (max_frontier) *max_frontier = front;
    return QV_OK;
}

qv_status qv_csr_create(qv_ctx* ctx, int64_t n_nodes, int64_t n_edges, const void* rowptr,
                        int32_t rowptr_bits, const int32_t* col, int32_t validate, qv_csr** out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_csr_create: ctx is NULL");
    if (!out) return fail(ctx, QV_EINVAL, "qv_csr_create: out is NULL");
    *out = nullptr;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31) || n_edges < 0 || !rowptr || (n_edges > 0 && !col))
        return fail(ctx, QV_EINVAL, "qv_csr_create: need 0 <= n_nodes < 2^31, n_edges >= 0, non-null arrays");
    if (rowptr_bits != 32 && rowptr_bits != 64)
        return fail(ctx, QV_EINVAL, "qv_csr_create: rowptr_bits must be 32 or 64");
    if (rowptr_bits == 32 && n_edges >= ((int64_t)1 << 31))
        return fail(ctx, QV_EINVAL, "qv_csr_create: int32 rowptr cannot index %lld edges", (long long)n_edges);
    // The arrays may live in pinned host memory mapped into the GPU (graphs beyond HBM): kernels
    // then read them over the host link.  Translate such pointers to their device view.
    for (const void** pp : {&rowptr, reinterpret_cast<const void**>(&col)}) {
        if (!*pp) continue;
        hipPointerAttribute_t attr;
        hipError_t pe = hipPointerGetAttributes(&attr, *pp);
        if (pe != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, QV_EINVAL, "qv_csr_create: an array is neither device memory nor pinned host memory (%s)",
                        hipGetErrorString(pe));
        }
        if (attr.type == hipMemoryTypeHost) {
            if (!attr.devicePointer) return fail(ctx, QV_EINVAL, "qv_csr_create: pinned host array is not mapped into the device");
            *pp = attr.devicePointer;
        }
    }
    if (validate) {
        qv_status pending = qv_ctx_sync(ctx);       // do not mix with an earlier deferred error
        if (pending != QV_OK) return pending;
        int blocks = grid_for(n_edges > n_nodes ? n_edges : n_nodes, 256 * 8, ctx->n_cu * 8);
        if (rowptr_bits == 32)
            hipLaunchKernelGGL(k_validate_csr<int32_t>, dim3(blocks), dim3(256), 0, ctx->stream, n_nodes,
                               n_edges, (const int32_t*)rowptr, col, ctx->d_status);
        else
            hipLaunchKernelGGL(k_validate_csr<int64_t>, dim3(blocks), dim3(256), 0, ctx->stream, n_nodes,
                               n_edges, (const int64_t*)rowptr, col, ctx->d_status);
        QV_LAUNCH_CHECK(ctx, "k_validate_csr");
        qv_status rc = qv_ctx_sync(ctx);
        if (rc == QV_EINVAL)
            return fail(ctx, QV_EINVAL, "qv_csr_create: malformed CSR (rowptr not monotone from 0 to n_edges, a row "
                                        "of 2^31 or more entries, or a column id outside [0, n_nodes))");
        if (rc != QV_OK) return rc;
    }
    qv_csr* g = new (std::nothrow) qv_csr{ctx, ctx->device, n_nodes, n_edges, rowptr, rowptr_bits, col};
    if (!g) return fail(ctx, QV_ENOMEM, "qv_csr_create: out of host memory");
    *out = g;
    return QV_OK;
}

const void* qv_csr_rowptr(const qv_csr* csr) { return csr ? csr->rowptr : nullptr; }
const int32_t* qv_csr_col(const qv_csr* csr) { return csr ? csr->col : nullptr; }
const void* qv_csr_fap_items(const qv_csr* csr, const int32_t** long_rows, int32_t* n_long, int64_t* n_items,
                             int32_t* block_log2) {
    const bool has = csr && csr->long_items;
    if (long_rows) *long_rows = has ? csr->long_rows : nullptr;
    if (n_long) *n_long = has ? csr->n_long : 0;
    if (n_items) *n_items = has ? csr->n_items : 0;
    if (block_log2) *block_log2 = has ? csr->long_block_log2 : 0;
    return has ? csr->long_items : nullptr;
}

void qv_csr_destroy(qv_csr* csr) {
    if (!csr) return;
    // owned arrays may still be read by work enqueued on the context's stream
    if (csr->owned_rowptr || csr->owned_col) {
        int prev = -1;
        if (hipGetDevice(&prev) == hipSuccess && prev != csr->device) (void)hipSetDevice(csr->device);
        (void)hipDeviceSynchronize();
        if (prev >= 0 && prev != csr->device) (void)hipSetDevice(prev);
    }
    if (csr->owned_rowptr) (void)hipFree(csr->owned_rowptr);
    if (csr->owned_col) (void)hipFree(csr->owned_col);
    if (csr->long_rows) (void)hipFree(csr->long_rows);
    if (csr->long_items) (void)hipFree(csr->long_items);
    delete csr;
}

}  // extern "C"
