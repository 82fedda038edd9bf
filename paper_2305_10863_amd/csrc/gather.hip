// Feature table (HBM tier + host-pinned tier + lookup table) and the row gather.
//
// Gather kernel: a group of LPR lanes (a power of two, up to the whole wave) copies one row with
// the widest vector the row starts allow (16, 8, 4 or 2 bytes per lane), one row per group per
// round with the next row's id already requested, up to kGatherJobs id lists per launch
// (blockIdx.y; a call with more lists is issued as several launches).  Rows of the host tier are
// read by the same loads through the device mapping of pinned host memory (zero-copy), so
// placement never changes the result.
//
// Row starts decide the vector width, not the row length: source tiers and the output may have a
// row stride larger than the row (a multiple of 128 bytes when the library lays the tier out
// itself), and a row whose length is not a multiple of the vector is finished with 2-byte pieces.
// Measured on MI355X, 8 x 157k rows per launch: 2,408-byte rows at a 2,408-byte stride (8-byte
// vectors, every row straddling lines) 3.7 TB/s; at a 2,432-byte stride (19 lines, 16-byte
// vectors) 5.4 TB/s.
#include "qv_internal.hpp"
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

namespace qv {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

constexpr int kGatherJobs = 64;     // id lists per launch: the job table travels in the kernel argument block (4 KB at most)

struct GatherArgs {
    const char* hot;
    const char* cold;
    const int32_t* loc;             // nullptr: row id == hot row
    int64_t n_rows;                 // rows of the table (range check)
    int64_t hot_stride, cold_stride;
    int64_t out_stride;
    int32_t vecs_per_row;           // whole vectors per row
    int32_t tail_pieces;            // 2-byte pieces after the last whole vector
    int32_t tail_at;                // index of the first tail piece (in 2-byte units)
    int32_t* status;
    GatherJob jobs[kGatherJobs];    // one id list / output per blockIdx.y
};

// Output rows are written once and not read again by this kernel: non-temporal stores keep them
// from displacing table lines in the caches.  Measured on MI355X (8 x 62.5k rows of 256 B):
// 53 us with plain stores and four rows in flight per group, 47 us with non-temporal stores and
// one row per group per round (more groups in flight instead of more rows per group).
template <typename V> __device__ __forceinline__ void store_streaming(V* p, V v) { __builtin_nontemporal_store(v, p); }

template <typename V, int LPR, bool TAIL>
__global__ void __launch_bounds__(256) k_gather(GatherArgs a) {
    const GatherJob& job = a.jobs[blockIdx.y];
    const int64_t n_host = job.n_ids;
    const int sub = threadIdx.x % LPR;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / LPR;
    const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / LPR;
    // The id of the first row is requested before the device-side count is known (the id list has
    // n_host entries whatever the count says), so the two loads overlap instead of queueing.
    int32_t id_next = group < n_host ? job.ids[group] : 0;
    int64_t n = n_host;
    if (job.n_ids_dev) { int64_t nd = *job.n_ids_dev; if (nd < n) n = nd; }
    for (int64_t r = group; r < n; r += n_groups) {
        const int32_t id = id_next;
        const int64_t rn = r + n_groups;
        id_next = rn < n ? job.ids[rn] : 0;
        if (id < 0 || (int64_t)id >= a.n_rows) {
            if (sub == 0) atomicOr(a.status, kStatRange);
            continue;
        }
        const char* p = a.hot + (int64_t)id * a.hot_stride;
        if (a.loc) {
            int32_t l = a.loc[id];
            p = l < 0 ? a.cold + (int64_t)(~l) * a.cold_stride : a.hot + (int64_t)l * a.hot_stride;
        }
        const V* src = reinterpret_cast<const V*>(p);
        V* dst = reinterpret_cast<V*>(job.out + r * a.out_stride);
        for (int i = sub; i < a.vecs_per_row; i += LPR) store_streaming(dst + i, src[i]);
        if (TAIL && sub < a.tail_pieces)
            reinterpret_cast<uint16_t*>(dst)[a.tail_at + sub] = reinterpret_cast<const uint16_t*>(src)[a.tail_at + sub];
    }
}

// Workgroups per id list.  A group of lanes that takes many rows one after the other has its next id on
// the way while it copies (and pays its start-up once), but the fewer the workgroups the longer the last
// ones run on after the rest: about 16 rounds of the workgroups the chip holds at once for a launch of
// well under a millisecond, 8 for longer ones, never more than the chip holds per list.  Measured with
// 64 lists per launch, of HBM peak: 256-byte rows 0.78 / 0.80 / 0.80 / 0.78 at 2,048 / 1,024 / 512 / 256
// workgroups per list, 2,408-byte rows 0.69 / 0.70 / 0.73 / 0.73, 400-byte rows 0.70 / 0.71 / 0.71 / 0.73.
static int gather_blocks_per_list(const qv_ctx* ctx, int n_jobs, int64_t bytes_bound) {
    const int resident = ctx->n_cu * 8;
    const int rounds = bytes_bound > ((int64_t)12 << 30) ? 8 : 16;
    int per_list = rounds * resident / n_jobs;
    if (per_list > resident) per_list = resident;
    return per_list < 1 ? 1 : per_list;
}

template <typename V, bool TAIL>
static void launch_gather_vt(qv_ctx* ctx, const GatherArgs& a, int lpr, int64_t max_ids, int n_jobs, int64_t bytes_bound) {
    int64_t threads = max_ids * lpr;
    dim3 grid((unsigned)grid_for(threads, 256, gather_blocks_per_list(ctx, n_jobs, bytes_bound)), (unsigned)n_jobs);
    switch (lpr) {
        case 8: hipLaunchKernelGGL((k_gather<V, 8, TAIL>), grid, dim3(256), 0, ctx->stream, a); break;
        case 16: hipLaunchKernelGGL((k_gather<V, 16, TAIL>), grid, dim3(256), 0, ctx->stream, a); break;
        case 32: hipLaunchKernelGGL((k_gather<V, 32, TAIL>), grid, dim3(256), 0, ctx->stream, a); break;
        default: hipLaunchKernelGGL((k_gather<V, 64, TAIL>), grid, dim3(256), 0, ctx->stream, a); break;
    }
}

template <typename V>
static void launch_gather_v(qv_ctx* ctx, const GatherArgs& a, int lpr, int64_t max_ids, int n_jobs, int64_t bytes_bound) {
    if (a.tail_pieces > 0) launch_gather_vt<V, true>(ctx, a, lpr, max_ids, n_jobs, bytes_bound);
    else launch_gather_vt<V, false>(ctx, a, lpr, max_ids, n_jobs, bytes_bound);
}

static qv_status launch_gather_some(qv_ctx* ctx, const GatherSource& s, const GatherJob* jobs, int n_jobs, int64_t out_stride);

qv_status launch_gather(qv_ctx* ctx, const GatherSource& s, const GatherJob* jobs, int n_jobs, int64_t out_stride) {
    for (int first = 0; first < n_jobs; first += kGatherJobs) {
        const int n = n_jobs - first < kGatherJobs ? n_jobs - first : kGatherJobs;
        const qv_status rc = launch_gather_some(ctx, s, jobs + first, n, out_stride);
        if (rc != QV_OK) return rc;
    }
    return QV_OK;
}

static qv_status launch_gather_some(qv_ctx* ctx, const GatherSource& s, const GatherJob* jobs, int n_jobs, int64_t out_stride) {
    // widest vector that divides every row start
    uintptr_t bits = (uintptr_t)s.hot_stride | (uintptr_t)out_stride | (uintptr_t)s.hot;
    if (s.cold) bits |= (uintptr_t)s.cold_stride | (uintptr_t)s.cold;     // a tier that does not exist constrains nothing
    int64_t max_ids = 0, sum_ids = 0;
    GatherArgs a{s.hot, s.cold, s.loc, s.n_rows, s.hot_stride, s.cold_stride, out_stride, 0, 0, 0, ctx->d_status, {}};
    for (int i = 0; i < n_jobs; ++i) {
        a.jobs[i] = jobs[i];
        if (jobs[i].n_ids > 0) bits |= (uintptr_t)jobs[i].out;
        if (jobs[i].n_ids > max_ids) max_ids = jobs[i].n_ids;
        sum_ids += jobs[i].n_ids;
    }
    const int64_t bytes_bound = 2 * sum_ids * s.row_bytes;      // read + written if every list is full
    if (max_ids == 0) return QV_OK;
    if (bits % 2 != 0 || s.row_bytes % 2 != 0) return fail(ctx, QV_EINVAL, "gather: rows must be 2-byte aligned");
    const int vec = (bits % 16 == 0) ? 16 : (bits % 8 == 0) ? 8 : (bits % 4 == 0) ? 4 : 2;
    a.vecs_per_row = (int32_t)(s.row_bytes / vec);
    a.tail_pieces = (int32_t)((s.row_bytes % vec) / 2);
    a.tail_at = (int32_t)((int64_t)a.vecs_per_row * vec / 2);
    int lpr = 8;                                        // at least 8 lanes so that a tail (< 16 bytes) fits
    while (lpr < 64 && lpr < a.vecs_per_row) lpr <<= 1;
    switch (vec) {
        case 16: launch_gather_v<v4u>(ctx, a, lpr, max_ids, n_jobs, bytes_bound); break;
        case 8: launch_gather_v<v2u>(ctx, a, lpr, max_ids, n_jobs, bytes_bound); break;
        case 4: launch_gather_v<uint32_t>(ctx, a, lpr, max_ids, n_jobs, bytes_bound); break;
        default: launch_gather_v<uint16_t>(ctx, a, lpr, max_ids, n_jobs, bytes_bound); break;
    }
    QV_LAUNCH_CHECK(ctx, "k_gather");
    return QV_OK;
}

// Row stride for a tier the library lays out itself: the next multiple of 128 bytes when that
// costs at most 1/32 more memory, else the row length rounded up to 16 bytes.
static int64_t owned_stride(int64_t row_bytes) {
    const int64_t lines = (row_bytes + 127) / 128 * 128;
    if ((lines - row_bytes) * 32 <= row_bytes) return lines;
    return (row_bytes + 15) / 16 * 16;
}

}  // namespace qv

using namespace qv;

extern "C" {

void qv_feat_destroy(qv_feat* f) {
    if (!f) return;
    // any context's stream may still be gathering from this table, and the creating context may be
    // gone already: wait for the device the memory lives on
    int prev = -1;
    if (hipGetDevice(&prev) == hipSuccess && prev != f->device) (void)hipSetDevice(f->device);
    (void)hipDeviceSynchronize();
    if (prev >= 0 && prev != f->device) (void)hipSetDevice(prev);
    if (f->hot_owned) (void)hipFree(f->hot_owned);
    if (f->cold_host) (void)hipHostFree(f->cold_host);
    if (f->loc) (void)hipFree(f->loc);
    delete f;
}

int64_t qv_feat_hot_rows(const qv_feat* f) { return f ? f->n_hot : 0; }
const int32_t* qv_feat_loc(const qv_feat* f) { return f ? f->loc : nullptr; }
int64_t qv_feat_row_stride(const qv_feat* f) { return f ? f->hot_stride : 0; }

qv_status qv_feat_create(qv_ctx* ctx, const void* table, int32_t table_on_device, int64_t n_rows, int32_t dim,
                         int32_t elem_bytes, int64_t hbm_budget_bytes, const int32_t* rank, int32_t flags,
                         qv_feat** out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_feat_create: ctx is NULL");
    if (!out) return fail(ctx, QV_EINVAL, "qv_feat_create: out is NULL");
    *out = nullptr;
    if (!table || n_rows < 0 || n_rows >= ((int64_t)1 << 31) || dim < 1 || (elem_bytes != 2 && elem_bytes != 4))
        return fail(ctx, QV_EINVAL, "qv_feat_create: need a table, 0 <= n_rows < 2^31, dim >= 1, elem_bytes 2 or 4");
    const int64_t row_bytes = (int64_t)dim * elem_bytes;
    const int64_t table_bytes = n_rows * row_bytes;
    const bool all_hot = hbm_budget_bytes < 0 || hbm_budget_bytes >= table_bytes;
    if (!all_hot && !rank) return fail(ctx, QV_EINVAL, "qv_feat_create: a budget below the table size needs `rank`");
    qv_feat* f = new (std::nothrow) qv_feat();
    if (!f) return fail(ctx, QV_ENOMEM, "qv_feat_create: out of host memory");
    f->ctx = ctx; f->device = ctx->device; f->n_rows = n_rows; f->dim = dim; f->elem_bytes = elem_bytes; f->row_bytes = row_bytes;
    f->hot = nullptr; f->hot_owned = nullptr; f->cold_host = nullptr; f->cold_dev = nullptr; f->loc = nullptr;
    f->hot_stride = row_bytes; f->cold_stride = row_bytes;
    f->n_hot = all_hot ? n_rows : hbm_budget_bytes / row_bytes;
    const int64_t pad_stride = owned_stride(row_bytes);
    qv_status rc = QV_OK;
    hipError_t e = hipSuccess;
#define FEAT_TRY(call)                                                                                   \
    if (rc == QV_OK && (e = (call)) != hipSuccess) {                                                      \
        (void)hipGetLastError();                                                                          \
        rc = fail(ctx, e == hipErrorOutOfMemory ? QV_ENOMEM : QV_EHIP, "qv_feat_create: %s failed: %s", #call, \
                  hipGetErrorString(e));                                                                  \
    }
    const GatherSource whole{(const char*)table, nullptr, nullptr, n_rows, row_bytes, row_bytes, row_bytes};
    if (all_hot) {
        const bool relayout = table_on_device && (flags & QV_FEAT_OWN_COPY) && pad_stride != row_bytes;
        if (table_on_device && !relayout) {
            f->hot = (const char*)table;                               // borrowed
        } else if (table_on_device) {
            // private copy with line-aligned rows: an identity gather into the padded layout
            f->hot_stride = pad_stride;
            int32_t* iota = nullptr;
            FEAT_TRY(hipMalloc((void**)&f->hot_owned, (size_t)(n_rows * pad_stride + 256)));
            FEAT_TRY(hipMalloc((void**)&iota, (size_t)n_rows * 4 + 256));
            if (rc == QV_OK) {
                std::vector<int32_t> h;
                try {
                    h.resize((size_t)n_rows);
                } catch (...) { rc = fail(ctx, QV_ENOMEM, "qv_feat_create: out of host memory"); }
                for (int64_t i = 0; i < n_rows && rc == QV_OK; ++i) h[(size_t)i] = (int32_t)i;
                FEAT_TRY(hipMemcpyAsync(iota, h.data(), (size_t)n_rows * 4, hipMemcpyHostToDevice, ctx->stream));
                FEAT_TRY(hipStreamSynchronize(ctx->stream));
            }
            if (rc == QV_OK) {
                GatherJob job{iota, n_rows, nullptr, f->hot_owned};
                rc = launch_gather(ctx, whole, &job, 1, pad_stride);
            }
            FEAT_TRY(hipStreamSynchronize(ctx->stream));
            if (iota) (void)hipFree(iota);
            f->hot = f->hot_owned;
        } else {
            f->hot_stride = pad_stride;
            FEAT_TRY(hipMalloc((void**)&f->hot_owned, (size_t)(n_rows * pad_stride + 256)));
            FEAT_TRY(hipMemcpy2DAsync(f->hot_owned, (size_t)pad_stride, table, (size_t)row_bytes, (size_t)row_bytes,
                                      (size_t)n_rows, hipMemcpyHostToDevice, ctx->stream));
            FEAT_TRY(hipStreamSynchronize(ctx->stream));
            f->hot = f->hot_owned;
        }
    } else {
        const int64_t n_hot = f->n_hot, n_cold = n_rows - n_hot;
        // the HBM tier holds floor(budget / row bytes) rows and never more bytes than the budget: rows are
        // padded to line-aligned strides only where the padded tier still fits
        const int64_t hot_stride = n_hot * pad_stride <= hbm_budget_bytes ? pad_stride : row_bytes;
        f->hot_stride = hot_stride; f->cold_stride = pad_stride;
        std::vector<int32_t> h_rank, h_loc, cold_ids;
        try {
            h_rank.resize((size_t)n_rows); h_loc.assign((size_t)n_rows, -1); cold_ids.reserve((size_t)n_cold);
        } catch (...) { rc = fail(ctx, QV_ENOMEM, "qv_feat_create: out of host memory"); }
        FEAT_TRY(hipMemcpyAsync(h_rank.data(), rank, (size_t)n_rows * 4, hipMemcpyDeviceToHost, ctx->stream));
        FEAT_TRY(hipStreamSynchronize(ctx->stream));
        if (rc == QV_OK) {
            // rank must be a permutation of the row ids
            std::vector<char> seen;
            try {
                seen.assign((size_t)n_rows, 0);
            } catch (...) { rc = fail(ctx, QV_ENOMEM, "qv_feat_create: out of host memory"); }
            for (int64_t i = 0; i < n_rows && rc == QV_OK; ++i) {
                int32_t id = h_rank[i];
                if (id < 0 || id >= n_rows || seen[id]) rc = fail(ctx, QV_EINVAL, "qv_feat_create: rank is not a permutation");
                else seen[id] = 1;
            }
        }
        if (rc == QV_OK) {
            for (int64_t i = 0; i < n_hot; ++i) h_loc[h_rank[i]] = (int32_t)i;
            int32_t c = 0;
            for (int64_t id = 0; id < n_rows; ++id)
                if (h_loc[id] < 0) { h_loc[id] = ~c; ++c; cold_ids.push_back((int32_t)id); }
        }
        FEAT_TRY(hipMalloc((void**)&f->loc, (size_t)n_rows * 4 + 256));
        FEAT_TRY(hipMemcpyAsync(f->loc, h_loc.data(), (size_t)n_rows * 4, hipMemcpyHostToDevice, ctx->stream));
        FEAT_TRY(hipMalloc((void**)&f->hot_owned, (size_t)(n_hot * hot_stride + 256)));
        FEAT_TRY(hipHostMalloc((void**)&f->cold_host, (size_t)(n_cold * pad_stride + 256), hipHostMallocMapped));
        FEAT_TRY(hipHostGetDevicePointer((void**)&f->cold_dev, f->cold_host, 0));
        f->hot = f->hot_owned;
        if (rc == QV_OK && table_on_device) {
            // both tiers are filled by the gather kernel itself (the cold tier through the mapping)
            int32_t* d_cold_ids = nullptr;
            FEAT_TRY(hipMalloc((void**)&d_cold_ids, (size_t)n_cold * 4 + 256));
            FEAT_TRY(hipMemcpyAsync(d_cold_ids, cold_ids.data(), (size_t)n_cold * 4, hipMemcpyHostToDevice, ctx->stream));
            if (rc == QV_OK) {
                GatherJob job{rank, n_hot, nullptr, f->hot_owned};
                rc = launch_gather(ctx, whole, &job, 1, hot_stride);
            }
            if (rc == QV_OK) {
                GatherJob job{d_cold_ids, n_cold, nullptr, (char*)f->cold_dev};
                rc = launch_gather(ctx, whole, &job, 1, pad_stride);
            }
            FEAT_TRY(hipStreamSynchronize(ctx->stream));
            if (d_cold_ids) (void)hipFree(d_cold_ids);
        } else if (rc == QV_OK) {
            const char* src = (const char*)table;
            for (int64_t c = 0; c < n_cold; ++c)
                std::memcpy(f->cold_host + c * pad_stride, src + (int64_t)cold_ids[c] * row_bytes, (size_t)row_bytes);
            // hot rows: stage through pinned memory in chunks
            const int64_t chunk_rows = std::max<int64_t>(1, (64ll << 20) / hot_stride);
            char* stage = nullptr;
            FEAT_TRY(hipHostMalloc((void**)&stage, (size_t)(chunk_rows * hot_stride), hipHostMallocDefault));
            for (int64_t i0 = 0; i0 < n_hot && rc == QV_OK; i0 += chunk_rows) {
                int64_t cnt = std::min(chunk_rows, n_hot - i0);
                for (int64_t i = 0; i < cnt; ++i)
                    std::memcpy(stage + i * hot_stride, src + (int64_t)h_rank[i0 + i] * row_bytes, (size_t)row_bytes);
                FEAT_TRY(hipMemcpyAsync(f->hot_owned + i0 * hot_stride, stage, (size_t)(cnt * hot_stride),
                                        hipMemcpyHostToDevice, ctx->stream));
                FEAT_TRY(hipStreamSynchronize(ctx->stream));
            }
            if (stage) (void)hipHostFree(stage);
        }
        FEAT_TRY(hipStreamSynchronize(ctx->stream));
    }
#undef FEAT_TRY
    if (rc != QV_OK) { std::string keep = ctx->err; qv_feat_destroy(f); ctx->err = keep; return rc; }
    *out = f;
    return QV_OK;
}

static qv_status check_stride(qv_ctx* ctx, const qv_feat* f, int64_t stride, const char* who) {
    if (stride < f->row_bytes || stride % f->elem_bytes != 0)
        return fail(ctx, QV_EINVAL, "%s: out_row_stride_bytes %lld must be >= %lld and a multiple of %d", who,
                    (long long)stride, (long long)f->row_bytes, f->elem_bytes);
    return QV_OK;
}

qv_status qv_gather(qv_ctx* ctx, const qv_feat* f, const int32_t* ids, int64_t n_ids, const int64_t* n_ids_dev,
                    void* out, int64_t out_row_stride_bytes) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_gather: ctx is NULL");
    if (!f || n_ids < 0 || (n_ids > 0 && (!ids || !out))) return fail(ctx, QV_EINVAL, "qv_gather: null or negative argument");
    qv_status rc = check_stride(ctx, f, out_row_stride_bytes, "qv_gather");
    if (rc != QV_OK) return rc;
    GatherJob job{ids, n_ids, n_ids_dev, (char*)out};
    const GatherSource s{f->hot, f->cold_dev, f->loc, f->n_rows, f->row_bytes, f->hot_stride, f->cold_stride};
    return launch_gather(ctx, s, &job, 1, out_row_stride_bytes);
}

qv_status qv_gather_many(qv_ctx* ctx, const qv_feat* f, int32_t n_batches, const int32_t* const* ids, const int64_t* n_ids,
                         const int64_t* const* n_ids_dev, void* const* outs, int64_t out_row_stride_bytes) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_gather_many: ctx is NULL");
    if (!f || !ids || !n_ids || !outs) return fail(ctx, QV_EINVAL, "qv_gather_many: null argument");
    if (n_batches < 1 || n_batches > kMaxBatch) return fail(ctx, QV_EINVAL, "qv_gather_many: n_batches %d outside [1, %d]", n_batches, kMaxBatch);
    qv_status rc = check_stride(ctx, f, out_row_stride_bytes, "qv_gather_many");
    if (rc != QV_OK) return rc;
    GatherJob jobs[kMaxBatch];
    for (int i = 0; i < n_batches; ++i) {
        if (n_ids[i] < 0 || (n_ids[i] > 0 && (!ids[i] || !outs[i]))) return fail(ctx, QV_EINVAL, "qv_gather_many: batch %d: null or negative argument", i);
        jobs[i] = GatherJob{ids[i], n_ids[i], n_ids_dev ? n_ids_dev[i] : nullptr, (char*)outs[i]};
    }
    const GatherSource s{f->hot, f->cold_dev, f->loc, f->n_rows, f->row_bytes, f->hot_stride, f->cold_stride};
    return launch_gather(ctx, s, jobs, n_batches, out_row_stride_bytes);
}

}  // extern "C"
