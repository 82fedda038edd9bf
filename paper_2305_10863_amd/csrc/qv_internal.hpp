// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdarg>
#include <string>
#include "../../include/qv.h"

namespace qv {

constexpr int kWave = 64;               // CDNA wavefront width
constexpr int kScanBlock = 256;         // threads per block of the scan kernels
constexpr int kMaxBatch = QV_MAX_BATCHES;
constexpr int kArgsRing = 8;            // staging slots for per-batch arguments uploaded to the device
// Rows of a graph longer than this are not left to one group of lanes by the whole-graph sweeps (a hub would
// hold its group for milliseconds after the rest of the grid is done): they get a workgroup each, or, in an
// in-edge CSR the library built, are visited block of sources by block of sources.
constexpr int64_t kLongRow = 8192;
constexpr int kFapItemEdges = 256;      // most edges of one work item of the blocked gather
struct FapItem {                        // edges [first, first + count) of col belong to row long_rows[k]
    int64_t first;
    int32_t k, count;
};

// deferred device status bits (qv_ctx::d_status[0])
constexpr int kStatRange = 1;
constexpr int kStatCapacity = 2;
constexpr int kStatInval = 4;

// Dedup table keyed by global node id: 16-byte slots {minpos, lid, lid_epoch}, in one of two forms:
//   direct  slot == node id (n_nodes slots): no probing, one fire-and-forget atomic per sampled
//           edge.  Used when n_nodes x 16 bytes x batches fits the context's table budget.
//   hashed  open addressing with linear probing over a power-of-two number of slots, with a
//           parallel array keyw[slot] = epoch << 32 | key; a slot whose epoch differs from the
//           call's is free.
// Fields:
//   minpos     smallest tagged position at which the key occurred in the newest stage of the
//              newest call: tag = (~epoch & 0xFFFFF) << 44 | (15 - stage) << 40 | position, so a
//              newer call or stage always wins an atomicMin and stale values never need a reset.
//   lid        local id of the key, meaningful only while lid_epoch equals the call's epoch.
// Nothing is cleared between calls; only when the epoch counter is exhausted.
struct alignas(16) TableSlot {
    uint64_t minpos;
    int32_t lid;
    uint32_t lid_epoch;
};
constexpr uint32_t kEpochLimit = 0xFFFFEu;          // epochs 1 .. kEpochLimit, then a full clear

// Sizes that only the device knows while a qv_sample call is in flight.
struct SampleMeta {
    int64_t node_off[QV_MAX_HOPS + 2];
    int64_t edge_off[QV_MAX_HOPS + 1];
    int64_t frontier_off[QV_MAX_HOPS + 2];
    int64_t stage_range[2];            // [begin, end) of the flat id array of stage 0
};

}  // namespace qv

struct qv_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    char* arena = nullptr;             // scratch; grown on demand, never shrunk
    size_t arena_bytes = 0;
    size_t arena_used = 0;             // bump pointer within one API call
    // hash tables live apart from the arena: their contents carry over between calls
    uint64_t* table_keyw = nullptr;    // hashed form only
    qv::TableSlot* table_slots = nullptr;
    size_t table_entries = 0;          // slots allocated (all batches of a call together)
    size_t table_keyw_entries = 0;     // entries allocated in keyw
    int64_t direct_budget_bytes = (int64_t)16 << 30;
    int dedup_form = 0;                // QV_DEDUP_AUTO / _TABLE / _PARTITIONED
    int part_log2 = -1;                // partitions per batch (log2) of the partitioned form, -1 = chosen per call
    int part_auto_log2 = -1;           // ... the count in use when it is chosen per call, and the call shape it was found for
    int64_t part_auto_bound = -1;
    bool part_stats_reset = true;      // the device's report words must be cleared before the next call
    int part_stable = 0;               // reports in a row that left the count alone
    unsigned part_calls = 0;
    int fap_direction = 0;             // qv_access_prob with an in-edge CSR: 0 choose per sweep, 1 gather only, 2 scatter only
    int fap_block_log2 = 0;            // qv_csr_transpose: node ids per block of the long rows' work items (log2), 0 = default
    uint32_t epoch = 0;
    // pinned staging ring for the per-batch arguments of calls with many batches
    void* args_ring = nullptr;
    hipEvent_t args_ev[qv::kArgsRing] = {};
    bool args_ev_live[qv::kArgsRing] = {};
    bool args_ev_used[qv::kArgsRing] = {};
    int args_next = 0;
    int32_t* d_status = nullptr;       // device status word
    int32_t* h_status = nullptr;       // pinned mirror
    int n_cu = 256;
    std::string err;
    // qv_step_many: the contexts (each with a stream of its own) that take the groups after the first,
    // made on first use; fork / join events
    qv_ctx* lanes[QV_STEP_LANES - 1] = {};
    hipEvent_t step_fork = nullptr;
    hipEvent_t lane_done[QV_STEP_LANES - 1] = {};
    bool owns_stream = false;          // a lane's stream belongs to it
};

struct qv_csr {
    qv_ctx* ctx;                       // the creating context (not dereferenced after creation: it may be destroyed first)
    int device = 0;
    int64_t n_nodes, n_edges;
    const void* rowptr;
    int rowptr_bits;
    const int32_t* col;
    void* owned_rowptr = nullptr;      // set when the library allocated the arrays (qv_csr_transpose)
    int32_t* owned_col = nullptr;
    // An in-edge CSR built by qv_csr_transpose lists every row's sources in ascending order.  Its rows
    // longer than qv::kLongRow are also cut into work items for qv_access_prob: runs of at most
    // qv::kFapItemEdges edges whose sources all lie in one block of 2^long_block_log2 node ids, listed block
    // by block, so that a sweep which takes the items in order reads one block's values at a time from the L2
    // caches.  Absent (null) when the graph has no such row or fits one block.
    int32_t* long_rows = nullptr;      // [n_long] the long rows, in no particular order
    qv::FapItem* long_items = nullptr; // [n_items]
    int32_t n_long = 0, long_blocks = 0, long_block_log2 = 0;
    int64_t n_items = 0;
    int64_t long_edges = 0;            // edges of the long rows together
};

struct qv_feat {
    qv_ctx* ctx;                       // the creating context (not dereferenced after creation: it may be destroyed first)
    int device;
    int64_t n_rows, n_hot;
    int32_t dim, elem_bytes;
    int64_t row_bytes;
    int64_t hot_stride, cold_stride;   // row strides of the two tiers (>= row_bytes)
    const char* hot;                   // HBM tier (borrowed or owned)
    char* hot_owned;
    char* cold_host;                   // pinned host allocation (owned)
    const char* cold_dev;              // the same memory as seen from the GPU
    int32_t* loc;                      // lookup table (owned) or nullptr
};

namespace qv {

qv_status fail(qv_ctx* ctx, qv_status code, const char* fmt, ...);
void set_global_error(const char* msg);

#define QV_HIP(ctx, call)                                                                   \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) {                                                             \
            (void)hipGetLastError(); /* reported here: a later launch check must not see it again */ \
            return qv::fail((ctx), e_ == hipErrorOutOfMemory ? QV_ENOMEM : QV_EHIP,         \
                            "%s failed: %s", #call, hipGetErrorString(e_));                 \
        }                                                                                   \
    } while (0)

#define QV_LAUNCH_CHECK(ctx, name)                                                          \
    do {                                                                                    \
        hipError_t e_ = hipGetLastError();                                                  \
        if (e_ != hipSuccess)                                                               \
            return qv::fail((ctx), QV_EHIP, "launch of %s failed: %s", name,                \
                            hipGetErrorString(e_));                                         \
    } while (0)

// scratch arena ---------------------------------------------------------------------------
qv_status arena_begin(qv_ctx* ctx, size_t total_bytes);     // ensure capacity, reset bump pointer
void* arena_take(qv_ctx* ctx, size_t bytes);                // 256-byte aligned slice
inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

inline int grid_for(int64_t work_items, int per_block, int cap) {
    int64_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (int)b;
}

// sample.hip: bind the fixed device scratch of qv_sample_hop_noalloc for the context's GPU (once
// per device; the device must be current)
qv_status static_scratch_bind(qv_ctx* ctx);

// gather.hip: raw row gather used by qv_gather and by tier construction
struct GatherJob {
    const int32_t* ids;
    int64_t n_ids;
    const int64_t* n_ids_dev;
    char* out;
};
struct GatherSource {
    const char* hot;
    const char* cold;
    const int32_t* loc;
    int64_t n_rows, row_bytes, hot_stride, cold_stride;
};
qv_status launch_gather(qv_ctx* ctx, const GatherSource& src, const GatherJob* jobs, int n_jobs,
                        int64_t out_stride);

}  // namespace qv
