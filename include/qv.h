/*
 * qv -- the data-parallel hot path of a GNN serving pipeline on one AMD MI355X (gfx950):
 * batched multi-hop neighbour sampling over a CSR graph, dedup + relabel of the sampled ids,
 * gather of the sampled nodes' feature rows into one dense tensor, and the two workload metrics
 * that govern the path: the probabilistic sampled sub-graph size (PSGS) per node and the
 * feature access probability (FAP) per node, which ranks feature rows for placement in HBM
 * versus host memory.  Paper: "Quiver: Supporting GPUs for Low-Latency, High-Throughput GNN
 * Serving with Workload Awareness", arXiv 2305.10863.
 *
 * General rules of this ABI
 *   - Plain C.  Every pointer argument is marked [dev] (device memory of the context's GPU),
 *     [host] (ordinary host memory) or [dev|host].  The caller owns every buffer it passes; the
 *     library owns only its handles and the scratch memory inside a context.
 *   - Every call returns a qv_status (0 = ok, negative = error) and never aborts or throws.
 *     qv_last_error() gives the text of the last error of a context (or, with NULL, of the last
 *     failed handle creation on this thread).
 *   - Work is enqueued on the context's HIP stream and is asynchronous.  Sizes that only the
 *     device knows (how many nodes, edges were produced) are written to device memory; the
 *     caller copies them back after synchronising.  Conditions only the device can detect (an id
 *     out of range, an output array too small) are recorded in a status word that qv_ctx_sync()
 *     returns; kernels never write outside the capacities they were given.
 *   - Graph and feature handles may be used by any context of the same GPU and may outlive the
 *     context that created them; destroying a handle whose memory the library owns waits for the
 *     whole device first.
 *   - One context serves one stream; calls on one context must not overlap.  Use several
 *     contexts (one per stream) to keep several batches in flight.  The context's GPU must be
 *     the calling thread's current device (qv_ctx_create makes it so; a caller that switches
 *     devices switches back before calling).
 *   - ids are int32 (graphs of fewer than 2^31 nodes); rowptr is int32 or int64; offsets int64.
 */
#ifndef QV_H
#define QV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct qv_ctx qv_ctx;    /* device, stream, scratch arena, status word            */
typedef struct qv_csr qv_csr;    /* view of a device-resident CSR graph (borrowed arrays) */
typedef struct qv_feat qv_feat;  /* feature table: HBM tier + host-pinned tier + lookup   */

typedef enum {
    QV_OK = 0,
    QV_EINVAL = -1,     /* bad argument (null pointer, fanout < 1, too many hops, ...)        */
    QV_ENOMEM = -2,     /* device or pinned-host allocation failed                           */
    QV_EHIP = -3,       /* a HIP call failed; text in qv_last_error                          */
    QV_ECAPACITY = -4,  /* an output array was too small; outputs are truncated, not overrun */
    QV_ERANGE = -5      /* a node / row id outside [0, n)                                    */
} qv_status;

#define QV_MAX_HOPS 8
#define QV_MAX_FANOUT 1024
#define QV_MAX_BATCHES 256   /* batches per qv_sample_many / qv_gather_many call */

/* ---------------------------------------------------------------------------------------------
 * Context
 * ------------------------------------------------------------------------------------------ */

/* Create a context on GPU `device` that enqueues on `hip_stream` (a hipStream_t; NULL = the
 * default stream).  The stream is borrowed and must outlive the context. */
qv_status qv_ctx_create(int device, void* hip_stream, qv_ctx** out);
void qv_ctx_destroy(qv_ctx* ctx);
const char* qv_last_error(const qv_ctx* ctx);

/* Wait for the context's stream, then return and clear the deferred device status:
 * QV_OK, QV_ERANGE or QV_ECAPACITY (or QV_EHIP if the stream reports a failure). */
qv_status qv_ctx_sync(qv_ctx* ctx);

/* Grow the scratch arena and the dedup tables now so that later qv_sample / qv_sample_many /
 * qv_reindex calls with at most `n_batches` batches of at most `n_seeds` seeds and these fanouts
 * on a graph of `n_nodes` nodes allocate nothing.  Optional.  1 <= n_batches <= QV_MAX_BATCHES. */
qv_status qv_ctx_reserve(qv_ctx* ctx, int64_t n_seeds, const int32_t* fanouts /*[host]*/,
                         int32_t n_hops, int64_t n_nodes, uint32_t flags /* as for qv_sample */,
                         int32_t n_batches);

/* Dedup tables come in two forms.  When n_nodes x 16 bytes x (batches in the call) is at most
 * `bytes`, the table is addressed directly by node id (no probing, one atomic per sampled
 * edge; the memory is held by the context).  Otherwise an open-addressing hash sized by the
 * batch is used.  Default 16 GiB; 0 selects the hash always.  Results are identical. */
qv_status qv_ctx_set_table_budget(qv_ctx* ctx, int64_t bytes);

/* Which dedup form qv_sample / qv_sample_many use (results are identical; this is a tuning and
 * testing aid).  QV_DEDUP_AUTO (default): the partitioned form (ids split by hash over
 * workgroups that dedup in LDS; nothing kept in HBM between calls) for calls that carry enough
 * edges to pay for its extra kernels (a-priori edge bound x batches >= 8 Mi), the tables above
 * otherwise.  QV_DEDUP_TABLE: always tables.  QV_DEDUP_PARTITIONED: the partitioned form
 * wherever it applies, i.e. layer frontiers with at most 4,194,304 ids per stage.
 * partitions_log2: partitions per batch of the partitioned form as a power of two, 0..8, or -1
 * to let the library settle on a count from what earlier calls report. */
#define QV_DEDUP_AUTO 0
#define QV_DEDUP_TABLE 1
#define QV_DEDUP_PARTITIONED 2
qv_status qv_ctx_set_dedup(qv_ctx* ctx, int32_t form, int32_t partitions_log2);

/* Testing / tuning aid for qv_access_prob when it is given the in-edge CSR: 0 (default) lets every
 * sweep choose between gathering over in-edges and scattering along the out-edges of the nodes
 * that carry mass; 1 always gathers; 2 always scatters.  Results agree to rounding. */
#define QV_FAP_CHOOSE 0
#define QV_FAP_GATHER 1
#define QV_FAP_SCATTER 2
qv_status qv_ctx_set_fap_direction(qv_ctx* ctx, int32_t direction);

/* Testing / tuning aid for qv_csr_transpose: the in-edge CSR it builds cuts every row with more than
 * 8,192 edges into work items whose sources lie in one block of 2^nodes_log2 consecutive node ids,
 * and qv_access_prob then sums those rows block by block (the values of one block stay in the L2
 * caches meanwhile).  0 restores the default (18: 2 MB of fp64 values per block); otherwise 6..30.
 * Graphs that fit one block get no items.  Applies to transposes made after the call. */
qv_status qv_ctx_set_fap_block(qv_ctx* ctx, int32_t nodes_log2);

/* Testing aid.  The dedup tables are never cleared between calls: every call stamps its entries
 * with a fresh epoch number, and only when the counter is exhausted (about 10^6 calls) are the
 * tables cleared once.  This sets the counter so that a test can cross that point quickly. */
qv_status qv_ctx_set_epoch(qv_ctx* ctx, uint32_t epoch);

/* A-priori output sizes of qv_sample (host arithmetic only): most distinct nodes, most edges
 * over all hops, most frontier entries over hops 0..n_hops.  Outputs sized to these bounds can
 * never report QV_ECAPACITY. */
qv_status qv_sample_bounds(int64_t n_seeds, const int32_t* fanouts /*[host]*/, int32_t n_hops,
                           int64_t n_nodes, uint32_t flags /* as for qv_sample */,
                           int64_t* max_nodes, int64_t* max_edges, int64_t* max_frontier);

/* ---------------------------------------------------------------------------------------------
 * Graph  (paper Section 3.2: the graph topology given at deployment)
 * ------------------------------------------------------------------------------------------ */

/* Wrap a CSR of OUT-edges: neighbours of v are col[rowptr[v] .. rowptr[v+1]).  rowptr [dev] has
 * n_nodes+1 entries of rowptr_bits (32 or 64) bits; col [dev] has n_edges int32 entries.  The
 * arrays are borrowed and must outlive the handle.  Either array may instead live in pinned host
 * memory (hipHostMalloc): the kernels then read the topology over the host link, zero-copy
 * (Section 4.3 (3): a graph shared from pinned host memory, for graphs larger than HBM).  With validate != 0 the arrays are checked
 * on the device (rowptr[0] == 0, non-decreasing, rowptr[n] == n_edges, 0 <= col < n_nodes) and
 * a malformed graph returns QV_EINVAL; this synchronises once. */
qv_status qv_csr_create(qv_ctx* ctx, int64_t n_nodes, int64_t n_edges, const void* rowptr,
                        int32_t rowptr_bits, const int32_t* col, int32_t validate, qv_csr** out);
void qv_csr_destroy(qv_csr* csr);

/* The in-edge CSR of a graph (Section 5.1 sums, for each node, over the edges that end at it):
 * row i of the result lists the sources j of the edges j -> i, in ascending order of j (parallel
 * edges stay parallel).  Built on the device (edge sources, one stable radix sort of the edge
 * list by destination, row boundaries from the sorted keys); the new arrays are device memory
 * owned by the handle (rowptr of the same width as the input's; (n_nodes+1)*width + 4*n_edges
 * bytes, plus the work items of the rows longer than 8,192 edges when the graph has more than 2^18
 * nodes: 16 bytes per such row and block of 2^18 node ids and per 256 of their edges, at most
 * 1 GiB) and are freed by qv_csr_destroy.  About 8*n_edges bytes more are held during the call.
 * Synchronises the context's stream.  A symmetric graph is its own in-edge CSR and needs none. */
qv_status qv_csr_transpose(qv_ctx* ctx, const qv_csr* csr, qv_csr** out);
/* Read-only views of a handle's arrays [dev] (for a transposed handle: the library's arrays). */
const void* qv_csr_rowptr(const qv_csr* csr);
const int32_t* qv_csr_col(const qv_csr* csr);
/* The work items of an in-edge CSR built by qv_csr_transpose, or NULL when it has none.  long_rows
 * [dev] int32[*n_long]: the rows with more than 8,192 edges, in no particular order.  Returns items
 * [dev], *n_items records of 16 bytes {int64 first; int32 k; int32 count}: the edges col[first ..
 * first + count) belong to row long_rows[k], 1 <= count <= 256, and their sources all lie in one
 * block of 2^*block_log2 node ids.  The items of a long row cover its edges exactly once; items are
 * listed in ascending order of their block. */
const void* qv_csr_fap_items(const qv_csr* csr, const int32_t** long_rows, int32_t* n_long, int64_t* n_items,
                             int32_t* block_log2);

/* ---------------------------------------------------------------------------------------------
 * Sampling  (paper Section 2.1, overview figure: seed -> layer-1 neighbours -> layer-2 ...;
 * Section 6: "k-hop neighbour sampling without replacement".  The paper prints no sampling
 * algorithm; the random choices are fixed as follows so that results are reproducible.)
 *
 * For frontier node v (global id) in hop k (1-based) with out-degree d and fanout l:
 *   d <= l : all d adjacency positions 0..d-1, in CSR order;
 *   d >  l : Floyd's selection of l distinct positions: for slot s = 0..l-1, j = d-l+s,
 *            t = rand_below(j+1), position = t unless an earlier slot already holds t, else j;
 *            output in slot order.
 *   rand_below(b) = high 64 bits of r64 * b, r64 = (x1 << 32) | x0 of Philox4x32-10 with
 *            key (lo32(rng_seed), hi32(rng_seed)) and counter (v, k, s, 0).
 * ------------------------------------------------------------------------------------------ */

/* One hop.  frontier [dev] int32[n_frontier] (order matters; ids may repeat).
 * off_out [dev] int64[n_frontier+1]: segment f of nbr_out starts at off_out[f];
 * off_out[n_frontier] = number of sampled neighbours.  nbr_out [dev] int32[nbr_cap] receives the
 * segments back to back; entries beyond nbr_cap are dropped and QV_ECAPACITY is deferred.
 * A frontier id outside [0, n_nodes) contributes an empty segment and defers QV_ERANGE. */
qv_status qv_sample_hop(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier,
                        int64_t n_frontier, int32_t fanout, uint64_t rng_seed, int32_t hop,
                        int32_t* nbr_out, int64_t nbr_cap, int64_t* off_out);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): qv_sample_hop with the same arguments and results, but
 * its scratch (row extents and segment offsets of the frontier, tile sums) lives in a fixed
 * device array of the library, about 16 MiB per GPU, held until the process ends.  The call
 * allocates and frees nothing.  n_frontier may be at most QV_NOALLOC_MAX_FRONTIER (QV_EINVAL
 * beyond).  All calls on one GPU share that array, whatever their context: calls that overlap
 * on one GPU race; serialise them (one stream, or events between streams). */
#define QV_NOALLOC_MAX_FRONTIER 1048576
qv_status qv_sample_hop_noalloc(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier,
                                int64_t n_frontier, int32_t fanout, uint64_t rng_seed, int32_t hop,
                                int32_t* nbr_out, int64_t nbr_cap, int64_t* off_out);

/* Output block of qv_sample.  All arrays are caller-allocated [dev] memory. */
typedef struct {
    int32_t* n_id;           /* distinct sampled nodes (global ids), the distinct seeds first,  */
    int64_t n_id_cap;        /*   then new nodes in order of first appearance; local id = index */
    int32_t* row_local;      /* per sampled edge: local id of the expanded node                 */
    int32_t* col_local;      /* per sampled edge: local id of the sampled neighbour             */
    int32_t* nbr_global;     /* per sampled edge: global id of the neighbour (may be NULL)      */
    int64_t edge_cap;        /* capacity of the three edge arrays                               */
    int32_t* frontier;       /* F_0 | F_1 | .. | F_K back to back (may be NULL): F_0 = distinct */
    int64_t frontier_cap;    /*   seeds, F_k = distinct neighbours produced by hop k            */
    int64_t* node_off;       /* [n_hops+2] node_off[0]=0, node_off[k+1] = |n_id| after hop k    */
    int64_t* edge_off;       /* [n_hops+1] hop k's edges are [edge_off[k-1], edge_off[k])       */
    int64_t* frontier_off;   /* [n_hops+2] F_k = frontier[frontier_off[k] .. frontier_off[k+1]) */
} qv_sample_out;

/* Multi-hop sampling + reindex for one batch of seeds [dev] int32[n_seeds] (repeats allowed;
 * they are merged, first occurrence first).  fanouts [host] int32[n_hops], each in
 * [1, QV_MAX_FANOUT]; 1 <= n_hops <= QV_MAX_HOPS.  Edges of a hop are ordered by the position
 * of the expanded node, then slot.  No host synchronisation happens inside the call.
 * flags = 0: hop k expands exactly F_{k-1}, the distinct nodes hop k-1 produced (layer
 *   frontiers: the process the PSGS / FAP recursions of Sections 4.1 and 5.1 model).
 * flags = QV_SAMPLE_CUMULATIVE: hop k expands every node sampled so far (n_id after hop k-1, in
 *   local-id order), which yields the nested bipartite blocks consumed by the GraphSAGE / GAT
 *   layers of the libraries whose samplers the paper adopts (Section 6).  A node expanded again
 *   in a later hop draws afresh (the hop number is part of the random stream).  `frontier` still
 *   receives the distinct neighbours of each hop. */
#define QV_SAMPLE_CUMULATIVE 1u
qv_status qv_sample(qv_ctx* ctx, const qv_csr* csr, const int32_t* seeds, int64_t n_seeds,
                    const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed, uint32_t flags,
                    const qv_sample_out* out);

/* Several independent batches through one set of kernel launches (Section 4.3 (1): several
 * pipelines are multiplexed on one processor so that small requests still fill it).  Batch b is
 * sampled exactly as qv_sample(seeds[b], n_seeds[b], rng_seeds[b], &outs[b]) would sample it; the
 * batches share nothing but the launches.  seeds: [host] array of n_batches [dev] pointers;
 * n_seeds, rng_seeds: [host] arrays; outs: [host] array of output blocks ([dev] arrays inside).
 * 1 <= n_batches <= QV_MAX_BATCHES.  Up to 8 batches travel in the kernel argument block; beyond
 * that the per-batch arguments are copied to the device once per call (a few microseconds).
 * Throughput grows with the batches per call (the fixed cost of a call's 14 launches is shared):
 * on a 111 M-node graph, 1,024 seeds, fanouts 15/10/5: 1.3 x 10^10 sampled edges/s at 32 batches
 * per call, 1.6 x 10^10 at 128, 1.7 x 10^10 at 256. */
qv_status qv_sample_many(qv_ctx* ctx, const qv_csr* csr, int32_t n_batches,
                         const int32_t* const* seeds, const int64_t* n_seeds,
                         const int32_t* fanouts, int32_t n_hops, const uint64_t* rng_seeds,
                         uint32_t flags, const qv_sample_out* outs);

/* Dedup + relabel (Section 2.1: the sampled nodes are collected once each and the sub-graph is
 * expressed over them).  known [dev] int32[n_known]: ids that already have local ids (local id
 * = index; entries must be distinct, else QV_EINVAL is deferred).  nbr [dev] int32[n_nbr].
 *   n_id_out     [dev] int32[n_id_cap]: known, then the ids of nbr not in known, in order of
 *                first appearance;  *n_id_len [dev] = its length
 *   local_out    [dev] int32[n_nbr]: local id of each nbr entry
 *   frontier_out [dev] int32[n_nbr] (may be NULL): the distinct ids of nbr in order of first
 *                appearance, whether known or not;  *frontier_len [dev] = its length */
qv_status qv_reindex(qv_ctx* ctx, const int32_t* known, int64_t n_known, const int32_t* nbr,
                     int64_t n_nbr, int64_t n_nodes /* ids must be < n_nodes; 0 = unchecked */,
                     int32_t* n_id_out, int64_t n_id_cap, int64_t* n_id_len, int32_t* local_out,
                     int32_t* frontier_out, int64_t* frontier_len);

/* ---------------------------------------------------------------------------------------------
 * Features  (Section 2.1: collect the features of all sampled nodes into one tensor;
 * Section 5.2 step (i) and Section 5.3: rows ranked by access probability, the most popular
 * placed in GPU memory, the rest in host memory read by the kernel itself (zero-copy), located
 * through a feature lookup table)
 * ------------------------------------------------------------------------------------------ */

/* Build a feature table of n_rows x dim elements of elem_bytes (2 or 4) bytes.
 *   table          [dev|host] (table_on_device says which) row-major, contiguous.
 *   hbm_budget_bytes  bytes of HBM the table may occupy; < 0 or >= the table size = all in HBM.
 *                  The HBM tier holds floor(budget / row bytes) rows and never exceeds the budget
 *                  (its rows are padded to a line-aligned stride only where that still fits).
 *   rank           [dev] int32[n_rows] placement order (most popular first, e.g. from
 *                  qv_place_rank); required when the budget is smaller than the table.
 *   flags          0, or QV_FEAT_OWN_COPY.
 * All rows in HBM, table on device, no QV_FEAT_OWN_COPY: the table is BORROWED (no copy) and
 * must outlive the handle.  Otherwise the library copies: the first floor(budget / row bytes)
 * rows of `rank` into an HBM tier it owns (hot row i = table[rank[i]]), the remaining rows, in
 * ascending id order, into host-pinned memory it owns and maps into the GPU; the caller's table
 * may be freed after the call returns (the call synchronises).  Tiers the library owns are laid
 * out with their rows starting on 128-byte boundaries when that costs at most 1/32 more memory
 * (e.g. 2,408-byte rows at a 2,432-byte stride), which the gather kernel rewards with wider
 * loads; QV_FEAT_OWN_COPY asks for such a private copy even where borrowing would do. */
#define QV_FEAT_OWN_COPY 1
qv_status qv_feat_create(qv_ctx* ctx, const void* table, int32_t table_on_device, int64_t n_rows,
                         int32_t dim, int32_t elem_bytes, int64_t hbm_budget_bytes,
                         const int32_t* rank, int32_t flags, qv_feat** out);
void qv_feat_destroy(qv_feat* feat);
/* Number of rows held in HBM (== n_rows when everything fits). */
int64_t qv_feat_hot_rows(const qv_feat* feat);
/* Row stride in bytes of the HBM tier (== row bytes for a borrowed table): a good choice for
 * out_row_stride_bytes of the gather calls as well. */
int64_t qv_feat_row_stride(const qv_feat* feat);
/* The lookup table [dev] int32[n_rows]: loc[id] >= 0 -> HBM row, < 0 -> host row ~loc[id];
 * NULL when every row is in HBM in id order. */
const int32_t* qv_feat_loc(const qv_feat* feat);

/* out[r, :] = table[ids[r], :] for r < n_ids, as raw bytes.  ids [dev] int32[n_ids], any order,
 * repeats allowed.  out [dev], row r at byte offset r * out_row_stride_bytes (>= row bytes, a
 * multiple of elem_bytes).  An id outside [0, n_rows) leaves its output row untouched and
 * defers QV_ERANGE.  `n_ids_dev` [dev] (may be NULL): if given, only min(*n_ids_dev, n_ids)
 * rows are gathered, so a gather can follow qv_sample without a host round trip. */
qv_status qv_gather(qv_ctx* ctx, const qv_feat* feat, const int32_t* ids, int64_t n_ids,
                    const int64_t* n_ids_dev, void* out, int64_t out_row_stride_bytes);

/* qv_gather for several id lists in one launch: ids, n_ids_dev, outs are [host] arrays of
 * n_batches [dev] pointers (n_ids_dev may be NULL, or hold NULL entries), n_ids a [host] array.
 * All outputs share out_row_stride_bytes.  1 <= n_batches <= QV_MAX_BATCHES. */
qv_status qv_gather_many(qv_ctx* ctx, const qv_feat* feat, int32_t n_batches,
                         const int32_t* const* ids, const int64_t* n_ids,
                         const int64_t* const* n_ids_dev, void* const* outs,
                         int64_t out_row_stride_bytes);

/* One serving step for many batches: qv_sample_many followed by the gather of every batch's
 * sampled nodes (Section 3.2, components 5 and 6 back to back), with the overlap done inside the
 * library.  Calls of more than QV_MAX_BATCHES batches are cut into up to QV_STEP_LANES groups of at
 * most QV_MAX_BATCHES; the first group runs on the context's stream, the others on streams the
 * context owns, so that the latency-bound sampling kernels of the groups run side by side
 * (Section 4.3 (1): pipelines multiplexed on one processor; worth 5 % at 1,024 batches per call on
 * a 111 M-node graph, nothing up to QV_MAX_BATCHES, where the call is the two calls).
 * Every internal stream starts after the work enqueued on the context's stream so far, and the
 * context's stream continues only after all of them: to the caller the call is ordered on the
 * context's stream like any other.  Batch b is sampled exactly as qv_sample_many would; then
 * rows_out[b] [dev] receives table[n_id[r]] for r < min(|n_id|, rows_cap[b], outs[b].n_id_cap) at
 * byte offset r * out_row_stride_bytes (the count is read on the device: no host round trip).
 * seeds, rows_out: [host] arrays of [dev] pointers; n_seeds, rng_seeds, rows_cap: [host] arrays.
 * 1 <= n_batches <= QV_MAX_STEP_BATCHES.  Deferred errors of all groups are reported by
 * qv_ctx_sync.  A host-side error (bad argument, allocation) returns at once with the failing
 * group's status and message; work of earlier groups may have been enqueued by then, and the
 * streams are joined all the same.  The internal contexts hold scratch of their own (as much as
 * the first group's) and are released with the context. */
#define QV_STEP_LANES 4
#define QV_MAX_STEP_BATCHES (QV_STEP_LANES * QV_MAX_BATCHES)
qv_status qv_step_many(qv_ctx* ctx, const qv_csr* csr, const qv_feat* feat, int32_t n_batches,
                       const int32_t* const* seeds, const int64_t* n_seeds, const int32_t* fanouts,
                       int32_t n_hops, const uint64_t* rng_seeds, uint32_t flags,
                       const qv_sample_out* outs, void* const* rows_out, const int64_t* rows_cap,
                       int64_t out_row_stride_bytes);

/* ---------------------------------------------------------------------------------------------
 * Workload metrics
 * ------------------------------------------------------------------------------------------ */

/* PSGS, Section 4.1:  Q[i] = sum_{k=0..K} q_k[i],  q_0 = 1,
 *   q_k[i] = sum_j delta_{k-1}(i,j) * min(deg(j), l_k),  delta_k = A_1 .. A_k,
 *   A_m[i][j] = min(deg(i), l_m) / deg(i) on every out-edge i->j (the probability that the edge
 *   is taken when min(deg, l_m) of deg neighbours are drawn without replacement).
 * psgs_out [dev] float[n_nodes].  Sums are accumulated in fp64 and stored in fp32. */
qv_status qv_psgs(qv_ctx* ctx, const qv_csr* csr, const int32_t* fanouts /*[host]*/,
                  int32_t n_hops, float* psgs_out);

/* Sum of PSGS over a batch of seeds (Section 4.2.2: the quantity compared with the chosen
 * threshold to decide where a batch is sampled).  psgs [dev] float[n_nodes], seeds [dev],
 * sum_out [dev] double[1]. */
qv_status qv_psgs_batch_sum(qv_ctx* ctx, const float* psgs, int64_t n_nodes, const int32_t* seeds,
                            int64_t n_seeds, double* sum_out);

/* FAP, Section 5.1:  P[i] = sum_{k=0..K} p_k[i],  p_0 = seed distribution,
 *   p_k[i] = sum_{j -> i} p_{k-1}[j] * A_k[j][i]   (A as above).
 * p0 [dev] float[n_nodes] or NULL for the uniform 1/n_nodes.  prob_out [dev] float[n_nodes].
 * Sums are accumulated in fp64 and stored in fp32.
 * csr_in: the in-edge CSR of the same graph (row i lists the sources j of the edges j -> i), or
 * NULL.  Without it every sweep scatters along out-edges with fp64 atomics.  With it each sweep
 * either gathers over in-edges (no atomics) or, when few nodes carry mass (a sparse p0, or a
 * graph where most nodes have no in-edges), scatters from those nodes only; the choice is made
 * on the device, the call stays asynchronous.  For a symmetric (undirected) graph pass the graph
 * itself; for any other, qv_csr_transpose builds one (and a gather over one it built is faster on
 * graphs with hub rows: those rows are summed block of sources by block of sources). */
qv_status qv_access_prob(qv_ctx* ctx, const qv_csr* csr, const qv_csr* csr_in,
                         const int32_t* fanouts /*[host]*/, int32_t n_hops, const float* p0,
                         float* prob_out);

/* Placement order, Section 5.2 step (i): node ids sorted by prob descending, ties by smaller id.
 * prob [dev] float[n] (no NaNs), rank_out [dev] int32[n]. */
qv_status qv_place_rank(qv_ctx* ctx, const float* prob, int64_t n, int32_t* rank_out);

#ifdef __cplusplus
}
#endif
#endif /* QV_H */
