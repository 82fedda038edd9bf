// Neighbour sampling (one sub-wave group per frontier node, Philox4x32-10 + Floyd's selection)
// and dedup / relabel.  The reindex has two forms with identical results:
//
//   partitioned  (calls that carry enough edges; layer frontiers): the ids of a stage are dealt by a
//                hash into P partitions per batch and every partition is deduplicated by one
//                workgroup in an LDS table; nothing is kept in HBM between stages or calls and no
//                global atomic is issued per edge.  Launches of a qv_sample / qv_sample_many call:
//                  stage 0:   k_part_seeds for batches of up to 2,048 seeds, else
//                             k_part_deal, k_part_dedup, k_part_assign        (seeds -> F_0, n_id)
//                  per hop k: k_sample, k_part_deal, k_part_dedup, k_part_assign
//                  k_relabel_links   (repeats of a node new in its hop take its local id; sizes exported)
//                See the comment above slot_hash for the three kernels.
//   table        (small calls, cumulative frontiers, stages beyond 4 Mi ids): a table in HBM keyed
//                by global id, addressed directly when the node count allows and by open-addressing
//                hash otherwise; first-occurrence order is recovered from the smallest position at
//                which each id occurs, found with one atomicMin per sampled edge.  Launches:
//                  k_insert_ids, k_flag, k_assign (stage 0); per hop k_sample, k_flag, k_assign; k_relabel.
//
// No host synchronisation anywhere; every kernel takes up to QV_MAX_BATCHES independent batches
// (blockIdx.y, or folded into blockIdx.x in k_part_seeds, k_part_dedup and k_relabel_links).
// A single-pass variant of k_flag + k_assign (tile scan with decoupled look-back) was measured
// and dropped: agent-scope atomics across the eight XCDs cost 1.5-2 us per dependent step, so
// the ticket + publish + look-back chain was slower (12-17 us per stage) than two short kernels
// (4-5 us each).
#include "qv_internal.hpp"
#include <cstring>
#include <mutex>
#include <new>

// Pointers that a kernel reads out of an argument record carry no address space, and the compiler
// then emits FLAT accesses for them.  A FLAT access counts against the LDS counter as well as the
// memory counter, so every wait for an LDS result also waits for all global loads and stores in
// flight.  Kernels therefore work on a copy of the record whose pointers are typed as global
// memory (BatchG below); on the host the qualifier is empty.
#if defined(__HIP_DEVICE_COMPILE__)
#define QV_G __attribute__((address_space(1)))
#else
#define QV_G
#endif

namespace qv {

template <typename T>
__device__ __forceinline__ T QV_G* gptr(T* p) { return (T QV_G*)p; }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load and store the wave has in flight (prefetches, fire-and-forget result stores), which costs a
// full memory round trip per barrier; the kernels that use this one exchange data between their
// threads through LDS alone.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter (node, hop, slot, 0), key = the 64-bit seed.
// Only words 0 and 1 of the output are used.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t philox_r64(uint64_t seed, uint32_t node, uint32_t hop, uint32_t slot) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t c0 = node, c1 = hop, c2 = slot, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32 x 32 -> 64 multiply per product (a single v_mad_u64_u32) instead of a high and a low half
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return ((uint64_t)c1 << 32) | c0;
}
__device__ __forceinline__ uint32_t rand_below(uint64_t seed, uint32_t node, uint32_t hop, uint32_t slot,
                                               uint32_t bound) {
    return (uint32_t)__umul64hi(philox_r64(seed, node, hop, slot), (uint64_t)bound);
}

// ---------------------------------------------------------------------------------------------
// Floyd's selection, all slots of one node at once.
// Slot s draws t_s in [0, base + s] (base = deg - fanout) and keeps it unless an earlier slot
// already holds that value, in which case it takes j_s = base + s.  j_s is larger than anything
// chosen before it, so slot s collides exactly when
//     some r < s drew the same value (t_r == t_s), or
//     t_s == j_r for an r < s that itself collided (only then is j_r in the set).
// The first test is a pairwise compare; the second is a dependency on one earlier slot, resolved
// by propagation (a chain can only point to lower slots, so it ends).
// Must be called by all 64 lanes of the wave; groups of G lanes are independent.
// `first_slot` is the slot number of sub-lane 0 (non-zero only for fanouts above 64, where the
// slots are processed 64 at a time and earlier picks are looked up by the caller).
// ---------------------------------------------------------------------------------------------
template <int G>
__device__ __forceinline__ uint32_t floyd_resolve(uint32_t t, bool active, bool pre_collided, uint32_t base,
                                                  int sub, int first_slot, int n_active) {
    bool dup = pre_collided;
    for (int r = 0; r + 1 < n_active; ++r) {
        uint32_t tr = __shfl(t, r, G);
        dup |= (r < sub) && (tr == t);
    }
    int s = first_slot + sub;
    int dep = -1;
    if (active && !dup && t >= base) {
        int r = (int)(t - base);                 // t == j_r
        if (r < s && r >= first_slot) dep = r - first_slot;
    }
    int known = (!active || dup || dep < 0) ? 1 : 0;
    int coll = (active && dup) ? 1 : 0;
    while (__any(!known)) {
        int src = dep < 0 ? sub : dep;
        int rk = __shfl(known, src, G), rc = __shfl(coll, src, G);
        if (!known && rk) { coll = rc; known = 1; }
    }
    return coll ? base + (uint32_t)s : t;
}

// ---------------------------------------------------------------------------------------------
// hash table
// ---------------------------------------------------------------------------------------------
struct TableView {
    uint64_t QV_G* keyw;            // hashed form only
    TableSlot QV_G* slots;
    uint32_t mask;
    int32_t shift;
    uint32_t epoch;
    int32_t direct;
};

__device__ __forceinline__ uint64_t pos_tag(uint32_t epoch, int stage) {
    return ((uint64_t)((~epoch) & 0xFFFFFu) << 44) | ((uint64_t)(15 - stage) << 40);
}

// Hashed form: returns the slot of `key`, inserting it if absent; 0xFFFFFFFF if the table is
// full.  A slot is free when the epoch in its key word is not the call's epoch.
__device__ __forceinline__ uint32_t table_insert(const TableView& t, uint32_t key) {
    const uint64_t mine = ((uint64_t)t.epoch << 32) | key;
    uint32_t h = ((key * 0x9E3779B1u) >> t.shift) & t.mask;
    for (uint32_t probes = 0; probes <= t.mask; ++probes) {
        unsigned long long* kw = reinterpret_cast<unsigned long long*>(&t.keyw[h]);
        uint64_t cur = __hip_atomic_load(kw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (;;) {
            if (cur == mine) return h;
            if ((uint32_t)(cur >> 32) == t.epoch) break;             // another key of this call
            uint64_t old = atomicCAS(kw, (unsigned long long)cur, (unsigned long long)mine);
            if (old == cur) return h;                                // claimed a free slot
            cur = old;                                               // lost a race: look again
        }
        h = (h + 1) & t.mask;
    }
    return 0xFFFFFFFFu;
}

// Register that `key` occurs at tagged position `tp`; returns the key's slot (0xFFFFFFFF: table
// full).  Direct form: the slot is the key itself and the atomicMin (result unused, so the wave
// does not wait for it) is the only table access per sampled edge.
__device__ __forceinline__ uint32_t table_touch(const TableView& t, uint32_t key, uint64_t tp) {
    const uint32_t slot = t.direct ? key : table_insert(t, key);
    if (slot != 0xFFFFFFFFu) atomicMin(reinterpret_cast<unsigned long long*>(&t.slots[slot].minpos), (unsigned long long)tp);
    return slot;
}

// full clear: after (re)allocation and when the epoch counter wraps
__global__ void k_table_clear(uint64_t* keyw, int64_t n_keyw, TableSlot* slots, int64_t n) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n_keyw; i += stride) keyw[i] = 0ull;            // epoch 0 = never used
    uint4 z;
    z.x = 0xFFFFFFFFu; z.y = 0xFFFFFFFFu; z.z = 0xFFFFFFFFu; z.w = 0u;        // minpos = max, lid = -1, lid_epoch = 0
    uint4* e = reinterpret_cast<uint4*>(slots);
    for (int64_t i = tid; i < n; i += stride) e[i] = z;
}

// ---------------------------------------------------------------------------------------------
// per-batch state and per-launch arguments
// ---------------------------------------------------------------------------------------------
struct BatchArgs {
    const int32_t* seeds;           // stage-0 ids
    int64_t n_seeds;
    uint64_t rng_seed;
    uint64_t* keyw; TableSlot* slots;                  // this batch's table region (slots == NULL: no dedup)
    SampleMeta* meta;
    uint32_t* seed_slot;            // table slot of each stage-0 id
    uint32_t* slot_of;              // table slot of each edge's neighbour
    int32_t* nbr;                   // global id per edge (caller's array or scratch)
    int32_t* row_local; int32_t* col_local;
    int64_t edge_cap;
    int32_t* n_id; int64_t n_id_cap;
    // working frontier F_0 | F_1 | .. (scratch, structure of arrays)
    int32_t* fr_id; int32_t* fr_lid; int64_t* fr_rs; uint32_t* fr_deg; uint32_t* fr_seg; int64_t fr_cap;
    int32_t* fr_user; int64_t fr_user_cap;
    uint16_t* seed_flags;           // stage-0 flags
    uint16_t* flags;                // per edge: first occurrence | new node << 1 | next-hop segment size << 2 | col_local written << 15
    uint32_t* partial;              // [kMaxTiles][3] per-tile counts of the stage being run
    // partitioned dedup (see k_part_dedup); all NULL in the table forms
    uint2* dealt;                   // the stage's (id, position) records, tile by tile, each tile sorted by partition
    int32_t* result;                // per record: what k_part_dedup found out about it (see there)
    uint16_t* run_off;              // [tile][P + 1] where each partition's records start inside the tile's 4096
    uint2* kdealt;                  // n_id dealt the same way, in tiles of 4,096 local ids: (id, local id) records
    uint16_t* krun_off;             // [tile of n_id][P + 1]
    uint32_t* pcount;               // [tile][partition][first, new] populations of the partition's earlier tiles
    uint32_t* tile_seg;             // [tile] next-hop edges produced by the tile's first occurrences
    uint16_t* fr_tile;              // per frontier entry: the tile that produced it (fr_seg is then tile-local)
    int64_t* node_off_out; int64_t* edge_off_out; int64_t* frontier_off_out;
    int64_t* n_id_len_out; int64_t* frontier_len_out;      // stand-alone reindex
};

// BatchArgs as the kernels see it: the same fields, pointers typed as global memory.
struct BatchG {
    const int32_t QV_G* seeds;
    int64_t n_seeds;
    uint64_t rng_seed;
    uint64_t QV_G* keyw;
    TableSlot QV_G* slots;
    SampleMeta QV_G* meta;
    uint32_t QV_G* seed_slot;
    uint32_t QV_G* slot_of;
    int32_t QV_G* nbr;
    int32_t QV_G* row_local;
    int32_t QV_G* col_local;
    int64_t edge_cap;
    int32_t QV_G* n_id;
    int64_t n_id_cap;
    int32_t QV_G* fr_id;
    int32_t QV_G* fr_lid;
    int64_t QV_G* fr_rs;
    uint32_t QV_G* fr_deg;
    uint32_t QV_G* fr_seg;
    int64_t fr_cap;
    int32_t QV_G* fr_user;
    int64_t fr_user_cap;
    uint16_t QV_G* seed_flags;
    uint16_t QV_G* flags;
    uint32_t QV_G* partial;
    uint2 QV_G* dealt;
    int32_t QV_G* result;
    uint16_t QV_G* run_off;
    uint2 QV_G* kdealt;
    uint16_t QV_G* krun_off;
    uint32_t QV_G* pcount;
    uint32_t QV_G* tile_seg;
    uint16_t QV_G* fr_tile;
    int64_t QV_G* node_off_out;
    int64_t QV_G* edge_off_out;
    int64_t QV_G* frontier_off_out;
    int64_t QV_G* n_id_len_out;
    int64_t QV_G* frontier_len_out;
    template <typename Rec>             // BatchArgs in the kernel argument block, or in global memory
    __device__ __forceinline__ explicit BatchG(const Rec& a)
        : seeds(gptr(a.seeds)),
          n_seeds(a.n_seeds),
          rng_seed(a.rng_seed),
          keyw(gptr(a.keyw)),
          slots(gptr(a.slots)),
          meta(gptr(a.meta)),
          seed_slot(gptr(a.seed_slot)),
          slot_of(gptr(a.slot_of)),
          nbr(gptr(a.nbr)),
          row_local(gptr(a.row_local)),
          col_local(gptr(a.col_local)),
          edge_cap(a.edge_cap),
          n_id(gptr(a.n_id)),
          n_id_cap(a.n_id_cap),
          fr_id(gptr(a.fr_id)),
          fr_lid(gptr(a.fr_lid)),
          fr_rs(gptr(a.fr_rs)),
          fr_deg(gptr(a.fr_deg)),
          fr_seg(gptr(a.fr_seg)),
          fr_cap(a.fr_cap),
          fr_user(gptr(a.fr_user)),
          fr_user_cap(a.fr_user_cap),
          seed_flags(gptr(a.seed_flags)),
          flags(gptr(a.flags)),
          partial(gptr(a.partial)),
          dealt(gptr(a.dealt)),
          result(gptr(a.result)),
          run_off(gptr(a.run_off)),
          kdealt(gptr(a.kdealt)),
          krun_off(gptr(a.krun_off)),
          pcount(gptr(a.pcount)),
          tile_seg(gptr(a.tile_seg)),
          fr_tile(gptr(a.fr_tile)),
          node_off_out(gptr(a.node_off_out)),
          edge_off_out(gptr(a.edge_off_out)),
          frontier_off_out(gptr(a.frontier_off_out)),
          n_id_len_out(gptr(a.n_id_len_out)),
          frontier_len_out(gptr(a.frontier_len_out)) {}
};

// BatchG of batch y with its size block addressed from the call header, so that the loads of the
// block do not wait for the argument record.
template <typename A>
__device__ __forceinline__ BatchG batch_of(const A& c, int y) {
    BatchG b(c.batch(y));
    b.meta = gptr(c.meta_base) + y;
    return b;
}



struct CallHeader {
    // graph
    const void* rowptr; const int32_t* col; int64_t n_nodes;
    // table geometry (same for every batch of the call)
    uint32_t mask; int32_t shift; uint32_t epoch; int32_t direct;
    // stage being run
    int32_t stage;                  // 0 = seeds / known ids, k >= 1 = hop k
    int32_t hop;                    // k_sample: hop number fed to the random stream (== stage in qv_sample)
    int32_t fanout;                 // k_sample: this hop's fanout
    int32_t next_fanout;            // k_dedup: fanout of the following hop, 0 = none
    int32_t n_hops;
    int32_t items_per_thread;       // k_flag / k_assign: tile = kScanBlock * items_per_thread positions
    int32_t cumulative;             // hop k expands every node sampled so far, not only F_{k-1}
    int32_t frontier_restart;       // stand-alone reindex: number this stage's frontier from 0
    int32_t expect_all_first;       // stand-alone reindex stage 0: ids must be distinct
    int32_t p_log2;                 // partitioned dedup: log2 of the partitions per batch
    int32_t p_tiles;                // ... and the tiles its per-tile arrays hold
    int32_t deal_all_nodes;         // k_part_deal: the partition count changed: deal all of n_id again, not only its new part
    int32_t deal_blocks;            // k_part_deal: workgroups (per batch) that deal the stage's ids; the rest deal n_id
    uint32_t* part_stats;           // [0] fullest LDS table of the call, [1] deepest split, [2] partitions_log2 + 1 (device, may be NULL)
    int32_t n_batches;
    int32_t* status;
    SampleMeta* meta_base;          // the batches' size blocks, one after the other: a kernel finds batch y's without its argument record
};

// The per-batch arguments travel in the kernel argument block while they fit (up to kInlineBatch
// batches: no upload, lowest latency) and in device memory beyond that (one small copy per call).
constexpr int kInlineBatch = 8;
struct CallInline : CallHeader {
    BatchArgs b[kInlineBatch];
    __device__ __forceinline__ const BatchArgs& batch(int y) const { return b[y]; }
};
struct CallDevice : CallHeader {
    const BatchArgs* b;
    __device__ __forceinline__ const BatchArgs QV_G& batch(int y) const { return *gptr(b + y); }
};
struct CallArgs : CallHeader {      // host side: header + every batch of the call
    BatchArgs b[kMaxBatch];
    const BatchArgs* b_dev = nullptr;       // device copy (calls of more than kInlineBatch batches)
};

__device__ __forceinline__ TableView table_of(const CallHeader& c, const BatchG& b) {
    return TableView{b.keyw, b.slots, c.mask, c.shift, c.epoch, c.direct};
}

// ---------------------------------------------------------------------------------------------
// k_insert_ids: a flat id array -> table, recording the smallest position of every id.
// The stage-0 launch is the first kernel of a call and also resets the scan state.
// ---------------------------------------------------------------------------------------------
template <typename A>
__global__ void __launch_bounds__(256) k_insert_ids(A c) {
    const BatchG b = batch_of(c, blockIdx.y);
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int32_t* ids;
    uint32_t* slot_of;
    int64_t n;
    if (c.stage == 0) {
        ids = b.seeds; slot_of = b.seed_slot; n = b.n_seeds;
        if (tid == 0) {
            SampleMeta* m = b.meta;
            for (int i = 0; i < QV_MAX_HOPS + 2; ++i) { m->node_off[i] = 0; m->frontier_off[i] = 0; }
            for (int i = 0; i < QV_MAX_HOPS + 1; ++i) m->edge_off[i] = 0;
            m->edge_off[1] = b.edge_cap;        // stand-alone reindex: stage 1 is the flat nbr array
            m->stage_range[0] = 0;
            m->stage_range[1] = b.n_seeds;
        }
    } else {                                    // stand-alone reindex, stage 1
        ids = b.nbr; slot_of = b.slot_of; n = b.edge_cap;
    }
    const TableView t = table_of(c, b);
    const uint64_t tag = pos_tag(c.epoch, c.stage);
    for (int64_t i = tid; i < n; i += stride) {
        int32_t id = ids[i];
        uint32_t slot = 0xFFFFFFFFu;
        if (id < 0 || (c.n_nodes >= 0 && (int64_t)id >= c.n_nodes)) {
            atomicOr(c.status, kStatRange);
        } else {
            slot = table_touch(t, (uint32_t)id, tag | (uint64_t)i);
            if (slot == 0xFFFFFFFFu) atomicOr(c.status, kStatCapacity);
        }
        if (!c.direct) slot_of[i] = slot;
    }
}

// ---------------------------------------------------------------------------------------------
// Geometry of the partitioned dedup (k_part_dedup / k_part_assign below)
// ---------------------------------------------------------------------------------------------
constexpr int kPTile = 4096;                        // positions per tile
constexpr int kPThreads = 512;                      // threads per workgroup of k_part_deal and k_part_assign
constexpr int kDThreads = 1024;                     // ... and of k_part_dedup (more waves to hide its LDS chains behind)
constexpr int kDKeys = 4;                           // ids / records a k_part_dedup thread has in flight
constexpr int kPKeys = kPTile / kPThreads;          // positions per thread and tile
constexpr int kPWords = kPTile / 64;                // 64-bit mask words per tile
constexpr int kPCapLog2 = 12;
constexpr int kPCap = 1 << kPCapLog2;               // entries of a partition's LDS table
constexpr uint32_t kPFillMax = kPCap / 8 * 7;       // a table fuller than this splits its partition further
constexpr int kPMaxTiles = 1024;                    // tiles per stage and batch (larger stages use the table forms)
constexpr int kPMaxLog2 = 8;                        // at most 256 partitions per batch
constexpr int kPMaxProbes = 128;                    // longer probe sequences count as overflow (unheard of below kPFillMax)
constexpr int kPMaxSplit = 12;                      // a partition is split into at most 2^12 sub-rounds
constexpr uint32_t kEmptyKey = 0xFFFFFFFFu;

// Partitioned form: a frontier entry carries its segment offset relative to the tile that produced
// it (fr_seg) and that tile's number (fr_tile); the tiles' edge counts (tile_seg) are scanned here,
// once per workgroup, into LDS.  Also publishes the hop's edge count.  All threads must call.
__device__ __forceinline__ void seg_base_prologue(const CallHeader& c, const BatchG& b, uint32_t* s_segbase,
                                                  uint32_t* s_wave, bool publish) {
    SampleMeta* m = b.meta;
    int64_t plen;
    if (c.stage == 1) {
        plen = b.n_seeds;
    } else {
        int64_t pe = m->edge_off[c.stage - 1];
        if (pe > b.edge_cap) pe = b.edge_cap;
        plen = pe - m->edge_off[c.stage - 2];
    }
    if (plen < 0) plen = 0;
    int n_tiles = (int)((plen + kPTile - 1) / kPTile);
    if (n_tiles > c.p_tiles) n_tiles = c.p_tiles;                     // <= kPMaxTiles (host check)
    const int nthr = (int)blockDim.x, tid = (int)threadIdx.x;
    if (n_tiles <= kWave) {                                           // the usual case: one wave scans them all
        if (tid < kWave) {
            const uint32_t x = tid < n_tiles ? b.tile_seg[tid] : 0u;
            uint32_t inc = x;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t y = __shfl_up(inc, o);
                if (tid >= o) inc += y;
            }
            if (tid < n_tiles) s_segbase[tid] = inc - x;
            if (publish && tid == kWave - 1) m->edge_off[c.stage] = m->edge_off[c.stage - 1] + (int64_t)inc;
        }
        lds_barrier();
        return;
    }
    const int per = (n_tiles + nthr - 1) / nthr;                      // consecutive tiles per thread
    uint32_t sum = 0;
    for (int i = 0; i < per; ++i) {
        const int t = tid * per + i;
        if (t < n_tiles) sum += b.tile_seg[t];
    }
    uint32_t inc = sum;
    const int lane = tid % kWave, wave = tid / kWave;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t x = __shfl_up(inc, o);
        if (lane >= o) inc += x;
    }
    if (lane == kWave - 1) s_wave[wave] = inc;
    lds_barrier();
    uint32_t pre = 0, total = 0;
    for (int w = 0; w < nthr / kWave; ++w) {
        if (w < wave) pre += s_wave[w];
        total += s_wave[w];
    }
    uint32_t run = pre + inc - sum;
    for (int i = 0; i < per; ++i) {
        const int t = tid * per + i;
        if (t < n_tiles) { s_segbase[t] = run; run += b.tile_seg[t]; }
    }
    if (publish && tid == 0) m->edge_off[c.stage] = m->edge_off[c.stage - 1] + (int64_t)total;
    lds_barrier();
}

// ---------------------------------------------------------------------------------------------
// k_sample: one group of G lanes per frontier node, fanout <= G
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void emit_edge(const CallHeader& c, const BatchG& b, const TableView& t, uint64_t tag,
                                          int64_t p, int32_t g, int32_t vl) {
    if (p < b.edge_cap) {
        b.nbr[p] = g;
        if (b.row_local) b.row_local[p] = vl;
        if (b.slots) {
            uint32_t slot = 0xFFFFFFFFu;
            if (g < 0 || (int64_t)g >= c.n_nodes) {
                atomicOr(c.status, kStatRange);
            } else {
                slot = table_touch(t, (uint32_t)g, tag | (uint64_t)p);
                if (slot == 0xFFFFFFFFu) atomicOr(c.status, kStatCapacity);
            }
            if (!c.direct) b.slot_of[p] = slot;
        }
    } else {
        atomicOr(c.status, kStatCapacity);
    }
}

// Per round a group of G lanes takes S consecutive frontier entries (S = 1, 2, 4 or 8): its first S
// lanes load one entry each, then the group works through them, one per sub-round, the entry's
// fields broadcast inside the group.  The neighbour ids of all S sub-rounds are requested before
// any is stored, so a wave keeps S random col reads per group in flight: with many entries the
// kernel's time is the latency of those reads.  S is what is left of the frontier divided by the
// groups of the grid, at most 8.
template <int G, typename A>
__global__ void __launch_bounds__(256) k_sample(A c) {
    const BatchG b = batch_of(c, blockIdx.y);
    const int lane = threadIdx.x % kWave, sub = lane % G;
    const SampleMeta QV_G* m = b.meta;
    const int64_t fbeg = c.cumulative ? 0 : m->frontier_off[c.stage - 1];
    const int64_t F = c.cumulative ? m->node_off[c.stage] : m->frontier_off[c.stage] - fbeg;
    const int64_t ebase = m->edge_off[c.stage - 1];
    const TableView t = table_of(c, b);
    const uint64_t tag = pos_tag(c.epoch, c.stage);
    const uint32_t l = (uint32_t)c.fanout;
    const int32_t QV_G* col = gptr(c.col);
    __shared__ uint32_t s_segbase[kPMaxTiles];
    __shared__ uint32_t s_wave[256 / kWave];
    const bool tiled = b.tile_seg != nullptr;
    if (tiled) seg_base_prologue(c, b, s_segbase, s_wave, blockIdx.x == 0);
    constexpr int kAhead = 8;                                   // most sub-rounds per round
    constexpr int groups_per_wave = kWave / G;
    const int64_t n_groups = (int64_t)gridDim.x * (256 / G);
    const int64_t wave_global = (int64_t)blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    // The loops are uniform over the grid: every lane runs the same number of iterations.  Every round
    // deals what is left evenly over all groups (S entries each, at most kAhead), so the last round keeps
    // the whole grid busy for a short while instead of a part of it for a full round.
    for (int64_t done = 0; done < F;) {
        const int64_t left = F - done;
        const int S = left >= n_groups * kAhead ? kAhead : (int)((left + n_groups - 1) / n_groups);
        const int64_t w0 = done + wave_global * (groups_per_wave * S);
        done += n_groups * S;
        const int64_t f = w0 + (int64_t)(lane / G) * S + sub;   // a group's S entries are consecutive
        uint32_t d_own = 0, off_own = 0, rs_lo = 0, rs_hi = 0;
        int32_t v_own = 0, vl_own = -1;
        if (sub < S && f < F) {
            v_own = b.fr_id[fbeg + f];
            const int64_t rs = b.fr_rs[fbeg + f];
            rs_lo = (uint32_t)rs; rs_hi = (uint32_t)((uint64_t)rs >> 32);
            d_own = b.fr_deg[fbeg + f];
            off_own = b.fr_seg[fbeg + f];
            if (tiled) off_own += s_segbase[b.fr_tile[fbeg + f]];
            vl_own = b.fr_lid[fbeg + f];
        }
        int32_t g[kAhead];
#pragma unroll
        for (int j = 0; j < kAhead; ++j) {                      // j: the group's lane whose entry is expanded
            if (j >= S) break;
            const uint32_t d = __shfl(d_own, j, G);
            const bool draw = d > l;
            const uint32_t mcount = draw ? l : d;
            uint32_t pos = (uint32_t)sub;
            if (__any(draw)) {
                const int32_t v = __shfl(v_own, j, G);
                const bool active = draw && (uint32_t)sub < l;
                const uint32_t base = d - l;                    // meaningful only where draw
                uint32_t tdraw = 0xFFFFFFFFu;
                if (active) tdraw = rand_below(b.rng_seed, (uint32_t)v, (uint32_t)c.hop, (uint32_t)sub, base + (uint32_t)sub + 1u);
                const uint32_t pick = floyd_resolve<G>(tdraw, active, false, base, sub, 0, (int)l);
                if (draw) pos = pick;
            }
            // (shuffles stay outside the branch: a lane that is switched off cannot be read from)
            const int64_t rs = (int64_t)(((uint64_t)__shfl(rs_hi, j, G) << 32) | __shfl(rs_lo, j, G));
            g[j] = 0;
            if ((uint32_t)sub < mcount) g[j] = col[rs + pos];
        }
#pragma unroll
        for (int j = 0; j < kAhead; ++j) {
            if (j >= S) break;
            const uint32_t d = __shfl(d_own, j, G);
            const uint32_t off = __shfl(off_own, j, G);
            const int32_t vl = __shfl(vl_own, j, G);
            const uint32_t mcount = d > l ? l : d;
            if ((uint32_t)sub < mcount) emit_edge(c, b, t, tag, ebase + off + sub, g[j], vl);
        }
    }
}

// Fanouts above 64: one wave (= one block) per frontier node, slots processed 64 at a time,
// earlier picks kept in LDS.
template <typename A>
__global__ void __launch_bounds__(64) k_sample_wide(A c) {
    __shared__ uint32_t picks[QV_MAX_FANOUT];
    const BatchG b = batch_of(c, blockIdx.y);
    const int lane = threadIdx.x;
    const SampleMeta* m = b.meta;
    const int64_t fbeg = c.cumulative ? 0 : m->frontier_off[c.stage - 1];
    const int64_t F = c.cumulative ? m->node_off[c.stage] : m->frontier_off[c.stage] - fbeg;
    const int64_t ebase = m->edge_off[c.stage - 1];
    const TableView t = table_of(c, b);
    const uint64_t tag = pos_tag(c.epoch, c.stage);
    const uint32_t l = (uint32_t)c.fanout;
    __shared__ uint32_t s_segbase[kPMaxTiles];
    __shared__ uint32_t s_wave[1];
    const bool tiled = b.tile_seg != nullptr;
    if (tiled) seg_base_prologue(c, b, s_segbase, s_wave, blockIdx.x == 0);
    for (int64_t f = blockIdx.x; f < F; f += gridDim.x) {
        const int32_t v = b.fr_id[fbeg + f];
        const int64_t rs = b.fr_rs[fbeg + f];
        const uint32_t d = b.fr_deg[fbeg + f];
        uint32_t off = b.fr_seg[fbeg + f];
        if (tiled) off += s_segbase[b.fr_tile[fbeg + f]];
        const int32_t vl = b.fr_lid[fbeg + f];
        const bool draw = d > l;
        const uint32_t mcount = draw ? l : d;
        const uint32_t base = d - l;
        for (uint32_t c0 = 0; c0 < mcount; c0 += kWave) {
            const uint32_t s = c0 + (uint32_t)lane;
            uint32_t pos = s;
            if (draw) {
                const bool active = s < l;
                uint32_t tdraw = 0xFFFFFFFFu;
                if (active) tdraw = rand_below(b.rng_seed, (uint32_t)v, (uint32_t)c.hop, s, base + s + 1u);
                bool pre = false;                       // already chosen by a slot of an earlier round?
                for (uint32_t r = 0; r < c0; ++r) pre |= (picks[r] == tdraw);
                const int n_active = (int)((l - c0) < (uint32_t)kWave ? (l - c0) : (uint32_t)kWave);
                pos = floyd_resolve<kWave>(tdraw, active, active && pre, base, lane, (int)c0, n_active);
                __syncthreads();
                if (active) picks[s] = pos;
                __syncthreads();
            }
            if (s < mcount) {
                const int32_t g = c.col[rs + pos];
                emit_edge(c, b, t, tag, ebase + off + s, g, vl);
            }
        }
        __syncthreads();                                // picks are reused by the next node
    }
}

// ---------------------------------------------------------------------------------------------
// block-wide exclusive scan of three counters (256 threads)
// ---------------------------------------------------------------------------------------------
struct Tri { uint32_t a, b, c; };

__device__ __forceinline__ Tri block_scan3(Tri v, Tri& total, uint32_t (*lds)[3]) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    Tri inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        uint32_t xa = __shfl_up(inc.a, o), xb = __shfl_up(inc.b, o), xc = __shfl_up(inc.c, o);
        if (lane >= o) { inc.a += xa; inc.b += xb; inc.c += xc; }
    }
    __syncthreads();                                    // lds may still be read from the last call
    if (lane == kWave - 1) { lds[wave][0] = inc.a; lds[wave][1] = inc.b; lds[wave][2] = inc.c; }
    __syncthreads();
    Tri pre = {0, 0, 0};
    total = {0, 0, 0};
    const int n_waves = blockDim.x / kWave;
    for (int w = 0; w < n_waves; ++w) {
        if (w < wave) { pre.a += lds[w][0]; pre.b += lds[w][1]; pre.c += lds[w][2]; }
        total.a += lds[w][0]; total.b += lds[w][1]; total.c += lds[w][2];
    }
    return {pre.a + inc.a - v.a, pre.b + inc.b - v.b, pre.c + inc.c - v.c};
}

// ---------------------------------------------------------------------------------------------
// k_flag / k_assign: first occurrences of a stage's ids -> frontier, n_id, local ids, extents.
// Position p of the stage is a first occurrence iff the table's smallest tagged position for
// its id is p itself; it is a new node iff that id has no local id yet.
// ---------------------------------------------------------------------------------------------
constexpr int kMaxTiles = 1024;         // tiles per stage (k_assign sums the counts of earlier tiles itself)

struct StageView {
    int64_t begin, end;
    const int32_t QV_G* ids;
    const uint32_t QV_G* slot_of;
    uint16_t QV_G* flags;
};

__device__ __forceinline__ StageView stage_view(const CallHeader& c, const BatchG& b) {
    StageView v;
    const SampleMeta* m = b.meta;
    if (c.stage == 0) {
        v.begin = m->stage_range[0]; v.end = m->stage_range[1];
        v.ids = b.seeds; v.slot_of = b.seed_slot; v.flags = b.seed_flags;
    } else {
        v.begin = m->edge_off[c.stage - 1]; v.end = m->edge_off[c.stage];
        if (v.end > b.edge_cap) v.end = b.edge_cap;
        v.ids = b.nbr; v.slot_of = b.slot_of; v.flags = b.flags;
    }
    if (v.end < v.begin) v.end = v.begin;
    return v;
}

// slot of the id at position p (0xFFFFFFFF: the id was out of range or the table was full)
__device__ __forceinline__ uint32_t slot_at(const CallHeader& c, const StageView& v, int64_t p, int32_t id) {
    if (!c.direct) return v.slot_of[p];
    return (id >= 0 && (c.n_nodes < 0 || (int64_t)id < c.n_nodes)) ? (uint32_t)id : 0xFFFFFFFFu;
}

template <typename RP, typename A>
__global__ void __launch_bounds__(kScanBlock) k_flag(A c) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const BatchG b = batch_of(c, blockIdx.y);
    const RP* __restrict__ rowptr = static_cast<const RP*>(c.rowptr);
    const StageView v = stage_view(c, b);
    const int64_t tile_size = (int64_t)kScanBlock * c.items_per_thread;
    const int64_t t0 = v.begin + (int64_t)blockIdx.x * tile_size;
    if (t0 >= v.end) return;
    const uint64_t tag = pos_tag(c.epoch, c.stage);
    Tri sum = {0, 0, 0};
    for (int it = 0; it < c.items_per_thread; ++it) {
        const int64_t p = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        if (p < v.end) {
            const int32_t id = v.ids[p];
            const uint32_t slot = slot_at(c, v, p, id);
            uint32_t first = 0, isnew = 0, seg = 0, resolved = 0;
            int32_t known_lid = -1;
            if (slot == 0xFFFFFFFFu) {
                resolved = 1;                                          // bad id: local id -1
            } else {
                // independent loads, issued together: one 16-byte slot, the row extent
                const uint4 sl = *reinterpret_cast<const uint4*>(&b.slots[slot]);
                int64_t rs = 0, re = 0;
                if (c.next_fanout > 0 && !c.cumulative) { rs = (int64_t)rowptr[id]; re = (int64_t)rowptr[id + 1]; }
                const uint64_t mp = ((uint64_t)sl.y << 32) | sl.x;
                first = (mp == (tag | (uint64_t)p)) ? 1u : 0u;
                isnew = (first && sl.w != c.epoch) ? 1u : 0u;          // no local id in this call yet
                if (sl.w == c.epoch) { resolved = 1; known_lid = (int32_t)sl.z; }   // numbered by an earlier stage
                if (first && !c.cumulative) {
                    const uint32_t d = (uint32_t)(re - rs);
                    seg = d < (uint32_t)c.next_fanout ? d : (uint32_t)c.next_fanout;
                }
            }
            if (resolved && c.stage > 0) b.col_local[p] = known_lid;
            v.flags[p] = (uint16_t)(first | (isnew << 1) | (seg << 2) | (resolved << 15));
            sum.a += first; sum.b += isnew; sum.c += seg;
        }
    }
    Tri total;
    block_scan3(sum, total, lds);
    if (threadIdx.x == 0) {
        b.partial[blockIdx.x * 3 + 0] = total.a;
        b.partial[blockIdx.x * 3 + 1] = total.b;
        b.partial[blockIdx.x * 3 + 2] = total.c;
    }
}

template <typename RP, typename A>
__global__ void __launch_bounds__(kScanBlock) k_assign(A c) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const BatchG b = batch_of(c, blockIdx.y);
    const RP* __restrict__ rowptr = static_cast<const RP*>(c.rowptr);
    SampleMeta* m = b.meta;
    const StageView v = stage_view(c, b);
    const int64_t tile_size = (int64_t)kScanBlock * c.items_per_thread;
    const int64_t t0 = v.begin + (int64_t)blockIdx.x * tile_size;
    const bool empty_stage = v.end <= v.begin;
    if (t0 >= v.end && !(empty_stage && blockIdx.x == 0)) return;
    const int64_t node_base = m->node_off[c.stage];
    const int64_t fr_base = m->frontier_off[c.stage];
    const int64_t edge_base = m->edge_off[c.stage];
    const int64_t fr_user_base = c.frontier_restart ? 0 : fr_base;
    // counts of all earlier tiles
    Tri pre = {0, 0, 0};
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kScanBlock) {
        pre.a += b.partial[i * 3 + 0]; pre.b += b.partial[i * 3 + 1]; pre.c += b.partial[i * 3 + 2];
    }
    Tri run;
    block_scan3(pre, run, lds);
    for (int it = 0; it < c.items_per_thread; ++it) {
        const int64_t p = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        const uint32_t f = (p < v.end) ? v.flags[p] : 0u;
        const Tri x = {f & 1u, (f >> 1) & 1u, (f >> 2) & 0x7FFu};
        // loads a first occurrence needs, issued before the scan's barriers
        int32_t id = 0, lid = -1;
        uint32_t slot = 0xFFFFFFFFu, deg = 0;
        int64_t rs = 0;
        if (x.a) {
            id = v.ids[p];
            slot = slot_at(c, v, p, id);
            if (!x.b) lid = b.slots[slot].lid;
            if (c.next_fanout > 0 && (!c.cumulative || x.b)) {
                rs = (int64_t)rowptr[id]; deg = (uint32_t)((int64_t)rowptr[id + 1] - rs);
            }
        }
        Tri tot;
        const Tri ex = block_scan3(x, tot, lds);
        if (x.a) {
            const int64_t u = node_base + run.b + ex.b;
            if (x.b) {
                lid = (int32_t)u;
                *reinterpret_cast<unsigned long long*>(&b.slots[slot].lid) =
                    ((unsigned long long)c.epoch << 32) | (unsigned long long)(uint32_t)lid;   // lid + lid_epoch, one store
                if (u < b.n_id_cap) b.n_id[u] = id;
                else atomicOr(c.status, kStatCapacity);
                if (c.stage > 0) b.col_local[p] = lid;
            }
            const int64_t j = (int64_t)run.a + ex.a;
            if (c.cumulative) {
                if (x.b && c.next_fanout > 0) {      // later hops expand every node: entry at its local id
                    const int64_t u = node_base + run.b + ex.b;
                    if (u < b.fr_cap) {
                        b.fr_id[u] = id; b.fr_lid[u] = lid; b.fr_rs[u] = rs; b.fr_deg[u] = deg;
                    } else {
                        atomicOr(c.status, kStatCapacity);
                    }
                }
            } else if (c.next_fanout > 0) {          // the next hop expands this entry
                if (fr_base + j < b.fr_cap) {
                    b.fr_id[fr_base + j] = id;
                    b.fr_lid[fr_base + j] = lid;
                    b.fr_rs[fr_base + j] = rs;
                    b.fr_deg[fr_base + j] = deg;
                    b.fr_seg[fr_base + j] = run.c + ex.c;
                } else {
                    atomicOr(c.status, kStatCapacity);
                }
            }
            if (b.fr_user) {
                if (fr_user_base + j < b.fr_user_cap) b.fr_user[fr_user_base + j] = id;
                else atomicOr(c.status, kStatCapacity);
            }
        }
        run.a += tot.a; run.b += tot.b; run.c += tot.c;
    }
    const bool last = empty_stage || (t0 + tile_size >= v.end);
    if (last && threadIdx.x == 0) {
        m->node_off[c.stage + 1] = node_base + run.b;
        m->frontier_off[c.stage + 1] = fr_base + run.a;
        if (c.next_fanout > 0 && !c.cumulative) m->edge_off[c.stage + 1] = edge_base + run.c;
        if (c.expect_all_first && (int64_t)run.a != v.end - v.begin) atomicOr(c.status, kStatInval);
    }
}

// ---------------------------------------------------------------------------------------------
// cumulative frontiers: before hop k, segment sizes min(deg, fanout_k) of ALL nodes sampled so
// far (entries indexed by local id) -> segment offsets and the hop's edge count
// ---------------------------------------------------------------------------------------------
template <typename A>
__global__ void __launch_bounds__(kScanBlock) k_cum_partial(A c) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const BatchG b = batch_of(c, blockIdx.y);
    const int64_t U = b.meta->node_off[c.stage];
    const int64_t t0 = (int64_t)blockIdx.x * kScanBlock * c.items_per_thread;
    if (t0 >= U) return;
    Tri sum = {0, 0, 0};
    for (int it = 0; it < c.items_per_thread; ++it) {
        const int64_t u = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        if (u < U && u < b.fr_cap) {
            const uint32_t d = b.fr_deg[u];
            sum.a += d < (uint32_t)c.fanout ? d : (uint32_t)c.fanout;
        }
    }
    Tri total;
    block_scan3(sum, total, lds);
    if (threadIdx.x == 0) b.partial[blockIdx.x * 3] = total.a;
}

template <typename A>
__global__ void __launch_bounds__(kScanBlock) k_cum_scan(A c) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const BatchG b = batch_of(c, blockIdx.y);
    SampleMeta* m = b.meta;
    const int64_t U = m->node_off[c.stage];
    const int64_t tile_size = (int64_t)kScanBlock * c.items_per_thread;
    const int64_t t0 = (int64_t)blockIdx.x * tile_size;
    if (t0 >= U && !(U == 0 && blockIdx.x == 0)) return;
    const int64_t edge_base = m->edge_off[c.stage - 1];
    Tri pre = {0, 0, 0}, run;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kScanBlock) pre.a += b.partial[i * 3];
    block_scan3(pre, run, lds);
    uint64_t running = run.a;
    for (int it = 0; it < c.items_per_thread; ++it) {
        const int64_t u = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        Tri v = {0, 0, 0}, tot;
        if (u < U && u < b.fr_cap) {
            const uint32_t d = b.fr_deg[u];
            v.a = d < (uint32_t)c.fanout ? d : (uint32_t)c.fanout;
        }
        const Tri ex = block_scan3(v, tot, lds);
        if (u < U && u < b.fr_cap) b.fr_seg[u] = (uint32_t)(running + ex.a);
        running += tot.a;
    }
    if (threadIdx.x == 0 && (U == 0 || t0 + tile_size >= U)) m->edge_off[c.stage] = edge_base + (int64_t)running;
}

// ---------------------------------------------------------------------------------------------
// k_relabel: local id of every edge's neighbour; export of the sizes
// ---------------------------------------------------------------------------------------------
template <typename A>
__global__ void __launch_bounds__(256) k_relabel(A c) {
    const BatchG b = batch_of(c, blockIdx.y);
    const SampleMeta* m = b.meta;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t end = m->edge_off[c.stage];                // c.stage = last stage
    if (end > b.edge_cap) end = b.edge_cap;
    for (int64_t p = tid; p < end; p += stride) {
        // only repeats of nodes that are new in their hop are still open: positions whose node was
        // numbered by an earlier stage were written by k_flag, first occurrences by k_assign
        const uint32_t f = b.flags[p];
        if ((f & 0x8000u) || (f & 3u) == 3u) continue;
        uint32_t slot;
        if (c.direct) {
            const int32_t g = b.nbr[p];
            slot = (g >= 0 && (c.n_nodes < 0 || (int64_t)g < c.n_nodes)) ? (uint32_t)g : 0xFFFFFFFFu;
        } else {
            slot = b.slot_of[p];
        }
        b.col_local[p] = slot == 0xFFFFFFFFu ? -1 : b.slots[slot].lid;
    }
    if (tid == 0) {
        if (b.node_off_out) for (int i = 0; i < c.n_hops + 2; ++i) b.node_off_out[i] = m->node_off[i];
        if (b.edge_off_out) for (int i = 0; i < c.n_hops + 1; ++i) b.edge_off_out[i] = m->edge_off[i];
        if (b.frontier_off_out) for (int i = 0; i < c.n_hops + 2; ++i) b.frontier_off_out[i] = m->frontier_off[i];
        if (b.n_id_len_out) *b.n_id_len_out = m->node_off[2];
        if (b.frontier_len_out) *b.frontier_len_out = m->frontier_off[2] - m->frontier_off[1];
    }
}

// ---------------------------------------------------------------------------------------------
// Partitioned dedup: the form qv_sample uses for layer frontiers.
//
// The ids of a stage (the seeds, or one hop's sampled neighbours) are split by a hash of the id into
// P partitions per batch, and each partition is deduplicated by one workgroup in a table in LDS.
// All random access of the dedup is thereby LDS access: nothing is kept in HBM between stages, no
// global atomic is issued per edge, and every global access is a coalesced stream.  Three kernels
// per stage:
//   k_part_deal    one workgroup per tile of 4,096 positions: a counting sort of the tile's
//                  (id, position) records by partition, through LDS, into the tile's own region
//                  of `dealt`; run_off says where each partition's run starts inside the tile.
//   k_part_dedup   one workgroup per (batch, partition): loads the nodes numbered by earlier stages
//                  into its table (from n_id, whose index is the local id; every workgroup reads all
//                  of n_id and keeps its share), then walks its runs, a wave per tile: pass 1
//                  registers every record (entry claimed if absent, smallest position by atomicMin),
//                  pass 2 writes one result word per record, beside it in `result`:
//                      >= 0   local id of a node numbered earlier | first occurrence in this stage << 30
//                      -1     first occurrence of a new node (k_part_assign numbers it)
//                      <= -2  repeat of a new node: -2 - (its first position); k_relabel_links follows it
//                  and counts the first occurrences and new nodes of every tile (pcount).
//   k_part_assign  one workgroup per tile: brings the results back into position order through LDS,
//                  ranks first occurrences and new nodes, writes local ids, n_id, the next frontier.
// A table that fills beyond kPFillMax (more distinct ids in the partition than LDS holds) makes
// k_part_dedup start over with its partition split into 2, 4, ... sub-rounds by further hash bits,
// one table fill per sub-round; results do not depend on P or on the split.  Its workgroups are
// numbered so that the partitions of one batch land on one XCD (workgroup w runs on XCD w mod 8).
// ---------------------------------------------------------------------------------------------
// Where an id goes inside its partition's table: multiplicative hashing (one multiply; its best bits
// are the top ones).  The table index is the top kPCapLog2 bits, the sub-round of a split partition the
// bits right below them.
__device__ __forceinline__ uint32_t slot_hash(uint32_t key) { return key * 0x9E3779B1u; }
__device__ __forceinline__ uint32_t slot_index(uint32_t h) { return h >> (32 - kPCapLog2); }
__device__ __forceinline__ uint32_t slot_round(uint32_t h, int split) {
    return (h >> (32 - kPCapLog2 - split)) & ((1u << split) - 1u);
}
static_assert(kPCapLog2 + kPMaxSplit <= 32, "table index and sub-round bits come out of one 32-bit hash");
// Partition of an id: full-rate shifts and xors only (a 32-bit multiply costs four of them, and
// k_part_dedup evaluates this for every known node in every workgroup).  Any spread will do:
// the table index inside a partition comes from slot_hash.
__device__ __forceinline__ uint32_t part_of(uint32_t key, int p_log2) {
    uint32_t h = key ^ (key >> 15);
    h ^= h >> 7;
    return h & ((1u << p_log2) - 1u);
}

// entry of `key` in the LDS table, claiming a free one if absent (then *claimed, the caller's own
// counter, goes up by one); -1 when none is found within kPMaxProbes entries, which callers treat
// like a full table (a table filling up would otherwise be walked end to end by every insertion)
__device__ __forceinline__ int lds_insert(uint32_t* t_key, uint32_t key, uint32_t start, uint32_t* claimed) {
    uint32_t s = start;
    for (int probes = 0; probes < kPMaxProbes; ++probes) {
        const uint32_t cur = atomicCAS(&t_key[s], kEmptyKey, key);
        if (cur == kEmptyKey) { ++*claimed; return (int)s; }
        if (cur == key) return (int)s;
        s = (s + 1) & (kPCap - 1);
    }
    return -1;
}

// [begin, end) of the stage's positions, its ids and the number of nodes numbered before it
struct PartStage {
    int64_t begin, end, known;
    const int32_t QV_G* ids;
};
__device__ __forceinline__ PartStage part_stage(const CallHeader& c, const BatchG& b) {
    PartStage v;
    const SampleMeta* m = b.meta;
    if (c.stage == 0) {                 // the size block is initialised by this very stage
        v.begin = 0; v.end = b.n_seeds; v.known = 0; v.ids = b.seeds;
    } else {
        v.begin = m->edge_off[c.stage - 1]; v.end = m->edge_off[c.stage];
        if (v.end > b.edge_cap) v.end = b.edge_cap;
        v.known = m->node_off[c.stage];
        if (v.known > b.n_id_cap) v.known = b.n_id_cap;
        v.ids = b.nbr;
    }
    if (v.end < v.begin) v.end = v.begin;
    const int64_t room = (int64_t)c.p_tiles * kPTile;          // what the per-tile arrays were sized for
    if (v.end - v.begin > room) v.end = v.begin + room;
    return v;
}

constexpr int32_t kResNone = INT32_MIN;            // k_part_assign: a position that was not dealt (id out of range)

template <typename A>
__global__ void __launch_bounds__(kPThreads) k_part_deal(A c) {
    __shared__ uint32_t hist[(1 << kPMaxLog2) + 1], offs[(1 << kPMaxLog2) + 1], wsum[(1 << kPMaxLog2) / kWave];
    static_assert((1 << kPMaxLog2) <= kPThreads, "a thread per partition in the scan");
    __shared__ uint2 sorted[kPTile];
    const BatchG b = batch_of(c, blockIdx.y);
    const int p_log2 = c.p_log2, P = 1 << p_log2;
    const int tid = (int)threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const PartStage v = part_stage(c, b);
    if (c.stage == 0 && blockIdx.x == 0 && tid == 0) {      // first kernel of a call: the size block starts at zero
        SampleMeta QV_G* m = b.meta;
        for (int i = 0; i < QV_MAX_HOPS + 2; ++i) { m->node_off[i] = 0; m->frontier_off[i] = 0; }
        for (int i = 0; i < QV_MAX_HOPS + 1; ++i) m->edge_off[i] = 0;
        m->stage_range[0] = 0; m->stage_range[1] = b.n_seeds;
    }
    const int64_t len = v.end - v.begin;
    const int n_tiles = (int)((len + kPTile - 1) / kPTile);
    const uint32_t n_valid = c.n_nodes >= 0 ? (uint32_t)c.n_nodes : 0x80000000u;   // ids are valid below this (as unsigned)
    // counting sort of the ids src[0 .. n) (n <= 4,096) by partition; the record of src[k] is (id, tag0 + k)
    auto deal_tile = [&](const int32_t QV_G* src, int64_t n, uint32_t tag0, uint2 QV_G* out, uint16_t QV_G* out_off) {
        if (tid <= P) hist[tid] = 0;
        lds_barrier();
        uint32_t key[kPKeys], where[kPKeys];                // where = partition << 16 | rank inside the partition's run
        bool bad = false;
#pragma unroll
        for (int i = 0; i < kPKeys; ++i) {
            const int rel = i * kPThreads + tid;
            key[i] = rel < n ? (uint32_t)src[rel] : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int i = 0; i < kPKeys; ++i) {
            where[i] = 0xFFFFFFFFu;
            if (key[i] < n_valid) {
                const uint32_t part = part_of(key[i], p_log2);
                where[i] = (part << 16) | atomicAdd(&hist[part], 1u);
            } else if (i * kPThreads + tid < n) {
                bad = true;
            }
        }
        if (bad) atomicOr((int*)gptr(c.status), kStatRange);
        lds_barrier();
        // exclusive scan of the run lengths: wave w takes partitions 64 w .. 64 w + 63
        const bool scans = wave * kWave < P;
        uint32_t x = 0, inc = 0;
        if (scans) {
            x = tid < P ? hist[tid] : 0u;
            inc = x;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t y = __shfl_up(inc, o);
                if (lane >= o) inc += y;
            }
            if (lane == kWave - 1) wsum[wave] = inc;
        }
        if (P > kWave) lds_barrier();                       // (uniform: P is a launch argument)
        if (scans) {
            for (int w = 0; w < wave; ++w) inc += wsum[w];
            if (tid < P) {
                offs[tid] = inc - x;
                out_off[tid] = (uint16_t)(inc - x);
            }
            if (tid == P - 1) {
                offs[P] = inc;
                out_off[P] = (uint16_t)inc;
            }
        }
        lds_barrier();
#pragma unroll
        for (int i = 0; i < kPKeys; ++i) {
            if (where[i] == 0xFFFFFFFFu) continue;
            sorted[offs[where[i] >> 16] + (where[i] & 0xFFFFu)] = make_uint2(key[i], tag0 + (uint32_t)(i * kPThreads + tid));
        }
        lds_barrier();
        const uint32_t total = offs[P];
        for (uint32_t k = (uint32_t)tid; k < total; k += kPThreads) out[k] = sorted[k];
        lds_barrier();                                      // hist, offs and sorted are reused by the next tile
    };
    // the stage's ids: records (id, position)
    const int stage_blocks = c.deal_blocks, node_blocks = (int)gridDim.x - stage_blocks;
    for (int t = (int)blockIdx.x; (int)blockIdx.x < stage_blocks && t < n_tiles; t += stage_blocks) {
        const int64_t rel0 = (int64_t)t * kPTile;
        deal_tile(v.ids + v.begin + rel0, len - rel0 < kPTile ? len - rel0 : kPTile, (uint32_t)(v.begin + rel0),
                  b.dealt + (size_t)t * kPTile, b.run_off + (size_t)t * (P + 1));
    }
    // the nodes the previous stage numbered: records (id, local id), in tiles of 4,096 local ids (the
    // tile the previous stage left unfinished is dealt again in full)
    if (c.stage > 0 && (int)blockIdx.x >= stage_blocks) {
        const SampleMeta QV_G* m = b.meta;
        int64_t known = m->node_off[c.stage], before = m->node_off[c.stage - 1];
        if (known > b.n_id_cap) known = b.n_id_cap;
        if (before > known) before = known;
        const int first = c.deal_all_nodes ? 0 : (int)(before / kPTile), end = (int)((known + kPTile - 1) / kPTile);
        for (int j = first + (int)blockIdx.x - stage_blocks; j < end; j += node_blocks) {
            const int64_t u0 = (int64_t)j * kPTile;
            deal_tile(b.n_id + u0, known - u0 < kPTile ? known - u0 : kPTile, (uint32_t)u0,
                      b.kdealt + (size_t)j * kPTile, b.krun_off + (size_t)j * (P + 1));
        }
    }
}

// shared state of one k_part_dedup workgroup
struct alignas(16) PartLds {
    uint32_t t_key[kPCap];                              // the partition's table: id,
    uint32_t t_min[kPCap];                              //   its smallest position in this stage,
    int32_t t_lid[kPCap];                               //   its local id if an earlier stage numbered it, else -1
    uint32_t run_at[kPMaxTiles + 1];                    // records of this partition before tile t (its runs laid end to end)
    uint16_t run_beg[kPMaxTiles];                       // where its run starts inside tile t
    uint32_t cnt[kPMaxTiles];                           // per tile: first occurrences | new nodes << 16 (a tile has 4,096 positions)
    uint32_t s_wave[kDThreads / kWave];
    uint32_t s_fill;                                    // entries claimed (+ kPCap for every insertion that found the table full)
};

template <typename A>
__global__ void __launch_bounds__(kDThreads, 8) k_part_dedup(A c) {     // 8 waves per SIMD: two workgroups per CU
    __shared__ PartLds S;
    const int p_log2 = c.p_log2, P = 1 << p_log2;
    const int q = (int)(blockIdx.x >> 3);
    const int batch = (int)(blockIdx.x & 7u) + 8 * (q >> p_log2);
    const uint32_t part = (uint32_t)(q & (P - 1));
    if (batch >= c.n_batches) return;
    const BatchG b = batch_of(c, batch);
    const int tid = (int)threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const PartStage v = part_stage(c, b);
    const int64_t len = v.end - v.begin;
    const int n_tiles = (int)((len + kPTile - 1) / kPTile);
    // The nodes numbered by earlier stages come from their dealt records, a wave per tile of n_id, a
    // lane per record of the run, kKnownAhead records of a lane requested together.  The order of the
    // insertions (these nodes, the stage's records) does not matter: pass 2 runs after all of them.
    constexpr int kKnownAhead = 3;
    const int n_ktiles = (int)((v.known + kPTile - 1) / kPTile);
    uint32_t kbeg0 = 0, kend0 = 0;                              // extents of the wave's first run of known nodes
    if (wave < n_ktiles) {
        kbeg0 = b.krun_off[(size_t)wave * (P + 1) + part];
        kend0 = b.krun_off[(size_t)wave * (P + 1) + part + 1];
    }
    // Where this partition's records are: its runs, one per tile, are numbered end to end, so that
    // the workgroup's threads can share them evenly whatever the runs' lengths (run_at = exclusive
    // scan of the run lengths).
    static_assert(kPMaxTiles <= kDThreads, "one tile per thread in the scan below");
    {
        uint32_t sum = 0;
        if (tid < n_tiles) {
            const uint32_t beg = b.run_off[(size_t)tid * (P + 1) + part];
            sum = b.run_off[(size_t)tid * (P + 1) + part + 1] - beg;
            S.run_beg[tid] = (uint16_t)beg;
        }
        uint32_t inc = sum;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        if (lane == kWave - 1) S.s_wave[wave] = inc;
        lds_barrier();
        uint32_t pre = 0;
        for (int w = 0; w < wave; ++w) pre += S.s_wave[w];
        if (tid < n_tiles) S.run_at[tid] = pre + inc - sum;
        if (tid == n_tiles - 1) S.run_at[n_tiles] = pre + inc;
        if (n_tiles == 0 && tid == 0) S.run_at[0] = 0;
    }
    lds_barrier();
    const uint32_t n_rec = S.run_at[n_tiles];
    // Index of record e (0 <= e < n_rec) in `dealt` / `result`; its tile is that index / kPTile.  The
    // runs of a partition are all about as long, so the tile is guessed in proportion and the guess
    // corrected against run_at (a step or two; a search would take log2(n_tiles) dependent LDS reads).
    const float tiles_per_rec = n_rec ? (float)n_tiles / (float)n_rec : 0.f;
    auto locate = [&](uint32_t e) -> uint32_t {
        int g = (int)((float)e * tiles_per_rec);
        if (g > n_tiles - 1) g = n_tiles - 1;
        while (S.run_at[g] > e) --g;                            // run_at[0] = 0 <= e
        while (S.run_at[g + 1] <= e) ++g;                       // run_at[n_tiles] = n_rec > e
        return (uint32_t)g * kPTile + S.run_beg[g] + (e - S.run_at[g]);
    };
    constexpr uint32_t kChunk = kDThreads * kDKeys;             // records the workgroup has in flight
    const uint32_t n_chunks = (n_rec + kChunk - 1) / kChunk;
    uint32_t fill = 0;
    int split = 0;
    for (;; ++split) {
        const uint32_t n_rounds = 1u << split;
        bool failed = false;
        for (uint32_t r = 0; r < n_rounds && !failed; ++r) {
            lds_barrier();                                      // the table is still being read
            static_assert(kPCap == 4 * kDThreads, "the clear below: four entries a thread");
            reinterpret_cast<uint4*>(S.t_key)[tid] = make_uint4(kEmptyKey, kEmptyKey, kEmptyKey, kEmptyKey);
            reinterpret_cast<uint4*>(S.t_min)[tid] = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
            reinterpret_cast<uint4*>(S.t_lid)[tid] = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
            if (r == 0) for (int t = tid; t < n_tiles; t += kDThreads) S.cnt[t] = 0;
            if (tid == 0) S.s_fill = 0;
            lds_barrier();
            uint32_t claimed = 0;
            auto add_known = [&](const uint2 rec) {
                if (rec.x == kEmptyKey) return;
                const uint32_t h = slot_hash(rec.x);
                if (split && slot_round(h, split) != r) return;
                const int s2 = lds_insert(S.t_key, rec.x, slot_index(h), &claimed);
                if (s2 < 0) claimed += (uint32_t)kPCap;
                else S.t_lid[s2] = (int32_t)rec.y;
            };
            // A chunk: kDKeys records per thread, requested together.  slot = the record's table entry,
            // -1 if it has none (no such record, not this sub-round's, table full).
            uint2 rec[kDKeys];
            uint32_t at[kDKeys];
            int slot[kDKeys];
            auto load_chunk = [&](uint32_t ci) {
#pragma unroll
                for (int i = 0; i < kDKeys; ++i) {
                    const uint32_t e = ci * kChunk + (uint32_t)(i * kDThreads + tid);
                    rec[i] = make_uint2(kEmptyKey, 0u); at[i] = 0;
                    if (e < n_rec) { at[i] = locate(e); rec[i] = b.dealt[at[i]]; }
                }
            };
            // pass 1: register every record
            for (uint32_t ci = 0; ci < n_chunks; ++ci) {
                load_chunk(ci);
#pragma unroll
                for (int i = 0; i < kDKeys; ++i) {
                    slot[i] = -1;
                    if (rec[i].x == kEmptyKey) continue;
                    const uint32_t h = slot_hash(rec[i].x);
                    if (split && slot_round(h, split) != r) continue;
                    slot[i] = lds_insert(S.t_key, rec[i].x, slot_index(h), &claimed);
                    if (slot[i] < 0) claimed += (uint32_t)kPCap;
                    else atomicMin(&S.t_min[slot[i]], rec[i].y);
                }
            }
            // the nodes numbered by earlier stages (after the stage's own records: the extents of the wave's
            // first run were requested at the start, so only the run itself is waited for here)
            for (int j = wave; j < n_ktiles; j += kDThreads / kWave) {
                const uint32_t beg = j == wave ? kbeg0 : b.krun_off[(size_t)j * (P + 1) + part];
                const uint32_t end = j == wave ? kend0 : b.krun_off[(size_t)j * (P + 1) + part + 1];
                for (uint32_t k0 = beg; k0 < end; k0 += kKnownAhead * kWave) {
                    uint2 more[kKnownAhead];
#pragma unroll
                    for (int i = 0; i < kKnownAhead; ++i) {
                        const uint32_t k = k0 + (uint32_t)(i * kWave + lane);
                        more[i] = make_uint2(kEmptyKey, 0u);
                        if (k < end) more[i] = b.kdealt[(size_t)j * kPTile + k];
                    }
#pragma unroll
                    for (int i = 0; i < kKnownAhead; ++i) add_known(more[i]);
                }
            }
            {   // one LDS atomic per wave, not one per lane on the same word
                uint32_t w = claimed;
#pragma unroll
                for (int o = kWave / 2; o > 0; o >>= 1) w += __shfl_down(w, o);
                if (lane == 0 && w) atomicAdd(&S.s_fill, w);
            }
            lds_barrier();
            fill = S.s_fill;
            if (fill > kPFillMax) { failed = true; break; }
            // pass 2: every id's smallest position is final.  The chunks are taken last to first: the
            // last one is still in registers with its table entries (mostly it is the only one).
            for (uint32_t ci = n_chunks; ci-- > 0;) {
                if (ci != n_chunks - 1) {
                    load_chunk(ci);
#pragma unroll
                    for (int i = 0; i < kDKeys; ++i) {
                        slot[i] = -1;
                        if (rec[i].x == kEmptyKey) continue;
                        const uint32_t h = slot_hash(rec[i].x);
                        if (split && slot_round(h, split) != r) continue;
                        uint32_t x = slot_index(h);
                        while (S.t_key[x] != rec[i].x) x = (x + 1) & (kPCap - 1);     // pass 1 put it there
                        slot[i] = (int)x;
                    }
                }
#pragma unroll
                for (int i = 0; i < kDKeys; ++i) {
                    const bool valid = slot[i] >= 0;
                    uint32_t mp = 0;
                    int32_t lid = -1;
                    if (valid) { mp = S.t_min[slot[i]]; lid = S.t_lid[slot[i]]; }
                    const bool first = valid && mp == rec[i].y;
                    const bool isnew = first && lid < 0;
                    if (valid) b.result[at[i]] = lid >= 0 ? (lid | (first ? 1 << 30 : 0)) : first ? -1 : -2 - (int32_t)mp;
                    // The tile's counters: the lanes of a wave hold consecutive records, so mostly one tile's;
                    // then one lane adds for all (LDS atomics on one word go one lane at a time).
                    const uint32_t tile = at[i] / kPTile;
                    const unsigned long long mf = __ballot(first), mn = __ballot(isnew);
                    if (mf) {
                        const int leader = __ffsll((long long)mf) - 1;
                        const uint32_t t0 = (uint32_t)__shfl((int)tile, leader);
                        if (__all(!first || tile == t0)) {
                            if (lane == leader) atomicAdd(&S.cnt[t0], (uint32_t)__popcll(mf) + ((uint32_t)__popcll(mn) << 16));
                        } else if (first) {
                            atomicAdd(&S.cnt[tile], isnew ? 0x10001u : 1u);
                        }
                    }
                }
            }
        }
        if (!failed) break;
        if (split == kPMaxSplit) {                              // 2^12 sub-rounds were not enough: give up loudly
            if (tid == 0) atomicOr((int*)gptr(c.status), kStatCapacity);
            break;
        }
    }
    lds_barrier();
    // What k_part_assign needs is the population of all tiles before its own: each partition writes its
    // populations scanned over the tiles (exclusive), so that the tile's workgroup adds up P numbers.
    {
        static_assert(kPMaxTiles <= kDThreads, "one tile per thread in the scan below");
        static_assert(kPTile < 65536, "two 16-bit counts per tile");
        const uint32_t both = tid < n_tiles ? S.cnt[tid] : 0u, f = both & 0xFFFFu, n = both >> 16;
        uint32_t fi = f, ni = n;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t yf = __shfl_up(fi, o), yn = __shfl_up(ni, o);
            if (lane >= o) { fi += yf; ni += yn; }
        }
        if (lane == kWave - 1) { S.s_wave[wave] = fi; S.run_at[wave] = ni; }    // (run_at is free by now)
        lds_barrier();
        uint32_t pf = 0, pn = 0;
        for (int w = 0; w < wave; ++w) { pf += S.s_wave[w]; pn += S.run_at[w]; }
        if (tid < n_tiles) {
            b.pcount[((size_t)tid * P + part) * 2] = pf + fi - f;
            b.pcount[((size_t)tid * P + part) * 2 + 1] = pn + ni - n;
        }
    }
    // what the host's choice of the partition count goes by: fullest table, deepest split
    if (tid == 0 && c.part_stats && c.stage == c.n_hops) {      // (the last stage holds the most nodes)
        // (looked at first: a thousand workgroups' atomics on one word would queue up behind each other,
        // and once a few calls have run hardly any workgroup has anything new to report)
        uint32_t QV_G* st = gptr(c.part_stats);
        if (split == 0) { if (fill > st[0]) atomicMax((uint32_t*)&st[0], fill); }
        else if ((uint32_t)split > st[1]) atomicMax((uint32_t*)&st[1], (uint32_t)split);
        if (st[2] != (uint32_t)p_log2 + 1u) st[2] = (uint32_t)p_log2 + 1u;
    }
}

// ---------------------------------------------------------------------------------------------
// k_part_assign: one workgroup per tile.  ORs the partitions' masks, ranks the first occurrences
// and the new nodes of the tile by popcount (the counts of earlier tiles give the base), and
// writes what k_assign writes in the table forms: n_id and local ids of the new nodes, the next
// hop's frontier entries (row extent read here; segment offset relative to the tile, the tile's
// total in tile_seg), the caller's frontier array, the sizes.
// ---------------------------------------------------------------------------------------------
template <typename RP, bool kNext, typename A>     // kNext: a next hop exists (frontier entries with row extents are built)
__global__ void __launch_bounds__(kPThreads, 4) k_part_assign(A c) {    // 4 waves per SIMD: two workgroups per CU
    __shared__ int32_t res[kPTile];                             // k_part_dedup's result word of every position of the tile
    __shared__ unsigned long long m_first[kPWords], m_new[kPWords];   // bit per position: first occurrence, new node
    __shared__ uint32_t pre_first[kPWords], pre_new[kPWords];
    __shared__ uint32_t seg_tot[kPWords], seg_pre[kPWords];
    __shared__ uint32_t s_tot[3], s_base[2];

    const BatchG b = batch_of(c, blockIdx.y);
    const RP* __restrict__ rowptr = static_cast<const RP*>(c.rowptr);
    SampleMeta* m = b.meta;
    const int P = 1 << c.p_log2;
    const int tid = (int)threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const PartStage v = part_stage(c, b);
    const int64_t len = v.end - v.begin;
    const int64_t node_base = m->node_off[c.stage];
    const int64_t fr_base = m->frontier_off[c.stage];
    // the grid holds fewer workgroups than the a-priori bound has tiles: each takes every gridDim.x-th tile
    for (int t = (int)blockIdx.x;; t += (int)gridDim.x) {
    const int64_t rel0 = (int64_t)t * kPTile;
    if (rel0 >= len && !(len == 0 && t == 0)) return;
    const bool have_tile = rel0 < len;

    // populations of the earlier tiles: every partition left its own, scanned over the tiles
    if (wave == 0) {
        const uint2 QV_G* pc = reinterpret_cast<const uint2 QV_G*>(b.pcount);
        uint32_t bf = 0, bn = 0;
        if (have_tile) for (int q = lane; q < P; q += kWave) { const uint2 x = pc[(size_t)t * P + q]; bf += x.x; bn += x.y; }
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) { bf += __shfl_down(bf, o); bn += __shfl_down(bn, o); }
        if (lane == 0) { s_base[0] = bf; s_base[1] = bn; }
    }
    for (int k = tid; k < kPTile; k += kPThreads) res[k] = kResNone;
    lds_barrier();
    const uint32_t base_first = s_base[0], base_new = s_base[1];
    // the tile's records are sorted by partition: bring their results back into position order
    if (have_tile) {
        const uint32_t total = b.run_off[(size_t)t * (P + 1) + P];
        const uint32_t pos0 = (uint32_t)(v.begin + rel0);
        // (all of a thread's records requested before the first is used)
        uint32_t where[kPKeys];
        int32_t rv[kPKeys];
#pragma unroll
        for (int i = 0; i < kPKeys; ++i) {
            const uint32_t k = (uint32_t)(i * kPThreads + tid);
            where[i] = 0; rv[i] = 0;
            if (k < total) {
                where[i] = reinterpret_cast<const uint32_t QV_G*>(b.dealt)[((size_t)t * kPTile + k) * 2 + 1];
                rv[i] = b.result[(size_t)t * kPTile + k];
            }
        }
#pragma unroll
        for (int i = 0; i < kPKeys; ++i)
            if ((uint32_t)(i * kPThreads + tid) < total) res[(where[i] - pos0) & (kPTile - 1)] = rv[i];
    }
    lds_barrier();
    int32_t rr[kPKeys];
#pragma unroll
    for (int i = 0; i < kPKeys; ++i) {
        rr[i] = res[i * kPThreads + tid];
        const bool first = rr[i] == -1 || (rr[i] >= 0 && ((rr[i] >> 30) & 1));
        const unsigned long long mf = __ballot(first), mn = __ballot(rr[i] == -1);
        if (lane == 0) { m_first[i * (kPThreads / kWave) + wave] = mf; m_new[i * (kPThreads / kWave) + wave] = mn; }
    }
    lds_barrier();
    if (wave < 2) {                                             // exclusive popcount prefixes over the 64 words
        const uint32_t x = (uint32_t)__popcll(wave ? m_new[lane] : m_first[lane]);
        uint32_t inc = x;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        (wave ? pre_new : pre_first)[lane] = inc - x;
        if (lane == kWave - 1) s_tot[wave] = inc;
    }
    lds_barrier();

    // my positions: what a first occurrence needs is requested for all of them before any is used
    const unsigned long long below = (1ull << lane) - 1ull;
    int32_t id[kPKeys], lid[kPKeys];
    int64_t rs[kPKeys];
    uint32_t deg[kPKeys], incl[kPKeys], flags = 0;
#pragma unroll
    for (int i = 0; i < kPKeys; ++i) {
        const int word = i * (kPThreads / kWave) + wave;
        const int64_t rel = rel0 + (int64_t)i * kPThreads + tid;
        const uint32_t first = (rel < len) ? (uint32_t)((m_first[word] >> lane) & 1ull) : 0u;
        const uint32_t isnew = first ? (uint32_t)((m_new[word] >> lane) & 1ull) : 0u;
        flags |= (first << i) | (isnew << (8 + i));
        id[i] = 0; lid[i] = -1; rs[i] = 0; deg[i] = 0;
        if (first) {
            id[i] = v.ids[v.begin + rel];
            if (!isnew) lid[i] = rr[i] & 0x3FFFFFFF;
        }
        // local id of every position that has one by now; a repeat of a new node keeps its link, a
        // position that was not dealt (id out of range) gets -1; new nodes are numbered below
        if (c.stage > 0 && rel < len && rr[i] != -1)
            b.col_local[v.begin + rel] = rr[i] >= 0 ? (rr[i] & 0x3FFFFFFF) : rr[i] == kResNone ? -1 : rr[i];
    }
    if (kNext) {
#pragma unroll
        for (int i = 0; i < kPKeys; ++i) {
            if ((flags >> i) & 1u) {
                rs[i] = (int64_t)rowptr[id[i]];
                deg[i] = (uint32_t)((int64_t)rowptr[id[i] + 1] - rs[i]);
            }
        }
    }
    // next-hop segment sizes, scanned in position order: within the wave here, across (slab, wave) below
    if (kNext) {
#pragma unroll
    for (int i = 0; i < kPKeys; ++i) {
        uint32_t seg = 0;
        if ((flags >> i) & 1u) seg = deg[i] < (uint32_t)c.next_fanout ? deg[i] : (uint32_t)c.next_fanout;
        uint32_t inc = seg;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        incl[i] = inc - seg;                                    // exclusive within the wave
        if (lane == kWave - 1) seg_tot[i * (kPThreads / kWave) + wave] = inc;
    }
    lds_barrier();
    if (wave == 0) {
        const uint32_t x = seg_tot[lane];
        uint32_t inc = x;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        seg_pre[lane] = inc - x;
        if (lane == kWave - 1) s_tot[2] = inc;
    }
    lds_barrier();
    }
    const uint32_t tot_first = have_tile ? s_tot[0] : 0u, tot_new = have_tile ? s_tot[1] : 0u;
    const int64_t fr_user_base = c.frontier_restart ? 0 : fr_base;
#pragma unroll
    for (int i = 0; i < kPKeys; ++i) {
        if (!((flags >> i) & 1u)) continue;
        const int word = i * (kPThreads / kWave) + wave;
        const int64_t pos = v.begin + rel0 + (int64_t)i * kPThreads + tid;
        const bool isnew = (flags >> (8 + i)) & 1u;
        const int64_t j = (int64_t)base_first + pre_first[word] + (uint32_t)__popcll(m_first[word] & below);
        int32_t l = lid[i];
        if (isnew) {
            const int64_t u = node_base + base_new + pre_new[word] + (uint32_t)__popcll(m_new[word] & below);
            l = (int32_t)u;
            if (u < b.n_id_cap) b.n_id[u] = id[i];
            else atomicOr(c.status, kStatCapacity);
            if (c.stage > 0) b.col_local[pos] = l;
        }
        if (kNext) {
            if (fr_base + j < b.fr_cap) {
                b.fr_id[fr_base + j] = id[i];
                b.fr_lid[fr_base + j] = l;
                b.fr_rs[fr_base + j] = rs[i];
                b.fr_deg[fr_base + j] = deg[i];
                b.fr_seg[fr_base + j] = seg_pre[word] + incl[i];
                b.fr_tile[fr_base + j] = (uint16_t)t;
            } else {
                atomicOr(c.status, kStatCapacity);
            }
        }
        if (b.fr_user) {
            if (fr_user_base + j < b.fr_user_cap) b.fr_user[fr_user_base + j] = id[i];
            else atomicOr(c.status, kStatCapacity);
        }
    }
    if (tid == 0) {
        if (kNext && have_tile) b.tile_seg[t] = s_tot[2];
        if (rel0 + kPTile >= len) {                             // the stage's last tile
            m->node_off[c.stage + 1] = node_base + base_new + tot_new;
            m->frontier_off[c.stage + 1] = fr_base + base_first + tot_first;
        }
    }
    lds_barrier();                                              // the shared arrays are reused by the next tile
    }
}

// ---------------------------------------------------------------------------------------------
// k_part_seeds: stage 0 of the partitioned form as one kernel, one workgroup per batch, for batches of
// at most kSeedMax seeds.  What k_part_deal, k_part_dedup and k_part_assign do for the seeds in three
// launches (each a chain of dependent memory round trips for a single tile) happens here in LDS: the
// seeds go into one hash table with their smallest position, first occurrences are ranked by ballot
// and popcount in position order, and n_id, the frontier entries of hop 1 (row extents read here), the
// caller's frontier array, the tile's edge total and the size block are written.  Same results.
// ---------------------------------------------------------------------------------------------
constexpr int kSeedThreads = 1024;
constexpr int kSeedKeys = 2;                                    // seeds per thread
constexpr int kSeedMax = kSeedThreads * kSeedKeys;              // 2,048
constexpr int kSeedCap = 2 * kSeedMax;                          // table entries: at most half full
constexpr int kSeedWords = kSeedMax / kWave;

template <typename RP, typename A>
__global__ void __launch_bounds__(kSeedThreads) k_part_seeds(A c) {
    __shared__ uint32_t t_key[kSeedCap], t_min[kSeedCap];
    __shared__ unsigned long long m_first[kSeedWords];
    __shared__ uint32_t pre_first[kSeedWords], seg_tot[kSeedWords], seg_pre[kSeedWords], s_tot[2];
    const BatchG b = batch_of(c, blockIdx.x);
    const RP* __restrict__ rowptr = static_cast<const RP*>(c.rowptr);
    SampleMeta QV_G* m = b.meta;
    const int tid = (int)threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int64_t n = b.n_seeds < kSeedMax ? b.n_seeds : kSeedMax;          // (the host sends larger batches the other way)
    const uint32_t n_valid = c.n_nodes >= 0 ? (uint32_t)c.n_nodes : 0x80000000u;
    // my seeds, requested before the table is cleared
    uint32_t key[kSeedKeys];
    bool valid[kSeedKeys], bad = false;
#pragma unroll
    for (int i = 0; i < kSeedKeys; ++i) {
        const int p = i * kSeedThreads + tid;
        key[i] = p < n ? (uint32_t)b.seeds[p] : 0xFFFFFFFFu;
    }
    for (int k = tid; k < kSeedCap; k += kSeedThreads) { t_key[k] = kEmptyKey; t_min[k] = 0xFFFFFFFFu; }
    lds_barrier();
    int slot[kSeedKeys];
#pragma unroll
    for (int i = 0; i < kSeedKeys; ++i) {
        const int p = i * kSeedThreads + tid;
        valid[i] = key[i] < n_valid;
        if (p < n && !valid[i]) bad = true;
        slot[i] = -1;
        if (valid[i]) {
            uint32_t x = slot_hash(key[i]) >> (32 - 12);            // kSeedCap = 2^12 entries
            static_assert(kSeedCap == 1 << 12, "the table index above");
            for (;;) {                                              // ends: the table is at most half full
                const uint32_t cur = atomicCAS(&t_key[x], kEmptyKey, key[i]);
                if (cur == kEmptyKey || cur == key[i]) break;
                x = (x + 1) & (kSeedCap - 1);
            }
            slot[i] = (int)x;
            atomicMin(&t_min[x], (uint32_t)p);
        }
    }
    if (bad) atomicOr((int*)gptr(c.status), kStatRange);
    lds_barrier();
    // first occurrences, a bit per position (position = word * 64 + lane)
    bool first[kSeedKeys];
#pragma unroll
    for (int i = 0; i < kSeedKeys; ++i) {
        first[i] = valid[i] && t_min[slot[i]] == (uint32_t)(i * kSeedThreads + tid);
        const unsigned long long mf = __ballot(first[i]);
        if (lane == 0) m_first[i * (kSeedThreads / kWave) + wave] = mf;
    }
    // row extents of the first occurrences (they are hop 1's frontier) and their segment sizes
    int64_t rs[kSeedKeys];
    uint32_t deg[kSeedKeys], incl[kSeedKeys];
#pragma unroll
    for (int i = 0; i < kSeedKeys; ++i) {
        rs[i] = 0; deg[i] = 0;
        if (first[i]) {
            rs[i] = (int64_t)rowptr[key[i]];
            deg[i] = (uint32_t)((int64_t)rowptr[key[i] + 1] - rs[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < kSeedKeys; ++i) {
        const uint32_t seg = first[i] ? (deg[i] < (uint32_t)c.next_fanout ? deg[i] : (uint32_t)c.next_fanout) : 0u;
        uint32_t inc = seg;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        incl[i] = inc - seg;
        if (lane == kWave - 1) seg_tot[i * (kSeedThreads / kWave) + wave] = inc;
    }
    lds_barrier();
    static_assert(kSeedWords <= kWave, "one wave scans the words");
    if (wave < 2) {                                                 // wave 0: ranks of the first occurrences; wave 1: segment offsets
        const uint32_t x = lane < kSeedWords ? (wave ? seg_tot[lane] : (uint32_t)__popcll(m_first[lane])) : 0u;
        uint32_t inc = x;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        if (lane < kSeedWords) (wave ? seg_pre : pre_first)[lane] = inc - x;
        if (lane == kWave - 1) s_tot[wave] = inc;
    }
    lds_barrier();
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < kSeedKeys; ++i) {
        if (!first[i]) continue;
        const int word = i * (kSeedThreads / kWave) + wave;
        const int64_t j = (int64_t)pre_first[word] + (uint32_t)__popcll(m_first[word] & below);   // local id and frontier index
        if (j < b.n_id_cap) b.n_id[j] = (int32_t)key[i];
        else atomicOr((int*)gptr(c.status), kStatCapacity);
        if (j < b.fr_cap) {
            b.fr_id[j] = (int32_t)key[i];
            b.fr_lid[j] = (int32_t)j;
            b.fr_rs[j] = rs[i];
            b.fr_deg[j] = deg[i];
            b.fr_seg[j] = seg_pre[word] + incl[i];
            b.fr_tile[j] = 0;
        } else {
            atomicOr((int*)gptr(c.status), kStatCapacity);
        }
        if (b.fr_user) {
            if (j < b.fr_user_cap) b.fr_user[j] = (int32_t)key[i];
            else atomicOr((int*)gptr(c.status), kStatCapacity);
        }
    }
    if (tid == 0) {                                                 // the size block starts here
        for (int i = 0; i < QV_MAX_HOPS + 2; ++i) { m->node_off[i] = 0; m->frontier_off[i] = 0; }
        for (int i = 0; i < QV_MAX_HOPS + 1; ++i) m->edge_off[i] = 0;
        m->stage_range[0] = 0; m->stage_range[1] = b.n_seeds;
        m->node_off[1] = s_tot[0];
        m->frontier_off[1] = s_tot[0];
        if (n > 0) b.tile_seg[0] = s_tot[1];
    }
}

// k_relabel_links: repeats of a node that was new in their hop point at its first position; follow
// the link (that position holds the local id by now).  Also exports the sizes.
template <typename A>
__global__ void __launch_bounds__(256) k_relabel_links(A c) {
    // Workgroup w runs on XCD w mod 8: the workgroups of a batch are numbered so that they share one,
    // whose L2 then holds the lines of first positions that the batch's repeats read again and again.
    const int per_batch = (int)(gridDim.x / (8u * (unsigned)((c.n_batches + 7) / 8)));
    const int q = (int)(blockIdx.x >> 3);
    const int batch = (int)(blockIdx.x & 7u) + 8 * (q / per_batch), chunk = q % per_batch;
    if (batch >= c.n_batches) return;
    const BatchG b = batch_of(c, batch);
    const SampleMeta* m = b.meta;
    const int64_t tid = (int64_t)chunk * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)per_batch * blockDim.x;
    int64_t end = m->edge_off[c.stage];                // c.stage = last stage
    if (end > b.edge_cap) end = b.edge_cap;
    constexpr int kU = 8;                               // positions a thread has in flight
    for (int64_t p0 = tid; p0 < end; p0 += kU * stride) {
        int32_t x[kU], y[kU];
#pragma unroll
        for (int k = 0; k < kU; ++k) { const int64_t p = p0 + k * stride; x[k] = p < end ? b.col_local[p] : 0; }
#pragma unroll
        for (int k = 0; k < kU; ++k) y[k] = x[k] <= -2 ? b.col_local[-2 - (int64_t)x[k]] : 0;
#pragma unroll
        for (int k = 0; k < kU; ++k) if (x[k] <= -2) b.col_local[p0 + k * stride] = y[k];
    }
    if (tid == 0) {
        if (b.node_off_out) for (int i = 0; i < c.n_hops + 2; ++i) b.node_off_out[i] = m->node_off[i];
        if (b.edge_off_out) for (int i = 0; i < c.n_hops + 1; ++i) b.edge_off_out[i] = m->edge_off[i];
        if (b.frontier_off_out) for (int i = 0; i < c.n_hops + 2; ++i) b.frontier_off_out[i] = m->frontier_off[i];
    }
}

// ---------------------------------------------------------------------------------------------
// stand-alone hop: row extents and segment offsets of a caller-given frontier (two-kernel scan)
// ---------------------------------------------------------------------------------------------
constexpr int kMaxDegTiles = 1024;

template <typename RP>
__global__ void __launch_bounds__(kScanBlock) k_deg_partial(const RP* __restrict__ rowptr, int64_t n_nodes,
                                                            const int32_t* __restrict__ frontier, int64_t F,
                                                            int32_t fanout, int32_t ipt, uint32_t* partial,
                                                            int32_t* status) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const int64_t t0 = (int64_t)blockIdx.x * kScanBlock * ipt;
    if (t0 >= F) return;
    Tri sum = {0, 0, 0};
    for (int it = 0; it < ipt; ++it) {
        int64_t f = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        if (f < F) {
            int32_t v = frontier[f];
            if (v >= 0 && (int64_t)v < n_nodes) {
                uint32_t d = (uint32_t)((int64_t)rowptr[v + 1] - (int64_t)rowptr[v]);
                sum.a += d < (uint32_t)fanout ? d : (uint32_t)fanout;
            } else {
                atomicOr(status, kStatRange);
            }
        }
    }
    Tri total;
    block_scan3(sum, total, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = total.a;
}

template <typename RP>
__global__ void __launch_bounds__(kScanBlock) k_deg_scan(const RP* __restrict__ rowptr, int64_t n_nodes,
                                                         const int32_t* __restrict__ frontier, int64_t F,
                                                         int32_t fanout, int32_t ipt, const uint32_t* partial,
                                                         int64_t* off_out, int64_t* fr_rs, uint32_t* fr_deg,
                                                         uint32_t* fr_seg, SampleMeta* meta) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const int64_t t0 = (int64_t)blockIdx.x * kScanBlock * ipt;
    if (t0 >= F && !(F == 0 && blockIdx.x == 0)) return;
    Tri pre = {0, 0, 0}, run;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kScanBlock) pre.a += partial[i];
    block_scan3(pre, run, lds);
    uint64_t running = run.a;
    for (int it = 0; it < ipt; ++it) {
        int64_t f = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        Tri v = {0, 0, 0}, tot;
        int64_t rs = 0;
        uint32_t d = 0;
        if (f < F) {
            int32_t x = frontier[f];
            if (x >= 0 && (int64_t)x < n_nodes) {
                rs = (int64_t)rowptr[x];
                d = (uint32_t)((int64_t)rowptr[x + 1] - rs);
                v.a = d < (uint32_t)fanout ? d : (uint32_t)fanout;
            }
        }
        Tri ex = block_scan3(v, tot, lds);
        if (f < F) {
            off_out[f] = (int64_t)(running + ex.a);
            fr_rs[f] = rs; fr_deg[f] = d; fr_seg[f] = (uint32_t)(running + ex.a);
        }
        running += tot.a;
    }
    if (threadIdx.x == 0 && (F == 0 || t0 + (int64_t)kScanBlock * ipt >= F)) {
        off_out[F] = (int64_t)running;
        meta->frontier_off[0] = 0; meta->frontier_off[1] = F;      // read by k_sample as stage 1
        meta->edge_off[0] = 0; meta->edge_off[1] = (int64_t)running;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct Bounds {
    int64_t nodes, edges, frontier;
    int64_t hop_edges[QV_MAX_HOPS + 1];     // [k] bound on hop k's edges (k >= 1)
    int64_t hop_front[QV_MAX_HOPS + 1];     // [k] bound on |F_k|
    int64_t nodes_after[QV_MAX_HOPS + 1];   // [k] bound on |n_id| after stage k
};

static qv_status compute_bounds(qv_ctx* ctx, int64_t n_seeds, const int32_t* fanouts, int n_hops,
                                int64_t n_nodes, bool cumulative, Bounds* b) {
    if (n_hops < 1 || n_hops > QV_MAX_HOPS) return fail(ctx, QV_EINVAL, "n_hops %d outside [1, %d]", n_hops, QV_MAX_HOPS);
    if (!fanouts) return fail(ctx, QV_EINVAL, "fanouts is NULL");
    if (n_seeds < 0 || n_seeds >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "n_seeds out of range");
    // hop_front[k] = most nodes hop k+1 may expand: |F_k| (layer frontiers) or |n_id| after hop k
    b->hop_front[0] = n_seeds;
    b->hop_edges[0] = 0;
    b->nodes = n_seeds < n_nodes ? n_seeds : n_nodes; b->edges = 0; b->frontier = n_seeds;
    b->nodes_after[0] = b->nodes;
    for (int k = 1; k <= n_hops; ++k) {
        int32_t l = fanouts[k - 1];
        if (l < 1 || l > QV_MAX_FANOUT) return fail(ctx, QV_EINVAL, "fanout %d outside [1, %d]", l, QV_MAX_FANOUT);
        int64_t e = b->hop_front[k - 1] * (int64_t)l;
        if (e >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "hop %d may produce 2^31 or more edges", k);
        b->hop_edges[k] = e;
        b->edges += e;
        b->frontier += e < n_nodes ? e : n_nodes;
        b->nodes = b->nodes + e < n_nodes ? b->nodes + e : n_nodes;
        b->hop_front[k] = cumulative ? b->nodes : (e < n_nodes ? e : n_nodes);
        b->nodes_after[k] = b->nodes;
    }
    return QV_OK;
}

static void table_geometry(int64_t max_keys, uint32_t* mask, int* shift) {
    int bits = 10;
    while (((int64_t)1 << bits) < 2 * max_keys && bits < 31) ++bits;
    *mask = (uint32_t)(((uint64_t)1 << bits) - 1);
    *shift = 32 - bits;
}

// Make sure the context owns n_tables tables of `slots` entries (with key words if hashed) and
// start a new epoch.
static qv_status table_prepare(qv_ctx* ctx, int n_tables, size_t slots, bool hashed) {
    const size_t need = (size_t)n_tables * slots;
    const size_t need_keyw = hashed ? need : 0;
    bool clear = false;
    if (need > ctx->table_entries || need_keyw > ctx->table_keyw_entries) {
        QV_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (need > ctx->table_entries) {
            if (ctx->table_slots) QV_HIP(ctx, hipFree(ctx->table_slots));
            ctx->table_slots = nullptr; ctx->table_entries = 0;
            QV_HIP(ctx, hipMalloc((void**)&ctx->table_slots, need * sizeof(TableSlot)));
            ctx->table_entries = need;
        }
        if (need_keyw > ctx->table_keyw_entries) {
            if (ctx->table_keyw) QV_HIP(ctx, hipFree(ctx->table_keyw));
            ctx->table_keyw = nullptr; ctx->table_keyw_entries = 0;
            QV_HIP(ctx, hipMalloc((void**)&ctx->table_keyw, need_keyw * sizeof(uint64_t)));
            ctx->table_keyw_entries = need_keyw;
        }
        clear = true;
    }
    if (ctx->epoch >= kEpochLimit) clear = true;
    if (clear) {
        const int64_t n_max = (int64_t)(ctx->table_entries > ctx->table_keyw_entries ? ctx->table_entries : ctx->table_keyw_entries);
        hipLaunchKernelGGL(k_table_clear, dim3(grid_for(n_max, 1024, ctx->n_cu * 16)), dim3(256), 0, ctx->stream,
                           ctx->table_keyw, (int64_t)ctx->table_keyw_entries, ctx->table_slots, (int64_t)ctx->table_entries);
        QV_LAUNCH_CHECK(ctx, "k_table_clear");
        ctx->epoch = 0;
    }
    ++ctx->epoch;
    return QV_OK;
}

// direct (slot == node id) when the arrays for all batches fit the context's budget
static bool use_direct(const qv_ctx* ctx, int64_t n_nodes, int n_tables) {
    return n_nodes > 0 && n_nodes * (int64_t)sizeof(TableSlot) * (int64_t)n_tables <= ctx->direct_budget_bytes;
}

struct Layout {                     // per-batch scratch sizes (elements)
    int64_t stage0, edges, frontier;
    bool part = false;              // partitioned dedup: no table, no per-edge flags
    int p_log2 = 0;                 // log2 of the partitions per batch
    int64_t p_tiles = 0;            // tiles of the largest stage
    int64_t k_tiles = 0;            // tiles of n_id
};

static void tile_shape(int64_t max_items, int* ipt, int* tiles) {
    int64_t per = (max_items + (int64_t)kScanBlock * kMaxTiles - 1) / ((int64_t)kScanBlock * kMaxTiles);
    if (per < 1) per = 1;
    int64_t t = (max_items + kScanBlock * per - 1) / (kScanBlock * per);
    if (t < 1) t = 1;
    *ipt = (int)per; *tiles = (int)t;
}

static size_t per_batch_bytes(const Layout& L) {
    size_t t = 0;
    t += align_up(sizeof(SampleMeta));
    if (L.part) {
        const size_t cells = (size_t)L.p_tiles << L.p_log2;                 // (tile, partition) pairs
        t += align_up((size_t)L.edges * 4);                                 // nbr
        t += 4 * align_up((size_t)L.frontier * 4) + align_up((size_t)L.frontier * 8) + align_up((size_t)L.frontier * 2);
        const size_t slots = (size_t)L.p_tiles * kPTile;                    // records of the largest stage
        t += align_up(slots * 8) + align_up(slots * 4);                     // dealt, result
        t += align_up(((size_t)L.p_tiles << L.p_log2) * 2 + (size_t)L.p_tiles * 2);     // run_off
        t += align_up((size_t)L.k_tiles * kPTile * 8);                      // kdealt
        t += align_up(((size_t)L.k_tiles << L.p_log2) * 2 + (size_t)L.k_tiles * 2);     // krun_off
        t += align_up(cells * 2 * 4) + align_up((size_t)L.p_tiles * 4);     // pcount, tile_seg
        return t + 2048;
    }
    t += align_up((size_t)L.stage0 * 4) + align_up((size_t)L.stage0 * 2);   // seed_slot, seed_flags
    t += 2 * align_up((size_t)L.edges * 4) + align_up((size_t)L.edges * 2); // slot_of, nbr, flags
    t += 4 * align_up((size_t)L.frontier * 4) + align_up((size_t)L.frontier * 8);   // fr_id, fr_lid, fr_deg, fr_seg, fr_rs
    t += align_up((size_t)kMaxTiles * 3 * 4);                               // partial
    return t + 2048;
}

static bool carve(qv_ctx* ctx, const Layout& L, BatchArgs* b) {
    b->meta = (SampleMeta*)arena_take(ctx, sizeof(SampleMeta));
    if (L.part) {
        const size_t cells = (size_t)L.p_tiles << L.p_log2;
        b->seed_slot = nullptr; b->seed_flags = nullptr; b->slot_of = nullptr; b->flags = nullptr; b->partial = nullptr;
        b->nbr = (int32_t*)arena_take(ctx, (size_t)L.edges * 4);
        b->fr_id = (int32_t*)arena_take(ctx, (size_t)L.frontier * 4);
        b->fr_lid = (int32_t*)arena_take(ctx, (size_t)L.frontier * 4);
        b->fr_rs = (int64_t*)arena_take(ctx, (size_t)L.frontier * 8);
        b->fr_deg = (uint32_t*)arena_take(ctx, (size_t)L.frontier * 4);
        b->fr_seg = (uint32_t*)arena_take(ctx, (size_t)L.frontier * 4);
        b->fr_tile = (uint16_t*)arena_take(ctx, (size_t)L.frontier * 2);
        const size_t slots = (size_t)L.p_tiles * kPTile;
        b->dealt = (uint2*)arena_take(ctx, slots * 8);
        b->result = (int32_t*)arena_take(ctx, slots * 4);
        b->run_off = (uint16_t*)arena_take(ctx, ((size_t)L.p_tiles << L.p_log2) * 2 + (size_t)L.p_tiles * 2);
        b->kdealt = (uint2*)arena_take(ctx, (size_t)L.k_tiles * kPTile * 8);
        b->krun_off = (uint16_t*)arena_take(ctx, ((size_t)L.k_tiles << L.p_log2) * 2 + (size_t)L.k_tiles * 2);
        b->pcount = (uint32_t*)arena_take(ctx, cells * 2 * 4);
        b->tile_seg = (uint32_t*)arena_take(ctx, (size_t)L.p_tiles * 4);
        b->fr_cap = L.frontier;
        return b->meta && b->nbr && b->fr_id && b->fr_lid && b->fr_rs && b->fr_deg && b->fr_seg && b->fr_tile && b->dealt && b->result && b->run_off && b->kdealt && b->krun_off &&
               b->pcount && b->tile_seg;
    }
    b->dealt = nullptr; b->result = nullptr; b->run_off = nullptr; b->kdealt = nullptr; b->krun_off = nullptr; b->pcount = nullptr; b->tile_seg = nullptr; b->fr_tile = nullptr;
    b->seed_slot = (uint32_t*)arena_take(ctx, (size_t)L.stage0 * 4);
    b->seed_flags = (uint16_t*)arena_take(ctx, (size_t)L.stage0 * 2);
    b->slot_of = (uint32_t*)arena_take(ctx, (size_t)L.edges * 4);
    b->nbr = (int32_t*)arena_take(ctx, (size_t)L.edges * 4);
    b->flags = (uint16_t*)arena_take(ctx, (size_t)L.edges * 2);
    b->fr_id = (int32_t*)arena_take(ctx, (size_t)L.frontier * 4);
    b->fr_lid = (int32_t*)arena_take(ctx, (size_t)L.frontier * 4);
    b->fr_rs = (int64_t*)arena_take(ctx, (size_t)L.frontier * 8);
    b->fr_deg = (uint32_t*)arena_take(ctx, (size_t)L.frontier * 4);
    b->fr_seg = (uint32_t*)arena_take(ctx, (size_t)L.frontier * 4);
    b->partial = (uint32_t*)arena_take(ctx, (size_t)kMaxTiles * 3 * 4);
    b->fr_cap = L.frontier;
    return b->meta && b->seed_slot && b->seed_flags && b->slot_of && b->nbr && b->flags && b->fr_id && b->fr_lid &&
           b->fr_rs && b->fr_deg && b->fr_seg && b->partial;
}

// Launch KERNEL<A> (QV_LAUNCH_A) or KERNEL<T1, A> (QV_LAUNCH_A1) with the argument form A that fits
// the call: per-batch arguments inside the kernel argument block, or a pointer to their device copy.
#define QV_LAUNCH_FORM(ctx, c, n_batches, grid, block, INLINE_KERNEL, DEVICE_KERNEL)                          \
    do {                                                                                                    \
        if ((n_batches) <= kInlineBatch) {                                                                  \
            CallInline a_;                                                                                  \
            static_cast<CallHeader&>(a_) = static_cast<const CallHeader&>(c);                               \
            for (int i_ = 0; i_ < (n_batches); ++i_) a_.b[i_] = (c).b[i_];                                   \
            hipLaunchKernelGGL(INLINE_KERNEL, grid, block, 0, (ctx)->stream, a_);                           \
        } else {                                                                                            \
            CallDevice a_;                                                                                  \
            static_cast<CallHeader&>(a_) = static_cast<const CallHeader&>(c);                               \
            a_.b = (c).b_dev;                                                                               \
            hipLaunchKernelGGL(DEVICE_KERNEL, grid, block, 0, (ctx)->stream, a_);                           \
        }                                                                                                   \
    } while (0)
#define QV_LAUNCH_A(ctx, c, n, grid, block, K) QV_LAUNCH_FORM(ctx, c, n, grid, block, (K<CallInline>), (K<CallDevice>))
#define QV_LAUNCH_A1(ctx, c, n, grid, block, K, T1) \
    QV_LAUNCH_FORM(ctx, c, n, grid, block, (K<T1, CallInline>), (K<T1, CallDevice>))

// Calls of more than kInlineBatch batches: copy the per-batch arguments to the device once, through
// a small ring of pinned staging slots (a slot is reused only after its copy has run).
static qv_status upload_batches(qv_ctx* ctx, CallArgs* c, int n_batches) {
    const size_t slot_bytes = sizeof(BatchArgs) * (size_t)kMaxBatch;
    if (!ctx->args_ring) {
        QV_HIP(ctx, hipHostMalloc((void**)&ctx->args_ring, slot_bytes * kArgsRing, hipHostMallocDefault));
        for (int i = 0; i < kArgsRing; ++i) {
            QV_HIP(ctx, hipEventCreateWithFlags(&ctx->args_ev[i], hipEventDisableTiming));
            ctx->args_ev_live[i] = true;
            ctx->args_ev_used[i] = false;
        }
    }
    const int slot = ctx->args_next;
    ctx->args_next = (slot + 1) % kArgsRing;
    if (ctx->args_ev_used[slot]) QV_HIP(ctx, hipEventSynchronize(ctx->args_ev[slot]));
    char* stage = (char*)ctx->args_ring + (size_t)slot * slot_bytes;
    std::memcpy(stage, c->b, sizeof(BatchArgs) * (size_t)n_batches);
    BatchArgs* dev = (BatchArgs*)arena_take(ctx, sizeof(BatchArgs) * (size_t)n_batches);
    if (!dev) return fail(ctx, QV_ENOMEM, "scratch arena too small for the batch arguments (internal sizing error)");
    QV_HIP(ctx, hipMemcpyAsync(dev, stage, sizeof(BatchArgs) * (size_t)n_batches, hipMemcpyHostToDevice, ctx->stream));
    QV_HIP(ctx, hipEventRecord(ctx->args_ev[slot], ctx->stream));
    ctx->args_ev_used[slot] = true;
    c->b_dev = dev;
    return QV_OK;
}

static qv_status launch_dedup(qv_ctx* ctx, CallArgs& c, int rowptr_bits, int64_t max_items, int n_batches) {
    int ipt, tiles;
    tile_shape(max_items, &ipt, &tiles);
    c.items_per_thread = ipt;
    dim3 grid((unsigned)tiles, (unsigned)n_batches);
    if (rowptr_bits == 32) {
        QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(kScanBlock), k_flag, int32_t);
        QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(kScanBlock), k_assign, int32_t);
    } else {
        QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(kScanBlock), k_flag, int64_t);
        QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(kScanBlock), k_assign, int64_t);
    }
    QV_LAUNCH_CHECK(ctx, "k_flag / k_assign");
    return QV_OK;
}

static qv_status launch_sample(qv_ctx* ctx, const CallArgs& c, int64_t max_frontier, int n_batches) {
    const int l = c.fanout;
    if (l > 64) {
        dim3 grid((unsigned)grid_for(max_frontier, 1, ctx->n_cu * 32), (unsigned)n_batches);
        QV_LAUNCH_A(ctx, c, n_batches, grid, dim3(64), k_sample_wide);
    } else {
        const int G = l <= 8 ? 8 : l <= 16 ? 16 : l <= 32 ? 32 : 64;
        // enough workgroups for one group per entry while the frontier is small; beyond the cap the
        // kernel gives every group up to 8 entries per round (its S)
        const int cap = n_batches >= 8 ? std::max(64, ctx->n_cu * 32 / n_batches) : ctx->n_cu * 8;
        dim3 grid((unsigned)grid_for(max_frontier, (256 / G) * (n_batches >= 8 ? 8 : 1), cap), (unsigned)n_batches);
        switch (G) {
            case 8: QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(256), k_sample, 8); break;
            case 16: QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(256), k_sample, 16); break;
            case 32: QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(256), k_sample, 32); break;
            default: QV_LAUNCH_A1(ctx, c, n_batches, grid, dim3(256), k_sample, 64); break;
        }
    }
    QV_LAUNCH_CHECK(ctx, "k_sample");
    return QV_OK;
}

// How many partitions per batch, when the caller leaves it open.  A partition's LDS table should
// end a call about half full: fuller tables probe longer and, past kPFillMax, split into sub-rounds
// that read the stage again; emptier ones mean more workgroups each reading the whole stage.  The
// a-priori node bound says little (sampled sub-graphs of skewed graphs repeat most of their nodes),
// so the kernels report the fullest table and the deepest split of a call (part_stats), the host
// copies the words back without waiting for them, and a later call moves the count one step.
// Results never depend on it.
constexpr int kStatsWord = 16;                      // part_stats = d_status + kStatsWord: fill, split, partitions_log2 + 1
static void part_adapt(qv_ctx* ctx, int64_t nodes_bound) {
    if (ctx->part_auto_log2 < 0 || ctx->part_auto_bound != nodes_bound) {   // first call, or another call shape
        int lg = 3;
        while (lg < kPMaxLog2 && ((int64_t)(kPCap / 2) << lg) < nodes_bound / 8) ++lg;
        ctx->part_auto_log2 = lg;
        ctx->part_auto_bound = nodes_bound;
        ctx->part_stats_reset = true;
        ctx->part_stable = 0;
        return;
    }
    volatile int32_t* h = ctx->h_status + kStatsWord;
    const uint32_t fill = (uint32_t)h[0], split = (uint32_t)h[1];
    if (h[2] != ctx->part_auto_log2 + 1 || (fill == 0 && split == 0)) return;  // nothing (new) has arrived
    int lg = ctx->part_auto_log2;
    if ((split > 0 || fill > kPCap * 3 / 4) && lg < kPMaxLog2) ++lg;
    else if (split == 0 && fill < kPCap * 9 / 32 && lg > 3) --lg;
    if (lg != ctx->part_auto_log2) {
        ctx->part_auto_log2 = lg;
        ctx->part_stats_reset = true;
        ctx->part_stable = 0;
    } else if (ctx->part_stable < 1000) {
        ++ctx->part_stable;
    }
}

// Sizes and dedup form of a qv_sample / qv_sample_many call.
// The partitioned form serves layer frontiers whose stages fit kPMaxTiles tiles; the cumulative
// variant, larger stages and a context told to use tables take the table forms.
static qv_status plan_sample(qv_ctx* ctx, int64_t max_seeds, const int32_t* fanouts, int n_hops, int64_t n_nodes,
                             bool cumulative, int n_batches, Bounds* bd, Layout* L) {
    qv_status rc = compute_bounds(ctx, max_seeds, fanouts, n_hops, n_nodes, cumulative, bd);
    if (rc != QV_OK) return rc;
    L->stage0 = max_seeds; L->edges = bd->edges;
    L->frontier = cumulative ? (bd->nodes > 0 ? bd->nodes : 1) : bd->frontier;   // cumulative: one entry per node, at its local id
    const int64_t max_stage = (int64_t)kPTile * kPMaxTiles;
    int64_t largest = max_seeds;
    for (int k = 1; k <= n_hops; ++k) largest = bd->hop_edges[k] > largest ? bd->hop_edges[k] : largest;
    // The partitioned form runs more kernels per stage (a fixed cost per call of some 0.1 ms) and does
    // less work per edge: it pays once a call carries enough edges (measured on a 111 M node graph,
    // batches of 1,024 seeds whose a-priori bound is 0.94 M edges each: 4 batches 135 us of sampling in
    // the table form against about 165 us, 8 batches 216 against 185 us, 12 batches 333 against 211 us).
    const bool big_call = bd->edges * (int64_t)n_batches >= (int64_t)7 << 20;
    L->part = (ctx->dedup_form == QV_DEDUP_PARTITIONED || (ctx->dedup_form == QV_DEDUP_AUTO && big_call)) && !cumulative &&
              largest <= max_stage;
    if (L->part) {
        L->p_tiles = (largest + kPTile - 1) / kPTile;
        if (L->p_tiles < 1) L->p_tiles = 1;
        L->k_tiles = (bd->nodes + kPTile - 1) / kPTile + 1;
        if (ctx->part_log2 >= 0) {
            L->p_log2 = ctx->part_log2;
        } else {
            part_adapt(ctx, bd->nodes);
            L->p_log2 = ctx->part_auto_log2;
        }
    }
    return QV_OK;
}

static qv_status launch_part_dedup(qv_ctx* ctx, CallArgs& c, int rowptr_bits, int64_t max_items, int n_batches) {
    const int P = 1 << c.p_log2;
    int64_t tiles = (max_items + kPTile - 1) / kPTile;
    if (tiles < 1) tiles = 1;
    dim3 grid((unsigned)tiles, (unsigned)n_batches);
    {   // the a-priori bounds are loose (most tiles do not exist): k_part_deal strides over the tiles
        const int64_t cap = n_batches >= 4 ? std::max(16, ctx->n_cu * 8 / n_batches) : ctx->n_cu * 2;
        c.deal_blocks = (int32_t)(tiles < cap ? tiles : cap);
        int node_blocks = c.stage == 0 ? 0 : n_batches >= 4 ? 8 : 32;            // workgroups of their own for the tiles of n_id
        // Workgroups go to the eight XCDs in turn by their linear index: with a width that is a multiple of
        // eight the x-th workgroup of every batch lands on the same XCD, and the stage's tiles and those of
        // n_id stay unevenly spread; an odd width rotates the batches over the XCDs (128 batches, hop 2:
        // 24 wide 28.6 us, 25 wide 24.4 us).
        if (node_blocks && (c.deal_blocks + node_blocks) % 2 == 0) ++node_blocks;
        dim3 deal_grid((unsigned)(c.deal_blocks + node_blocks), (unsigned)n_batches);
        QV_LAUNCH_A(ctx, c, n_batches, deal_grid, dim3(kPThreads), k_part_deal);
    }
    const unsigned wgs = 8u * (unsigned)((n_batches + 7) / 8) * (unsigned)P;    // (XCD, batch within XCD, partition)
    QV_LAUNCH_A(ctx, c, n_batches, dim3(wgs), dim3(kDThreads), k_part_dedup);
    const bool next = c.next_fanout > 0;
    if (rowptr_bits == 32) {
        if (next) QV_LAUNCH_FORM(ctx, c, n_batches, grid, dim3(kPThreads), (k_part_assign<int32_t, true, CallInline>), (k_part_assign<int32_t, true, CallDevice>));
        else QV_LAUNCH_FORM(ctx, c, n_batches, grid, dim3(kPThreads), (k_part_assign<int32_t, false, CallInline>), (k_part_assign<int32_t, false, CallDevice>));
    } else {
        if (next) QV_LAUNCH_FORM(ctx, c, n_batches, grid, dim3(kPThreads), (k_part_assign<int64_t, true, CallInline>), (k_part_assign<int64_t, true, CallDevice>));
        else QV_LAUNCH_FORM(ctx, c, n_batches, grid, dim3(kPThreads), (k_part_assign<int64_t, false, CallInline>), (k_part_assign<int64_t, false, CallDevice>));
    }
    QV_LAUNCH_CHECK(ctx, "k_part_deal / k_part_dedup / k_part_assign");
    return QV_OK;
}

static qv_status sample_many(qv_ctx* ctx, const qv_csr* csr, int n_batches, const int32_t* const* seeds,
                             const int64_t* n_seeds, const int32_t* fanouts, int n_hops, const uint64_t* rng_seeds,
                             uint32_t flags, const qv_sample_out* outs, const char* who) {
    if (flags & ~(uint32_t)QV_SAMPLE_CUMULATIVE) return fail(ctx, QV_EINVAL, "%s: unknown flag bits 0x%x", who, flags);
    const bool cumulative = (flags & QV_SAMPLE_CUMULATIVE) != 0;
    if (!csr || !outs || !seeds || !n_seeds || !rng_seeds) return fail(ctx, QV_EINVAL, "%s: null argument", who);
    if (n_batches < 1 || n_batches > kMaxBatch) return fail(ctx, QV_EINVAL, "%s: n_batches %d outside [1, %d]", who, n_batches, kMaxBatch);
    int64_t max_seeds = 0;
    for (int i = 0; i < n_batches; ++i) {
        const qv_sample_out& o = outs[i];
        if (n_seeds[i] < 0 || (n_seeds[i] > 0 && !seeds[i])) return fail(ctx, QV_EINVAL, "%s: batch %d has no seeds array", who, i);
        if (!o.n_id || !o.row_local || !o.col_local || !o.node_off || !o.edge_off || !o.frontier_off)
            return fail(ctx, QV_EINVAL, "%s: n_id, row_local, col_local and the three offset arrays are required", who);
        if (o.n_id_cap < 0 || o.edge_cap < 0 || (o.frontier && o.frontier_cap < 0)) return fail(ctx, QV_EINVAL, "%s: negative capacity", who);
        if (n_seeds[i] > max_seeds) max_seeds = n_seeds[i];
    }
    Bounds bd;
    Layout L;
    qv_status rc = plan_sample(ctx, max_seeds, fanouts, n_hops, csr->n_nodes, cumulative, n_batches, &bd, &L);
    if (rc != QV_OK) return rc;
    rc = arena_begin(ctx, per_batch_bytes(L) * n_batches + align_up(sizeof(BatchArgs) * (size_t)kMaxBatch) +
                              align_up(sizeof(SampleMeta) * (size_t)kMaxBatch));
    if (rc != QV_OK) return rc;
    CallArgs c{};
    c.rowptr = csr->rowptr; c.col = csr->col; c.n_nodes = csr->n_nodes;
    size_t table_slots = 0;
    if (!L.part) {
        table_geometry(bd.nodes, &c.mask, &c.shift);
        c.direct = use_direct(ctx, csr->n_nodes, n_batches) ? 1 : 0;
        table_slots = c.direct ? (size_t)csr->n_nodes : (size_t)c.mask + 1;
        rc = table_prepare(ctx, n_batches, table_slots, !c.direct);
        if (rc != QV_OK) return rc;
    }
    c.epoch = ctx->epoch; c.n_hops = n_hops; c.status = ctx->d_status; c.cumulative = cumulative ? 1 : 0;
    c.p_log2 = L.p_log2; c.p_tiles = (int32_t)L.p_tiles; c.n_batches = n_batches;
    const bool adaptive = L.part && ctx->part_log2 < 0;
    if (adaptive) {
        c.part_stats = reinterpret_cast<uint32_t*>(ctx->d_status + kStatsWord);
        if (ctx->part_stats_reset) {                // the count changed: earlier reports no longer apply
            QV_HIP(ctx, hipMemsetAsync(ctx->d_status + kStatsWord, 0, 3 * sizeof(int32_t), ctx->stream));
            ctx->h_status[kStatsWord] = 0; ctx->h_status[kStatsWord + 1] = 0; ctx->h_status[kStatsWord + 2] = 0;
            ctx->part_stats_reset = false;
        }
    }
    c.meta_base = (SampleMeta*)arena_take(ctx, sizeof(SampleMeta) * (size_t)n_batches);
    if (!c.meta_base) return fail(ctx, QV_ENOMEM, "%s: scratch arena too small (internal sizing error)", who);
    for (int i = 0; i < n_batches; ++i) {
        BatchArgs& b = c.b[i];
        if (!carve(ctx, L, &b)) return fail(ctx, QV_ENOMEM, "%s: scratch arena too small (internal sizing error)", who);
        b.meta = c.meta_base + i;
        const qv_sample_out& o = outs[i];
        b.seeds = seeds[i]; b.n_seeds = n_seeds[i]; b.rng_seed = rng_seeds[i];
        b.keyw = (L.part || c.direct) ? nullptr : ctx->table_keyw + (size_t)i * table_slots;
        b.slots = L.part ? nullptr : ctx->table_slots + (size_t)i * table_slots;
        if (o.nbr_global) b.nbr = o.nbr_global;
        b.row_local = o.row_local; b.col_local = o.col_local;
        b.edge_cap = bd.edges < o.edge_cap ? bd.edges : o.edge_cap;
        b.n_id = o.n_id; b.n_id_cap = o.n_id_cap;
        b.fr_user = o.frontier; b.fr_user_cap = o.frontier ? o.frontier_cap : 0;
        b.node_off_out = o.node_off; b.edge_off_out = o.edge_off; b.frontier_off_out = o.frontier_off;
        b.n_id_len_out = nullptr; b.frontier_len_out = nullptr;
    }
    if (n_batches > kInlineBatch) {
        rc = upload_batches(ctx, &c, n_batches);
        if (rc != QV_OK) return rc;
    }
    if (L.part) {
        // Partitioned form: per stage k_part_deal + k_part_dedup + k_part_assign; k_sample only writes
        // the edges.  Early stages hold few nodes and take fewer partitions (every partition is a
        // workgroup with a table to clear): the last stage's count scaled by the a-priori node bounds,
        // times eight because those bounds are the looser the later the stage.
        auto stage_p_log2 = [&](int k) {
            int lg = 0;
            while (lg < L.p_log2 && (bd.nodes << lg) < 8 * (bd.nodes_after[k] << L.p_log2)) ++lg;
            return lg;
        };
        c.stage = 0; c.next_fanout = fanouts[0]; c.p_log2 = stage_p_log2(0); c.deal_all_nodes = 0;
        if (max_seeds <= kSeedMax) {                                // the seeds of a batch fit one workgroup's LDS table
            if (csr->rowptr_bits == 32)
                QV_LAUNCH_FORM(ctx, c, n_batches, dim3((unsigned)n_batches), dim3(kSeedThreads), (k_part_seeds<int32_t, CallInline>),
                               (k_part_seeds<int32_t, CallDevice>));
            else
                QV_LAUNCH_FORM(ctx, c, n_batches, dim3((unsigned)n_batches), dim3(kSeedThreads), (k_part_seeds<int64_t, CallInline>),
                               (k_part_seeds<int64_t, CallDevice>));
            QV_LAUNCH_CHECK(ctx, "k_part_seeds");
        } else {
            rc = launch_part_dedup(ctx, c, csr->rowptr_bits, max_seeds, n_batches);
            if (rc != QV_OK) return rc;
        }
        for (int k = 1; k <= n_hops; ++k) {
            c.stage = k; c.hop = k; c.fanout = fanouts[k - 1]; c.next_fanout = k < n_hops ? fanouts[k] : 0;
            const int lg = stage_p_log2(k);
            c.deal_all_nodes = lg != c.p_log2;
            rc = launch_sample(ctx, c, bd.hop_front[k - 1], n_batches);
            if (rc != QV_OK) return rc;
            c.p_log2 = lg;
            rc = launch_part_dedup(ctx, c, csr->rowptr_bits, bd.hop_edges[k], n_batches);
            if (rc != QV_OK) return rc;
        }
        c.stage = n_hops;
        const unsigned per_batch = (unsigned)grid_for(bd.edges, 256 * 32, ctx->n_cu * 4);
        dim3 grid(per_batch * 8u * (unsigned)((n_batches + 7) / 8));          // (XCD, batch within XCD, chunk)
        QV_LAUNCH_A(ctx, c, n_batches, grid, dim3(256), k_relabel_links);
        QV_LAUNCH_CHECK(ctx, "k_relabel_links");
        // report back: every call while the count is still moving, every 32nd once it has settled
        if (adaptive && (ctx->part_stable < 8 || (++ctx->part_calls & 31) == 0))
            QV_HIP(ctx, hipMemcpyAsync(ctx->h_status + kStatsWord, ctx->d_status + kStatsWord, 3 * sizeof(int32_t),
                                       hipMemcpyDeviceToHost, ctx->stream));
        return QV_OK;
    }
    // stage 0: the seeds
    c.stage = 0; c.next_fanout = fanouts[0];
    {
        dim3 grid((unsigned)grid_for(max_seeds, 256, ctx->n_cu * 4), (unsigned)n_batches);
        QV_LAUNCH_A(ctx, c, n_batches, grid, dim3(256), k_insert_ids);
        QV_LAUNCH_CHECK(ctx, "k_insert_ids");
    }
    // edge_off[1] is preset by k_insert_ids for the stand-alone reindex; stage 0 overwrites it here
    rc = launch_dedup(ctx, c, csr->rowptr_bits, max_seeds, n_batches);
    if (rc != QV_OK) return rc;
    for (int k = 1; k <= n_hops; ++k) {
        c.stage = k; c.hop = k; c.fanout = fanouts[k - 1]; c.next_fanout = k < n_hops ? fanouts[k] : 0;
        if (cumulative) {                       // segment offsets of every node sampled so far
            int ipt, tiles;
            tile_shape(bd.hop_front[k - 1], &ipt, &tiles);
            c.items_per_thread = ipt;
            dim3 grid((unsigned)tiles, (unsigned)n_batches);
            QV_LAUNCH_A(ctx, c, n_batches, grid, dim3(kScanBlock), k_cum_partial);
            QV_LAUNCH_A(ctx, c, n_batches, grid, dim3(kScanBlock), k_cum_scan);
            QV_LAUNCH_CHECK(ctx, "k_cum_scan");
        }
        rc = launch_sample(ctx, c, bd.hop_front[k - 1], n_batches);
        if (rc != QV_OK) return rc;
        rc = launch_dedup(ctx, c, csr->rowptr_bits, bd.hop_edges[k], n_batches);
        if (rc != QV_OK) return rc;
    }
    c.stage = n_hops;
    dim3 grid((unsigned)grid_for(bd.edges, 256 * 4, ctx->n_cu * 4), (unsigned)n_batches);
    QV_LAUNCH_A(ctx, c, n_batches, grid, dim3(256), k_relabel);
    QV_LAUNCH_CHECK(ctx, "k_relabel");
    return QV_OK;
}

// ---------------------------------------------------------------------------------------------
// stand-alone hop, shared by qv_sample_hop (scratch from the context's arena) and
// qv_sample_hop_noalloc (scratch in a fixed device array)
// ---------------------------------------------------------------------------------------------
struct HopScratch {
    SampleMeta* meta;
    uint32_t* partial;          // [kMaxDegTiles]
    int64_t* fr_rs;             // [n_frontier] row start
    uint32_t* fr_deg;           // [n_frontier] degree
    uint32_t* fr_seg;           // [n_frontier] segment offset
};

static size_t hop_scratch_bytes(int64_t n_frontier) {
    const size_t F = (size_t)n_frontier;
    return align_up(sizeof(SampleMeta)) + align_up(kMaxDegTiles * 4) + align_up(F * 8) + 2 * align_up(F * 4) + 4096;
}

static qv_status check_hop_args(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier, int64_t n_frontier, int32_t fanout,
                                int32_t hop, const int32_t* nbr_out, int64_t nbr_cap, const int64_t* off_out, const char* who) {
    if (!csr || !off_out || (n_frontier > 0 && !frontier) || n_frontier < 0 || nbr_cap < 0 || (nbr_cap > 0 && !nbr_out))
        return fail(ctx, QV_EINVAL, "%s: null or negative argument", who);
    if (fanout < 1 || fanout > QV_MAX_FANOUT) return fail(ctx, QV_EINVAL, "%s: fanout %d outside [1, %d]", who, fanout, QV_MAX_FANOUT);
    if (hop < 1) return fail(ctx, QV_EINVAL, "%s: hop is 1-based", who);
    if (n_frontier * (int64_t)fanout >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "%s: 2^31 or more edges possible", who);
    return QV_OK;
}

static qv_status sample_hop_run(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier, int64_t n_frontier, int32_t fanout,
                                uint64_t rng_seed, int32_t hop, int32_t* nbr_out, int64_t nbr_cap, int64_t* off_out,
                                const HopScratch& s) {
    if (!s.meta || !s.partial || !s.fr_rs || !s.fr_deg || !s.fr_seg)
        return fail(ctx, QV_ENOMEM, "qv_sample_hop: scratch too small (internal sizing error)");
    int64_t per = (n_frontier + (int64_t)kScanBlock * kMaxDegTiles - 1) / ((int64_t)kScanBlock * kMaxDegTiles);
    if (per < 1) per = 1;
    int64_t tiles = (n_frontier + kScanBlock * per - 1) / (kScanBlock * per);
    if (tiles < 1) tiles = 1;
    const int ipt = (int)per;
    if (csr->rowptr_bits == 32) {
        hipLaunchKernelGGL(k_deg_partial<int32_t>, dim3((unsigned)tiles), dim3(kScanBlock), 0, ctx->stream, (const int32_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, s.partial, ctx->d_status);
        hipLaunchKernelGGL(k_deg_scan<int32_t>, dim3((unsigned)tiles), dim3(kScanBlock), 0, ctx->stream, (const int32_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, s.partial, off_out, s.fr_rs, s.fr_deg, s.fr_seg, s.meta);
    } else {
        hipLaunchKernelGGL(k_deg_partial<int64_t>, dim3((unsigned)tiles), dim3(kScanBlock), 0, ctx->stream, (const int64_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, s.partial, ctx->d_status);
        hipLaunchKernelGGL(k_deg_scan<int64_t>, dim3((unsigned)tiles), dim3(kScanBlock), 0, ctx->stream, (const int64_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, s.partial, off_out, s.fr_rs, s.fr_deg, s.fr_seg, s.meta);
    }
    QV_LAUNCH_CHECK(ctx, "k_deg_scan");
    if (n_frontier == 0) return QV_OK;
    CallArgs c{};
    c.rowptr = csr->rowptr; c.col = csr->col; c.n_nodes = csr->n_nodes;
    c.stage = 1; c.hop = hop; c.fanout = fanout; c.status = ctx->d_status;
    BatchArgs& b = c.b[0];
    b.rng_seed = rng_seed; b.meta = s.meta; c.meta_base = s.meta;
    b.fr_id = const_cast<int32_t*>(frontier); b.fr_lid = const_cast<int32_t*>(frontier);   // local ids unused (row_local == NULL)
    b.fr_rs = s.fr_rs; b.fr_deg = s.fr_deg; b.fr_seg = s.fr_seg;
    b.nbr = nbr_out; b.row_local = nullptr; b.slot_of = nullptr; b.edge_cap = nbr_cap;
    return launch_sample(ctx, c, n_frontier, 1);
}

// ---------------------------------------------------------------------------------------------
// Fixed scratch of qv_sample_hop_noalloc: one array per GPU, held until the process ends.  In
// host code the array's name is only a stand-in; its device address is asked for once per device
// (static_scratch_bind, called from qv_ctx_create with that device current) and kept here.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes =
    ((sizeof(SampleMeta) + 255) / 256 * 256) + (((size_t)kMaxDegTiles * 4 + 255) / 256 * 256) +
    (size_t)QV_NOALLOC_MAX_FRONTIER * 16 + 3 * 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[kMaxDevices] = {};

qv_status static_scratch_bind(qv_ctx* ctx) {
    if (ctx->device < 0 || ctx->device >= kMaxDevices) return QV_OK;      // such a device simply has no no-alloc entry point
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[ctx->device]) return QV_OK;
    void* p = nullptr;
    QV_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch_ptr[ctx->device] = (char*)p;
    return QV_OK;
}

static qv_status static_scratch_of(qv_ctx* ctx, char** out) {
    char* p = nullptr;
    if (ctx->device >= 0 && ctx->device < kMaxDevices) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[ctx->device];
    }
    if (!p) return fail(ctx, QV_EHIP, "qv_sample_hop_noalloc: the fixed scratch of GPU %d was not bound at context creation", ctx->device);
    *out = p;
    return QV_OK;
}

}  // namespace qv

using namespace qv;

extern "C" {

qv_status qv_ctx_reserve(qv_ctx* ctx, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops, int64_t n_nodes,
                         uint32_t flags, int32_t n_batches) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_reserve: ctx is NULL");
    if (n_batches < 1 || n_batches > kMaxBatch) return fail(ctx, QV_EINVAL, "qv_ctx_reserve: n_batches %d outside [1, %d]", n_batches, kMaxBatch);
    const bool cumulative = (flags & QV_SAMPLE_CUMULATIVE) != 0;
    Bounds bd;
    Layout L;
    qv_status rc = plan_sample(ctx, n_seeds, fanouts, n_hops, n_nodes, cumulative, n_batches, &bd, &L);
    if (rc != QV_OK) return rc;
    const size_t want = per_batch_bytes(L) * (size_t)n_batches + align_up(sizeof(BatchArgs) * (size_t)kMaxBatch) +
                        align_up(sizeof(SampleMeta) * (size_t)kMaxBatch);
    if (want > ctx->arena_bytes) {
        rc = arena_begin(ctx, want);
        if (rc != QV_OK) return rc;
    }
    if (L.part) return QV_OK;                       // the partitioned form keeps nothing in HBM between calls
    uint32_t mask; int shift;
    table_geometry(bd.nodes, &mask, &shift);
    const bool direct = use_direct(ctx, n_nodes, n_batches);
    return table_prepare(ctx, n_batches, direct ? (size_t)n_nodes : (size_t)mask + 1, !direct);
}

qv_status qv_sample_hop(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier, int64_t n_frontier,
                        int32_t fanout, uint64_t rng_seed, int32_t hop, int32_t* nbr_out, int64_t nbr_cap,
                        int64_t* off_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_sample_hop: ctx is NULL");
    qv_status rc = check_hop_args(ctx, csr, frontier, n_frontier, fanout, hop, nbr_out, nbr_cap, off_out, "qv_sample_hop");
    if (rc != QV_OK) return rc;
    rc = arena_begin(ctx, hop_scratch_bytes(n_frontier));
    if (rc != QV_OK) return rc;
    HopScratch s;
    const size_t F = (size_t)n_frontier;
    s.meta = (SampleMeta*)arena_take(ctx, sizeof(SampleMeta));
    s.partial = (uint32_t*)arena_take(ctx, kMaxDegTiles * 4);
    s.fr_rs = (int64_t*)arena_take(ctx, F * 8);
    s.fr_deg = (uint32_t*)arena_take(ctx, F * 4);
    s.fr_seg = (uint32_t*)arena_take(ctx, F * 4);
    return sample_hop_run(ctx, csr, frontier, n_frontier, fanout, rng_seed, hop, nbr_out, nbr_cap, off_out, s);
}

qv_status qv_sample_hop_noalloc(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier, int64_t n_frontier,
                                int32_t fanout, uint64_t rng_seed, int32_t hop, int32_t* nbr_out, int64_t nbr_cap,
                                int64_t* off_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_sample_hop_noalloc: ctx is NULL");
    qv_status rc = check_hop_args(ctx, csr, frontier, n_frontier, fanout, hop, nbr_out, nbr_cap, off_out, "qv_sample_hop_noalloc");
    if (rc != QV_OK) return rc;
    if (n_frontier > QV_NOALLOC_MAX_FRONTIER)
        return fail(ctx, QV_EINVAL, "qv_sample_hop_noalloc: n_frontier %lld exceeds the fixed scratch (%d entries); use qv_sample_hop",
                    (long long)n_frontier, QV_NOALLOC_MAX_FRONTIER);
    char* base = nullptr;
    rc = static_scratch_of(ctx, &base);
    if (rc != QV_OK) return rc;
    // carve the device's fixed array: the same five pieces qv_sample_hop takes from the arena, each at
    // its place for the largest frontier, so nothing depends on the sizes of earlier calls
    constexpr size_t Fmax = (size_t)QV_NOALLOC_MAX_FRONTIER;
    HopScratch s;
    size_t at = 0;
    s.meta = (SampleMeta*)(base + at);     at += align_up(sizeof(SampleMeta));
    s.partial = (uint32_t*)(base + at);    at += align_up(kMaxDegTiles * 4);
    s.fr_rs = (int64_t*)(base + at);       at += align_up(Fmax * 8);
    s.fr_deg = (uint32_t*)(base + at);     at += align_up(Fmax * 4);
    s.fr_seg = (uint32_t*)(base + at);
    return sample_hop_run(ctx, csr, frontier, n_frontier, fanout, rng_seed, hop, nbr_out, nbr_cap, off_out, s);
}

qv_status qv_sample(qv_ctx* ctx, const qv_csr* csr, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts,
                    int32_t n_hops, uint64_t rng_seed, uint32_t flags, const qv_sample_out* out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_sample: ctx is NULL");
    if (!out) return fail(ctx, QV_EINVAL, "qv_sample: null argument");
    return sample_many(ctx, csr, 1, &seeds, &n_seeds, fanouts, n_hops, &rng_seed, flags, out, "qv_sample");
}

qv_status qv_sample_many(qv_ctx* ctx, const qv_csr* csr, int32_t n_batches, const int32_t* const* seeds,
                         const int64_t* n_seeds, const int32_t* fanouts, int32_t n_hops, const uint64_t* rng_seeds,
                         uint32_t flags, const qv_sample_out* outs) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_sample_many: ctx is NULL");
    return sample_many(ctx, csr, n_batches, seeds, n_seeds, fanouts, n_hops, rng_seeds, flags, outs, "qv_sample_many");
}

qv_status qv_reindex(qv_ctx* ctx, const int32_t* known, int64_t n_known, const int32_t* nbr, int64_t n_nbr,
                     int64_t n_nodes, int32_t* n_id_out, int64_t n_id_cap, int64_t* n_id_len, int32_t* local_out,
                     int32_t* frontier_out, int64_t* frontier_len) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_reindex: ctx is NULL");
    if (n_known < 0 || n_nbr < 0 || n_id_cap < 0 || (n_known > 0 && !known) || (n_nbr > 0 && (!nbr || !local_out)) ||
        !n_id_out || !n_id_len || (frontier_out && !frontier_len))
        return fail(ctx, QV_EINVAL, "qv_reindex: null or negative argument");
    if (n_known >= ((int64_t)1 << 31) || n_nbr >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "qv_reindex: too many ids");
    Layout L;
    L.stage0 = n_known; L.edges = n_nbr; L.frontier = 1;
    qv_status rc = arena_begin(ctx, per_batch_bytes(L));
    if (rc != QV_OK) return rc;
    CallArgs c{};
    c.rowptr = nullptr; c.col = nullptr; c.n_nodes = n_nodes > 0 ? n_nodes : -1;
    table_geometry(n_known + n_nbr, &c.mask, &c.shift);
    c.direct = use_direct(ctx, n_nodes, 1) ? 1 : 0;
    rc = table_prepare(ctx, 1, c.direct ? (size_t)n_nodes : (size_t)c.mask + 1, !c.direct);
    if (rc != QV_OK) return rc;
    c.epoch = ctx->epoch; c.n_hops = 1; c.status = ctx->d_status;
    BatchArgs& b = c.b[0];
    if (!carve(ctx, L, &b)) return fail(ctx, QV_ENOMEM, "qv_reindex: scratch arena too small (internal sizing error)");
    c.meta_base = b.meta;
    b.seeds = known; b.n_seeds = n_known; b.rng_seed = 0;
    b.keyw = c.direct ? nullptr : ctx->table_keyw; b.slots = ctx->table_slots;
    b.nbr = const_cast<int32_t*>(nbr);                   // read only on this path
    b.row_local = nullptr; b.col_local = local_out; b.edge_cap = n_nbr;
    b.n_id = n_id_out; b.n_id_cap = n_id_cap;
    b.fr_user = nullptr; b.fr_user_cap = 0;
    b.node_off_out = nullptr; b.edge_off_out = nullptr; b.frontier_off_out = nullptr;
    b.n_id_len_out = n_id_len; b.frontier_len_out = frontier_len;
    // stage 0: the known ids
    c.stage = 0; c.next_fanout = 0; c.frontier_restart = 0; c.expect_all_first = 1;
    {
        QV_LAUNCH_A(ctx, c, 1, dim3(grid_for(n_known, 256, ctx->n_cu * 4)), dim3(256), k_insert_ids);
        QV_LAUNCH_CHECK(ctx, "k_insert_ids");
    }
    rc = launch_dedup(ctx, c, 32, n_known, 1);
    if (rc != QV_OK) return rc;
    // stage 1: the neighbour ids
    c.stage = 1; c.frontier_restart = 1; c.expect_all_first = 0;
    b.fr_user = frontier_out; b.fr_user_cap = frontier_out ? n_nbr : 0;
    if (n_nbr > 0) {
        QV_LAUNCH_A(ctx, c, 1, dim3(grid_for(n_nbr, 256, ctx->n_cu * 4)), dim3(256), k_insert_ids);
        QV_LAUNCH_CHECK(ctx, "k_insert_ids");
    }
    rc = launch_dedup(ctx, c, 32, n_nbr, 1);
    if (rc != QV_OK) return rc;
    QV_LAUNCH_A(ctx, c, 1, dim3(grid_for(n_nbr, 256 * 4, ctx->n_cu * 4)), dim3(256), k_relabel);
    QV_LAUNCH_CHECK(ctx, "k_relabel");
    return QV_OK;
}

}  // extern "C"
