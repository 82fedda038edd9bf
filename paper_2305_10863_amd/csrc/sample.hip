// Neighbour sampling (one sub-wave group per frontier node, Philox4x32-10 + Floyd's selection)
// and dedup / relabel (open-addressing hash in HBM keyed by global id, first-occurrence order
// recovered from the smallest position at which each id occurs).
//
// Stage structure of one qv_sample call (no host synchronisation anywhere):
//   k_init        clear the table, initialise the device-side size block
//   k_insert_ids  seeds -> table                                  (stage 0)
//   k_flag / k_assign  first occurrences -> F_0, n_id, local ids, segment offsets of hop 1
//   per hop k:   k_sample (pick neighbours, write edges, insert into the table)
//                k_flag / k_assign  -> F_k, n_id growth, segment offsets of hop k+1
//   k_relabel     col_local for all edges, export of the size block
#include "qv_internal.hpp"
#include <new>

namespace qv {

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter (node, hop, slot, 0), key = the 64-bit seed.
// Only words 0 and 1 of the output are used.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t philox_r64(uint64_t seed, uint32_t node, uint32_t hop, uint32_t slot) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t c0 = node, c1 = hop, c2 = slot, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
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
__device__ __forceinline__ uint32_t table_home(uint32_t key, int shift) { return (key * 0x9E3779B1u) >> shift; }

// Returns the slot of `key`, inserting it if absent; 0xFFFFFFFF if the table is full.
__device__ __forceinline__ uint32_t table_insert(HashEntry* table, uint32_t mask, int shift, uint32_t key) {
    uint32_t h = table_home(key, shift) & mask;
    for (uint32_t probes = 0; probes <= mask; ++probes) {
        uint32_t k = __hip_atomic_load(&table[h].key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (k == key) return h;
        if (k == kEmptyKey) {
            uint32_t old = atomicCAS(&table[h].key, kEmptyKey, key);
            if (old == kEmptyKey || old == key) return h;
        }
        h = (h + 1) & mask;
    }
    return 0xFFFFFFFFu;
}

struct TableRef {
    HashEntry* entries;
    uint32_t mask;
    int shift;
};

// ---------------------------------------------------------------------------------------------
// k_init: clear the table and write the initial size block
// ---------------------------------------------------------------------------------------------
__global__ void k_init(TableRef tab, SampleMeta* meta, int64_t stage0_len, int64_t edge1_len) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    uint4 empty;
    empty.x = kEmptyKey; empty.y = 0xFFFFFFFFu; empty.z = 0xFFFFFFFFu; empty.w = 0xFFFFFFFFu;
    uint4* e = reinterpret_cast<uint4*>(tab.entries);
    for (int64_t i = tid; i <= (int64_t)tab.mask; i += stride) e[i] = empty;
    if (tid == 0) {
        for (int i = 0; i < QV_MAX_HOPS + 2; ++i) { meta->node_off[i] = 0; meta->frontier_off[i] = 0; }
        for (int i = 0; i < QV_MAX_HOPS + 1; ++i) meta->edge_off[i] = 0;
        meta->edge_off[1] = edge1_len;           // used by the stand-alone reindex only
        meta->stage_range[0] = 0;
        meta->stage_range[1] = stage0_len;
    }
}

// ---------------------------------------------------------------------------------------------
// k_insert_ids: a flat id array -> table, recording the smallest position of every id
// ---------------------------------------------------------------------------------------------
__global__ void k_insert_ids(const int32_t* __restrict__ ids, int64_t n, int64_t n_nodes, TableRef tab,
                             uint64_t tag, uint32_t* __restrict__ slot_of, int32_t* status) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) {
        int32_t id = ids[i];
        uint32_t slot = 0xFFFFFFFFu;
        if (id < 0 || (n_nodes >= 0 && (int64_t)id >= n_nodes)) {
            atomicOr(status, kStatRange);
        } else {
            slot = table_insert(tab.entries, tab.mask, tab.shift, (uint32_t)id);
            if (slot == 0xFFFFFFFFu) atomicOr(status, kStatCapacity);
            else atomicMin(reinterpret_cast<unsigned long long*>(&tab.entries[slot].minpos),
                           (unsigned long long)(tag | (uint64_t)i));
        }
        slot_of[i] = slot;
    }
}

// ---------------------------------------------------------------------------------------------
// k_sample: one group of G lanes per frontier node, fanout <= G
// ---------------------------------------------------------------------------------------------
struct SampleArgs {
    const void* rowptr;
    const int32_t* col;
    int64_t n_nodes;
    const int32_t* frontier;        // global ids
    const int32_t* frontier_lid;    // local ids of the frontier entries (nullable)
    const int64_t* seg_off;         // start of each frontier entry's segment, relative to the hop's base
    const int64_t* fr_range;        // device [begin, end) into the three arrays above; NULL = [0, n_frontier)
    int64_t n_frontier;
    const int64_t* edge_base;       // device: first edge index of this hop; NULL = 0
    int32_t fanout, hop;
    uint64_t seed;
    int32_t* nbr_out;               // global id per edge
    int32_t* row_local;             // nullable
    int64_t cap;
    TableRef tab;                   // entries == nullptr: no dedup bookkeeping
    uint32_t* slot_of;
    uint64_t tag;
    int32_t* status;
};

template <int G, typename RP>
__global__ void __launch_bounds__(256) k_sample(SampleArgs a) {
    const RP* __restrict__ rowptr = static_cast<const RP*>(a.rowptr);
    const int sub = threadIdx.x % G;
    const int groups_per_block = 256 / G;
    int64_t fbeg = 0, F = a.n_frontier;
    if (a.fr_range) { fbeg = a.fr_range[0]; F = a.fr_range[1] - fbeg; }
    const int64_t ebase = a.edge_base ? *a.edge_base : 0;
    const int64_t stride = (int64_t)gridDim.x * groups_per_block;
    const int group_in_wave = (threadIdx.x % kWave) / G;
    // the loop is uniform over the wave: every lane runs the same number of iterations
    int64_t f0 = (int64_t)blockIdx.x * groups_per_block + (threadIdx.x / kWave) * (kWave / G);
    for (; f0 < F; f0 += stride) {
        int64_t f = f0 + group_in_wave;
        uint32_t d = 0;
        int64_t rs = 0, off = 0;
        int32_t v = -1, vl = -1;
        if (f < F) {
            v = a.frontier[fbeg + f];
            if (v < 0 || (int64_t)v >= a.n_nodes) {
                if (sub == 0) atomicOr(a.status, kStatRange);
                v = -1;
            } else {
                rs = (int64_t)rowptr[v];
                d = (uint32_t)((int64_t)rowptr[v + 1] - rs);
                off = a.seg_off[fbeg + f];
                if (a.frontier_lid) vl = a.frontier_lid[fbeg + f];
            }
        }
        const uint32_t l = (uint32_t)a.fanout;
        const bool draw = d > l;
        const uint32_t m = draw ? l : d;
        uint32_t pos = (uint32_t)sub;
        if (__any(draw)) {
            bool active = draw && (uint32_t)sub < l;
            uint32_t base = d - l;                      // meaningful only where draw
            uint32_t t = 0xFFFFFFFFu;
            if (active) t = rand_below(a.seed, (uint32_t)v, (uint32_t)a.hop, (uint32_t)sub, base + (uint32_t)sub + 1u);
            uint32_t pick = floyd_resolve<G>(t, active, false, base, sub, 0, (int)l);
            if (draw) pos = pick;
        }
        if ((uint32_t)sub < m) {
            int64_t p = ebase + off + sub;
            if (p < a.cap) {
                int32_t g = a.col[rs + pos];
                a.nbr_out[p] = g;
                if (a.row_local) a.row_local[p] = vl;
                if (a.tab.entries) {
                    uint32_t slot = 0xFFFFFFFFu;
                    if (g < 0 || (int64_t)g >= a.n_nodes) {
                        atomicOr(a.status, kStatRange);
                    } else {
                        slot = table_insert(a.tab.entries, a.tab.mask, a.tab.shift, (uint32_t)g);
                        if (slot == 0xFFFFFFFFu) atomicOr(a.status, kStatCapacity);
                        else atomicMin(reinterpret_cast<unsigned long long*>(&a.tab.entries[slot].minpos),
                                       (unsigned long long)(a.tag | (uint64_t)p));
                    }
                    a.slot_of[p] = slot;
                }
            } else {
                atomicOr(a.status, kStatCapacity);
            }
        }
    }
}

// Fanouts above 64: one wave (= one block) per frontier node, slots processed 64 at a time,
// earlier picks kept in LDS.
template <typename RP>
__global__ void __launch_bounds__(64) k_sample_wide(SampleArgs a) {
    __shared__ uint32_t picks[QV_MAX_FANOUT];
    const RP* __restrict__ rowptr = static_cast<const RP*>(a.rowptr);
    const int lane = threadIdx.x;
    int64_t fbeg = 0, F = a.n_frontier;
    if (a.fr_range) { fbeg = a.fr_range[0]; F = a.fr_range[1] - fbeg; }
    const int64_t ebase = a.edge_base ? *a.edge_base : 0;
    const uint32_t l = (uint32_t)a.fanout;
    for (int64_t f = blockIdx.x; f < F; f += gridDim.x) {
        int32_t v = a.frontier[fbeg + f];
        if (v < 0 || (int64_t)v >= a.n_nodes) {
            if (lane == 0) atomicOr(a.status, kStatRange);
            continue;
        }
        const int64_t rs = (int64_t)rowptr[v];
        const uint32_t d = (uint32_t)((int64_t)rowptr[v + 1] - rs);
        const int64_t off = a.seg_off[fbeg + f];
        const int32_t vl = a.frontier_lid ? a.frontier_lid[fbeg + f] : -1;
        const bool draw = d > l;
        const uint32_t m = draw ? l : d;
        const uint32_t base = d - l;
        for (uint32_t c0 = 0; c0 < m; c0 += kWave) {
            uint32_t s = c0 + (uint32_t)lane;
            uint32_t pos = s;
            if (draw) {
                bool active = s < l;
                uint32_t t = 0xFFFFFFFFu;
                if (active) t = rand_below(a.seed, (uint32_t)v, (uint32_t)a.hop, s, base + s + 1u);
                bool pre = false;                       // t already chosen by a slot of an earlier round?
                for (uint32_t r = 0; r < c0; ++r) pre |= (picks[r] == t);
                int n_active = (int)((l - c0) < (uint32_t)kWave ? (l - c0) : (uint32_t)kWave);
                pos = floyd_resolve<kWave>(t, active, active && pre, base, lane, (int)c0, n_active);
                __syncthreads();
                if (active) picks[s] = pos;
                __syncthreads();
            }
            if (s < m) {
                int64_t p = ebase + off + s;
                if (p < a.cap) {
                    int32_t g = a.col[rs + pos];
                    a.nbr_out[p] = g;
                    if (a.row_local) a.row_local[p] = vl;
                    if (a.tab.entries) {
                        uint32_t slot = 0xFFFFFFFFu;
                        if (g < 0 || (int64_t)g >= a.n_nodes) {
                            atomicOr(a.status, kStatRange);
                        } else {
                            slot = table_insert(a.tab.entries, a.tab.mask, a.tab.shift, (uint32_t)g);
                            if (slot == 0xFFFFFFFFu) atomicOr(a.status, kStatCapacity);
                            else atomicMin(reinterpret_cast<unsigned long long*>(&a.tab.entries[slot].minpos),
                                           (unsigned long long)(a.tag | (uint64_t)p));
                        }
                        a.slot_of[p] = slot;
                    }
                } else {
                    atomicOr(a.status, kStatCapacity);
                }
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
// k_flag / k_assign: first occurrences of a stage's ids -> frontier, n_id, local ids, offsets
// ---------------------------------------------------------------------------------------------
struct StageArgs {
    const void* rowptr;             // for the degree of first occurrences (next hop's segment sizes)
    int64_t n_nodes;
    const int32_t* ids;             // the stage's id array (seeds, or global neighbour ids)
    const uint32_t* slot_of;
    uint16_t* flags;
    uint32_t* partial;              // [kMaxTiles][3]
    SampleMeta* meta;
    int32_t stage;                  // 0 = seeds / known ids, k >= 1 = hop k
    int32_t next_fanout;            // 0: no further hop
    int32_t items_per_thread;
    int32_t frontier_restart;       // stand-alone reindex: number the stage's frontier from 0
    int32_t expect_all_first;       // stand-alone reindex stage 0: known ids must be distinct
    int64_t ids_cap;                // positions at or above this were dropped
    HashEntry* table;
    uint64_t tag;
    int32_t* n_id; int64_t n_id_cap;
    int32_t* fr_ids; int32_t* fr_lid; int64_t* fr_seg; int64_t fr_cap;      // working frontier (scratch)
    int32_t* fr_user; int64_t fr_user_cap;                                  // caller's copy (nullable)
    int32_t* status;
};

__device__ __forceinline__ void stage_range(const StageArgs& a, int64_t& begin, int64_t& end) {
    if (a.stage == 0) { begin = a.meta->stage_range[0]; end = a.meta->stage_range[1]; }
    else { begin = a.meta->edge_off[a.stage - 1]; end = a.meta->edge_off[a.stage]; }
    if (end > a.ids_cap) end = a.ids_cap;
    if (end < begin) end = begin;
}

template <typename RP>
__global__ void __launch_bounds__(kScanBlock) k_flag(StageArgs a) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    const RP* __restrict__ rowptr = static_cast<const RP*>(a.rowptr);
    int64_t begin, end;
    stage_range(a, begin, end);
    const int64_t tile_size = (int64_t)kScanBlock * a.items_per_thread;
    const int64_t t0 = begin + (int64_t)blockIdx.x * tile_size;
    if (t0 >= end) return;
    Tri sum = {0, 0, 0};
    for (int it = 0; it < a.items_per_thread; ++it) {
        int64_t p = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        if (p < end) {
            uint32_t slot = a.slot_of[p];
            uint32_t first = 0, isnew = 0, m = 0;
            if (slot != 0xFFFFFFFFu) {
                HashEntry e = a.table[slot];
                first = (e.minpos == (a.tag | (uint64_t)p)) ? 1u : 0u;
                isnew = (first && e.lid < 0) ? 1u : 0u;
                if (first && a.next_fanout > 0) {
                    int32_t g = a.ids[p];
                    uint32_t d = (uint32_t)((int64_t)rowptr[g + 1] - (int64_t)rowptr[g]);
                    m = d < (uint32_t)a.next_fanout ? d : (uint32_t)a.next_fanout;
                }
            }
            a.flags[p] = (uint16_t)(first | (isnew << 1) | (m << 2));
            sum.a += first; sum.b += isnew; sum.c += m;
        }
    }
    Tri total;
    block_scan3(sum, total, lds);
    if (threadIdx.x == 0) {
        a.partial[blockIdx.x * 3 + 0] = total.a;
        a.partial[blockIdx.x * 3 + 1] = total.b;
        a.partial[blockIdx.x * 3 + 2] = total.c;
    }
}

__global__ void __launch_bounds__(kScanBlock) k_assign(StageArgs a) {
    __shared__ uint32_t lds[kScanBlock / kWave][3];
    int64_t begin, end;
    stage_range(a, begin, end);
    const int64_t tile_size = (int64_t)kScanBlock * a.items_per_thread;
    const int64_t t0 = begin + (int64_t)blockIdx.x * tile_size;
    const bool empty_stage = end <= begin;
    if (t0 >= end && !(empty_stage && blockIdx.x == 0)) return;
    // totals of all earlier tiles
    Tri pre = {0, 0, 0};
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kScanBlock) {
        pre.a += a.partial[i * 3 + 0]; pre.b += a.partial[i * 3 + 1]; pre.c += a.partial[i * 3 + 2];
    }
    Tri run;
    block_scan3(pre, run, lds);
    const int64_t node_base = a.meta->node_off[a.stage];
    const int64_t fr_base = a.meta->frontier_off[a.stage];
    const int64_t fr_user_base = a.frontier_restart ? 0 : fr_base;
    for (int it = 0; it < a.items_per_thread; ++it) {
        int64_t p = t0 + (int64_t)it * kScanBlock + threadIdx.x;
        uint32_t f = (p < end) ? a.flags[p] : 0u;
        Tri v = {f & 1u, (f >> 1) & 1u, f >> 2};
        Tri tot;
        Tri ex = block_scan3(v, tot, lds);
        if (v.a) {
            uint32_t slot = a.slot_of[p];
            int32_t id = a.ids[p];
            int64_t u = node_base + run.b + ex.b;
            int32_t lid;
            if (v.b) {
                lid = (int32_t)u;
                a.table[slot].lid = lid;
                if (u < a.n_id_cap) a.n_id[u] = id;
                else atomicOr(a.status, kStatCapacity);
            } else {
                lid = a.table[slot].lid;
            }
            int64_t j = (int64_t)run.a + ex.a;
            if (fr_base + j < a.fr_cap) {
                a.fr_ids[fr_base + j] = id;
                a.fr_lid[fr_base + j] = lid;
                a.fr_seg[fr_base + j] = (int64_t)run.c + ex.c;
            } else {
                atomicOr(a.status, kStatCapacity);
            }
            if (a.fr_user) {
                if (fr_user_base + j < a.fr_user_cap) a.fr_user[fr_user_base + j] = id;
                else atomicOr(a.status, kStatCapacity);
            }
        }
        run.a += tot.a; run.b += tot.b; run.c += tot.c;
    }
    const bool last = empty_stage || (t0 + tile_size >= end);
    if (last && threadIdx.x == 0) {
        a.meta->node_off[a.stage + 1] = node_base + run.b;
        a.meta->frontier_off[a.stage + 1] = fr_base + run.a;
        if (a.next_fanout > 0) a.meta->edge_off[a.stage + 1] = a.meta->edge_off[a.stage] + run.c;
        if (a.expect_all_first && (int64_t)run.a != end - begin) atomicOr(a.status, kStatInval);
    }
}

// ---------------------------------------------------------------------------------------------
// k_relabel: local id of every edge's neighbour; export of the sizes
// ---------------------------------------------------------------------------------------------
struct RelabelArgs {
    const uint32_t* slot_of;
    const HashEntry* table;
    const SampleMeta* meta;
    int32_t last_stage;             // edges are [edge_off[first_stage-1].. edge_off[last_stage])
    int64_t cap;
    int32_t* col_local;
    // exports (all nullable)
    int64_t* node_off; int64_t* edge_off; int64_t* frontier_off; int32_t n_hops;
    int64_t* n_id_len; int64_t* frontier_len;      // stand-alone reindex
};

__global__ void k_relabel(RelabelArgs a) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t end = a.meta->edge_off[a.last_stage];
    if (end > a.cap) end = a.cap;
    for (int64_t p = tid; p < end; p += stride) {
        uint32_t slot = a.slot_of[p];
        a.col_local[p] = slot == 0xFFFFFFFFu ? -1 : a.table[slot].lid;
    }
    if (tid == 0) {
        if (a.node_off) for (int i = 0; i < a.n_hops + 2; ++i) a.node_off[i] = a.meta->node_off[i];
        if (a.edge_off) for (int i = 0; i < a.n_hops + 1; ++i) a.edge_off[i] = a.meta->edge_off[i];
        if (a.frontier_off) for (int i = 0; i < a.n_hops + 2; ++i) a.frontier_off[i] = a.meta->frontier_off[i];
        if (a.n_id_len) *a.n_id_len = a.meta->node_off[2];
        if (a.frontier_len) *a.frontier_len = a.meta->frontier_off[2] - (a.meta->frontier_off[1]);
    }
}

// ---------------------------------------------------------------------------------------------
// stand-alone hop: segment sizes -> offsets (two-kernel tile scan)
// ---------------------------------------------------------------------------------------------
template <typename RP>
__global__ void __launch_bounds__(kScanBlock) k_deg_partial(const RP* __restrict__ rowptr, int64_t n_nodes,
                                                            const int32_t* __restrict__ frontier, int64_t F,
                                                            int32_t fanout, int32_t ipt, uint32_t* partial) {
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
                                                         int64_t* off_out) {
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
        if (f < F) {
            int32_t x = frontier[f];
            if (x >= 0 && (int64_t)x < n_nodes) {
                uint32_t d = (uint32_t)((int64_t)rowptr[x + 1] - (int64_t)rowptr[x]);
                v.a = d < (uint32_t)fanout ? d : (uint32_t)fanout;
            }
        }
        Tri ex = block_scan3(v, tot, lds);
        if (f < F) off_out[f] = (int64_t)(running + ex.a);
        running += tot.a;
    }
    if (threadIdx.x == 0 && (F == 0 || t0 + (int64_t)kScanBlock * ipt >= F)) off_out[F] = (int64_t)running;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct Bounds {
    int64_t nodes, edges, frontier;
    int64_t hop_edges[QV_MAX_HOPS + 1];     // [k] bound on hop k's edges (k >= 1)
    int64_t hop_front[QV_MAX_HOPS + 1];     // [k] bound on |F_k|
};

static qv_status compute_bounds(qv_ctx* ctx, int64_t n_seeds, const int32_t* fanouts, int n_hops,
                                int64_t n_nodes, Bounds* b) {
    if (n_hops < 1 || n_hops > QV_MAX_HOPS) return fail(ctx, QV_EINVAL, "n_hops %d outside [1, %d]", n_hops, QV_MAX_HOPS);
    if (!fanouts) return fail(ctx, QV_EINVAL, "fanouts is NULL");
    if (n_seeds < 0 || n_seeds >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "n_seeds out of range");
    b->hop_front[0] = n_seeds;
    b->hop_edges[0] = 0;
    b->nodes = n_seeds; b->edges = 0; b->frontier = n_seeds;
    for (int k = 1; k <= n_hops; ++k) {
        int32_t l = fanouts[k - 1];
        if (l < 1 || l > QV_MAX_FANOUT) return fail(ctx, QV_EINVAL, "fanout %d outside [1, %d]", l, QV_MAX_FANOUT);
        int64_t e = b->hop_front[k - 1] * (int64_t)l;
        if (e >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "hop %d may produce 2^31 or more edges", k);
        b->hop_edges[k] = e;
        b->hop_front[k] = e < n_nodes ? e : n_nodes;
        b->edges += e; b->frontier += b->hop_front[k]; b->nodes += e;
    }
    if (b->nodes > n_nodes) b->nodes = n_nodes;
    return QV_OK;
}

static void table_geometry(int64_t max_keys, uint32_t* mask, int* shift) {
    int bits = 10;
    while (((int64_t)1 << bits) < 2 * max_keys && bits < 31) ++bits;
    *mask = (uint32_t)(((uint64_t)1 << bits) - 1);
    *shift = 32 - bits;
}

struct Scratch {
    TableRef tab;
    SampleMeta* meta;
    uint32_t *seed_slot, *slot_of, *partial;
    uint16_t *seed_flags, *flags;
    int32_t *nbr, *fr_ids, *fr_lid;
    int64_t* fr_seg;
    int64_t edge_room, fr_room;
};

static size_t scratch_bytes(int64_t stage0, int64_t edges, int64_t frontier, int64_t max_keys) {
    uint32_t mask; int shift;
    table_geometry(max_keys, &mask, &shift);
    size_t t = 0;
    t += align_up(((size_t)mask + 1) * sizeof(HashEntry));
    t += align_up(sizeof(SampleMeta));
    t += align_up((size_t)stage0 * 4) + align_up((size_t)stage0 * 2);
    t += align_up((size_t)edges * 4) * 2 + align_up((size_t)edges * 2);
    t += align_up((size_t)frontier * 4) * 2 + align_up((size_t)frontier * 8);
    t += align_up((size_t)kMaxTiles * 3 * 4);
    return t + 4096;
}

size_t sample_scratch_bytes(int64_t n_seeds, const int32_t* fanouts, int n_hops, int64_t n_nodes) {
    Bounds b;
    if (compute_bounds(nullptr, n_seeds, fanouts, n_hops, n_nodes, &b) != QV_OK) return 0;
    return scratch_bytes(n_seeds, b.edges, b.frontier, b.nodes);
}

static qv_status take_scratch(qv_ctx* ctx, int64_t stage0, int64_t edges, int64_t frontier, int64_t max_keys,
                              Scratch* s) {
    qv_status rc = arena_begin(ctx, scratch_bytes(stage0, edges, frontier, max_keys));
    if (rc != QV_OK) return rc;
    table_geometry(max_keys, &s->tab.mask, &s->tab.shift);
    s->tab.entries = (HashEntry*)arena_take(ctx, ((size_t)s->tab.mask + 1) * sizeof(HashEntry));
    s->meta = (SampleMeta*)arena_take(ctx, sizeof(SampleMeta));
    s->seed_slot = (uint32_t*)arena_take(ctx, (size_t)stage0 * 4);
    s->seed_flags = (uint16_t*)arena_take(ctx, (size_t)stage0 * 2);
    s->slot_of = (uint32_t*)arena_take(ctx, (size_t)edges * 4);
    s->nbr = (int32_t*)arena_take(ctx, (size_t)edges * 4);
    s->flags = (uint16_t*)arena_take(ctx, (size_t)edges * 2);
    s->fr_ids = (int32_t*)arena_take(ctx, (size_t)frontier * 4);
    s->fr_lid = (int32_t*)arena_take(ctx, (size_t)frontier * 4);
    s->fr_seg = (int64_t*)arena_take(ctx, (size_t)frontier * 8);
    s->partial = (uint32_t*)arena_take(ctx, (size_t)kMaxTiles * 3 * 4);
    s->edge_room = edges; s->fr_room = frontier;
    if (!s->tab.entries || !s->meta || !s->seed_slot || !s->seed_flags || !s->slot_of || !s->nbr || !s->flags ||
        !s->fr_ids || !s->fr_lid || !s->fr_seg || !s->partial)
        return fail(ctx, QV_ENOMEM, "scratch arena too small (internal sizing error)");
    return QV_OK;
}

static void tile_shape(int64_t max_items, int* ipt, int* tiles) {
    int64_t per = (max_items + (int64_t)kScanBlock * kMaxTiles - 1) / ((int64_t)kScanBlock * kMaxTiles);
    if (per < 1) per = 1;
    int64_t t = (max_items + kScanBlock * per - 1) / (kScanBlock * per);
    if (t < 1) t = 1;
    *ipt = (int)per; *tiles = (int)t;
}

static qv_status run_stage(qv_ctx* ctx, StageArgs a, int rowptr_bits, int64_t max_items) {
    int ipt, tiles;
    tile_shape(max_items, &ipt, &tiles);
    a.items_per_thread = ipt;
    if (rowptr_bits == 32) hipLaunchKernelGGL(k_flag<int32_t>, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, a);
    else hipLaunchKernelGGL(k_flag<int64_t>, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, a);
    QV_LAUNCH_CHECK(ctx, "k_flag");
    hipLaunchKernelGGL(k_assign, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, a);
    QV_LAUNCH_CHECK(ctx, "k_assign");
    return QV_OK;
}

template <typename RP>
static void launch_sample_rp(qv_ctx* ctx, const SampleArgs& a, int64_t max_frontier) {
    int l = a.fanout;
    if (l > 64) {
        int blocks = grid_for(max_frontier, 1, ctx->n_cu * 32);
        hipLaunchKernelGGL(k_sample_wide<RP>, dim3(blocks), dim3(64), 0, ctx->stream, a);
        return;
    }
    int G = l <= 8 ? 8 : l <= 16 ? 16 : l <= 32 ? 32 : 64;
    int blocks = grid_for(max_frontier, 256 / G, ctx->n_cu * 16);
    switch (G) {
        case 8: hipLaunchKernelGGL((k_sample<8, RP>), dim3(blocks), dim3(256), 0, ctx->stream, a); break;
        case 16: hipLaunchKernelGGL((k_sample<16, RP>), dim3(blocks), dim3(256), 0, ctx->stream, a); break;
        case 32: hipLaunchKernelGGL((k_sample<32, RP>), dim3(blocks), dim3(256), 0, ctx->stream, a); break;
        default: hipLaunchKernelGGL((k_sample<64, RP>), dim3(blocks), dim3(256), 0, ctx->stream, a); break;
    }
}

static qv_status launch_sample(qv_ctx* ctx, const SampleArgs& a, int rowptr_bits, int64_t max_frontier) {
    if (rowptr_bits == 32) launch_sample_rp<int32_t>(ctx, a, max_frontier);
    else launch_sample_rp<int64_t>(ctx, a, max_frontier);
    QV_LAUNCH_CHECK(ctx, "k_sample");
    return QV_OK;
}

static inline uint64_t stage_tag(int stage) { return (uint64_t)(255 - stage) << 48; }   // newer stage = smaller tag

}  // namespace qv

using namespace qv;

extern "C" {

qv_status qv_ctx_reserve(qv_ctx* ctx, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops, int64_t n_nodes) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_ctx_reserve: ctx is NULL");
    Bounds b;
    qv_status rc = compute_bounds(ctx, n_seeds, fanouts, n_hops, n_nodes, &b);
    if (rc != QV_OK) return rc;
    return arena_begin(ctx, scratch_bytes(n_seeds, b.edges, b.frontier, b.nodes));
}

qv_status qv_sample_hop(qv_ctx* ctx, const qv_csr* csr, const int32_t* frontier, int64_t n_frontier,
                        int32_t fanout, uint64_t rng_seed, int32_t hop, int32_t* nbr_out, int64_t nbr_cap,
                        int64_t* off_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_sample_hop: ctx is NULL");
    if (!csr || !off_out || (n_frontier > 0 && !frontier) || n_frontier < 0 || nbr_cap < 0 || (nbr_cap > 0 && !nbr_out))
        return fail(ctx, QV_EINVAL, "qv_sample_hop: null or negative argument");
    if (fanout < 1 || fanout > QV_MAX_FANOUT) return fail(ctx, QV_EINVAL, "qv_sample_hop: fanout %d outside [1, %d]", fanout, QV_MAX_FANOUT);
    if (hop < 1) return fail(ctx, QV_EINVAL, "qv_sample_hop: hop is 1-based");
    if (n_frontier * (int64_t)fanout >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "qv_sample_hop: 2^31 or more edges possible");
    qv_status rc = arena_begin(ctx, align_up((size_t)kMaxTiles * 4) + 4096);
    if (rc != QV_OK) return rc;
    uint32_t* partial = (uint32_t*)arena_take(ctx, (size_t)kMaxTiles * 4);
    int ipt, tiles;
    tile_shape(n_frontier, &ipt, &tiles);
    if (csr->rowptr_bits == 32) {
        hipLaunchKernelGGL(k_deg_partial<int32_t>, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, (const int32_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, partial);
        hipLaunchKernelGGL(k_deg_scan<int32_t>, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, (const int32_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, partial, off_out);
    } else {
        hipLaunchKernelGGL(k_deg_partial<int64_t>, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, (const int64_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, partial);
        hipLaunchKernelGGL(k_deg_scan<int64_t>, dim3(tiles), dim3(kScanBlock), 0, ctx->stream, (const int64_t*)csr->rowptr,
                           csr->n_nodes, frontier, n_frontier, fanout, ipt, partial, off_out);
    }
    QV_LAUNCH_CHECK(ctx, "k_deg_scan");
    if (n_frontier == 0) return QV_OK;
    SampleArgs a{};
    a.rowptr = csr->rowptr; a.col = csr->col; a.n_nodes = csr->n_nodes;
    a.frontier = frontier; a.frontier_lid = nullptr; a.seg_off = off_out; a.fr_range = nullptr;
    a.n_frontier = n_frontier; a.edge_base = nullptr; a.fanout = fanout; a.hop = hop; a.seed = rng_seed;
    a.nbr_out = nbr_out; a.row_local = nullptr; a.cap = nbr_cap;
    a.tab.entries = nullptr; a.tab.mask = 0; a.tab.shift = 0; a.slot_of = nullptr; a.tag = 0; a.status = ctx->d_status;
    return launch_sample(ctx, a, csr->rowptr_bits, n_frontier);
}

qv_status qv_sample(qv_ctx* ctx, const qv_csr* csr, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts,
                    int32_t n_hops, uint64_t rng_seed, const qv_sample_out* out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_sample: ctx is NULL");
    if (!csr || !out || (n_seeds > 0 && !seeds)) return fail(ctx, QV_EINVAL, "qv_sample: null argument");
    if (!out->n_id || !out->row_local || !out->col_local || !out->node_off || !out->edge_off || !out->frontier_off)
        return fail(ctx, QV_EINVAL, "qv_sample: n_id, row_local, col_local and the three offset arrays are required");
    if (out->n_id_cap < 0 || out->edge_cap < 0 || (out->frontier && out->frontier_cap < 0))
        return fail(ctx, QV_EINVAL, "qv_sample: negative capacity");
    Bounds b;
    qv_status rc = compute_bounds(ctx, n_seeds, fanouts, n_hops, csr->n_nodes, &b);
    if (rc != QV_OK) return rc;
    const int64_t edge_room = b.edges < out->edge_cap ? b.edges : out->edge_cap;
    Scratch s;
    rc = take_scratch(ctx, n_seeds, edge_room, b.frontier, b.nodes, &s);
    if (rc != QV_OK) return rc;
    int32_t* nbr = out->nbr_global ? out->nbr_global : s.nbr;

    int init_blocks = grid_for((int64_t)s.tab.mask + 1, 256 * 4, ctx->n_cu * 8);
    hipLaunchKernelGGL(k_init, dim3(init_blocks), dim3(256), 0, ctx->stream, s.tab, s.meta, n_seeds, (int64_t)0);
    QV_LAUNCH_CHECK(ctx, "k_init");
    if (n_seeds > 0) {
        hipLaunchKernelGGL(k_insert_ids, dim3(grid_for(n_seeds, 256, ctx->n_cu * 8)), dim3(256), 0, ctx->stream, seeds,
                           n_seeds, csr->n_nodes, s.tab, stage_tag(0), s.seed_slot, ctx->d_status);
        QV_LAUNCH_CHECK(ctx, "k_insert_ids");
    }
    StageArgs st{};
    st.rowptr = csr->rowptr; st.n_nodes = csr->n_nodes; st.partial = s.partial; st.meta = s.meta;
    st.table = s.tab.entries; st.n_id = out->n_id; st.n_id_cap = out->n_id_cap;
    st.fr_ids = s.fr_ids; st.fr_lid = s.fr_lid; st.fr_seg = s.fr_seg; st.fr_cap = s.fr_room;
    st.fr_user = out->frontier; st.fr_user_cap = out->frontier ? out->frontier_cap : 0;
    st.status = ctx->d_status; st.frontier_restart = 0; st.expect_all_first = 0;
    // stage 0: the seeds
    st.ids = seeds; st.slot_of = s.seed_slot; st.flags = s.seed_flags; st.stage = 0; st.next_fanout = fanouts[0];
    st.ids_cap = n_seeds; st.tag = stage_tag(0);
    rc = run_stage(ctx, st, csr->rowptr_bits, n_seeds);
    if (rc != QV_OK) return rc;
    for (int k = 1; k <= n_hops; ++k) {
        SampleArgs a{};
        a.rowptr = csr->rowptr; a.col = csr->col; a.n_nodes = csr->n_nodes;
        a.frontier = s.fr_ids; a.frontier_lid = s.fr_lid; a.seg_off = s.fr_seg;
        a.fr_range = &s.meta->frontier_off[k - 1]; a.n_frontier = 0; a.edge_base = &s.meta->edge_off[k - 1];
        a.fanout = fanouts[k - 1]; a.hop = k; a.seed = rng_seed;
        a.nbr_out = nbr; a.row_local = out->row_local; a.cap = edge_room;
        a.tab = s.tab; a.slot_of = s.slot_of; a.tag = stage_tag(k); a.status = ctx->d_status;
        rc = launch_sample(ctx, a, csr->rowptr_bits, b.hop_front[k - 1]);
        if (rc != QV_OK) return rc;
        st.ids = nbr; st.slot_of = s.slot_of; st.flags = s.flags; st.stage = k;
        st.next_fanout = k < n_hops ? fanouts[k] : 0; st.ids_cap = edge_room; st.tag = stage_tag(k);
        rc = run_stage(ctx, st, csr->rowptr_bits, b.hop_edges[k]);
        if (rc != QV_OK) return rc;
    }
    RelabelArgs r{};
    r.slot_of = s.slot_of; r.table = s.tab.entries; r.meta = s.meta; r.last_stage = n_hops; r.cap = edge_room;
    r.col_local = out->col_local; r.node_off = out->node_off; r.edge_off = out->edge_off;
    r.frontier_off = out->frontier_off; r.n_hops = n_hops; r.n_id_len = nullptr; r.frontier_len = nullptr;
    hipLaunchKernelGGL(k_relabel, dim3(grid_for(b.edges, 256 * 4, ctx->n_cu * 8)), dim3(256), 0, ctx->stream, r);
    QV_LAUNCH_CHECK(ctx, "k_relabel");
    if (b.edges > out->edge_cap) {
        // the device flags an overflow only if it happens; nothing to do here
    }
    return QV_OK;
}

qv_status qv_reindex(qv_ctx* ctx, const int32_t* known, int64_t n_known, const int32_t* nbr, int64_t n_nbr,
                     int64_t n_nodes, int32_t* n_id_out, int64_t n_id_cap, int64_t* n_id_len, int32_t* local_out,
                     int32_t* frontier_out, int64_t* frontier_len) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_reindex: ctx is NULL");
    if (n_known < 0 || n_nbr < 0 || n_id_cap < 0 || (n_known > 0 && !known) || (n_nbr > 0 && (!nbr || !local_out)) ||
        !n_id_out || !n_id_len || (frontier_out && !frontier_len))
        return fail(ctx, QV_EINVAL, "qv_reindex: null or negative argument");
    if (n_known >= ((int64_t)1 << 31) || n_nbr >= ((int64_t)1 << 31)) return fail(ctx, QV_EINVAL, "qv_reindex: too many ids");
    if (n_nodes <= 0) n_nodes = -1;                     // unchecked
    Scratch s;
    int64_t keys = n_known + n_nbr;
    qv_status rc = take_scratch(ctx, n_known, n_nbr, n_known + n_nbr, keys, &s);
    if (rc != QV_OK) return rc;
    int init_blocks = grid_for((int64_t)s.tab.mask + 1, 256 * 4, ctx->n_cu * 8);
    hipLaunchKernelGGL(k_init, dim3(init_blocks), dim3(256), 0, ctx->stream, s.tab, s.meta, n_known, n_nbr);
    QV_LAUNCH_CHECK(ctx, "k_init");
    StageArgs st{};
    st.rowptr = nullptr; st.n_nodes = n_nodes; st.partial = s.partial; st.meta = s.meta; st.table = s.tab.entries;
    st.n_id = n_id_out; st.n_id_cap = n_id_cap;
    st.fr_ids = s.fr_ids; st.fr_lid = s.fr_lid; st.fr_seg = s.fr_seg; st.fr_cap = s.fr_room;
    st.status = ctx->d_status; st.next_fanout = 0;
    if (n_known > 0) {
        hipLaunchKernelGGL(k_insert_ids, dim3(grid_for(n_known, 256, ctx->n_cu * 8)), dim3(256), 0, ctx->stream, known,
                           n_known, n_nodes, s.tab, stage_tag(0), s.seed_slot, ctx->d_status);
        QV_LAUNCH_CHECK(ctx, "k_insert_ids");
    }
    st.ids = known; st.slot_of = s.seed_slot; st.flags = s.seed_flags; st.stage = 0; st.ids_cap = n_known;
    st.tag = stage_tag(0); st.fr_user = nullptr; st.fr_user_cap = 0; st.frontier_restart = 0; st.expect_all_first = 1;
    rc = run_stage(ctx, st, 32, n_known);
    if (rc != QV_OK) return rc;
    if (n_nbr > 0) {
        hipLaunchKernelGGL(k_insert_ids, dim3(grid_for(n_nbr, 256, ctx->n_cu * 8)), dim3(256), 0, ctx->stream, nbr, n_nbr,
                           n_nodes, s.tab, stage_tag(1), s.slot_of, ctx->d_status);
        QV_LAUNCH_CHECK(ctx, "k_insert_ids");
    }
    st.ids = nbr; st.slot_of = s.slot_of; st.flags = s.flags; st.stage = 1; st.ids_cap = n_nbr; st.tag = stage_tag(1);
    st.fr_user = frontier_out; st.fr_user_cap = n_nbr; st.frontier_restart = 1; st.expect_all_first = 0;
    rc = run_stage(ctx, st, 32, n_nbr);
    if (rc != QV_OK) return rc;
    RelabelArgs r{};
    r.slot_of = s.slot_of; r.table = s.tab.entries; r.meta = s.meta; r.last_stage = 1; r.cap = n_nbr;
    r.col_local = local_out; r.node_off = nullptr; r.edge_off = nullptr; r.frontier_off = nullptr; r.n_hops = 0;
    r.n_id_len = n_id_len; r.frontier_len = frontier_len;
    hipLaunchKernelGGL(k_relabel, dim3(grid_for(n_nbr, 256 * 4, ctx->n_cu * 8)), dim3(256), 0, ctx->stream, r);
    QV_LAUNCH_CHECK(ctx, "k_relabel");
    return QV_OK;
}

}  // extern "C"
