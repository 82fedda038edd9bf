// Workload metrics over the whole graph: PSGS (pull sweeps over out-edges), feature access
// probability (push sweeps with fp64 hardware atomics) and the placement order (radix sort).
//
// Both metrics are K sparse matrix-VECTOR sweeps, not a K-th matrix power: the sums the paper
// defines re-associate so that only one value per node is carried between hops.
//   PSGS:  S_m[i] = min(deg i, l_m) + (min(deg i, l_m)/deg i) * sum_{j in N+(i)} S_{m+1}[j],
//          S_{K+1} = 0,  Q = 1 + S_1.
//   FAP:   p_k[i] = sum_{j -> i} p_{k-1}[j] * min(deg j, l_k)/deg j,  P = sum_k p_k.
// Row sums run to 10^5 terms and in-degree sums to 10^6 and more, so partial sums are kept in
// fp64 (vector fp64 adds are far from the bottleneck next to the memory traffic); values carried
// between PSGS sweeps and all outputs are fp32.
#include "qv_internal.hpp"
#include <cstring>
#include <string.h>
#include <rocprim/rocprim.hpp>

namespace qv {

template <int G>
__device__ __forceinline__ double group_sum(double v) {
#pragma unroll
    for (int o = G / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, G);
    return v;
}

// One PSGS sweep: group of G lanes per row.  s_next == nullptr is the innermost hop (no edges read).
// Long rows are left to k_psgs_long; the first edge-reading sweep of a call lists them (collect != 0),
// the later ones only skip them (the list depends on the graph alone).
template <int G, typename RP>
__global__ void __launch_bounds__(256) k_psgs_sweep(const RP* __restrict__ rowptr, const int32_t* __restrict__ col,
                                                    int64_t n, int32_t fanout, const float* __restrict__ s_next,
                                                    float* __restrict__ s_out, float add, int32_t* __restrict__ long_rows,
                                                    int32_t* n_long, int32_t long_cap, int32_t collect) {
    const int sub = threadIdx.x % G;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / G;
    const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / G;
    for (int64_t i = group; i < n; i += n_groups) {
        const int64_t rs = (int64_t)rowptr[i], re = (int64_t)rowptr[i + 1];
        const int64_t deg = re - rs;
        const double m = (double)(deg < fanout ? deg : (int64_t)fanout);
        double val = m;
        if (s_next && deg > kLongRow) {
            if (collect && sub == 0) {
                const int32_t k = atomicAdd(n_long, 1);
                if (k < long_cap) long_rows[k] = (int32_t)i;
            }
            continue;
        }
        if (s_next && deg > 0) {
            // kAhead neighbours, then their kAhead values, are requested before the first is used
            constexpr int kAhead = 8;
            double acc0 = 0.0, acc1 = 0.0;
            for (int64_t e = rs + sub; e < re; e += kAhead * G) {
                int32_t nb[kAhead];
#pragma unroll
                for (int j = 0; j < kAhead; ++j) nb[j] = e + j * G < re ? col[e + j * G] : -1;
                float x[kAhead];
#pragma unroll
                for (int j = 0; j < kAhead; ++j) x[j] = nb[j] >= 0 ? s_next[nb[j]] : 0.0f;
#pragma unroll
                for (int j = 0; j < kAhead; j += 2) { acc0 += (double)x[j]; acc1 += (double)x[j + 1]; }
            }
            double acc = group_sum<G>(acc0 + acc1);
            val = m + (m / (double)deg) * acc;
        }
        if (sub == 0) s_out[i] = (float)(val + (double)add);
    }
}

// the listed long rows of a PSGS sweep, a workgroup per row, four loads a thread in flight
template <typename RP>
__global__ void __launch_bounds__(256) k_psgs_long(const RP* __restrict__ rowptr, const int32_t* __restrict__ col,
                                                   int32_t fanout, const float* __restrict__ s_next,
                                                   float* __restrict__ s_out, float add,
                                                   const int32_t* __restrict__ long_rows, const int32_t* n_long,
                                                   int32_t long_cap) {
    __shared__ double part[256 / kWave];
    int32_t count = *n_long;
    if (count > long_cap) count = long_cap;
    for (int32_t k = blockIdx.x; k < count; k += gridDim.x) {
        const int64_t i = long_rows[k];
        const int64_t rs = (int64_t)rowptr[i], re = (int64_t)rowptr[i + 1];
        const int64_t deg = re - rs;
        double acc0 = 0.0, acc1 = 0.0;
        int64_t e = rs + threadIdx.x;
        for (; e + 768 < re; e += 1024) {
            const float x0 = s_next[col[e]], x1 = s_next[col[e + 256]], x2 = s_next[col[e + 512]], x3 = s_next[col[e + 768]];
            acc0 += (double)x0 + (double)x2; acc1 += (double)x1 + (double)x3;
        }
        for (; e < re; e += 256) acc0 += (double)s_next[col[e]];
        const double w = group_sum<kWave>(acc0 + acc1);
        __syncthreads();
        if (threadIdx.x % kWave == 0) part[threadIdx.x / kWave] = w;
        __syncthreads();
        if (threadIdx.x == 0) {
            double acc = 0.0;
            for (int q = 0; q < 256 / kWave; ++q) acc += part[q];
            const double m = (double)(deg < fanout ? deg : (int64_t)fanout);
            s_out[i] = (float)(m + (m / (double)deg) * acc + (double)add);
        }
    }
}

__global__ void k_psgs_control_clear(int32_t* n_long) { *n_long = 0; }

__global__ void k_psgs_batch_sum(const float* __restrict__ psgs, int64_t n_nodes, const int32_t* __restrict__ seeds,
                                 int64_t n_seeds, double* out, int32_t* status) {
    __shared__ double part[256 / kWave];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n_seeds; i += blockDim.x) {
        int32_t s = seeds[i];
        if (s < 0 || (int64_t)s >= n_nodes) atomicOr(status, kStatRange);
        else acc += (double)psgs[s];
    }
    acc = group_sum<kWave>(acc);
    if (threadIdx.x % kWave == 0) part[threadIdx.x / kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < (int)(blockDim.x / kWave); ++w) t += part[w];
        *out = t;
    }
}

// FAP ------------------------------------------------------------------------------------------
__global__ void k_fap_init(int64_t n, const float* __restrict__ p0, double uniform, double* __restrict__ p_cur,
                           double* __restrict__ p_nxt, double* __restrict__ p_tot) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) {
        double v = p0 ? (double)p0[i] : uniform;
        p_cur[i] = v; p_tot[i] = v; p_nxt[i] = 0.0;
    }
}

// push: every out-edge j -> i adds p_cur[j] * w(j) to p_nxt[i]
template <int G, typename RP>
__global__ void __launch_bounds__(256) k_fap_push(const RP* __restrict__ rowptr, const int32_t* __restrict__ col,
                                                  int64_t n, int32_t fanout, const double* __restrict__ p_cur,
                                                  double* __restrict__ p_nxt) {
    const int sub = threadIdx.x % G;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / G;
    const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / G;
    for (int64_t j = group; j < n; j += n_groups) {
        const int64_t rs = (int64_t)rowptr[j], re = (int64_t)rowptr[j + 1];
        const int64_t deg = re - rs;
        if (deg == 0) continue;
        const double m = (double)(deg < fanout ? deg : (int64_t)fanout);
        const double c = p_cur[j] * (m / (double)deg);
        if (c == 0.0) continue;
        for (int64_t e = rs + sub; e < re; e += G) unsafeAtomicAdd(&p_nxt[col[e]], c);
    }
}

// fold the finished layer into the total, clear the buffer the next sweep will add into
__global__ void k_fap_fold(int64_t n, const double* __restrict__ p_new, double* __restrict__ p_tot,
                           double* __restrict__ p_old, float* __restrict__ out) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) {
        double t = p_tot[i] + p_new[i];
        p_tot[i] = t;
        p_old[i] = 0.0;
        if (out) out[i] = (float)t;
    }
}

// FAP with the in-edge CSR at hand.
//   c_k[j]   = p_{k-1}[j] * min(deg_out j, l_k) / deg_out j      (what node j sends along each out-edge)
//   p_k[i]   = sum over in-neighbours j of c_k[j]
// Every sweep runs in one of two directions, chosen on the device from the number of out-edges that
// leave nodes with mass (counted while the previous sweep finishes its rows):
//   gather  (k_fap_pull, k_fap_pull_long): row i sums c_k over its in-row; no atomics; reads all edges.
//   scatter (k_fap_scatter + k_fap_scatter_fold): nodes with mass add c_k[j] along their out-edges
//           with fp64 atomics; reads only those edges.
// A random atomic costs about 2.5 random loads on this GPU, so scatter is taken when 2.5 x the active
// edges is below what the gather costs in random loads (a sparse p_0; the later sweeps of a
// citation-like graph, where two thirds of the nodes are never cited and so carry no mass after the
// first sweep).
// Both kernels of both directions are launched every sweep; the ones not chosen return at once.
// Rows longer than kLongRow are left out by k_fap_pull so that one hub does not hold a 16-lane group
// for milliseconds.  An in-edge CSR that carries the long rows' work items (one the library built: its
// rows list their sources in ascending order) has them summed block of sources by block of sources
// (k_fap_pull_items): all long rows' edges into block b are visited while the 2 MB of c values of
// block b sit in the L2 caches, instead of one 128-byte line fetched from HBM per edge.  Any other
// in-edge CSR gets a workgroup per long row (k_fap_pull_long).
constexpr double kAtomicPerLoadCost = 2.5;
constexpr double kBlockedEdgeCost = 0.2;            // an edge of the blocked gather, in random loads from HBM

struct FapControl {
    double active_edges;    // out-edges of nodes whose c of the coming sweep is non-zero (exact: integers below 2^53)
    int32_t scatter;        // direction of the sweep being run
    int32_t n_long;         // rows handed to k_fap_pull_long
};

template <typename RPF>
__device__ __forceinline__ double send_weight(const RPF* __restrict__ rowptr_f, int64_t i, int32_t fanout, double* deg_out) {
    const int64_t deg = (int64_t)rowptr_f[i + 1] - (int64_t)rowptr_f[i];
    *deg_out = (double)deg;
    if (deg <= 0 || fanout <= 0) return 0.0;
    return (double)(deg < fanout ? deg : (int64_t)fanout) / (double)deg;
}

// every lane of the wave calls this once, at the end of the kernel
__device__ __forceinline__ void add_active(FapControl* ctl, double local) {
    const double w = group_sum<kWave>(local);
    if (threadIdx.x % kWave == 0 && w != 0.0) unsafeAtomicAdd(&ctl->active_edges, w);
}

template <typename RPF>
__global__ void k_fap_pull_init(int64_t n, const float* __restrict__ p0, double uniform, const RPF* __restrict__ rowptr_f,
                                int32_t fanout1, double* __restrict__ c_cur, double* __restrict__ p_tot, FapControl* ctl) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    double active = 0.0;
    for (int64_t i = tid; i < n; i += stride) {
        const double v = p0 ? (double)p0[i] : uniform;
        double deg;
        const double c = v * send_weight(rowptr_f, i, fanout1, &deg);
        p_tot[i] = v;
        c_cur[i] = c;
        if (c != 0.0) active += deg;
    }
    add_active(ctl, active);
}

__global__ void k_fap_control_clear(FapControl* ctl) { ctl->active_edges = 0.0; ctl->scatter = 0; ctl->n_long = 0; }

// before each sweep: fix its direction, restart the counters the sweep fills for the next one
__global__ void k_fap_decide(FapControl* ctl, double n_edges, int32_t allow_scatter) {
    ctl->scatter = (allow_scatter && ctl->active_edges * kAtomicPerLoadCost < n_edges) ? 1 : 0;
    ctl->active_edges = 0.0;
    ctl->n_long = 0;
}

// p = p_k[i]: fold into the total, prepare c_{k+1}[i]; returns the out-edges i activates in the next sweep
template <typename RPF>
__device__ __forceinline__ double fap_finish_row(int64_t i, double p, const RPF* __restrict__ rowptr_f, int32_t next_fanout,
                                                 double* __restrict__ c_nxt, double* __restrict__ p_tot,
                                                 float* __restrict__ out) {
    const double t = p_tot[i] + p;
    p_tot[i] = t;
    if (out) out[i] = (float)t;
    if (next_fanout <= 0) return 0.0;
    double deg;
    const double c = p * send_weight(rowptr_f, i, next_fanout, &deg);
    c_nxt[i] = c;
    return c != 0.0 ? deg : 0.0;
}

template <int G, typename RPT, typename RPF>
__global__ void __launch_bounds__(256) k_fap_pull(const RPT* __restrict__ rowptr_t, const int32_t* __restrict__ col_t,
                                                  const RPF* __restrict__ rowptr_f, int64_t n, int32_t next_fanout,
                                                  const double* __restrict__ c_cur, double* __restrict__ c_nxt,
                                                  double* __restrict__ p_tot, float* __restrict__ out,
                                                  int32_t* __restrict__ long_rows, FapControl* ctl, int32_t long_cap) {
    // (long_rows == nullptr: the long rows are known already and only skipped here)
    if (ctl->scatter) return;
    const int sub = threadIdx.x % G;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / G;
    const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / G;
    double active = 0.0;
    for (int64_t i = group; i < n; i += n_groups) {
        const int64_t rs = (int64_t)rowptr_t[i], re = (int64_t)rowptr_t[i + 1];
        if (re - rs > kLongRow) {
            if (sub == 0 && long_rows) {
                const int32_t k = atomicAdd(&ctl->n_long, 1);
                if (k < long_cap) long_rows[k] = (int32_t)i;
            }
            continue;
        }
        // kAhead sources, then their kAhead values, are requested before the first is used: most rows are
        // done in one round, and the sweep's time is how many of these random reads are in flight
        constexpr int kAhead = 8;
        double acc0 = 0.0, acc1 = 0.0;
        for (int64_t e = rs + sub; e < re; e += kAhead * G) {
            int32_t src[kAhead];
#pragma unroll
            for (int j = 0; j < kAhead; ++j) src[j] = e + j * G < re ? col_t[e + j * G] : -1;
            double x[kAhead];
#pragma unroll
            for (int j = 0; j < kAhead; ++j) x[j] = src[j] >= 0 ? c_cur[src[j]] : 0.0;
#pragma unroll
            for (int j = 0; j < kAhead; j += 2) { acc0 += x[j]; acc1 += x[j + 1]; }
        }
        const double p = group_sum<G>(acc0 + acc1);
        if (sub == 0) active += fap_finish_row(i, p, rowptr_f, next_fanout, c_nxt, p_tot, out);
    }
    add_active(ctl, active);
}

template <typename RPT, typename RPF>
__global__ void __launch_bounds__(256) k_fap_pull_long(const RPT* __restrict__ rowptr_t, const int32_t* __restrict__ col_t,
                                                       const RPF* __restrict__ rowptr_f, int32_t next_fanout,
                                                       const double* __restrict__ c_cur, double* __restrict__ c_nxt,
                                                       double* __restrict__ p_tot, float* __restrict__ out,
                                                       const int32_t* __restrict__ long_rows, FapControl* ctl,
                                                       int32_t long_cap) {
    __shared__ double part[256 / kWave];
    if (ctl->scatter) return;
    int32_t count = ctl->n_long;
    if (count > long_cap) count = long_cap;
    double active = 0.0;
    for (int32_t k = blockIdx.x; k < count; k += gridDim.x) {
        const int64_t i = long_rows[k];
        const int64_t rs = (int64_t)rowptr_t[i], re = (int64_t)rowptr_t[i + 1];
        double acc0 = 0.0, acc1 = 0.0;
        int64_t e = rs + threadIdx.x;
        for (; e + 256 < re; e += 512) {
            const double x0 = c_cur[col_t[e]], x1 = c_cur[col_t[e + 256]];
            acc0 += x0; acc1 += x1;
        }
        if (e < re) acc0 += c_cur[col_t[e]];
        const double w = group_sum<kWave>(acc0 + acc1);
        __syncthreads();
        if (threadIdx.x % kWave == 0) part[threadIdx.x / kWave] = w;
        __syncthreads();
        if (threadIdx.x == 0) {
            double p = 0.0;
            for (int q = 0; q < 256 / kWave; ++q) p += part[q];
            active += fap_finish_row(i, p, rowptr_f, next_fanout, c_nxt, p_tot, out);
        }
    }
    add_active(ctl, active);
}

// Long rows, block of sources by block of sources: one group of 32 lanes per work item (at most 256
// edges of one long row whose sources lie in one block; the in-edge CSR lists them block by block).
// Workgroups start in the order of their index, so the items being worked on at any time are about as
// many consecutive ones as the chip holds groups, i.e. they read one or two blocks of c.  A lane
// requests all its sources, then all their values, then adds; the item's sum goes to psum[k] with one
// fp64 atomic.
constexpr int kItemLanes = 32;
__global__ void __launch_bounds__(256) k_fap_pull_items(const int32_t* __restrict__ col_t, const FapItem* __restrict__ items,
                                                        int64_t n_items, const double* __restrict__ c_cur,
                                                        double* __restrict__ psum, const FapControl* ctl) {
    if (ctl->scatter) return;
    constexpr int kPer = kFapItemEdges / kItemLanes;
    const int sub = threadIdx.x % kItemLanes;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kItemLanes;
    FapItem it{0, 0, 0};
    if (group < n_items) it = items[group];
    int32_t src[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int at = j * kItemLanes + sub;
        src[j] = at < it.count ? __builtin_nontemporal_load(&col_t[it.first + at]) : -1;
    }
    double x[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) x[j] = src[j] >= 0 ? c_cur[src[j]] : 0.0;
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) acc += x[j];
    const double p = group_sum<kItemLanes>(acc);
    if (sub == 0 && p != 0.0) unsafeAtomicAdd(&psum[it.k], p);
}

// ... then every long row is finished from its sum, which goes back to zero for the next sweep
template <typename RPF>
__global__ void __launch_bounds__(256) k_fap_long_finish(const int32_t* __restrict__ long_rows, int32_t n_long,
                                                         double* __restrict__ psum, const RPF* __restrict__ rowptr_f,
                                                         int32_t next_fanout, double* __restrict__ c_nxt,
                                                         double* __restrict__ p_tot, float* __restrict__ out, FapControl* ctl) {
    if (ctl->scatter) return;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    double active = 0.0;
    for (int64_t k = tid; k < n_long; k += stride) {
        const double p = psum[k];
        psum[k] = 0.0;
        active += fap_finish_row((int64_t)long_rows[k], p, rowptr_f, next_fanout, c_nxt, p_tot, out);
    }
    add_active(ctl, active);
}

__global__ void k_fap_zero(double* __restrict__ v, int64_t n) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) v[i] = 0.0;
}

// scatter direction, step 1: the accumulator (the next sweep's c array) starts at zero
__global__ void k_fap_scatter_clear(int64_t n, double* __restrict__ c_nxt, const FapControl* ctl) {
    if (!ctl->scatter) return;
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) c_nxt[i] = 0.0;
}

// step 2: nodes with mass add what they send to each out-neighbour's accumulator
template <int G, typename RPF>
__global__ void __launch_bounds__(256) k_fap_scatter(const RPF* __restrict__ rowptr_f, const int32_t* __restrict__ col_f, int64_t n,
                                                     const double* __restrict__ c_cur, double* __restrict__ acc,
                                                     const FapControl* ctl) {
    if (!ctl->scatter) return;
    const int sub = threadIdx.x % G;
    const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / G;
    const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / G;
    for (int64_t j = group; j < n; j += n_groups) {
        const double c = c_cur[j];
        if (c == 0.0) continue;
        const int64_t rs = (int64_t)rowptr_f[j], re = (int64_t)rowptr_f[j + 1];
        for (int64_t e = rs + sub; e < re; e += G) unsafeAtomicAdd(&acc[col_f[e]], c);
    }
}

// step 3: the accumulator holds p_k; finish every row in place (acc[i] becomes c_{k+1}[i])
template <typename RPF>
__global__ void k_fap_scatter_fold(int64_t n, const RPF* __restrict__ rowptr_f, int32_t next_fanout, double* acc,
                                   double* __restrict__ p_tot, float* __restrict__ out, FapControl* ctl) {
    if (!ctl->scatter) return;
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    double active = 0.0;
    for (int64_t i = tid; i < n; i += stride) {
        const double p = acc[i];
        const double t = p_tot[i] + p;
        p_tot[i] = t;
        if (out) out[i] = (float)t;
        if (next_fanout > 0) {
            double deg;
            const double c = p * send_weight(rowptr_f, i, next_fanout, &deg);
            acc[i] = c;
            if (c != 0.0) active += deg;
        }
    }
    add_active(ctl, active);
}

// placement keys: ascending order of the key == descending prob, ties by ascending id
__global__ void k_rank_keys(int64_t n, const float* __restrict__ prob, uint64_t* __restrict__ keys) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) {
        float f = prob[i];
        if (f == 0.0f) f = 0.0f;                                  // -0 and +0 compare equal
        uint32_t b = __float_as_uint(f);
        uint32_t asc = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
        keys[i] = ((uint64_t)(~asc) << 32) | (uint64_t)(uint32_t)i;
    }
}
__global__ void k_rank_ids(int64_t n, const uint64_t* __restrict__ keys, int32_t* __restrict__ rank) {
    int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n; i += stride) rank[i] = (int32_t)(uint32_t)keys[i];
}

static int group_width_for(int64_t n, int64_t e) {
    double avg = n > 0 ? (double)e / (double)n : 0.0;
    return avg < 12 ? 4 : avg < 24 ? 8 : avg < 48 ? 16 : avg < 96 ? 32 : 64;
}

template <typename RP>
static void launch_psgs_sweep(qv_ctx* ctx, const qv_csr* g, int G, int32_t fanout, const float* s_next, float* s_out,
                              float add, int32_t* long_rows, int32_t* n_long, int32_t long_cap, int32_t collect) {
    int blocks = grid_for(g->n_nodes * G, 256, ctx->n_cu * 32);
    const RP* rp = (const RP*)g->rowptr;
#define QV_SWEEP(GW)                                                                                                   \
    hipLaunchKernelGGL((k_psgs_sweep<GW, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, g->col, g->n_nodes, fanout,    \
                       s_next, s_out, add, long_rows, n_long, long_cap, collect)
    switch (G) {
        case 4: QV_SWEEP(4); break;
        case 8: QV_SWEEP(8); break;
        case 16: QV_SWEEP(16); break;
        case 32: QV_SWEEP(32); break;
        default: QV_SWEEP(64); break;
    }
#undef QV_SWEEP
    if (s_next)
        hipLaunchKernelGGL((k_psgs_long<RP>), dim3(grid_for(long_cap, 1, ctx->n_cu * 4)), dim3(256), 0, ctx->stream, rp, g->col,
                           fanout, s_next, s_out, add, (const int32_t*)long_rows, (const int32_t*)n_long, long_cap);
}

template <typename RP>
static void launch_fap_push(qv_ctx* ctx, const qv_csr* g, int G, int32_t fanout, const double* p_cur, double* p_nxt) {
    int blocks = grid_for(g->n_nodes * G, 256, ctx->n_cu * 32);
    const RP* rp = (const RP*)g->rowptr;
    switch (G) {
        case 4: hipLaunchKernelGGL((k_fap_push<4, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, g->col, g->n_nodes, fanout, p_cur, p_nxt); break;
        case 8: hipLaunchKernelGGL((k_fap_push<8, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, g->col, g->n_nodes, fanout, p_cur, p_nxt); break;
        case 16: hipLaunchKernelGGL((k_fap_push<16, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, g->col, g->n_nodes, fanout, p_cur, p_nxt); break;
        case 32: hipLaunchKernelGGL((k_fap_push<32, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, g->col, g->n_nodes, fanout, p_cur, p_nxt); break;
        default: hipLaunchKernelGGL((k_fap_push<64, RP>), dim3(blocks), dim3(256), 0, ctx->stream, rp, g->col, g->n_nodes, fanout, p_cur, p_nxt); break;
    }
}

static qv_status check_fanouts(qv_ctx* ctx, const char* who, const int32_t* fanouts, int n_hops) {
    if (!fanouts || n_hops < 1 || n_hops > QV_MAX_HOPS) return fail(ctx, QV_EINVAL, "%s: need 1 <= n_hops <= %d and fanouts", who, QV_MAX_HOPS);
    for (int k = 0; k < n_hops; ++k)
        if (fanouts[k] < 1) return fail(ctx, QV_EINVAL, "%s: fanout %d < 1", who, fanouts[k]);
    return QV_OK;
}

}  // namespace qv

using namespace qv;

template <typename RPT, typename RPF>
static qv_status fap_pull(qv_ctx* ctx, const qv_csr* g, const qv_csr* gin, const int32_t* fanouts, int n_hops,
                          const float* p0, float* prob_out) {
    const int64_t n = g->n_nodes;
    const int64_t long_cap64 = gin->n_edges / kLongRow + 1;
    const int32_t long_cap = (int32_t)long_cap64;
    const bool blocked = gin->long_items != nullptr;        // the long rows came with the in-edge CSR, cut into work items
    qv_status rc = arena_begin(ctx, 3 * align_up((size_t)n * 8) + align_up((size_t)long_cap * 4) +
                                        align_up((size_t)gin->n_long * 8) + 4096);
    if (rc != QV_OK) return rc;
    double* c_cur = (double*)arena_take(ctx, (size_t)n * 8);
    double* c_nxt = (double*)arena_take(ctx, (size_t)n * 8);
    double* p_tot = (double*)arena_take(ctx, (size_t)n * 8);
    int32_t* long_rows = blocked ? (int32_t*)nullptr : (int32_t*)arena_take(ctx, (size_t)long_cap * 4);
    double* psum = blocked ? (double*)arena_take(ctx, (size_t)gin->n_long * 8) : (double*)nullptr;
    FapControl* ctl = (FapControl*)arena_take(ctx, sizeof(FapControl));
    const RPT* rpt = (const RPT*)gin->rowptr;
    const RPF* rpf = (const RPF*)g->rowptr;
    const int ew = grid_for(n, 256 * 4, ctx->n_cu * 16);
    hipLaunchKernelGGL(k_fap_control_clear, dim3(1), dim3(1), 0, ctx->stream, ctl);
    hipLaunchKernelGGL((k_fap_pull_init<RPF>), dim3(ew), dim3(256), 0, ctx->stream, n, p0, 1.0 / (double)n, rpf, fanouts[0],
                       c_cur, p_tot, ctl);
    QV_LAUNCH_CHECK(ctx, "k_fap_pull_init");
    const int G = group_width_for(n, gin->n_edges - (blocked ? gin->long_edges : 0));      // lanes per row that k_fap_pull sums
    const int Gf = group_width_for(n, g->n_edges);
    const int blocks = grid_for(n * G, 256, ctx->n_cu * 32);
    const int blocks_f = grid_for(n * Gf, 256, ctx->n_cu * 32);
    const int32_t allow_scatter = ctx->fap_direction != 1;          // 1: gather only (testing aid)
    // what a gather sweep costs, in random loads from HBM; 2: scatter whenever possible
    const double gather_cost = blocked ? (double)(gin->n_edges - gin->long_edges) + kBlockedEdgeCost * (double)gin->long_edges
                                       : (double)gin->n_edges;
    const double edges_for_choice = ctx->fap_direction == 2 ? 1e300 : gather_cost;
    if (blocked) {
        hipLaunchKernelGGL(k_fap_zero, dim3(grid_for(gin->n_long, 256, ctx->n_cu * 4)), dim3(256), 0, ctx->stream, psum,
                           (int64_t)gin->n_long);
        QV_LAUNCH_CHECK(ctx, "k_fap_zero");
    }
    for (int k = 1; k <= n_hops; ++k) {
        const int32_t nf = k < n_hops ? fanouts[k] : 0;
        float* out = k == n_hops ? prob_out : (float*)nullptr;
        hipLaunchKernelGGL(k_fap_decide, dim3(1), dim3(1), 0, ctx->stream, ctl, edges_for_choice, allow_scatter);
#define QV_PULL(GW)                                                                                                    \
    hipLaunchKernelGGL((k_fap_pull<GW, RPT, RPF>), dim3(blocks), dim3(256), 0, ctx->stream, rpt, gin->col, rpf, n, nf,     \
                       (const double*)c_cur, c_nxt, p_tot, out, long_rows, ctl, long_cap)
        switch (G) {
            case 4: QV_PULL(4); break;
            case 8: QV_PULL(8); break;
            case 16: QV_PULL(16); break;
            case 32: QV_PULL(32); break;
            default: QV_PULL(64); break;
        }
#undef QV_PULL
        QV_LAUNCH_CHECK(ctx, "k_fap_pull");
        if (blocked) {
            const int per_block = 256 / kItemLanes;
            hipLaunchKernelGGL(k_fap_pull_items, dim3((unsigned)((gin->n_items + per_block - 1) / per_block)), dim3(256), 0,
                               ctx->stream, gin->col, (const FapItem*)gin->long_items, gin->n_items, (const double*)c_cur, psum,
                               (const FapControl*)ctl);
            QV_LAUNCH_CHECK(ctx, "k_fap_pull_items");
            hipLaunchKernelGGL((k_fap_long_finish<RPF>), dim3(grid_for(gin->n_long, 256, ctx->n_cu * 4)), dim3(256), 0, ctx->stream,
                               (const int32_t*)gin->long_rows, gin->n_long, psum, rpf, nf, c_nxt, p_tot, out, ctl);
            QV_LAUNCH_CHECK(ctx, "k_fap_long_finish");
        } else {
            hipLaunchKernelGGL((k_fap_pull_long<RPT, RPF>), dim3(grid_for(long_cap, 1, ctx->n_cu * 4)), dim3(256), 0, ctx->stream,
                               rpt, gin->col, rpf, nf, (const double*)c_cur, c_nxt, p_tot, out, (const int32_t*)long_rows, ctl,
                               long_cap);
            QV_LAUNCH_CHECK(ctx, "k_fap_pull_long");
        }
        hipLaunchKernelGGL(k_fap_scatter_clear, dim3(ew), dim3(256), 0, ctx->stream, n, c_nxt, (const FapControl*)ctl);
#define QV_SCAT(GW)                                                                                                    \
    hipLaunchKernelGGL((k_fap_scatter<GW, RPF>), dim3(blocks_f), dim3(256), 0, ctx->stream, rpf, g->col, n,                \
                       (const double*)c_cur, c_nxt, (const FapControl*)ctl)
        switch (Gf) {
            case 4: QV_SCAT(4); break;
            case 8: QV_SCAT(8); break;
            case 16: QV_SCAT(16); break;
            case 32: QV_SCAT(32); break;
            default: QV_SCAT(64); break;
        }
#undef QV_SCAT
        QV_LAUNCH_CHECK(ctx, "k_fap_scatter");
        hipLaunchKernelGGL((k_fap_scatter_fold<RPF>), dim3(ew), dim3(256), 0, ctx->stream, n, rpf, nf, c_nxt, p_tot, out, ctl);
        QV_LAUNCH_CHECK(ctx, "k_fap_scatter_fold");
        double* t = c_cur; c_cur = c_nxt; c_nxt = t;
    }
    return QV_OK;
}

extern "C" {

qv_status qv_psgs(qv_ctx* ctx, const qv_csr* g, const int32_t* fanouts, int32_t n_hops, float* psgs_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_psgs: ctx is NULL");
    if (!g || !psgs_out) return fail(ctx, QV_EINVAL, "qv_psgs: null argument");
    qv_status rc = check_fanouts(ctx, "qv_psgs", fanouts, n_hops);
    if (rc != QV_OK) return rc;
    const int64_t n = g->n_nodes;
    if (n == 0) return QV_OK;
    const int32_t long_cap = (int32_t)(g->n_edges / kLongRow + 1);
    rc = arena_begin(ctx, align_up((size_t)n * 4) + align_up((size_t)long_cap * 4) + 4096);
    if (rc != QV_OK) return rc;
    float* tmp = (float*)arena_take(ctx, (size_t)n * 4);
    int32_t* long_rows = (int32_t*)arena_take(ctx, (size_t)long_cap * 4);
    int32_t* n_long = (int32_t*)arena_take(ctx, 4);
    hipLaunchKernelGGL(k_psgs_control_clear, dim3(1), dim3(1), 0, ctx->stream, n_long);
    bool listed = false;
    const int G = group_width_for(n, g->n_edges);
    const float* prev = nullptr;
    for (int j = 0; j < n_hops; ++j) {                 // hop m = K - j
        const int m = n_hops - j;
        float* dst = ((n_hops - 1 - j) % 2 == 0) ? psgs_out : tmp;
        const float add = (m == 1) ? 1.0f : 0.0f;
        const int Gj = prev ? G : 4;                   // the innermost hop reads no edges
        const int32_t collect = (prev && !listed) ? 1 : 0;
        if (g->rowptr_bits == 32) launch_psgs_sweep<int32_t>(ctx, g, Gj, fanouts[m - 1], prev, dst, add, long_rows, n_long, long_cap, collect);
        else launch_psgs_sweep<int64_t>(ctx, g, Gj, fanouts[m - 1], prev, dst, add, long_rows, n_long, long_cap, collect);
        QV_LAUNCH_CHECK(ctx, "k_psgs_sweep");
        if (prev) listed = true;
        prev = dst;
    }
    return QV_OK;
}

qv_status qv_psgs_batch_sum(qv_ctx* ctx, const float* psgs, int64_t n_nodes, const int32_t* seeds, int64_t n_seeds,
                            double* sum_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_psgs_batch_sum: ctx is NULL");
    if (!psgs || !sum_out || n_seeds < 0 || (n_seeds > 0 && !seeds)) return fail(ctx, QV_EINVAL, "qv_psgs_batch_sum: null or negative argument");
    hipLaunchKernelGGL(k_psgs_batch_sum, dim3(1), dim3(256), 0, ctx->stream, psgs, n_nodes, seeds, n_seeds, sum_out, ctx->d_status);
    QV_LAUNCH_CHECK(ctx, "k_psgs_batch_sum");
    return QV_OK;
}

qv_status qv_access_prob(qv_ctx* ctx, const qv_csr* g, const qv_csr* g_in, const int32_t* fanouts, int32_t n_hops,
                         const float* p0, float* prob_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_access_prob: ctx is NULL");
    if (!g || !prob_out) return fail(ctx, QV_EINVAL, "qv_access_prob: null argument");
    qv_status rc = check_fanouts(ctx, "qv_access_prob", fanouts, n_hops);
    if (rc != QV_OK) return rc;
    const int64_t n = g->n_nodes;
    if (n == 0) return QV_OK;
    if (g_in) {
        if (g_in->n_nodes != n || g_in->n_edges != g->n_edges)
            return fail(ctx, QV_EINVAL, "qv_access_prob: the in-edge CSR must have the node and edge counts of the graph");
        if (g_in->rowptr_bits == 32) return g->rowptr_bits == 32 ? fap_pull<int32_t, int32_t>(ctx, g, g_in, fanouts, n_hops, p0, prob_out)
                                                                   : fap_pull<int32_t, int64_t>(ctx, g, g_in, fanouts, n_hops, p0, prob_out);
        return g->rowptr_bits == 32 ? fap_pull<int64_t, int32_t>(ctx, g, g_in, fanouts, n_hops, p0, prob_out)
                                     : fap_pull<int64_t, int64_t>(ctx, g, g_in, fanouts, n_hops, p0, prob_out);
    }
    rc = arena_begin(ctx, 3 * align_up((size_t)n * 8) + 4096);
    if (rc != QV_OK) return rc;
    double* p_cur = (double*)arena_take(ctx, (size_t)n * 8);
    double* p_nxt = (double*)arena_take(ctx, (size_t)n * 8);
    double* p_tot = (double*)arena_take(ctx, (size_t)n * 8);
    const int ew = grid_for(n, 256 * 4, ctx->n_cu * 16);
    hipLaunchKernelGGL(k_fap_init, dim3(ew), dim3(256), 0, ctx->stream, n, p0, 1.0 / (double)n, p_cur, p_nxt, p_tot);
    QV_LAUNCH_CHECK(ctx, "k_fap_init");
    const int G = group_width_for(n, g->n_edges);
    for (int k = 1; k <= n_hops; ++k) {
        if (g->rowptr_bits == 32) launch_fap_push<int32_t>(ctx, g, G, fanouts[k - 1], p_cur, p_nxt);
        else launch_fap_push<int64_t>(ctx, g, G, fanouts[k - 1], p_cur, p_nxt);
        QV_LAUNCH_CHECK(ctx, "k_fap_push");
        hipLaunchKernelGGL(k_fap_fold, dim3(ew), dim3(256), 0, ctx->stream, n, (const double*)p_nxt, p_tot, p_cur,
                           k == n_hops ? prob_out : (float*)nullptr);
        QV_LAUNCH_CHECK(ctx, "k_fap_fold");
        double* t = p_cur; p_cur = p_nxt; p_nxt = t;
    }
    return QV_OK;
}

qv_status qv_place_rank(qv_ctx* ctx, const float* prob, int64_t n, int32_t* rank_out) {
    if (!ctx) return fail(nullptr, QV_EINVAL, "qv_place_rank: ctx is NULL");
    if (n < 0 || n >= ((int64_t)1 << 31) || (n > 0 && (!prob || !rank_out))) return fail(ctx, QV_EINVAL, "qv_place_rank: bad argument");
    if (n == 0) return QV_OK;
    size_t temp_bytes = 0;
    hipError_t e = rocprim::radix_sort_keys((void*)nullptr, temp_bytes, (uint64_t*)nullptr, (uint64_t*)nullptr, (size_t)n,
                                            0, 64, ctx->stream);
    if (e != hipSuccess) return fail(ctx, QV_EHIP, "qv_place_rank: sort sizing failed: %s", hipGetErrorString(e));
    qv_status rc = arena_begin(ctx, 2 * align_up((size_t)n * 8) + align_up(temp_bytes) + 4096);
    if (rc != QV_OK) return rc;
    uint64_t* keys_in = (uint64_t*)arena_take(ctx, (size_t)n * 8);
    uint64_t* keys_out = (uint64_t*)arena_take(ctx, (size_t)n * 8);
    void* temp = arena_take(ctx, temp_bytes);
    const int ew = grid_for(n, 256 * 4, ctx->n_cu * 16);
    hipLaunchKernelGGL(k_rank_keys, dim3(ew), dim3(256), 0, ctx->stream, n, prob, keys_in);
    QV_LAUNCH_CHECK(ctx, "k_rank_keys");
    e = rocprim::radix_sort_keys(temp, temp_bytes, keys_in, keys_out, (size_t)n, 0, 64, ctx->stream);
    if (e != hipSuccess) return fail(ctx, QV_EHIP, "qv_place_rank: sort failed: %s", hipGetErrorString(e));
    hipLaunchKernelGGL(k_rank_ids, dim3(ew), dim3(256), 0, ctx->stream, n, (const uint64_t*)keys_out, rank_out);
    QV_LAUNCH_CHECK(ctx, "k_rank_ids");
    return QV_OK;
}

}  // extern "C"
