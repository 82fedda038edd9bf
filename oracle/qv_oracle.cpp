// CPU oracle for the sampling -> reindex -> gather path and for the two workload metrics
// (PSGS, feature access probability) of the Quiver paper (arXiv 2305.10863).
//
// THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded statement of what the path
// computes.  Only the tests, the smoke check and the bench's cpu_baseline leg may call it; the
// product (the HIP library) never does, and the two share no code.
//
// Conventions
//   graph     CSR of out-edges: neighbours of v are col[rowptr[v] .. rowptr[v+1]); sampling walks
//             out-edges, as the metric definitions do (Section 4.1, N+).
//   sampling  k-hop uniform neighbour sampling without replacement with a per-hop fanout list
//             (Section 2.1, overview figure narration; Section 6 "k-hop neighbour sampling
//             without replacement").  The paper adopts existing samplers and prints no
//             algorithm, so the random choices are fixed by the contract below.
//   PSGS      Section 4.1, Q_K[i] = sum_k q_k[i].
//   FAP       Section 5.1, P_K[i] = sum_k p_k[i].
//   placement Section 5.2 step (i) sort by FAP, one GPU / one host tier.
//
// Random-choice contract (ours; the paper is silent):
//   Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).  key = (lo32(seed), hi32(seed)),
//   counter = (node, hop, slot, 0): node = global id of the frontier node being expanded, hop is
//   1-based, slot 0-based.  r64 = (x1 << 32) | x0.  rand_below(b) = high 64 bits of r64 * b.
//   deg <= fanout: every adjacency position, in CSR order.
//   deg >  fanout: Floyd's selection (Bentley & Floyd, CACM 30(9), 1987), output in slot order.
//
// Parity pins: see tests/test_oracle_*.py.  The particular random subgraph for a given seed is
// "parity unpinned" by the paper (it prints none); what is pinned is the generator (published
// known-answer vectors), the selection law (uniformity, invariants, brute force) and the metrics
// (the paper's two worked examples, closed forms, exhaustive enumeration).
#include <cstdint>
#include <cstring>
#include <vector>
#include <unordered_map>
#include <unordered_set>
#include <algorithm>

namespace {

// ---- Philox4x32-10 -------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;   // multiplier for word 0
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;   // multiplier for word 2
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;                          // key schedule (golden ratio)
        k1 += 0xBB67AE85u;                          // key schedule (sqrt 3 - 1)
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint64_t rand_below(uint64_t seed, uint32_t node, uint32_t hop, uint32_t slot, uint64_t bound) {
    uint32_t ctr[4] = {node, hop, slot, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    philox4x32_10(ctr, key, x);
    uint64_t r64 = ((uint64_t)x[1] << 32) | x[0];
    unsigned __int128 prod = (unsigned __int128)r64 * bound;
    return (uint64_t)(prod >> 64);
}

// Adjacency positions chosen for one node in one hop, in output order.
void sample_positions(uint64_t seed, int32_t node, int32_t hop, int64_t deg, int32_t fanout,
                      std::vector<int64_t>& pos) {
    pos.clear();
    if (deg <= fanout) {
        for (int64_t i = 0; i < deg; ++i) pos.push_back(i);
        return;
    }
    // Floyd: for j = deg-fanout .. deg-1 draw t in [0, j]; take t unless already taken, else j.
    for (int32_t s = 0; s < fanout; ++s) {
        int64_t j = deg - fanout + s;
        int64_t t = (int64_t)rand_below(seed, (uint32_t)node, (uint32_t)hop, (uint32_t)s,
                                        (uint64_t)(j + 1));
        bool taken = std::find(pos.begin(), pos.end(), t) != pos.end();
        pos.push_back(taken ? j : t);
    }
}

inline double incl_weight(int64_t deg, int32_t fanout, int mode) {
    // mode 0: inclusion probability of one out-edge when min(deg, fanout) of deg are taken
    //         uniformly without replacement -- the reading under which Q is an expected size.
    // mode 1: plain row-stochastic 1/deg (kept only so that tests can show it is NOT the
    //         reading that reproduces the paper's expected-size semantics).
    if (deg <= 0) return 0.0;
    if (mode == 1) return 1.0 / (double)deg;
    return (double)std::min<int64_t>(deg, fanout) / (double)deg;
}

}  // namespace

extern "C" {

void o_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

uint64_t o_rand_below(uint64_t seed, uint32_t node, uint32_t hop, uint32_t slot, uint64_t bound) {
    return rand_below(seed, node, hop, slot, bound);
}

// Positions picked for one node; returns how many (min(deg, fanout)).
int64_t o_sample_positions(uint64_t seed, int32_t node, int32_t hop, int64_t deg, int32_t fanout,
                           int64_t* pos_out) {
    std::vector<int64_t> pos;
    sample_positions(seed, node, hop, deg, fanout, pos);
    for (size_t i = 0; i < pos.size(); ++i) pos_out[i] = pos[i];
    return (int64_t)pos.size();
}

// One hop over a frontier (order matters).  nbr_out holds the segments back to back in frontier
// order; off_out[f] is where frontier[f]'s segment starts, off_out[n_frontier] the total.
// nbr_out may be NULL to obtain only the offsets.  Returns the total, or -1 on a bad node id.
int64_t o_sample_hop(int64_t n_nodes, const int64_t* rowptr, const int32_t* col,
                     const int32_t* frontier, int64_t n_frontier, int32_t fanout, uint64_t seed,
                     int32_t hop, int32_t* nbr_out, int64_t* off_out) {
    std::vector<int64_t> pos;
    int64_t total = 0;
    for (int64_t f = 0; f < n_frontier; ++f) {
        int32_t v = frontier[f];
        if (v < 0 || v >= n_nodes) return -1;
        off_out[f] = total;
        int64_t start = rowptr[v], deg = rowptr[v + 1] - rowptr[v];
        sample_positions(seed, v, hop, deg, fanout, pos);
        for (int64_t p : pos) {
            if (nbr_out) nbr_out[total] = col[start + p];
            ++total;
        }
    }
    off_out[n_frontier] = total;
    return total;
}

// Dedup + relabel.  `known` is the list of ids that already have local ids (local id = index,
// entries distinct).  Scanning nbr in order, an id not seen before is appended to the id list.
// Outputs: n_id_out = known followed by the new ids in order of first appearance;
// local_out[e] = local id of nbr[e]; frontier_out = the distinct ids of nbr in order of first
// appearance within nbr (whether or not they were known before).
// Returns 0, or -1 if `known` holds a repeated id.
int o_reindex(const int32_t* known, int64_t n_known, const int32_t* nbr, int64_t n_nbr,
              int32_t* n_id_out, int64_t* n_id_len, int32_t* local_out, int32_t* frontier_out,
              int64_t* frontier_len) {
    std::unordered_map<int32_t, int32_t> local;
    int64_t n = 0;
    for (int64_t i = 0; i < n_known; ++i) {
        if (!local.emplace(known[i], (int32_t)n).second) return -1;
        n_id_out[n++] = known[i];
    }
    std::unordered_set<int32_t> seen_here;
    int64_t nf = 0;
    for (int64_t e = 0; e < n_nbr; ++e) {
        int32_t g = nbr[e];
        auto it = local.find(g);
        if (it == local.end()) {
            it = local.emplace(g, (int32_t)n).first;
            n_id_out[n++] = g;
        }
        local_out[e] = it->second;
        if (seen_here.insert(g).second) frontier_out[nf++] = g;
    }
    *n_id_len = n;
    *frontier_len = nf;
    return 0;
}

// Multi-hop sampling.  cumulative == 0 (layer frontiers): hop k expands exactly the distinct nodes
// that hop k-1 produced (hop 0 = the distinct seeds), which is the process the PSGS and FAP
// recursions model (q_k is driven by the hop k-1 set; p_k by p_{k-1}).  cumulative != 0: hop k
// expands every node sampled so far (n_id after hop k-1, in local-id order), which yields the
// nested bipartite blocks that GraphSAGE / GAT layers consume in the libraries whose samplers the
// paper adopts (Section 6); a node expanded again in a later hop draws afresh (the hop number is
// part of the random stream).  `frontier` holds the distinct neighbours of each hop either way.
//   n_id          all distinct sampled nodes, seeds first, in order of first appearance
//   row/col_local per edge: local id of the expanded node / of the sampled neighbour
//   nbr_global    per edge: global id of the sampled neighbour
//   frontier      F_0, F_1, .., F_K back to back; frontier_off[K+2]
//   node_off[K+2] node_off[0] = 0, node_off[k+1] = size of n_id after hop k (k = 0: the seeds)
//   edge_off[K+1] edge range of hop k is [edge_off[k-1], edge_off[k])
// Output arrays must be large enough (bounds: see the binding).  Returns 0, -1 on a bad id.
int o_sample(int64_t n_nodes, const int64_t* rowptr, const int32_t* col, const int32_t* seeds,
             int64_t n_seeds, const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed,
             int32_t cumulative, int32_t* n_id, int32_t* row_local, int32_t* col_local, int32_t* nbr_global,
             int32_t* frontier, int64_t* node_off, int64_t* edge_off, int64_t* frontier_off) {
    std::unordered_map<int32_t, int32_t> local;
    std::vector<int32_t> cur;                       // F_{k-1}
    int64_t n_nodes_out = 0, n_edges = 0, n_front = 0;
    node_off[0] = 0; edge_off[0] = 0; frontier_off[0] = 0;
    for (int64_t i = 0; i < n_seeds; ++i) {
        int32_t s = seeds[i];
        if (s < 0 || s >= n_nodes) return -1;
        if (local.emplace(s, (int32_t)n_nodes_out).second) {
            n_id[n_nodes_out++] = s;
            cur.push_back(s);
            frontier[n_front++] = s;
        }
    }
    node_off[1] = n_nodes_out; frontier_off[1] = n_front;
    std::vector<int64_t> pos;
    for (int32_t k = 1; k <= n_hops; ++k) {
        std::vector<int32_t> next;
        std::unordered_set<int32_t> seen_here;
        if (cumulative) cur.assign(n_id, n_id + n_nodes_out);       // everything sampled so far
        for (int32_t v : cur) {
            int64_t start = rowptr[v], deg = rowptr[v + 1] - rowptr[v];
            sample_positions(rng_seed, v, k, deg, fanouts[k - 1], pos);
            int32_t v_local = local.at(v);
            for (int64_t p : pos) {
                int32_t g = col[start + p];
                auto it = local.find(g);
                if (it == local.end()) {
                    it = local.emplace(g, (int32_t)n_nodes_out).first;
                    n_id[n_nodes_out++] = g;
                }
                row_local[n_edges] = v_local;
                col_local[n_edges] = it->second;
                nbr_global[n_edges] = g;
                ++n_edges;
                if (seen_here.insert(g).second) next.push_back(g);
            }
        }
        for (int32_t g : next) frontier[n_front++] = g;
        node_off[k + 1] = n_nodes_out;
        edge_off[k] = n_edges;
        frontier_off[k + 1] = n_front;
        if (!cumulative) cur.swap(next);
    }
    return 0;
}

// Feature aggregation: out[r] = table[ids[r]] as raw bytes (Section 2.1: collect the features of
// all sampled nodes into one tensor).  Where a row physically lives never changes the result.
int o_gather(const uint8_t* table, int64_t n_rows, int64_t row_bytes, const int32_t* ids,
             int64_t n_ids, uint8_t* out) {
    for (int64_t r = 0; r < n_ids; ++r) {
        if (ids[r] < 0 || ids[r] >= n_rows) return -1;
        std::memcpy(out + r * row_bytes, table + (int64_t)ids[r] * row_bytes, (size_t)row_bytes);
    }
    return 0;
}

// PSGS (Section 4.1).  Q[i] = sum_{k=0..K} q_k[i], q_0 = 1,
//   q_k[i] = sum_j delta_{k-1}(i,j) * min(deg(j), l_k),   delta_0 = identity,
//   delta_k = A_1 A_2 .. A_k with A_m[i][j] = w_m(i) on every out-edge i->j.
// For all nodes at once the sum is taken from the far end (the same terms, re-associated):
//   S_m[i] = min(deg i, l_m) + w_m(i) * sum_{j in N+(i)} S_{m+1}[j],  S_{K+1} = 0,  Q = 1 + S_1,
// where S_m[i] is the expected number of nodes sampled in hops m..K below a node i that sits in
// hop m-1.  o_psgs_forward below evaluates the printed formula in its printed order for one
// start node; the tests require the two to agree.
void o_psgs(int64_t n, const int64_t* rowptr, const int32_t* col, const int32_t* fanouts,
            int32_t n_hops, int32_t weight_mode, double* Q) {
    std::vector<double> S_next((size_t)n, 0.0), S((size_t)n, 0.0);
    for (int32_t m = n_hops; m >= 1; --m) {
        int32_t l = fanouts[m - 1];
        for (int64_t i = 0; i < n; ++i) {
            int64_t deg = rowptr[i + 1] - rowptr[i];
            double acc = 0.0;
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) acc += S_next[col[e]];
            S[i] = (double)std::min<int64_t>(deg, l) + incl_weight(deg, l, weight_mode) * acc;
        }
        S.swap(S_next);
    }
    for (int64_t i = 0; i < n; ++i) Q[i] = 1.0 + S_next[i];
}

// The printed formula in its own order, for one start node: carry row i of delta_{k-1} as a
// dense vector, q_k[i] = sum_j delta_{k-1}(i,j) min(deg j, l_k).  O(K (N + E)) per start node.
// q_out[0..K] receives q_0..q_K.
void o_psgs_forward(int64_t n, const int64_t* rowptr, const int32_t* col, const int32_t* fanouts,
                    int32_t n_hops, int32_t weight_mode, int64_t start, double* q_out) {
    std::vector<double> delta((size_t)n, 0.0), nxt((size_t)n, 0.0);
    delta[start] = 1.0;
    q_out[0] = 1.0;
    for (int32_t k = 1; k <= n_hops; ++k) {
        int32_t l = fanouts[k - 1];
        double qk = 0.0;
        std::fill(nxt.begin(), nxt.end(), 0.0);
        for (int64_t j = 0; j < n; ++j) {
            if (delta[j] == 0.0) continue;
            int64_t deg = rowptr[j + 1] - rowptr[j];
            qk += delta[j] * (double)std::min<int64_t>(deg, l);
            double w = incl_weight(deg, l, weight_mode);
            for (int64_t e = rowptr[j]; e < rowptr[j + 1]; ++e) nxt[col[e]] += delta[j] * w;
        }
        q_out[k] = qk;
        delta.swap(nxt);
    }
}

// FAP (Section 5.1).  P[i] = sum_{k=0..K} p_k[i];  p_0 = seed distribution (NULL = 1/N);
//   p_k[i] = sum_j p_0[j] delta_k(j,i)  with delta_k = A_1 .. A_k  as above, i.e.
//   p_k[i] = sum_{j -> i} p_{k-1}[j] * w_k(j).
// p_layers (may be NULL) receives p_0..p_K as (K+1) x N, row-major.
void o_access_prob(int64_t n, const int64_t* rowptr, const int32_t* col, const int32_t* fanouts,
                   int32_t n_hops, const double* p0, int32_t weight_mode, double* P,
                   double* p_layers) {
    std::vector<double> p((size_t)n), nxt((size_t)n);
    for (int64_t i = 0; i < n; ++i) p[i] = p0 ? p0[i] : 1.0 / (double)n;
    for (int64_t i = 0; i < n; ++i) P[i] = p[i];
    if (p_layers) std::memcpy(p_layers, p.data(), sizeof(double) * (size_t)n);
    for (int32_t k = 1; k <= n_hops; ++k) {
        int32_t l = fanouts[k - 1];
        std::fill(nxt.begin(), nxt.end(), 0.0);
        for (int64_t j = 0; j < n; ++j) {
            int64_t deg = rowptr[j + 1] - rowptr[j];
            double c = p[j] * incl_weight(deg, l, weight_mode);
            if (c == 0.0) continue;
            for (int64_t e = rowptr[j]; e < rowptr[j + 1]; ++e) nxt[col[e]] += c;
        }
        p.swap(nxt);
        for (int64_t i = 0; i < n; ++i) P[i] += p[i];
        if (p_layers) std::memcpy(p_layers + (size_t)k * n, p.data(), sizeof(double) * (size_t)n);
    }
}

// Placement, single GPU + host memory (Section 5.2 step (i), and the lookup table of
// Section 5.3): order ids by access probability, highest first, ties by smaller id; the first
// n_hot go to the GPU tier.  loc[id] = hot row index, or ~(cold row index) with the cold rows
// kept in ascending id order.
void o_place(const float* prob, int64_t n, int64_t n_hot, int32_t* rank_out, int32_t* loc_out) {
    std::vector<int32_t> order((size_t)n);
    for (int64_t i = 0; i < n; ++i) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return prob[a] > prob[b]; });
    for (int64_t i = 0; i < n; ++i) rank_out[i] = order[i];
    if (!loc_out) return;
    if (n_hot > n) n_hot = n;
    std::vector<char> hot((size_t)n, 0);
    for (int64_t i = 0; i < n_hot; ++i) { loc_out[order[i]] = (int32_t)i; hot[order[i]] = 1; }
    int32_t c = 0;
    for (int64_t id = 0; id < n; ++id) if (!hot[id]) loc_out[id] = ~(c++);
}

}  // extern "C"
