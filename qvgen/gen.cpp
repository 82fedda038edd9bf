// Seeded synthetic inputs: power-law CSR graphs, feature tables, seed batches.
//
// This module only makes DATA.  It holds none of the method's arithmetic (no sampler, no
// Philox, no metric) and is the one piece of code that both the CPU oracle's tests and the GPU
// library's tests may call, so that both sides see identical arrays.
//
// Everything is a pure function of (seed, indices) through a 64-bit counter hash, so results do
// not depend on the number of threads used.
#include <cstdint>
#include <cstring>
#include <cmath>
#include <vector>
#include <thread>
#include <atomic>
#include <algorithm>

namespace {

inline uint64_t mix64(uint64_t x) {            // splitmix64 finaliser
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}
inline uint64_t hash4(uint64_t seed, uint64_t dom, uint64_t a, uint64_t b) {
    uint64_t x = mix64(seed ^ (dom * 0xD6E8FEB86659FD93ull + 0x9E3779B97F4A7C15ull));
    x = mix64(x + a * 0x9E3779B97F4A7C15ull + 1);
    x = mix64(x ^ (b * 0xC2B2AE3D27D4EB4Full + 2));
    return x;
}
inline double u01(uint64_t h) { return (double)(h >> 11) * (1.0 / 9007199254740992.0); }

// Stateless pseudo-random permutation of [0, n): 4-round Feistel on 2*half bits + cycle walking.
struct Perm {
    uint64_t n, seed; int half; uint64_t mask;
    Perm(uint64_t n_, uint64_t seed_) : n(n_), seed(seed_) {
        int bits = 2; while ((1ull << bits) < n) bits += 2;
        half = bits / 2; mask = (1ull << half) - 1;
    }
    inline uint64_t once(uint64_t x) const {
        uint64_t L = x >> half, R = x & mask;
        for (int r = 0; r < 4; ++r) {
            uint64_t F = mix64(R + seed * 0x9E3779B97F4A7C15ull + (uint64_t)r * 0xD1B54A32D192ED03ull) & mask;
            uint64_t nl = R; R = L ^ F; L = nl;
        }
        return (L << half) | R;
    }
    inline uint64_t operator()(uint64_t x) const {
        do { x = once(x); } while (x >= n);
        return x;
    }
};

template <class Fn>
void parallel_chunks(int64_t n, int64_t chunk, int n_threads, Fn fn) {
    if (n_threads < 1) n_threads = 1;
    std::atomic<int64_t> next(0);
    auto worker = [&]() {
        for (;;) {
            int64_t b = next.fetch_add(chunk);
            if (b >= n) break;
            fn(b, std::min(n, b + chunk));
        }
    };
    std::vector<std::thread> th;
    for (int t = 1; t < n_threads; ++t) th.emplace_back(worker);
    worker();
    for (auto& t : th) t.join();
}

struct GraphSpec {
    int64_t n; double deg_c; double deg_s; int64_t dmin, dmax;
    int endpoint_mode;       // 0 uniform, 1 shifted power law (Zipf-Mandelbrot) over a permutation
    double ep_s, ep_q; uint64_t seed;
};

inline int64_t degree_of_rank(const GraphSpec& g, uint64_t r /*1-based*/) {
    double d = std::floor(g.deg_c * std::pow((double)r, -g.deg_s));
    if (d < (double)g.dmin) d = (double)g.dmin;
    if (d > (double)g.dmax) d = (double)g.dmax;
    return (int64_t)d;
}

// sum over ranks of the clamped degree, from the counts of ranks at or above each level
double degree_sum_estimate(int64_t n, double c, double s, int64_t dmin, int64_t dmax) {
    double tot = (double)n * (double)dmin;
    for (int64_t k = dmin + 1; k <= dmax; ++k) {
        double r = std::floor(std::pow(c / (double)k, 1.0 / s));
        if (r <= 0) break;
        tot += std::min((double)n, r);
    }
    return tot;
}

inline uint16_t f32_to_f16_rne(float f) {
    uint32_t x; std::memcpy(&x, &f, 4);
    uint32_t sign = (x >> 16) & 0x8000u;
    int32_t e = (int32_t)((x >> 23) & 0xFF) - 127 + 15;
    uint32_t m = x & 0x7FFFFFu;
    if (e >= 31) return (uint16_t)(sign | 0x7C00u);                    // overflow -> inf
    if (e <= 0) {                                                       // subnormal or zero
        if (e < -10) return (uint16_t)sign;
        m |= 0x800000u;
        int shift = 14 - e;                                             // 14..24
        uint32_t half = m >> shift, rem = m & ((1u << shift) - 1), mid = 1u << (shift - 1);
        if (rem > mid || (rem == mid && (half & 1))) ++half;
        return (uint16_t)(sign | half);
    }
    uint32_t half = ((uint32_t)e << 10) | (m >> 13), rem = m & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (half & 1))) ++half;        // may carry into exponent
    return (uint16_t)(sign | half);
}

// Feature element (i, j): Irwin-Hall(4) of 16-bit fields, centred, scaled to unit variance.
// Integer-exact up to one fp32 multiply, so a device kernel can regenerate it bit for bit.
inline float feature_value(uint64_t seed, uint64_t i, uint64_t j) {
    uint64_t h = hash4(seed, 3, i, j);
    int32_t s = (int32_t)(h & 0xFFFF) + (int32_t)((h >> 16) & 0xFFFF) +
                (int32_t)((h >> 32) & 0xFFFF) + (int32_t)(h >> 48) - 131070;
    return (float)s * 2.6428998e-5f;                                    // 1 / 37837.227 = 1 / sd of the sum
}

}  // namespace

extern "C" {

uint64_t qg_hash(uint64_t seed, uint64_t dom, uint64_t a, uint64_t b) { return hash4(seed, dom, a, b); }
uint64_t qg_perm(uint64_t n, uint64_t seed, uint64_t x) { return Perm(n, seed)(x); }

// Find the scale C of the rank-degree law d(r) = clamp(floor(C r^-s), dmin, dmax) whose degree
// sum is closest to `edge_target` (bisection on C).
double qg_calibrate_degree_scale(int64_t n, double s, int64_t dmin, int64_t dmax, double edge_target) {
    double lo = 1e-3, hi = 1.0;
    while (degree_sum_estimate(n, hi, s, dmin, dmax) < edge_target && hi < 1e30) hi *= 2;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (degree_sum_estimate(n, mid, s, dmin, dmax) < edge_target) lo = mid; else hi = mid;
    }
    return hi;
}

// rowptr[n+1] of the directed graph: node v has the degree of rank perm(v)+1.
int64_t qg_graph_rowptr(int64_t n, double deg_c, double deg_s, int64_t dmin, int64_t dmax,
                        uint64_t seed, int n_threads, int64_t* rowptr) {
    GraphSpec g{n, deg_c, deg_s, dmin, std::min<int64_t>(dmax, n), 0, 0, 0, seed};
    Perm perm((uint64_t)n, seed ^ 0x1111);
    parallel_chunks(n, 1 << 16, n_threads, [&](int64_t b, int64_t e) {
        for (int64_t v = b; v < e; ++v) rowptr[v + 1] = degree_of_rank(g, perm((uint64_t)v) + 1);
    });
    rowptr[0] = 0;
    for (int64_t v = 0; v < n; ++v) rowptr[v + 1] += rowptr[v];
    return rowptr[n];
}

// Fill col for the rows of rowptr: distinct endpoints per row, ascending within the row.
// endpoint_mode 0: uniform over nodes.  1: rank x in [0,n) with density ~ (x + q)^-s, mapped to
// a node through a second permutation (a power-law in-degree skew with a flattened head).
void qg_graph_col(int64_t n, const int64_t* rowptr, int endpoint_mode, double ep_s, double ep_q,
                  uint64_t seed, int n_threads, int32_t* col) {
    Perm perm2((uint64_t)n, seed ^ 0x2222);
    const double one_m_s = 1.0 - ep_s;
    const bool log_law = std::fabs(one_m_s) < 1e-9;
    const double a = log_law ? std::log(ep_q) : std::pow(ep_q, one_m_s);
    const double bq = log_law ? std::log((double)n + ep_q) : std::pow((double)n + ep_q, one_m_s);
    parallel_chunks(n, 1 << 12, n_threads, [&](int64_t b, int64_t e) {
        std::vector<int32_t> set;                      // open-addressing set for long rows
        for (int64_t v = b; v < e; ++v) {
            int64_t start = rowptr[v], deg = rowptr[v + 1] - start;
            int32_t* row = col + start;
            bool use_set = deg > 24;
            size_t cap = 0;
            if (use_set) {
                cap = 64; while ((int64_t)cap < 2 * deg) cap <<= 1;
                set.assign(cap, -1);
            }
            for (int64_t j = 0; j < deg; ++j) {
                for (uint64_t attempt = 0;; ++attempt) {
                    uint64_t h = hash4(seed, 2, (uint64_t)v, (uint64_t)j | (attempt << 40));
                    int64_t node;
                    if (endpoint_mode == 0) {
                        node = (int64_t)(((unsigned __int128)h * (uint64_t)n) >> 64);
                    } else {
                        double u = u01(h);
                        double t = a - u * (a - bq);
                        double x = (log_law ? std::exp(t) : std::pow(t, 1.0 / one_m_s)) - ep_q;
                        int64_t r = (int64_t)x;
                        if (r < 0) r = 0;
                        if (r >= n) r = n - 1;
                        node = (int64_t)perm2((uint64_t)r);
                    }
                    bool dup = false;
                    if (use_set) {
                        size_t s = (size_t)mix64((uint64_t)node) & (cap - 1);
                        while (set[s] != -1) {
                            if (set[s] == (int32_t)node) { dup = true; break; }
                            s = (s + 1) & (cap - 1);
                        }
                        if (!dup) set[s] = (int32_t)node;
                    } else {
                        for (int64_t q = 0; q < j; ++q) if (row[q] == (int32_t)node) { dup = true; break; }
                    }
                    if (!dup) { row[j] = (int32_t)node; break; }
                }
            }
            std::sort(row, row + deg);
        }
    });
}

// Symmetrise: out-rows become sorted(unique(out U in)).  Two calls: first with new_col == NULL
// fills new_rowptr (n+1) and returns the new edge count; the second fills new_col.
int64_t qg_symmetrise(int64_t n, const int64_t* rowptr, const int32_t* col, int64_t* new_rowptr,
                      int32_t* new_col, int n_threads) {
    int64_t E = rowptr[n];
    std::vector<int64_t> tptr((size_t)n + 1, 0);
    for (int64_t e = 0; e < E; ++e) tptr[col[e] + 1]++;
    for (int64_t v = 0; v < n; ++v) tptr[v + 1] += tptr[v];
    std::vector<int32_t> tcol((size_t)E);
    {
        std::vector<int64_t> cur(tptr.begin(), tptr.end() - 1);
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) tcol[cur[col[e]]++] = (int32_t)v;
    }   // sources arrive in ascending order, so each transposed row is already sorted
    auto merge_row = [&](int64_t v, int32_t* out) -> int64_t {
        const int32_t *a = col + rowptr[v], *ae = col + rowptr[v + 1];
        const int32_t *b = tcol.data() + tptr[v], *be = tcol.data() + tptr[v + 1];
        int64_t k = 0;
        while (a < ae || b < be) {
            int32_t x;
            if (b >= be || (a < ae && *a < *b)) x = *a++;
            else if (a >= ae || *b < *a) x = *b++;
            else { x = *a; ++a; ++b; }
            if (out) out[k] = x;
            ++k;
        }
        return k;
    };
    if (!new_col) {
        parallel_chunks(n, 1 << 14, n_threads, [&](int64_t b, int64_t e) {
            for (int64_t v = b; v < e; ++v) new_rowptr[v + 1] = merge_row(v, nullptr);
        });
        new_rowptr[0] = 0;
        for (int64_t v = 0; v < n; ++v) new_rowptr[v + 1] += new_rowptr[v];
        return new_rowptr[n];
    }
    parallel_chunks(n, 1 << 14, n_threads, [&](int64_t b, int64_t e) {
        for (int64_t v = b; v < e; ++v) merge_row(v, new_col + new_rowptr[v]);
    });
    return new_rowptr[n];
}

// Feature rows [row_begin, row_end) of an n x dim table, elem_bytes 4 (fp32) or 2 (fp16, RNE).
void qg_features(uint64_t seed, int64_t row_begin, int64_t row_end, int64_t dim, int elem_bytes,
                 int n_threads, void* out) {
    parallel_chunks(row_end - row_begin, 1 << 10, n_threads, [&](int64_t b, int64_t e) {
        for (int64_t r = b; r < e; ++r) {
            uint64_t i = (uint64_t)(row_begin + r);
            if (elem_bytes == 4) {
                float* o = (float*)out + r * dim;
                for (int64_t j = 0; j < dim; ++j) o[j] = feature_value(seed, i, (uint64_t)j);
            } else {
                uint16_t* o = (uint16_t*)out + r * dim;
                for (int64_t j = 0; j < dim; ++j) o[j] = f32_to_f16_rne(feature_value(seed, i, (uint64_t)j));
            }
        }
    });
}

// Feature rows of listed ids (for checking a gather without holding the table).
void qg_feature_rows(uint64_t seed, const int32_t* ids, int64_t n_ids, int64_t dim, int elem_bytes,
                     int n_threads, void* out) {
    parallel_chunks(n_ids, 1 << 8, n_threads, [&](int64_t b, int64_t e) {
        for (int64_t r = b; r < e; ++r) {
            uint64_t i = (uint64_t)ids[r];
            if (elem_bytes == 4) {
                float* o = (float*)out + r * dim;
                for (int64_t j = 0; j < dim; ++j) o[j] = feature_value(seed, i, (uint64_t)j);
            } else {
                uint16_t* o = (uint16_t*)out + r * dim;
                for (int64_t j = 0; j < dim; ++j) o[j] = f32_to_f16_rne(feature_value(seed, i, (uint64_t)j));
            }
        }
    });
}

// Seed batch `batch`: n_seeds node ids.  mode 0 uniform with replacement; mode 1 popularity
// ~ 1/(rank + 1) (Zipf s = 1) over a third permutation of the nodes.
void qg_seeds(uint64_t seed, int64_t n_nodes, int64_t batch, int64_t n_seeds, int mode, int32_t* out) {
    Perm perm3((uint64_t)n_nodes, seed ^ 0x3333);
    for (int64_t i = 0; i < n_seeds; ++i) {
        uint64_t h = hash4(seed, 4, (uint64_t)batch, (uint64_t)i);
        if (mode == 0) {
            out[i] = (int32_t)(((unsigned __int128)h * (uint64_t)n_nodes) >> 64);
        } else {
            double x = std::exp(u01(h) * std::log((double)n_nodes + 1.0)) - 1.0;  // density ~ 1/(x+1)
            int64_t r = (int64_t)x;
            if (r < 0) r = 0;
            if (r >= n_nodes) r = n_nodes - 1;
            out[i] = (int32_t)perm3((uint64_t)r);
        }
    }
}

// The seed distribution of mode 1 as a probability vector over nodes (sums to 1).
void qg_seed_popularity(uint64_t seed, int64_t n_nodes, int n_threads, double* p0) {
    Perm perm3((uint64_t)n_nodes, seed ^ 0x3333);
    double norm = std::log((double)n_nodes + 1.0);
    parallel_chunks(n_nodes, 1 << 16, n_threads, [&](int64_t b, int64_t e) {
        for (int64_t r = b; r < e; ++r)
            p0[perm3((uint64_t)r)] = (std::log((double)r + 2.0) - std::log((double)r + 1.0)) / norm;
    });
}

uint64_t qg_batch_rng_seed(uint64_t seed, int64_t batch) { return hash4(seed, 5, (uint64_t)batch, 0); }

}  // extern "C"
