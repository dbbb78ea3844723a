// Seeded synthetic graph generators (input data only).
//
// This file produces the *inputs* of the backward-aggregation path: an undirected
// random graph (Chung-Lu power law or R-MAT), symmetrised, with self-loops, vertex
// ids randomly permuted, stored as a pull-mode CSR with ascending unique columns.
// It contains none of the method's arithmetic (no frontier expansion, no path
// extraction, no aggregation); both the CPU oracle and the GPU library receive the
// arrays written here as plain inputs.
//
// Every random number is a pure function of (seed, stream, counter), so the result
// does not depend on the number of threads.
//
// Build: g++ -O2 -fopenmp -shared -fPIC graphgen.cpp -o libgraphgen.so

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>
#include <omp.h>
#include <parallel/algorithm>

namespace {

// splitmix64 finaliser used as a counter-based generator: u64(seed, stream, i).
inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
inline uint64_t rnd64(uint64_t seed, uint64_t stream, uint64_t i) {
    return mix64(mix64(seed ^ (stream * 0xD6E8FEB86659FD93ull)) + i * 0x9E3779B97F4A7C15ull);
}
inline double u01(uint64_t r) { return (double)(r >> 11) * (1.0 / 9007199254740992.0); }

struct Rec { uint64_t key; uint64_t idx; };
inline bool rec_less(const Rec& a, const Rec& b) {
    return a.key < b.key || (a.key == b.key && a.idx < b.idx);
}

struct Graph {
    int64_t n = 0;
    int64_t n_undirected = 0;     // distinct undirected non-loop edges
    int64_t raw_draws = 0;        // candidate pairs drawn (incl. rejected / duplicate)
    std::vector<int32_t> rowptr;  // n+1  (nnz < 2^31 enforced)
    std::vector<int32_t> col;
    std::vector<float> val;
};

enum { KIND_CHUNG_LU = 0, KIND_RMAT = 1 };

struct Sampler {
    int kind;
    int64_t n;
    uint64_t seed;
    // Chung-Lu
    std::vector<double> cdf;  // cumulative weights, cdf[n-1] == total
    // R-MAT
    int scale;
    uint32_t ta, tab, tabc;  // 16-bit cumulative thresholds for quadrants a, a+b, a+b+c

    int64_t pick_cl(double u) const {
        double x = u * cdf[n - 1];
        int64_t lo = 0, hi = n - 1;  // first index with cdf[idx] > x
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (cdf[mid] > x) hi = mid; else lo = mid + 1;
        }
        return lo;
    }
    // Candidate number i -> canonical key (min<<32|max), or ~0 when rejected.
    uint64_t draw(uint64_t i) const {
        int64_t a, b;
        if (kind == KIND_CHUNG_LU) {
            a = pick_cl(u01(rnd64(seed, 1, 2 * i)));
            b = pick_cl(u01(rnd64(seed, 1, 2 * i + 1)));
        } else {
            a = 0; b = 0;
            int words = (scale + 3) / 4;
            int lvl = 0;
            for (int w = 0; w < words; ++w) {
                uint64_t r = rnd64(seed, 2, i * (uint64_t)words + w);
                for (int q = 0; q < 4 && lvl < scale; ++q, ++lvl) {
                    uint32_t x = (uint32_t)(r >> (16 * q)) & 0xFFFFu;
                    int qa = (x >= ta) + (x >= tab) + (x >= tabc);  // 0:a 1:b 2:c 3:d
                    a = (a << 1) | (qa >> 1);
                    b = (b << 1) | (qa & 1);
                }
            }
            if (a >= n || b >= n) return ~0ull;
        }
        if (a == b) return ~0ull;
        uint64_t lo = (uint64_t)std::min(a, b), hi = (uint64_t)std::max(a, b);
        return (lo << 32) | hi;
    }
};

// Draw candidates [first, first+count) and return the accepted ones sorted by (key, idx),
// one record per distinct key (smallest idx).
std::vector<Rec> draw_round(const Sampler& s, uint64_t first, uint64_t count) {
    int nt = omp_get_max_threads();
    std::vector<std::vector<Rec>> parts(nt);
#pragma omp parallel
    {
        int t = omp_get_thread_num();
        std::vector<Rec>& mine = parts[t];
        mine.reserve(count / nt + 16);
#pragma omp for schedule(static)
        for (int64_t j = 0; j < (int64_t)count; ++j) {
            uint64_t k = s.draw(first + j);
            if (k != ~0ull) mine.push_back(Rec{k, first + (uint64_t)j});
        }
    }
    size_t tot = 0;
    for (auto& p : parts) tot += p.size();
    std::vector<Rec> all;
    all.reserve(tot);
    for (auto& p : parts) { all.insert(all.end(), p.begin(), p.end()); std::vector<Rec>().swap(p); }
    __gnu_parallel::sort(all.begin(), all.end(), rec_less);
    size_t w = 0;
    for (size_t r = 0; r < all.size(); ++r)
        if (w == 0 || all[r].key != all[w - 1].key) all[w++] = all[r];
    all.resize(w);
    return all;
}

// Merge two key-sorted distinct lists, keeping the smaller idx on equal keys.
std::vector<Rec> merge_unique(const std::vector<Rec>& a, const std::vector<Rec>& b) {
    std::vector<Rec> out;
    out.reserve(a.size() + b.size());
    size_t i = 0, j = 0;
    while (i < a.size() && j < b.size()) {
        if (a[i].key < b[j].key) out.push_back(a[i++]);
        else if (b[j].key < a[i].key) out.push_back(b[j++]);
        else { out.push_back(a[i].idx < b[j].idx ? a[i] : b[j]); ++i; ++j; }
    }
    while (i < a.size()) out.push_back(a[i++]);
    while (j < b.size()) out.push_back(b[j++]);
    return out;
}

}  // namespace

extern "C" {

// kind: 0 Chung-Lu (p0 = gamma), 1 R-MAT (p0=a, p1=b, p2=c; scale = ceil(log2 n)).
// target_edges > 0: keep exactly the first `target_edges` distinct pairs in draw order.
// target_edges == 0: draw exactly `raw_draws` candidates and keep all distinct ones.
// permute != 0: relabel vertices by a seeded random permutation.
// Returns an opaque handle (NULL on failure).
void* gg_build(int kind, int64_t n, double p0, double p1, double p2, int64_t target_edges,
               int64_t raw_draws, uint64_t seed, int permute) {
    if (n < 1 || n > 0x7FFFFFFFll) return nullptr;
    Sampler s;
    s.kind = kind; s.n = n; s.seed = seed; s.scale = 0; s.ta = s.tab = s.tabc = 0;
    if (kind == KIND_CHUNG_LU) {
        s.cdf.resize(n);
        double ex = -1.0 / (p0 - 1.0), acc = 0.0;
        for (int64_t i = 0; i < n; ++i) { acc += std::pow((double)(i + 1), ex); s.cdf[i] = acc; }
    } else if (kind == KIND_RMAT) {
        while ((1ll << s.scale) < n) ++s.scale;
        s.ta = (uint32_t)std::lround(p0 * 65536.0);
        s.tab = (uint32_t)std::lround((p0 + p1) * 65536.0);
        s.tabc = (uint32_t)std::lround((p0 + p1 + p2) * 65536.0);
    } else return nullptr;

    std::vector<Rec> uniq;
    uint64_t drawn = 0;
    if (target_edges > 0) {
        double yield = 0.9;
        int rounds = 0;
        while ((int64_t)uniq.size() < target_edges) {
            if (++rounds > 200) return nullptr;  // graph cannot hold that many distinct edges
            int64_t need = target_edges - (int64_t)uniq.size();
            uint64_t m = (uint64_t)((double)need / std::max(yield, 0.02) * 1.05) + 1024;
            std::vector<Rec> fresh = draw_round(s, drawn, m);
            size_t before = uniq.size();
            uniq = uniq.empty() ? std::move(fresh) : merge_unique(uniq, fresh);
            drawn += m;
            yield = (double)(uniq.size() - before) / (double)m;
        }
        if ((int64_t)uniq.size() > target_edges) {
            std::vector<uint64_t> idx(uniq.size());
            for (size_t i = 0; i < uniq.size(); ++i) idx[i] = uniq[i].idx;
            std::nth_element(idx.begin(), idx.begin() + (target_edges - 1), idx.end());
            uint64_t thr = idx[target_edges - 1];
            size_t w = 0;
            for (size_t r = 0; r < uniq.size(); ++r) if (uniq[r].idx <= thr) uniq[w++] = uniq[r];
            uniq.resize(w);
        }
    } else {
        uniq = draw_round(s, 0, (uint64_t)raw_draws);
        drawn = (uint64_t)raw_draws;
    }
    std::vector<double>().swap(s.cdf);

    const int64_t E = (int64_t)uniq.size();
    const int64_t nnz = 2 * E + n;
    if (nnz >= 0x7FFFFFFFll) return nullptr;

    // Vertex relabelling: rank of each vertex under a hashed key.
    std::vector<int32_t> label(n);
    if (permute) {
        std::vector<Rec> pk(n);
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < n; ++v) pk[v] = Rec{rnd64(seed, 3, (uint64_t)v), (uint64_t)v};
        __gnu_parallel::sort(pk.begin(), pk.end(), rec_less);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < n; ++r) label[pk[r].idx] = (int32_t)r;
    } else {
        for (int64_t v = 0; v < n; ++v) label[v] = (int32_t)v;
    }

    Graph* g = new Graph();
    g->n = n; g->n_undirected = E; g->raw_draws = (int64_t)drawn;
    g->rowptr.assign(n + 1, 0);
    std::vector<int32_t> deg(n, 1);  // self-loop
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < E; ++e) {
        int32_t a = label[uniq[e].key >> 32], b = label[uniq[e].key & 0xFFFFFFFFull];
#pragma omp atomic
        deg[a]++;
#pragma omp atomic
        deg[b]++;
    }
    for (int64_t v = 0; v < n; ++v) g->rowptr[v + 1] = g->rowptr[v] + deg[v];
    g->col.resize(nnz);
    std::vector<int32_t> cur(g->rowptr.begin(), g->rowptr.end() - 1);
    for (int64_t v = 0; v < n; ++v) g->col[cur[v]++] = (int32_t)v;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < E; ++e) {
        int32_t a = label[uniq[e].key >> 32], b = label[uniq[e].key & 0xFFFFFFFFull];
        int32_t pa, pb;
#pragma omp atomic capture
        pa = cur[a]++;
#pragma omp atomic capture
        pb = cur[b]++;
        g->col[pa] = b;
        g->col[pb] = a;
    }
    std::vector<Rec>().swap(uniq);
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t v = 0; v < n; ++v)
        std::sort(g->col.begin() + g->rowptr[v], g->col.begin() + g->rowptr[v + 1]);

    // Symmetric normalisation with self-loops: e_vu = 1 / sqrt(d_v d_u), d = row length.
    g->val.resize(nnz);
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t v = 0; v < n; ++v)
        for (int32_t j = g->rowptr[v]; j < g->rowptr[v + 1]; ++j)
            g->val[j] = (float)(1.0 / std::sqrt((double)deg[v] * (double)deg[g->col[j]]));
    return g;
}

int64_t gg_n(void* h) { return ((Graph*)h)->n; }
int64_t gg_nnz(void* h) { return (int64_t)((Graph*)h)->col.size(); }
int64_t gg_undirected_edges(void* h) { return ((Graph*)h)->n_undirected; }
int64_t gg_raw_draws(void* h) { return ((Graph*)h)->raw_draws; }

void gg_export(void* h, int32_t* rowptr, int32_t* col, float* val) {
    Graph* g = (Graph*)h;
    std::memcpy(rowptr, g->rowptr.data(), g->rowptr.size() * sizeof(int32_t));
    std::memcpy(col, g->col.data(), g->col.size() * sizeof(int32_t));
    std::memcpy(val, g->val.data(), g->val.size() * sizeof(float));
}

void gg_free(void* h) { delete (Graph*)h; }

// Standard-normal fill of selected rows of a zeroed row-major n x F fp32 matrix:
// out[v, f] = N(0,1) for member[v] != 0, else untouched. Box-Muller on counter-based
// uniforms, so element (v, f) depends on (seed, v, f) only.
void gg_normal_rows(float* out, int64_t n, int64_t F, const uint8_t* member, uint64_t seed) {
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t v = 0; v < n; ++v) {
        if (member && !member[v]) continue;
        float* row = out + v * F;
        for (int64_t f = 0; f < F; f += 2) {
            uint64_t c = (uint64_t)v * (uint64_t)((F + 1) / 2) + (uint64_t)(f >> 1);
            double u1 = 1.0 - u01(rnd64(seed, 4, 2 * c));  // (0, 1]
            double u2 = u01(rnd64(seed, 4, 2 * c + 1));
            double r = std::sqrt(-2.0 * std::log(u1));
            double a = 6.283185307179586476925 * u2;
            row[f] = (float)(r * std::cos(a));
            if (f + 1 < F) row[f + 1] = (float)(r * std::sin(a));
        }
    }
}

}  // extern "C"
