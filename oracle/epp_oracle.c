/* CPU oracle for partially-active backward aggregation (TEST INFRASTRUCTURE ONLY).
 *
 * Plain, slow, obviously-correct C written from the paper.  It shares no code with the
 * HIP library and must never be called from the product path; only the tests, the smoke
 * check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes
 *   - active sets  N^k_{V_t}, k = 0..L   (Sec. 3, Theorem 1: the k-neighbour sets of V_t)
 *   - execution paths SG_l               (Sec. 4: vertex set N^{L-l}, edge set
 *                                         N(v) ∩ N^{L-l-1} for every v in N^{L-l})
 *   - all-active backward aggregation    (Alg. 1, backward aggregation loop)
 *   - partially-active aggregation       (Alg. 2, aggregation loop)
 *
 * The graph is a pull-mode CSR of the backward operator: row v lists the vertices u whose
 * gradient rows v accumulates, with weight e_vu.  Sums are accumulated in double in CSR
 * order and rounded once to float.  Rows are independent, so the OpenMP row split used for
 * timing does not change any result.
 *
 * Parity status: every function here is pinned by tests (paper's worked example, dense
 * brute force, closed forms, a sparse-library product, Theorem 1 invariants).
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC epp_oracle.c -o libepp_oracle.so
 */
#include <stdint.h>
#include <string.h>

/* N^0 = V_t (set semantics: duplicates collapse).  member0[v] in {0,1}.
 * Returns -1 if any id is outside [0, n). */
int oracle_mark_training(int64_t n, const int32_t* train_ids, int64_t n_train, uint8_t* member0) {
    memset(member0, 0, (size_t)n);
    for (int64_t i = 0; i < n_train; ++i) {
        if (train_ids[i] < 0 || train_ids[i] >= n) return -1;
        member0[train_ids[i]] = 1;
    }
    return 0;
}

/* One expansion step of Theorem 1's induction: v is in N^{k+1} iff some entry u of row v
 * is in N^k (v accumulates a possibly non-zero row).  The image is NOT united with N^k;
 * with self-loops in the graph the union happens by itself. */
void oracle_expand(int64_t n, const int32_t* rowptr, const int32_t* col, const uint8_t* member_k,
                   uint8_t* member_k1) {
    for (int64_t v = 0; v < n; ++v) {
        uint8_t hit = 0;
        for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j)
            if (member_k[col[j]]) { hit = 1; break; }
        member_k1[v] = hit;
    }
}

/* Size of SG with rows N^{k+1} (member_rows) and sources N^k (member_src). */
void oracle_path_size(int64_t n, const int32_t* rowptr, const int32_t* col, const uint8_t* member_rows,
                      const uint8_t* member_src, int64_t* n_rows, int64_t* nnz) {
    int64_t r = 0, e = 0;
    for (int64_t v = 0; v < n; ++v) {
        if (!member_rows[v]) continue;
        ++r;
        for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) e += member_src[col[j]] != 0;
    }
    *n_rows = r;
    *nnz = e;
}

/* Execution path in canonical form: destination vertices ascending (row_ids), each with
 * its neighbour list filtered by the source set, entries in input order, original ids. */
void oracle_path_extract(int64_t n, const int32_t* rowptr, const int32_t* col, const float* val,
                         const uint8_t* member_rows, const uint8_t* member_src, int32_t* p_row_ids,
                         int32_t* p_rowptr, int32_t* p_col, float* p_val) {
    int64_t r = 0, e = 0;
    p_rowptr[0] = 0;
    for (int64_t v = 0; v < n; ++v) {
        if (!member_rows[v]) continue;
        for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
            if (member_src[col[j]]) { p_col[e] = col[j]; p_val[e] = val[j]; ++e; }
        }
        p_row_ids[r] = (int32_t)v;
        p_rowptr[r + 1] = (int32_t)e;
        ++r;
    }
}

/* Aggregation over a CSR whose r-th row belongs to vertex row_ids[r] (row_ids == NULL:
 * r-th row is vertex r):   out[v, :] = sum_j val[j] * in[col[j], :].
 * Only the listed rows of `out` are written.  `stride` selects every stride-th row
 * starting at `first` (first = 0, stride = 1: all rows), used for bounded timing samples. */
void oracle_aggregate(int64_t n_rows, const int32_t* row_ids, const int32_t* rowptr, const int32_t* col,
                      const float* val, const float* in, float* out, int64_t F, int64_t first,
                      int64_t stride) {
#pragma omp parallel
    {
        double acc[512];
#pragma omp for schedule(dynamic, 256)
        for (int64_t r = first; r < n_rows; r += stride) {
            int64_t v = row_ids ? row_ids[r] : r;
            for (int64_t f0 = 0; f0 < F; f0 += 512) {
                int64_t fw = F - f0 < 512 ? F - f0 : 512;
                for (int64_t f = 0; f < fw; ++f) acc[f] = 0.0;
                for (int32_t j = rowptr[r]; j < rowptr[r + 1]; ++j) {
                    const float* src = in + (int64_t)col[j] * F + f0;
                    double w = (double)val[j];
                    for (int64_t f = 0; f < fw; ++f) acc[f] += w * (double)src[f];
                }
                for (int64_t f = 0; f < fw; ++f) out[v * F + f0 + f] = (float)acc[f];
            }
        }
    }
}

/* Alg. 2's aggregation loop written directly on the input graph: for v in N^{L-l}
 * (member_rows), for u in N(v) ∩ N^{L-l-1} (member_src): X'_v += e_vu * Y'_u.
 * Every row of `out` (n x F) is written; rows outside member_rows become zero. */
void oracle_partial_aggregate(int64_t n, const int32_t* rowptr, const int32_t* col, const float* val,
                              const uint8_t* member_rows, const uint8_t* member_src, const float* in,
                              float* out, int64_t F) {
#pragma omp parallel
    {
        double acc[512];
#pragma omp for schedule(dynamic, 256)
        for (int64_t v = 0; v < n; ++v) {
            for (int64_t f0 = 0; f0 < F; f0 += 512) {
                int64_t fw = F - f0 < 512 ? F - f0 : 512;
                for (int64_t f = 0; f < fw; ++f) acc[f] = 0.0;
                if (member_rows[v]) {
                    for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
                        if (!member_src[col[j]]) continue;
                        const float* src = in + (int64_t)col[j] * F + f0;
                        double w = (double)val[j];
                        for (int64_t f = 0; f < fw; ++f) acc[f] += w * (double)src[f];
                    }
                }
                for (int64_t f = 0; f < fw; ++f) out[v * F + f0 + f] = (float)acc[f];
            }
        }
    }
}

/* Thread control for the timing leg (results never depend on it). */
#ifdef _OPENMP
#include <omp.h>
int oracle_max_threads(void) { return omp_get_max_threads(); }
void oracle_set_threads(int t) { if (t > 0) omp_set_num_threads(t); }
#else
int oracle_max_threads(void) { return 1; }
void oracle_set_threads(int t) { (void)t; }
#endif
