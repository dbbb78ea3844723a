/* The CPU side of the build (the C oracle and the input generator) under AddressSanitizer and
 * UndefinedBehaviorSanitizer: this driver is compiled together with oracle/epp_oracle.c and linked
 * against graphgen/graphgen.cpp, both built with -fsanitize=address,undefined, and walks every entry
 * point of the two on generated graphs (both generators, with and without a target edge count,
 * widths that cross the oracle's 512-column blocks, strided row samples, an out-of-range training id).
 * Any out-of-bounds access, use after free, signed overflow or misaligned access aborts the run.
 * Plain invariants are checked on the way (the sanitizers are the point, the pins live in the Python tests). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

/* oracle/epp_oracle.c */
int oracle_mark_training(int64_t n, const int32_t* train_ids, int64_t n_train, uint8_t* member0);
void oracle_expand(int64_t n, const int32_t* rowptr, const int32_t* col, const uint8_t* member_k, uint8_t* member_k1);
void oracle_path_size(int64_t n, const int32_t* rowptr, const int32_t* col, const uint8_t* member_rows,
                      const uint8_t* member_src, int64_t* n_rows, int64_t* nnz);
void oracle_path_extract(int64_t n, const int32_t* rowptr, const int32_t* col, const float* val,
                         const uint8_t* member_rows, const uint8_t* member_src, int32_t* p_row_ids, int32_t* p_rowptr,
                         int32_t* p_col, float* p_val);
void oracle_aggregate(int64_t n_rows, const int32_t* row_ids, const int32_t* rowptr, const int32_t* col,
                      const float* val, const float* in, float* out, int64_t F, int64_t first, int64_t stride);
void oracle_partial_aggregate(int64_t n, const int32_t* rowptr, const int32_t* col, const float* val,
                              const uint8_t* member_rows, const uint8_t* member_src, const float* in, float* out,
                              int64_t F);
int oracle_max_threads(void);
void oracle_set_threads(int t);

/* graphgen/graphgen.cpp */
void* gg_build(int kind, int64_t n, double p0, double p1, double p2, int64_t target_edges, int64_t raw_draws,
               uint64_t seed, int permute);
int64_t gg_n(void* h);
int64_t gg_nnz(void* h);
int64_t gg_undirected_edges(void* h);
int64_t gg_raw_draws(void* h);
void gg_export(void* h, int32_t* rowptr, int32_t* col, float* val);
void gg_free(void* h);
void gg_normal_rows(float* out, int64_t n, int64_t F, const uint8_t* member, uint64_t seed);

#define CHECK(cond)                                          \
    do {                                                     \
        if (!(cond)) {                                       \
            printf("FAILED line %d: %s\n", __LINE__, #cond); \
            exit(1);                                         \
        }                                                    \
    } while (0)

static void one_graph(int kind, int64_t n, int64_t target_edges, int64_t raw_draws, int L, int64_t F) {
    void* h = kind == 0 ? gg_build(0, n, 2.5, 0.0, 0.0, target_edges, raw_draws, 77u + (uint64_t)n, 1)
                        : gg_build(1, n, 0.57, 0.19, 0.19, target_edges, raw_draws, 78u + (uint64_t)n, 1);
    CHECK(h != NULL);
    CHECK(gg_n(h) == n);
    const int64_t nnz = gg_nnz(h);
    CHECK(nnz >= n); /* self-loops */
    CHECK(gg_undirected_edges(h) >= 0 && gg_raw_draws(h) >= 0);
    int32_t* rowptr = malloc((size_t)(n + 1) * 4);
    int32_t* col = malloc((size_t)nnz * 4);
    float* val = malloc((size_t)nnz * 4);
    gg_export(h, rowptr, col, val);
    gg_free(h);
    CHECK(rowptr[0] == 0 && rowptr[n] == nnz);

    /* training set: every 7th vertex, with a duplicate */
    int64_t n_train = n / 7 + 2;
    int32_t* train = malloc((size_t)n_train * 4);
    for (int64_t i = 0; i < n_train; ++i) train[i] = (int32_t)((i * 7) % n);
    uint8_t** sets = malloc((size_t)(L + 1) * sizeof(uint8_t*));
    for (int k = 0; k <= L; ++k) sets[k] = malloc((size_t)n);
    CHECK(oracle_mark_training(n, train, n_train, sets[0]) == 0);
    train[1] = (int32_t)n; /* out of range: refused, nothing written out of bounds */
    uint8_t* junk = malloc((size_t)n);
    CHECK(oracle_mark_training(n, train, n_train, junk) == -1);
    free(junk);
    for (int k = 0; k < L; ++k) oracle_expand(n, rowptr, col, sets[k], sets[k + 1]);

    float* in = malloc((size_t)n * (size_t)F * 4);
    float* full = calloc((size_t)n * (size_t)F, 4);
    float* part = malloc((size_t)n * (size_t)F * 4);
    float* path_out = calloc((size_t)n * (size_t)F, 4);
    for (int k = 0; k < L; ++k) {
        int64_t R = 0, E = 0;
        oracle_path_size(n, rowptr, col, sets[k + 1], sets[k], &R, &E);
        int32_t* prow = malloc((size_t)(R > 0 ? R : 1) * 4);
        int32_t* pptr = malloc((size_t)(R + 1) * 4);
        int32_t* pcol = malloc((size_t)(E > 0 ? E : 1) * 4);
        float* pval = malloc((size_t)(E > 0 ? E : 1) * 4);
        oracle_path_extract(n, rowptr, col, val, sets[k + 1], sets[k], prow, pptr, pcol, pval);
        CHECK(pptr[0] == 0 && pptr[R] == E);
        memset(in, 0, (size_t)n * (size_t)F * 4); /* the generator fills the member rows only */
        gg_normal_rows(in, n, F, sets[k], 1000u + (uint64_t)k);
        oracle_aggregate(n, NULL, rowptr, col, val, in, full, F, 0, 1);
        oracle_partial_aggregate(n, rowptr, col, val, sets[k + 1], sets[k], in, part, F);
        memset(path_out, 0, (size_t)n * (size_t)F * 4);
        oracle_aggregate(R, prow, pptr, pcol, pval, in, path_out, F, 0, 1);
        /* Theorem 1 / Alg. 2: the three agree (skipped terms are exact zeros) */
        for (int64_t i = 0; i < n * F; ++i) CHECK(full[i] == part[i] && part[i] == path_out[i]);
        /* strided sample: the sampled rows equal the full result, the others stay untouched */
        memset(path_out, 0, (size_t)n * (size_t)F * 4);
        oracle_aggregate(R, prow, pptr, pcol, pval, in, path_out, F, 1, 3);
        for (int64_t r = 0; r < R; ++r)
            for (int64_t f = 0; f < F; ++f) {
                const float x = path_out[(int64_t)prow[r] * F + f];
                CHECK(r % 3 == 1 ? x == part[(int64_t)prow[r] * F + f] : x == 0.0f);
            }
        free(prow); free(pptr); free(pcol); free(pval);
    }
    free(in); free(full); free(part); free(path_out);
    for (int k = 0; k <= L; ++k) free(sets[k]);
    free(sets); free(train); free(rowptr); free(col); free(val);
}

int main(void) {
    oracle_set_threads(2);
    CHECK(oracle_max_threads() >= 1);
    one_graph(0, 700, 2000, 0, 2, 7);      /* Chung-Lu, exact edge count */
    one_graph(1, 1000, 0, 9000, 3, 41);    /* R-MAT, all distinct pairs of a fixed number of draws */
    one_graph(1, 257, 600, 0, 2, 600);     /* width beyond one 512-column block of the oracle */
    one_graph(0, 1, 0, 0, 1, 3);           /* a single vertex */
    printf("ok\n");
    return 0;
}
