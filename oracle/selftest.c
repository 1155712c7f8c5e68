/*
 * TEST INFRASTRUCTURE.  A plain C driver that walks every routine of embedpart_oracle.c over small
 * seeded inputs with ragged sizes, empty rows, empty clusters, duplicate points and labels to reject,
 * so that a build with -fsanitize=address,undefined sees every access and every arithmetic operation
 * of the oracle (tests/test_oracle_sanitized.py builds and runs it).  It checks only invariants that
 * hold by definition (counts add up to n, a permutation is a permutation, the rewritten graph keeps its
 * gap sum); the pins proper live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int or_init_indices(uint64_t seed, int64_t n, int32_t k, int64_t *idx);
double or_round_bf16(double v);
double or_assign(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld, const double *C, int round_bf16,
                 int32_t *labels, double *best, double *second);
int32_t or_update(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld, const int32_t *labels, double *C,
                  int64_t *counts);
void or_validate_labels(int64_t n, int32_t k, const int32_t *labels, int64_t *out);
int or_lloyd(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld, int32_t iters, const int64_t *idx,
             int flags, double *C, int32_t *labels, int64_t *counts, double *obj_hist, double *obj_final);
int or_lloyd_bounds(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld, int32_t iters, const int64_t *idx,
                    int flags, int audit, double *C, int32_t *labels, int64_t *counts, double *obj_hist,
                    int64_t *skipped, int64_t *moved, int64_t *violations);
int or_sampled_kmeans(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld, int64_t m, const int64_t *rows,
                      int32_t iters, int flags, double *C, int32_t *labels, int64_t *counts, double *obj_hist,
                      double *obj_full);
int or_partition_quality(int64_t n, int32_t k, const int64_t *rowptr, const int32_t *colidx, const int32_t *labels,
                         int64_t *cut, int64_t *sizes);
double or_edge_cut_ratio(int64_t cut, int64_t nnz);
double or_vertex_balance(int32_t k, const int64_t *sizes);
int or_balance(int64_t n, int32_t k, const int64_t *rowptr, const uint8_t *vclass, int32_t class_id, double beta,
               uint64_t seed, int32_t max_rounds, int32_t *labels, int64_t *stats);
int or_permutation(int64_t n, int32_t k, const int32_t *labels, int32_t *new_id, int32_t *order);
uint64_t or_edge_gap_sum(int64_t n, const int64_t *rowptr, const int32_t *colidx, const int32_t *new_id);
uint64_t or_vertex_bandwidth_sum(int64_t n, const int64_t *rowptr, const int32_t *colidx, const int32_t *new_id);
int or_reorder_csr(int64_t n, const int64_t *rowptr, const int32_t *colidx, const int32_t *new_id,
                   int64_t *new_rowptr, int32_t *new_colidx);

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static uint64_t rng(void)   /* xorshift64*: inputs only, not part of the method */
{
    rng_state ^= rng_state >> 12;
    rng_state ^= rng_state << 25;
    rng_state ^= rng_state >> 27;
    return rng_state * 0x2545F4914F6CDD1Dull;
}
static double unit(void) { return (double)(rng() >> 11) * (1.0 / 9007199254740992.0); }

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            fprintf(stderr, "selftest: %s failed at line %d\n", #cond, __LINE__);    \
            exit(1);                                                                 \
        }                                                                            \
    } while (0)

static void kmeans_case(int64_t n, int32_t d, int32_t k, int64_t pad, int flags)
{
    const int64_t ld = d + pad;
    float *X = (float *)malloc((size_t)n * ld * sizeof(float));
    for (int64_t i = 0; i < n; ++i)
        for (int64_t m = 0; m < ld; ++m)   /* a few blobs, some exact duplicates */
            X[i * ld + m] = (float)((double)(i % 5) * 3.0 + (i % 7 == 0 ? 0.0 : unit() - 0.5));
    int64_t *idx = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    CHECK(or_init_indices(11 + (uint64_t)n, n, k, idx) == 0);
    double *C = (double *)malloc((size_t)k * d * sizeof(double)), *C2 = (double *)malloc((size_t)k * d * sizeof(double));
    int32_t *lab = (int32_t *)malloc((size_t)n * sizeof(int32_t)), *lab2 = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int64_t *cnt = (int64_t *)malloc((size_t)k * sizeof(int64_t)), *cnt2 = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    const int32_t iters = 6;
    double hist[8], hist2[8], fin = 0.0;
    CHECK(or_lloyd(n, d, k, X, ld, iters, idx, flags, C, lab, cnt, hist, &fin) == 0);
    int64_t total = 0;
    for (int32_t j = 0; j < k; ++j) total += cnt[j];
    CHECK(total == n);
    for (int32_t t = 1; t < iters; ++t) CHECK(hist[t] <= hist[t - 1] * (1.0 + 1e-12) + 1e-9 || (flags & 2));
    int64_t skipped[8], moved[8], viol = -1;
    CHECK(or_lloyd_bounds(n, d, k, X, ld, iters, idx, flags & 2, 1, C2, lab2, cnt2, hist2, skipped, moved, &viol) == 0);
    CHECK(viol == 0);
    CHECK(memcmp(lab, lab2, (size_t)n * sizeof(int32_t)) == 0);

    /* assignment with both optional outputs, the label check, then an update that meets an empty cluster */
    double *best = (double *)malloc((size_t)n * sizeof(double)), *second = (double *)malloc((size_t)n * sizeof(double));
    const double obj = or_assign(n, d, k, X, ld, C, flags & 2 ? 1 : 0, lab, best, second);
    CHECK(obj >= 0.0);
    (void)or_assign(n, d, k, X, ld, C, 0, lab2, NULL, NULL);
    for (int64_t i = 0; i < n; i += 3) lab[i] = (i % 2) ? -1 : k + 5;
    for (int64_t i = 0; i < n; ++i)
        if (lab[i] == k - 1) lab[i] = 0;   /* cluster k - 1 is empty now (k >= 2), or stays as it is (k == 1) */
    int64_t bad[2];
    or_validate_labels(n, k, lab, bad);
    CHECK(bad[0] >= 1 && bad[1] == 0);
    for (int64_t i = 0; i < n; i += 3) lab[i] = 0;   /* or_update takes valid labels only (its wrapper checks) */
    or_validate_labels(n, k, lab, bad);
    CHECK(bad[0] == 0 && bad[1] == n);
    CHECK(or_update(n, d, k, X, ld, lab, C, cnt) >= (k >= 2 ? 1 : 0));   /* cluster k - 1 has no points */

    /* sample-trained variant on the first rows drawn */
    const int64_t m = n < 4 * (int64_t)k ? n : 4 * (int64_t)k;
    int64_t *rows = (int64_t *)malloc((size_t)m * sizeof(int64_t));
    CHECK(or_init_indices(5, n, (int32_t)m, rows) == 0);
    double full = 0.0;
    CHECK(or_sampled_kmeans(n, d, k, X, ld, m, rows, 3, flags & 2, C, lab, cnt, hist, &full) == 0);

    free(rows); free(best); free(second); free(cnt); free(cnt2); free(lab); free(lab2); free(C); free(C2); free(idx); free(X);
}

static void graph_case(int64_t n, int32_t k, int max_deg)
{
    int64_t *rowptr = (int64_t *)malloc((size_t)(n + 1) * sizeof(int64_t));
    rowptr[0] = 0;
    for (int64_t v = 0; v < n; ++v)   /* runs of empty rows and a hub */
        rowptr[v + 1] = rowptr[v] + (v % 4 == 1 ? 0 : (v == n / 2 ? 3 * max_deg : (int64_t)(rng() % (uint64_t)(max_deg + 1))));
    const int64_t nnz = rowptr[n];
    int32_t *colidx = (int32_t *)malloc((size_t)(nnz + 1) * sizeof(int32_t));
    for (int64_t e = 0; e < nnz; ++e) colidx[e] = (int32_t)(rng() % (uint64_t)n);   /* self-loops and repeats allowed */
    int32_t *lab = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    for (int64_t v = 0; v < n; ++v) lab[v] = (int32_t)((rng() % 3 == 0) ? 0 : rng() % (uint64_t)k);   /* partition 0 overloaded */
    int64_t cut = -1, *sizes = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    CHECK(or_partition_quality(n, k, rowptr, colidx, lab, &cut, sizes) == 0);
    CHECK(cut >= 0 && cut <= nnz);
    (void)or_edge_cut_ratio(cut, nnz);
    (void)or_edge_cut_ratio(0, 0);
    CHECK(or_vertex_balance(k, sizes) >= 1.0 - 1e-12);

    uint8_t *vclass = (uint8_t *)malloc((size_t)n);
    for (int64_t v = 0; v < n; ++v) vclass[v] = (uint8_t)(rng() % 3);
    int64_t stats[3];
    for (int32_t cls = 0; cls < 3; ++cls) CHECK(or_balance(n, k, rowptr, vclass, cls, 1.05, 99, 16, lab, stats) == 0);
    CHECK(or_balance(n, k, rowptr, vclass, 0, 1.0, 7, 4, lab, stats) == 0);

    int32_t *new_id = (int32_t *)malloc((size_t)n * sizeof(int32_t)), *order = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    CHECK(or_permutation(n, k, lab, new_id, order) == 0);
    for (int64_t v = 0; v < n; ++v) CHECK(order[new_id[v]] == v);
    const uint64_t gap = or_edge_gap_sum(n, rowptr, colidx, new_id);
    const uint64_t bw = or_vertex_bandwidth_sum(n, rowptr, colidx, new_id);
    int64_t *rp2 = (int64_t *)malloc((size_t)(n + 1) * sizeof(int64_t));
    int32_t *ci2 = (int32_t *)malloc((size_t)(nnz + 1) * sizeof(int32_t)), *ident = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    CHECK(or_reorder_csr(n, rowptr, colidx, new_id, rp2, ci2) == 0);
    CHECK(rp2[n] == nnz);
    for (int64_t v = 0; v < n; ++v) ident[v] = (int32_t)v;
    CHECK(or_edge_gap_sum(n, rp2, ci2, ident) == gap);
    CHECK(or_vertex_bandwidth_sum(n, rp2, ci2, ident) == bw);

    free(ident); free(ci2); free(rp2); free(order); free(new_id); free(vclass); free(sizes); free(lab); free(colidx); free(rowptr);
}

int main(void)
{
    for (int v = 0; v < 8; ++v) {   /* bf16 rounding: ordinary values, halfway cases, zeros, the largest finite value */
        const double x[8] = {1.0, 1.00390625, -3.14159, 0.0, -0.0, 3.3895313892515355e38, 1e-40, 65504.0};
        const double r = or_round_bf16(x[v]);
        CHECK(r == r && fabs(r - x[v]) <= fabs(x[v]) * 0.00390625 + 1e-38);
    }
    kmeans_case(1, 1, 1, 0, 0);
    kmeans_case(7, 3, 7, 1, 0);      /* k == n */
    kmeans_case(97, 5, 4, 3, 0);
    kmeans_case(333, 16, 9, 0, 2);   /* centroids rounded to bf16 for the distances */
    kmeans_case(1000, 8, 2, 0, 1);   /* one further assignment at the end */
    graph_case(1, 1, 2);
    graph_case(50, 3, 6);
    graph_case(501, 7, 9);
    printf("oracle selftest ok\n");
    return 0;
}
