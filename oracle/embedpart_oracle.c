/*
 * EmbedPart phase-2 oracle: a plain, slow, fp64 CPU statement of what the
 * clustering hot path computes.
 *
 * THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load it.  It shares no code, header,
 * table or helper with the HIP library and neither side includes the other.
 *
 * What it follows (EmbedPart paper):
 *   - Alg. 3, first step  P <- KMeans(E, k): cluster one dense embedding per
 *     vertex into exactly k groups; the clusters are the partitions
 *     (Sec. "Phase 2: Clustering and Balancing").
 *   - Sec. "Implementation": the centroids are computed on a sample of the
 *     embeddings (2^9 per cluster), then every vertex is assigned.
 *   - Alg. 3 (the balancing loops) with the migration policy of Alg. 4:
 *     vertices move from overloaded to underloaded partitions, smallest degree
 *     first, destinations drawn in proportion to free capacity.
 *   - Sec. "Partitioning quality metrics": an edge (u,v) is cut iff
 *     pid(u) != pid(v); ECR = |C|/|E|; vertex balance = max|P_i| / mean|P_i|.
 *   - Sec. "Extension to Graph Reordering": gap xi_pi(u,v) = |pi(u)-pi(v)|,
 *     vertex bandwidth = max gap over a vertex's neighbours, average graph
 *     bandwidth = its mean over vertices; the reordering gives vertices of
 *     one partition consecutive ids, and the ids are the positions in memory:
 *     the graph is rewritten under the new ids.
 *
 * The paper names K-Means but none of its details.  The readings taken here
 * (squared Euclidean distance in its direct form, lowest index wins ties, an
 * empty cluster keeps its previous centroid, Lloyd iterations over all points
 * from k distinct seeded rows) are listed in the design notes of this
 * repository; each function below says which reading it implements.
 *
 * Pins (tests marked "not gpu"): brute force on integer coordinates, a
 * hand-worked 1-D Lloyd run, k = 1 and k = N special cases, separated blobs,
 * a hand-counted label vector with ids outside [0, k); the rounds with bounds:
 * equal to the plain rounds on every input tried, a hand-worked 1-D case
 * with the skipped points named, an audit that searches every skipped point,
 * translation / permutation equivariance, monotone objective, mean property,
 * closed-form cuts on paths / cycles / complete graphs / matchings,
 * adjacency-matrix brute force, balance extremes, permutation bijectivity;
 * sample-trained run: identity sample = Lloyd + one re-assignment, labels are
 * the brute-force nearest centroid, rows outside the sample do not move C;
 * balancing: a hand-worked two-partition case, balanced input untouched, the
 * movers are the smallest-degree members (independent argsort), loads within
 * capacity afterwards, destinations in proportion to free capacity, the draw
 * function restated with Python integers; rewriting the graph under pi: the
 * permuted sparse matrix of a library routine, gap / bandwidth / cut carried
 * over unchanged, identity and inverse permutations, a hand-worked graph.
 * Numerical parity with figures printed in the paper is unpinned: every such
 * figure depends on datasets and trained weights that are not available.
 *
 * Arithmetic: fp64 throughout; inputs arrive as the exact fp32 values the
 * device sees (bf16 inputs are widened to fp32 by the caller, which is exact).
 * Sums run in index order.  The only parallel loop is the per-point search of
 * the assignment step, whose iterations are independent.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define OR_FLAG_FINAL_REASSIGN 1
#define OR_FLAG_BF16_CENTROIDS 2

int or_version(void) { return 1; }

/* ---- seeded choice of k distinct rows -------------------------------- */

/* splitmix64 (Steele, Lea, Flood 2014; Vigna's public-domain constants). */
static uint64_t splitmix64_next(uint64_t *state)
{
    uint64_t z = (*state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/*
 * Initial centroids are k distinct rows.  Reading: distinct row indices,
 * drawn as (splitmix64 output mod n) from a stream started at `seed`,
 * repeats rejected, draw order kept as centroid order.
 * Returns 0, or -1 when k > n or an argument is out of range.
 */
int or_init_indices(uint64_t seed, int64_t n, int32_t k, int64_t *idx)
{
    if (n < 1 || k < 1 || (int64_t)k > n || !idx) return -1;
    uint64_t state = seed;
    int32_t have = 0;
    while (have < k) {
        int64_t r = (int64_t)(splitmix64_next(&state) % (uint64_t)n);
        int seen = 0;
        for (int32_t j = 0; j < have; ++j)
            if (idx[j] == r) { seen = 1; break; }
        if (!seen) idx[have++] = r;
    }
    return 0;
}

/* ---- bf16 rounding of a centroid coordinate --------------------------- */

/*
 * Round to bfloat16 (8 exponent bits, 7 stored mantissa bits), nearest-even,
 * in the precision path the device uses: the fp64 master value is first
 * rounded to fp32 (the device's master copy), then the fp32 value to bf16.
 * NaN/Inf do not occur for finite centroids of finite data.
 */
double or_round_bf16(double v)
{
    float f = (float)v;                 /* fp64 -> fp32, nearest-even */
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;      /* last kept bit */
    u += 0x7FFFu + lsb;                 /* nearest, ties to even */
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* ---- assignment step --------------------------------------------------- */

/*
 * For every point i: squared Euclidean distance to every centroid in the
 * direct form sum_m (x_im - c_jm)^2, m ascending; the label is the first j
 * that attains the minimum (strict < while j ascends).  best[i] is that
 * minimum, second[i] the second-smallest distance (HUGE_VAL when k == 1);
 * both may be NULL.  With round_bf16 != 0 the centroids used for distances
 * are the bf16-rounded copies, C itself is not modified.
 * Returns the objective sum_i best[i], added in index order.
 */
double or_assign(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld,
                 const double *C, int round_bf16,
                 int32_t *labels, double *best, double *second)
{
    double *Cq = (double *)malloc((size_t)k * d * sizeof(double));
    double *b = best ? best : (double *)malloc((size_t)n * sizeof(double));
    for (int64_t t = 0; t < (int64_t)k * d; ++t)
        Cq[t] = round_bf16 ? or_round_bf16(C[t]) : C[t];

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float *x = X + i * ld;
        double dmin = HUGE_VAL, dsec = HUGE_VAL;
        int32_t jmin = 0;
        for (int32_t j = 0; j < k; ++j) {
            const double *c = Cq + (int64_t)j * d;
            double d2 = 0.0;
            for (int32_t m = 0; m < d; ++m) {
                double diff = (double)x[m] - c[m];
                d2 += diff * diff;
            }
            if (d2 < dmin) { dsec = dmin; dmin = d2; jmin = j; }
            else if (d2 < dsec) { dsec = d2; }
        }
        labels[i] = jmin;
        b[i] = dmin;
        if (second) second[i] = dsec;
    }

    double obj = 0.0;
    for (int64_t i = 0; i < n; ++i) obj += b[i];
    if (!best) free(b);
    free(Cq);
    return obj;
}

/* ---- update step --------------------------------------------------------- */

/*
 * c_j <- mean of the points labelled j (sums in index order); a cluster with
 * no points keeps its previous centroid and gets count 0.  C is updated in
 * place.  Returns the number of empty clusters.
 */
int32_t or_update(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld,
                  const int32_t *labels, double *C, int64_t *counts)
{
    double *sum = (double *)calloc((size_t)k * d, sizeof(double));
    for (int32_t j = 0; j < k; ++j) counts[j] = 0;
    for (int64_t i = 0; i < n; ++i) {
        const float *x = X + i * ld;
        double *s = sum + (int64_t)labels[i] * d;
        for (int32_t m = 0; m < d; ++m) s[m] += (double)x[m];
        counts[labels[i]] += 1;
    }
    int32_t empty = 0;
    for (int32_t j = 0; j < k; ++j) {
        if (counts[j] == 0) { ++empty; continue; }
        for (int32_t m = 0; m < d; ++m)
            C[(int64_t)j * d + m] = sum[(int64_t)j * d + m] / (double)counts[j];
    }
    free(sum);
    return empty;
}

/*
 * Every vertex carries exactly one of the k partition ids (Sec. "Graph
 * Partitioning": the partitions are disjoint and cover V).  out[0] = number
 * of labels outside [0, k), out[1] = index of the first one (n if none).
 */
void or_validate_labels(int64_t n, int32_t k, const int32_t *labels, int64_t *out)
{
    out[0] = 0;
    out[1] = n;
    for (int64_t i = 0; i < n; ++i) {
        if (labels[i] >= 0 && labels[i] < k) continue;
        if (out[0] == 0) out[1] = i;
        out[0] += 1;
    }
}

/* ---- Lloyd iterations ---------------------------------------------------- */

/*
 * KMeans(E, k) of Alg. 3 read as `iters` Lloyd rounds (assign, then update)
 * from the rows idx[0..k) as initial centroids.
 *   labels  : labels of the last assignment step run
 *   C       : k x d centroids, means of the labels of the iters-th assignment
 *   counts  : sizes of those clusters
 *   obj_hist: objective of each of the `iters` assignment steps (may be NULL)
 * OR_FLAG_FINAL_REASSIGN: one more assignment against the final C; labels
 *   then hold that assignment, and *obj_final its objective.  counts and C
 *   still describe the iters-th round.
 * OR_FLAG_BF16_CENTROIDS: distances use bf16-rounded centroids.
 */
int or_lloyd(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld,
             int32_t iters, const int64_t *idx, int flags,
             double *C, int32_t *labels, int64_t *counts,
             double *obj_hist, double *obj_final)
{
    if (n < 1 || d < 1 || k < 1 || (int64_t)k > n || ld < d || iters < 0) return -1;
    for (int32_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || idx[j] >= n) return -1;
        for (int32_t m = 0; m < d; ++m)
            C[(int64_t)j * d + m] = (double)X[idx[j] * ld + m];
    }
    int q = (flags & OR_FLAG_BF16_CENTROIDS) ? 1 : 0;
    for (int32_t t = 0; t < iters; ++t) {
        double obj = or_assign(n, d, k, X, ld, C, q, labels, NULL, NULL);
        if (obj_hist) obj_hist[t] = obj;
        or_update(n, d, k, X, ld, labels, C, counts);
    }
    if (flags & OR_FLAG_FINAL_REASSIGN) {
        double obj = or_assign(n, d, k, X, ld, C, q, labels, NULL, NULL);
        if (obj_final) *obj_final = obj;
    }
    return 0;
}

/* ---- Lloyd rounds with bounds and incremental sums ------------------------------ */

/*
 * The same Lloyd rounds as or_lloyd, reached with less work: an exact
 * acceleration (the paper's contribution list and Sec. "Phase 2: Clustering
 * and Balancing" leave the clustering algorithm of Phase 2 open to more
 * advanced ones).  The scheme is the published one of Hamerly ("Making
 * k-means even faster", SDM 2010), restated:
 *   every point keeps  u >= distance to its own centroid  and
 *                      l <= distance to every other centroid;
 *   when the centroids move by delta_j, u grows by delta of the own centroid
 *   and l shrinks by the largest delta among the others (triangle
 *   inequality); a point with u < l cannot change its label and is skipped;
 *   any other point is searched in full, which also renews its bounds;
 *   the sums are kept between rounds: only a point that changes its label
 *   is taken out of one sum and put into another.
 * Round 1 is a full round.  The distances, and so the bounds, are those to
 * the centroids as the distances use them (bf16-rounded with the flag).
 * A relative slack of 1e-12 on the test keeps fp64 rounding of the bounds
 * from ever deciding a label.
 *   skipped[t], moved[t] : points not searched / points that changed label in
 *                          round t (t = 0 .. iters-1; skipped[0] = 0); may be NULL
 *   *violations          : with `audit` != 0 every skipped point is searched
 *                          anyway and counted here if its label would have
 *                          changed (must stay 0); may be NULL
 * Outputs otherwise as or_lloyd (obj_hist by the definition, over all
 * points).  OR_FLAG_FINAL_REASSIGN is not supported here (returns -1).
 */
int or_lloyd_bounds(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld,
                    int32_t iters, const int64_t *idx, int flags, int audit,
                    double *C, int32_t *labels, int64_t *counts, double *obj_hist,
                    int64_t *skipped, int64_t *moved, int64_t *violations)
{
    if (n < 1 || d < 1 || k < 1 || (int64_t)k > n || ld < d || iters < 0) return -1;
    if (flags & OR_FLAG_FINAL_REASSIGN) return -1;
    for (int32_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || idx[j] >= n) return -1;
        for (int32_t m = 0; m < d; ++m)
            C[(int64_t)j * d + m] = (double)X[idx[j] * ld + m];
    }
    const int q = (flags & OR_FLAG_BF16_CENTROIDS) ? 1 : 0;
    const size_t kd = (size_t)k * d;
    double *u = (double *)malloc((size_t)n * sizeof(double));
    double *l = (double *)malloc((size_t)n * sizeof(double));
    double *sum = (double *)calloc(kd, sizeof(double));
    double *Cu = (double *)malloc(kd * sizeof(double));      /* centroids as the distances use them */
    double *Cu_old = (double *)malloc(kd * sizeof(double));
    double *delta = (double *)malloc((size_t)k * sizeof(double));
    if (violations) *violations = 0;
    for (int32_t j = 0; j < k; ++j) counts[j] = 0;

    for (int32_t t = 0; t < iters; ++t) {
        for (size_t e = 0; e < kd; ++e) Cu[e] = q ? or_round_bf16(C[e]) : C[e];
        int64_t n_skipped = 0, n_moved = 0;
        if (t == 0) {
            /* a full round: nearest and second-nearest distance of every point, sums from scratch */
            or_assign(n, d, k, X, ld, C, q, labels, u, l);
            for (int64_t i = 0; i < n; ++i) {
                u[i] = sqrt(u[i]);
                l[i] = sqrt(l[i]);                       /* HUGE_VAL when k == 1 */
                for (int32_t m = 0; m < d; ++m) sum[(int64_t)labels[i] * d + m] += (double)X[i * ld + m];
                counts[labels[i]] += 1;
            }
            n_moved = n;
        } else {
            /* the centroids moved since the bounds were taken */
            double first = 0.0, second = 0.0;            /* largest and second-largest movement */
            int32_t jfirst = -1;
            for (int32_t j = 0; j < k; ++j) {
                double s2 = 0.0;
                for (int32_t m = 0; m < d; ++m) {
                    double diff = Cu[(int64_t)j * d + m] - Cu_old[(int64_t)j * d + m];
                    s2 += diff * diff;
                }
                delta[j] = sqrt(s2);
                if (delta[j] > first) { second = first; first = delta[j]; jfirst = j; }
                else if (delta[j] > second) { second = delta[j]; }
            }
            for (int64_t i = 0; i < n; ++i) {
                const float *x = X + i * ld;
                const int32_t a = labels[i];
                u[i] += delta[a];
                l[i] -= (a == jfirst) ? second : first;
                const int skip = u[i] < l[i] * (1.0 - 1e-12);
                if (skip && !audit) { ++n_skipped; continue; }
                /* full search, as in or_assign */
                double dmin = HUGE_VAL, dsec = HUGE_VAL;
                int32_t jmin = 0;
                for (int32_t j = 0; j < k; ++j) {
                    const double *c = Cu + (int64_t)j * d;
                    double d2 = 0.0;
                    for (int32_t m = 0; m < d; ++m) {
                        double diff = (double)x[m] - c[m];
                        d2 += diff * diff;
                    }
                    if (d2 < dmin) { dsec = dmin; dmin = d2; jmin = j; }
                    else if (d2 < dsec) { dsec = d2; }
                }
                if (skip) {                               /* audit: the bounds promised that nothing changes */
                    ++n_skipped;
                    if (jmin != a && violations) *violations += 1;
                    continue;
                }
                u[i] = sqrt(dmin);
                l[i] = sqrt(dsec);
                if (jmin != a) {
                    for (int32_t m = 0; m < d; ++m) {
                        sum[(int64_t)a * d + m] -= (double)x[m];
                        sum[(int64_t)jmin * d + m] += (double)x[m];
                    }
                    counts[a] -= 1;
                    counts[jmin] += 1;
                    labels[i] = jmin;
                    ++n_moved;
                }
            }
        }
        if (obj_hist) {                                   /* by the definition, over all points */
            double obj = 0.0;
            for (int64_t i = 0; i < n; ++i) {
                const double *c = Cu + (int64_t)labels[i] * d;
                double d2 = 0.0;
                for (int32_t m = 0; m < d; ++m) {
                    double diff = (double)X[i * ld + m] - c[m];
                    d2 += diff * diff;
                }
                obj += d2;
            }
            obj_hist[t] = obj;
        }
        if (skipped) skipped[t] = n_skipped;
        if (moved) moved[t] = n_moved;
        /* update step from the kept sums; an empty cluster keeps its centroid */
        memcpy(Cu_old, Cu, kd * sizeof(double));
        for (int32_t j = 0; j < k; ++j) {
            if (counts[j] == 0) continue;
            for (int32_t m = 0; m < d; ++m)
                C[(int64_t)j * d + m] = sum[(int64_t)j * d + m] / (double)counts[j];
        }
    }
    free(u); free(l); free(sum); free(Cu); free(Cu_old); free(delta);
    return 0;
}

/* ---- sample-trained K-Means ------------------------------------------------ */

/*
 * The clustering as the paper's Sec. "Implementation" runs it: the centroids
 * are computed on a sample of the embeddings (2^9 per cluster there), and every
 * vertex then gets the partition of its nearest centroid.
 * Reading taken (the paper gives no further detail): the sample is the m rows
 * rows[0..m) of X in that order; Lloyd runs `iters` rounds on it from its
 * first k rows as initial centroids; then one assignment of all n rows
 * against the trained centroids.
 *   C        : k x d trained centroids (means over the SAMPLE)
 *   counts   : sizes of the sample's clusters in the last round
 *   obj_hist : the sample's objective per round (may be NULL)
 *   labels   : n labels of the full assignment;  *obj_full its objective
 * Returns 0, or -1 on bad arguments (m < k, m > n, a row out of range).
 */
int or_sampled_kmeans(int64_t n, int32_t d, int32_t k, const float *X, int64_t ld,
                      int64_t m, const int64_t *rows, int32_t iters, int flags,
                      double *C, int32_t *labels, int64_t *counts,
                      double *obj_hist, double *obj_full)
{
    if (n < 1 || d < 1 || k < 1 || m < (int64_t)k || m > n || ld < d || iters < 0) return -1;
    for (int64_t i = 0; i < m; ++i)
        if (rows[i] < 0 || rows[i] >= n) return -1;
    float *S = (float *)malloc((size_t)m * (size_t)d * sizeof(float));
    int32_t *sample_labels = (int32_t *)malloc((size_t)m * sizeof(int32_t));
    int64_t *first = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    if (!S || !sample_labels || !first) { free(S); free(sample_labels); free(first); return -1; }
    for (int64_t i = 0; i < m; ++i)
        for (int32_t c = 0; c < d; ++c) S[i * d + c] = X[rows[i] * ld + c];
    for (int32_t j = 0; j < k; ++j) first[j] = j;
    int rc = or_lloyd(m, d, k, S, d, iters, first, flags & OR_FLAG_BF16_CENTROIDS,
                      C, sample_labels, counts, obj_hist, NULL);
    if (rc == 0) {
        double obj = or_assign(n, d, k, X, ld, C, (flags & OR_FLAG_BF16_CENTROIDS) ? 1 : 0,
                               labels, NULL, NULL);
        if (obj_full) *obj_full = obj;
    }
    free(S); free(sample_labels); free(first);
    return rc;
}

/* ---- partition quality over a CSR graph ---------------------------------- */

/*
 * cut   = number of stored CSR entries (u,v) with pid(u) != pid(v)
 *         (an undirected edge stored in both directions counts twice, so
 *         cut / nnz is the edge-cut ratio either way);
 * sizes = |P_p| for p in [0,k).
 * Returns 0, or -1 if a label or a column index is out of range.
 */
int or_partition_quality(int64_t n, int32_t k, const int64_t *rowptr,
                         const int32_t *colidx, const int32_t *labels,
                         int64_t *cut, int64_t *sizes)
{
    for (int32_t p = 0; p < k; ++p) sizes[p] = 0;
    int64_t c = 0;
    for (int64_t u = 0; u < n; ++u) {
        if (labels[u] < 0 || labels[u] >= k) return -1;
        sizes[labels[u]] += 1;
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            int32_t v = colidx[e];
            if (v < 0 || v >= n) return -1;
            if (labels[u] != labels[v]) ++c;
        }
    }
    *cut = c;
    return 0;
}

/* ECR = |C| / |E| and vertex balance = max / mean of the partition sizes. */
double or_edge_cut_ratio(int64_t cut, int64_t nnz)
{
    return nnz > 0 ? (double)cut / (double)nnz : 0.0;
}

double or_vertex_balance(int32_t k, const int64_t *sizes)
{
    int64_t mx = 0, total = 0;
    for (int32_t p = 0; p < k; ++p) {
        total += sizes[p];
        if (sizes[p] > mx) mx = sizes[p];
    }
    return (double)mx / ((double)total / (double)k);
}

/* ---- balancing (Alg. 3 loops, Alg. 4 migration policy) ---------------------- */

/*
 * One stateless draw: the destination of vertex v in migration round `round`
 * is decided by a 64-bit mix of (seed, round, v), so the order in which the
 * vertices are visited does not matter.  The mix is the splitmix64 output
 * function applied to seed + (round * 2^32 + v + 1) * golden-ratio increment.
 */
static uint64_t draw64(uint64_t seed, uint32_t round, int64_t v)
{
    uint64_t z = seed + (((uint64_t)round << 32) + (uint64_t)v + 1ULL) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

typedef struct { int64_t degree; int64_t v; } or_cand;
static int cand_less(const void *a, const void *b)
{
    const or_cand *x = (const or_cand *)a, *y = (const or_cand *)b;
    if (x->degree != y->degree) return x->degree < y->degree ? -1 : 1;
    return x->v < y->v ? -1 : (x->v > y->v ? 1 : 0);
}

/*
 * Balancing of one vertex class (one of the three while-loops of Alg. 3) with
 * the migration policy of Alg. 4.
 *   S          = {v : vclass == NULL or vclass[v] == class_id}, the candidate set
 *   capacity   C = max(floor(beta * |S| / k), ceil(|S| / k)) for every partition
 *                (Alg. 3: a partition is overloaded iff its load exceeds
 *                beta * |S| / k; the second term only keeps the target reachable
 *                when beta is so close to 1 that k * floor(..) < |S|)
 *   per round  loads L_i over S; O = {L_i > C}, U = {L_i < C}; f_i = C - L_i on U,
 *              F = sum f_i; from every i in O the m_i = L_i - C members of S with
 *              the smallest degree move (reading: ties by smaller vertex id; the
 *              degree is the stored row length rowptr[v+1] - rowptr[v]); each
 *              goes to j in U with probability f_j / F: r = draw64 mod F, j = the
 *              partition whose interval of the running sum of f (partitions in
 *              index order) holds r.  All draws of a round use that round's L.
 *   rounds     repeat while some partition is overloaded, at most max_rounds.
 * stats[0] = rounds run, stats[1] = vertices moved in total, stats[2] = partitions
 * still overloaded at the end.  Returns 0, or -1 on bad arguments.
 */
int or_balance(int64_t n, int32_t k, const int64_t *rowptr, const uint8_t *vclass,
               int32_t class_id, double beta, uint64_t seed, int32_t max_rounds,
               int32_t *labels, int64_t *stats)
{
    if (n < 1 || k < 1 || k > 255 || !rowptr || !labels || !stats || max_rounds < 0 || !(beta >= 1.0)) return -1;
    for (int64_t v = 0; v < n; ++v)
        if (labels[v] < 0 || labels[v] >= k) return -1;
    int64_t *L = (int64_t *)calloc((size_t)k, sizeof(int64_t));
    int64_t *cumf = (int64_t *)calloc((size_t)k, sizeof(int64_t));
    or_cand *cand = (or_cand *)malloc((size_t)n * sizeof(or_cand));
    int32_t *dest = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    if (!L || !cumf || !cand || !dest) { free(L); free(cumf); free(cand); free(dest); return -1; }
    stats[0] = stats[1] = stats[2] = 0;
    for (int32_t round = 0;; ++round) {
        int64_t total = 0;
        for (int32_t i = 0; i < k; ++i) L[i] = 0;
        for (int64_t v = 0; v < n; ++v)
            if (!vclass || vclass[v] == class_id) { L[labels[v]]++; total++; }
        int64_t C = (int64_t)floor(beta * (double)total / (double)k);
        const int64_t reach = (total + k - 1) / k;
        if (C < reach) C = reach;
        int64_t F = 0, over = 0;
        for (int32_t i = 0; i < k; ++i) {
            if (L[i] < C) F += C - L[i];
            cumf[i] = F;                       /* running sum of the free capacities */
            if (L[i] > C) over++;
        }
        stats[2] = over;
        if (over == 0 || round >= max_rounds) break;
        stats[0] = round + 1;
        for (int64_t v = 0; v < n; ++v) dest[v] = -1;
        for (int32_t i = 0; i < k; ++i) {
            if (L[i] <= C) continue;
            int64_t cnt = 0;
            for (int64_t v = 0; v < n; ++v)
                if ((!vclass || vclass[v] == class_id) && labels[v] == i) {
                    cand[cnt].degree = rowptr[v + 1] - rowptr[v];
                    cand[cnt].v = v;
                    cnt++;
                }
            qsort(cand, (size_t)cnt, sizeof(or_cand), cand_less);
            const int64_t m = L[i] - C;
            for (int64_t q = 0; q < m; ++q) {
                const int64_t v = cand[q].v;
                const uint64_t r = draw64(seed, (uint32_t)round, v) % (uint64_t)F;
                int32_t j = 0;
                while ((uint64_t)cumf[j] <= r) ++j;   /* first partition whose running sum exceeds r */
                dest[v] = j;
            }
        }
        for (int64_t v = 0; v < n; ++v)
            if (dest[v] >= 0) { labels[v] = dest[v]; stats[1]++; }
    }
    free(L); free(cumf); free(cand); free(dest);
    return 0;
}

/* ---- reordering ------------------------------------------------------------ */

/*
 * Vertices of one partition get consecutive new ids.  Reading that makes the
 * result unique: partitions in increasing id, vertices inside a partition in
 * increasing original id.  new_id[v] = pi(v); order[pi(v)] = v.
 */
int or_permutation(int64_t n, int32_t k, const int32_t *labels,
                   int32_t *new_id, int32_t *order)
{
    int64_t *next = (int64_t *)calloc((size_t)k + 1, sizeof(int64_t));
    for (int64_t v = 0; v < n; ++v) {
        if (labels[v] < 0 || labels[v] >= k) { free(next); return -1; }
        next[labels[v] + 1] += 1;
    }
    for (int32_t p = 0; p < k; ++p) next[p + 1] += next[p];  /* next[p] = first id of p */
    for (int64_t v = 0; v < n; ++v) {
        int64_t id = next[labels[v]]++;
        new_id[v] = (int32_t)id;
        order[id] = (int32_t)v;
    }
    free(next);
    return 0;
}

/* Sum over stored CSR entries of |pi(u) - pi(v)|; pi = identity when NULL. */
uint64_t or_edge_gap_sum(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                         const int32_t *new_id)
{
    uint64_t total = 0;
    for (int64_t u = 0; u < n; ++u) {
        int64_t pu = new_id ? new_id[u] : u;
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            int64_t pv = new_id ? new_id[colidx[e]] : colidx[e];
            total += (uint64_t)(pu > pv ? pu - pv : pv - pu);
        }
    }
    return total;
}

/*
 * Sum over vertices of the vertex bandwidth max_{u in N(v)} |pi(v) - pi(u)|
 * (0 for an isolated vertex); divided by |V| it is the average graph
 * bandwidth.
 */
uint64_t or_vertex_bandwidth_sum(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                                 const int32_t *new_id)
{
    uint64_t total = 0;
    for (int64_t u = 0; u < n; ++u) {
        int64_t pu = new_id ? new_id[u] : u;
        int64_t widest = 0;
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            int64_t pv = new_id ? new_id[colidx[e]] : colidx[e];
            int64_t gap = pu > pv ? pu - pv : pv - pu;
            if (gap > widest) widest = gap;
        }
        total += (uint64_t)widest;
    }
    return total;
}

/*
 * The graph rewritten under the new ids (Sec. "Extension to Graph
 * Reordering": the id of a vertex is its position in memory, so relabelling
 * means moving the rows).  Row pi(v) of the result holds the neighbours of v
 * under their new ids.  Reading that makes the result unique: the entries of a
 * row come in ascending new id (parallel edges stay, side by side).
 * new_rowptr has n + 1 entries, new_colidx as many as colidx.
 */
static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int or_reorder_csr(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                   const int32_t *new_id, int64_t *new_rowptr, int32_t *new_colidx)
{
    int32_t *order = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    for (int64_t r = 0; r < n; ++r) order[r] = -1;
    for (int64_t v = 0; v < n; ++v) {
        if (new_id[v] < 0 || new_id[v] >= n || order[new_id[v]] != -1) { free(order); return -1; }
        order[new_id[v]] = (int32_t)v;
    }
    new_rowptr[0] = 0;
    for (int64_t r = 0; r < n; ++r) {
        int64_t v = order[r], len = rowptr[v + 1] - rowptr[v], at = new_rowptr[r];
        for (int64_t j = 0; j < len; ++j) {
            int32_t u = colidx[rowptr[v] + j];
            if (u < 0 || u >= n) { free(order); return -1; }
            new_colidx[at + j] = new_id[u];
        }
        qsort(new_colidx + at, (size_t)len, sizeof(int32_t), cmp_i32);
        new_rowptr[r + 1] = at + len;
    }
    free(order);
    return 0;
}
