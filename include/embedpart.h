/*
 * embedpart.h -- C ABI of the MI355X (gfx950) clustering hot path of EmbedPart.
 *
 * The library implements the dense, data-parallel part of the paper's Phase 2
 * (Alg. 3, first step: P <- KMeans(E, k); Sec. "Phase 2: Clustering and
 * Balancing": one embedding per vertex is clustered into exactly k groups and
 * the clusters are the graph partitions), the integer evaluation of the
 * resulting partition (Sec. "Partitioning quality metrics": cut edges and
 * partition sizes, from which ECR = |C|/|E| and the vertex balance follow) and
 * the relabelling used for graph reordering (Sec. "Adapting EmbedPart for
 * Reordering": vertices of one partition get consecutive ids; Eq. gap:
 * xi_pi(u,v) = |pi(u) - pi(v)|).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name ends in `_host`.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; no call synchronises, so outputs are valid
 *     once the caller has synchronised the stream.
 *   - The caller owns every buffer, including the workspace `ws`, which must be
 *     256-byte aligned and at least as large as the matching *_workspace_bytes
 *     call reports.  The library allocates nothing, frees nothing and keeps no
 *     pointer after a call returns.  Its only global state is the code of the
 *     last failing HIP call (ep_last_hip_error) and the static workspace of
 *     kmeans_run_noalloc.  (The benchmark aids of embedpart_bench.h, which are not
 *     part of the method, add one more.)
 *   - Partition / cluster ids are 0-based, in [0, k).  (The paper numbers
 *     partitions 1..k.)
 *   - Return value: EP_OK (0) or a negative EP_E* code.  Arguments are checked
 *     on the host before any HIP call is made; no exception crosses the ABI.
 *   - Results are bit-reproducible from run to run: no floating-point atomics
 *     are used and every reduction has a fixed order.
 */
#ifndef EMBEDPART_H
#define EMBEDPART_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EP_OK            0
#define EP_EINVAL       (-1)  /* null pointer, size out of range, k > n, ld < d, misaligned buffer */
#define EP_EUNSUPPORTED (-2)  /* shape or dtype no kernel of this build covers */
#define EP_EWORKSPACE   (-3)  /* workspace missing, misaligned or too small */
#define EP_EHIP         (-4)  /* a HIP runtime call failed: see ep_last_hip_error() */

#define EP_F32  0             /* embeddings stored as IEEE binary32 */
#define EP_BF16 1             /* embeddings stored as bfloat16; all accumulation is fp32 or wider */
#define EP_F16  2             /* embeddings stored as IEEE binary16: widened to fp32 on arrival (exact), then as EP_F32 */

/* kmeans_run flags */
#define EP_RUN_FINAL_REASSIGN 1  /* one more assignment against the final centroids */
#define EP_RUN_BOUNDS         2  /* skip points whose distance bounds show that their label cannot change */

/* kmeans_update flags */
#define EP_UPDATE_ACCUMULATE 1   /* add this call's rows to the sums and counts that earlier calls left in ws */
#define EP_UPDATE_FINALIZE   2   /* form the means (C_out, counts) from everything accumulated */

/* Limits of this build. */
#define EP_MAX_D          1024
#define EP_MAX_K          65536
#define EP_MAX_N          ((int64_t)1 << 31)   /* vertex ids and labels are int32; n < 2^31 */
#define EP_BALANCE_MAX_K      255              /* partition_balance: partition-scale k only */
#define EP_BALANCE_MAX_ROUNDS 1024

/* The clustering problem: n embeddings of dimension d, row-major with row
 * stride ld (elements, ld >= d), to be grouped into k clusters.
 * X must be 16-byte aligned; ld must be a multiple of 4 (EP_F32) or of 8
 * (EP_BF16, EP_F16), so that every row starts 16-byte aligned. */
typedef struct ep_problem {
    int64_t n;
    int64_t ld;
    int32_t d;
    int32_t k;
    int32_t dtype;     /* EP_F32, EP_BF16 or EP_F16 */
    int32_t reserved;  /* must be 0 */
} ep_problem;

/* Library version (major * 100 + minor). */
int ep_version(void);

/* Static, human-readable text for a return code. */
const char *ep_strerror(int code);

/* hipError_t value of the most recent failing HIP call of this process (0 if none). */
int ep_last_hip_error(void);

/*
 * Seeded choice of the k initial rows.  The paper leaves K-Means'
 * initialisation open; here the initial centroids are k distinct rows:
 * a splitmix64 stream started at `seed` is reduced mod n, repeats are
 * rejected and the draw order is the centroid order.
 * idx_host: k entries, host memory, written.   Host-only, no HIP call.
 */
int kmeans_init_indices(uint64_t seed, int64_t n, int32_t k, int64_t *idx_host);

/* Bytes of workspace that kmeans_init / assign / update / run need for `p`. */
int kmeans_workspace_bytes(const ep_problem *p, size_t *bytes_host);

/*
 * Initial centroids (the paper's Alg. 3 begins with P <- KMeans(E, k) and leaves the start of
 * K-Means open; here it starts from k rows of E): C[j, :] = X[idx_host[j], :] widened to fp32.
 * idx_host: k row indices in [0, n) on the host.  They are copied to the device during the call
 * from pageable host memory: the call may wait on the host until earlier work on `stream` has
 * drained, and it cannot be recorded into a stream capture (every other call of the K-Means
 * group only enqueues).
 * C: k x d fp32, dense (row stride d), written.
 */
int kmeans_init(const ep_problem *p, const void *X, const int64_t *idx_host,
                float *C, void *ws, size_t ws_bytes, void *stream);

/*
 * Assignment step of K-Means (Alg. 3, P <- KMeans(E, k); Sec. "Phase 2: Clustering and
 * Balancing": every vertex joins the cluster, i.e. the partition, of its nearest centroid):
 * labels[i] = argmin_j ||x_i - c_j||^2 (squared Euclidean; the lowest j wins an exact tie),
 * evaluated as ||c_j||^2 - 2 x_i.c_j in fp32.  With EP_BF16 the centroids are rounded to
 * bf16 (nearest-even) for the x.c products, which accumulate in fp32.
 *   C         k x d fp32, read
 *   labels    n int32, 16-byte aligned, written
 *   min_d2    n fp32 or NULL: ||x_i - c_label||^2 (clamped at 0), written
 *   objective 1 double or NULL: sum_i ||x_i - c_label||^2, written (not added to)
 * Row ranges: rows are independent, so the rows [b, e) of a larger matrix are assigned by a call
 * with n = e - b, X + b * ld (elements), labels + b and min_d2 + b (b a multiple of 4 keeps labels
 * aligned); `objective` is then the range's own sum and the caller adds the ranges up.  For such a
 * call k may exceed n.  A matrix that does not fit the device is streamed this way, chunk by
 * chunk, with kmeans_update's flags for the other half of the round.
 */
int kmeans_assign(const ep_problem *p, const void *X, const float *C,
                  int32_t *labels, float *min_d2, double *objective,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * Update step of K-Means (Alg. 3, P <- KMeans(E, k): a centroid moves to the mean of the
 * embeddings assigned to it): C_out[j] = mean of the rows labelled j; a cluster without rows
 * keeps C_prev[j] and gets count 0.  Sums are fp32 over bounded runs of rows, combined in fp64 in
 * a fixed order.
 *   labels  n int32 in [0, k), read (a label outside the range is undefined behaviour
 *           in the sense of a wrong result, never of an out-of-bounds access: such
 *           rows are skipped; ep_validate_labels counts them)
 *   C_prev  k x d fp32, read;  C_out k x d fp32, written (may alias C_prev)
 *   counts  k int64, written
 *   flags   EP_UPDATE_FINALIZE: the whole update in one call, as described above.
 *           Over row ranges (chunks of a matrix that is streamed through the device, in any sizes;
 *           k may exceed a chunk's n): the first chunk with flags 0, the following ones with
 *           EP_UPDATE_ACCUMULATE, the last one with EP_UPDATE_ACCUMULATE | EP_UPDATE_FINALIZE.
 *           Between those calls the fp64 sums and the counts live at the start of `ws`, at a place
 *           that depends on k and d only: pass the same ws (sized for the largest chunk) to all of
 *           them; kmeans_assign calls in between leave it alone, any other call may not.  C_prev,
 *           C_out and counts are used by the finalizing call only.  The result is the mean over all
 *           chunks and, for given chunk boundaries, bit-reproducible.
 */
int kmeans_update(const ep_problem *p, const void *X, const int32_t *labels,
                  const float *C_prev, float *C_out, int64_t *counts, int flags,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * Check of a label vector against the paper's contract that every vertex carries exactly one
 * partition id (Sec. "Graph Partitioning": the partitions are disjoint and cover V; ids here are 0 .. k-1).
 * The hot calls skip labels outside [0, k) instead of testing for them; this call counts them.
 *   result  2 int64, 8-byte aligned, written: [0] = number of labels outside [0, k),
 *           [1] = index of the first one (n if there is none)
 */
int ep_validate_labels(int64_t n, int32_t k, const int32_t *labels, int64_t *result, void *stream);

/*
 * `iters` Lloyd rounds (assign, then update: the K-Means of Alg. 3's first step, run for a fixed
 * number of rounds) starting from the centroids in C.
 *   C               k x d fp32: initial centroids in, final centroids out
 *   labels          n int32, 16-byte aligned, written: the labels of the last assignment performed
 *   counts          k int64, written: cluster sizes of round `iters`, of which C holds the means
 *   objective_hist  iters + 1 doubles or NULL: [t] = objective of round t's assignment;
 *                   [iters] is written only with EP_RUN_FINAL_REASSIGN
 * Without the flag, C is exactly the mean of the rows carrying each returned label.
 * With it, labels come from one further assignment against the final C
 * (train-then-assign use); counts and C still describe round `iters`.
 * iters may be 0 (then only the optional final assignment runs).
 */
int kmeans_run(const ep_problem *p, const void *X, int32_t iters, float *C,
               int32_t *labels, int64_t *counts, double *objective_hist, int flags,
               void *ws, size_t ws_bytes, void *stream);

/*
 * EP_RUN_BOUNDS: the same Lloyd rounds reached with less work (the paper's contribution list and
 * Sec. "Phase 2: Clustering and Balancing" leave Phase 2 open to more advanced clustering
 * algorithms; this is the exact one of Hamerly, "Making k-means even faster", SDM 2010).  Every
 * point keeps an upper bound on the distance to its own centroid and a lower bound on the distance
 * to all others; after an update the bounds are moved by how far the centroids moved, and a point
 * whose bounds still separate is not read at all in the next round.  The per-cluster sums are kept
 * in fp64 between rounds and only rows that change label are moved between them.  The first three
 * rounds are ordinary ones; the third also takes every point's bounds (from its best and second-best
 * score) and keeps the sums.
 *   Results: a searched point goes through the score arithmetic of the plain rounds and the bounds
 *   leave room for its rounding, so from equal centroids a round gives the labels of the plain round
 *   bit for bit.  The centroids themselves agree with the plain run's to the order of the fp64
 *   additions (about 1e-7 relative: kept sums against sums from scratch), which can decide a near-tie
 *   the other way in a later round; every round still is an exact Lloyd round of its own centroids.
 *   A run of T1 rounds followed by one of T2 is therefore not bit-equal to T1 + T2 rounds in one run,
 *   as it is without the flag; the run itself is bit-reproducible.
 *   Shapes: k in [2, 64], d = 64 or 128, fp32, fp16 or bfloat16 rows, iters >= 4; for any other shape the
 *   flag is accepted and the rounds run in full.
 *   When it pays: a bounded round is five launches where a plain round is two, and what it saves is
 *   reading rows from memory, so it is for matrices well beyond the chip's 256 MB of cache (measured:
 *   1.45x at 57 GB, 2.1x at 1.25 GB; at 87 MB and below the plain rounds are faster).
 *   Workspace: kmeans_run_workspace_bytes(p, iters, flags), which grows by 12 bytes per row.
 * kmeans_run_workspace_bytes with flags without EP_RUN_BOUNDS equals kmeans_workspace_bytes.
 * kmeans_run_searched copies out, from the workspace of a finished kmeans_run with EP_RUN_BOUNDS
 * (same p, iters, flags), the number of rows whose distances were evaluated in each round:
 *   searched  iters int64, 8-byte aligned, written (n for the full rounds);
 *   EP_EUNSUPPORTED when the flag has no effect on this shape.
 */
int kmeans_run_workspace_bytes(const ep_problem *p, int32_t iters, int flags, size_t *bytes_host);
int kmeans_run_searched(const ep_problem *p, int32_t iters, int flags, const void *ws, size_t ws_bytes,
                        int64_t *searched, void *stream);

/*
 * kmeans_run for callers that cannot allocate device memory or carry a workspace: code under
 * stream capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels
 * and results (bit for bit) as kmeans_run, without `ws`: the workspace is a static device array
 * of EP_NOALLOC_SCRATCH_BYTES inside the library, which every GPU the library runs on holds until
 * the process ends.  The call allocates and frees nothing.
 *   Limit: kmeans_workspace_bytes(p) <= EP_NOALLOC_SCRATCH_BYTES, else EP_EWORKSPACE.  Every shape of
 *   the fused kernels (k <= 64 with d <= 128, k <= 16 with d <= 256, any n) fits; other shapes fit
 *   for small n only, because their workspace grows with n.
 *   The array is looked up once per device, at the first call made with that device current; the
 *   current device must be the one `stream` belongs to.
 *   All calls on one GPU share the array and it keeps the last call's contents (no call relies on
 *   them): two calls whose work overlaps on one GPU (different streams, or threads) race.
 */
#define EP_NOALLOC_SCRATCH_BYTES (34 * 1024 * 1024)
int kmeans_run_noalloc(const ep_problem *p, const void *X, int32_t iters, float *C,
                       int32_t *labels, int64_t *counts, double *objective_hist, int flags,
                       void *stream);

/*
 * Sample-trained K-Means: the clustering as the paper's Sec. "Implementation" runs it. The
 * centroids are computed on a sample of the embeddings (2^9 per cluster there) and every vertex
 * then takes the partition of its nearest centroid.
 *   m, sample_rows_host  the sample: m row indices of X (k <= m <= n, each in [0, n); they
 *                        should be distinct, e.g. from kmeans_init_indices(seed, n, m)), HOST memory
 *   iters                Lloyd rounds on the sample, starting from its first k rows
 *   C                    k x d fp32, written: the trained centroids (means over the sample)
 *   labels               n int32, 16-byte aligned, written: nearest trained centroid of every row of X
 *   counts               k int64, written: the sample's cluster sizes in the last round
 *   objective_hist       iters + 1 doubles or NULL: [t] = the sample's objective in round t,
 *                        [iters] = the objective of the full assignment
 *   ws                   kmeans_sampled_workspace_bytes(p, m) bytes; holds the dense copy of the sample
 * sample_rows_host is copied to the device during the call from pageable host memory: like
 * kmeans_init, the call may wait on the host for earlier work on `stream` and cannot be captured.
 * Errors as kmeans_run; EP_EINVAL also for m outside [k, n] or a row index outside [0, n).
 */
int kmeans_sampled_workspace_bytes(const ep_problem *p, int64_t m, size_t *bytes_host);
int kmeans_run_sampled(const ep_problem *p, const void *X, int64_t m, const int64_t *sample_rows_host,
                       int32_t iters, float *C, int32_t *labels, int64_t *counts, double *objective_hist,
                       void *ws, size_t ws_bytes, void *stream);

/* Bytes of workspace that the graph calls below need. */
int graph_workspace_bytes(int64_t n, int64_t nnz, int32_t k, size_t *bytes_host);

/*
 * Quality of a partition over a CSR graph, in integers (Sec. "Partitioning quality metrics": an
 * edge (u,v) is cut iff pid(u) != pid(v); edge-cut ratio |C| / |E|; vertex balance
 * max |P_i| / mean |P_i|).
 *   rowptr   n + 1 offsets, int32 or int64 (rowptr_is_i64), rowptr[n] == nnz
 *   colidx   nnz int32 column indices in [0, n), 16-byte aligned
 *   labels   n int32 partition ids in [0, k)
 *   cut      1 int64, written: stored entries (u,v) with labels[u] != labels[v]
 *            (an undirected edge stored in both directions counts twice; divide
 *            by nnz for the edge-cut ratio)
 *   sizes    k int64, written: vertices per partition (max * k / n is the vertex balance)
 * Entries whose column index or whose labels fall outside their range are skipped.
 */
int partition_quality(int64_t n, int64_t nnz, int32_t k, const void *rowptr, int rowptr_is_i64,
                      const int32_t *colidx, const int32_t *labels,
                      int64_t *cut, int64_t *sizes, void *ws, size_t ws_bytes, void *stream);

/*
 * Reordering (Sec. "Adapting EmbedPart for Reordering": vertices of one partition get
 * consecutive ids): partitions in increasing id, vertices inside a partition in increasing
 * original id.  Vertices whose label is outside [0, k) come last, in increasing id.
 *   new_id  n int32, written: pi(v)
 *   order   n int32, written: order[pi(v)] = v
 */
int partition_permutation(int64_t n, int32_t k, const int32_t *labels,
                          int32_t *new_id, int32_t *order, void *ws, size_t ws_bytes, void *stream);

/*
 * Sum over stored CSR entries (u,v) of the gap xi_pi(u,v) = |pi(u) - pi(v)| (Eq. gap of the
 * reordering section); new_id == NULL means the identity.  gap_sum: 1 uint64, written.  Divide by nnz for the mean gap.
 */
int edge_gap_sum(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64,
                 const int32_t *colidx, const int32_t *new_id,
                 uint64_t *gap_sum, void *ws, size_t ws_bytes, void *stream);

/*
 * Balancing of a partition for ONE vertex class: one of the three loops of the paper's Alg. 3
 * (training, validation, remaining vertices) with the migration policy of Alg. 4. While some
 * partition holds more than C = max(floor(beta |S| / k), ceil(|S| / k)) members of the class S,
 * every overloaded partition gives up its L_i - C members of smallest degree (equal degrees:
 * smaller vertex id first; degree = rowptr[v+1] - rowptr[v], degrees of 2^24 and more count as
 * equal), and each of them goes to an underloaded partition drawn with probability proportional
 * to its free capacity: r = mix64(seed, round, v) mod F over the running sum of the free
 * capacities in partition order (mix64 = the splitmix64 output function applied to
 * seed + (round * 2^32 + v + 1) * 0x9E3779B97F4A7C15).  All draws of a round use the loads at its
 * start.  At most max_rounds rounds are enqueued; rounds after the last needed one do nothing.
 *   rowptr     n + 1 offsets, int32 or int64 (rowptr_is_i64); only the row lengths are used
 *   vclass     n bytes, class of every vertex, or NULL: all vertices form the class
 *   class_id   the class to balance (0..255)
 *   beta       imbalance factor, >= 1
 *   labels     n int32 in [0, k), updated in place
 *   stats      3 int64, written: rounds that moved vertices, vertices moved, partitions still
 *              overloaded after the last round (0 = balanced)
 *   ws         balance_workspace_bytes(n) bytes
 * k <= EP_BALANCE_MAX_K (else EP_EUNSUPPORTED); 0 <= max_rounds <= EP_BALANCE_MAX_ROUNDS.
 * Integer arithmetic and a counter-based draw: the result is bit-reproducible.
 */
int balance_workspace_bytes(int64_t n, size_t *bytes_host);
int partition_balance(int64_t n, int32_t k, const void *rowptr, int rowptr_is_i64,
                      const uint8_t *vclass, int32_t class_id, double beta, uint64_t seed,
                      int32_t max_rounds, int32_t *labels, int64_t *stats,
                      void *ws, size_t ws_bytes, void *stream);

/*
 * Phase 2 of the method in one call (the paper's Alg. 3, ClusterAndBalance): P <- KMeans(E, k),
 * then the three balancing loops over the training, validation and remaining vertices, each
 * with its own imbalance factor.  It enqueues exactly what kmeans_init + kmeans_run (or
 * kmeans_run_sampled) + three partition_balance calls would, in that order, and returns the
 * same results bit for bit.
 *   rows_host  sample_rows == 0: k distinct row indices, the initial centroids (kmeans_init);
 *              sample_rows == m > 0: the m sample rows of kmeans_run_sampled
 *   vclass     n bytes: 0 training, 1 validation, 2 remaining vertex; NULL: every vertex counts
 *              as remaining (one loop, beta[2])
 *   C          k * d fp32, written: the centroids K-Means ended with
 *   labels     n int32, 16-byte aligned, written: the partition of every vertex after balancing
 *   counts     k int64, written: the cluster sizes K-Means ended with (before balancing)
 *   stats      9 int64, written: the three partition_balance statistics of class 0, 1, 2 (with
 *              vclass == NULL only the last three)
 *   ws         cluster_and_balance_workspace_bytes(p, sample_rows) bytes
 * Errors: as the calls it is made of; k > EP_BALANCE_MAX_K gives EP_EUNSUPPORTED.
 */
typedef struct ep_phase2 {
    double beta[3];      /* imbalance factors beta_train, beta_val, beta_rest (>= 1) */
    uint64_t seed;       /* class c draws its destinations with seed + c */
    int32_t iters;       /* Lloyd rounds */
    int32_t max_rounds;  /* migration rounds per class, at most EP_BALANCE_MAX_ROUNDS */
    int64_t sample_rows; /* 0: Lloyd over all rows; m: centroids trained on m sample rows */
} ep_phase2;
int cluster_and_balance_workspace_bytes(const ep_problem *p, int64_t sample_rows, size_t *bytes_host);
int cluster_and_balance(const ep_problem *p, const void *X, const void *rowptr, int rowptr_is_i64,
                        const uint8_t *vclass, const ep_phase2 *opt, const int64_t *rows_host,
                        float *C, int32_t *labels, int64_t *counts, int64_t *stats,
                        void *ws, size_t ws_bytes, void *stream);

/*
 * Sum over vertices of the vertex bandwidth max_{u in N(v)} |pi(v) - pi(u)|
 * (0 for a vertex without neighbours); divided by n it is the average graph
 * bandwidth of the paper's reordering evaluation.  bw_sum: 1 uint64, written.
 */
int vertex_bandwidth_sum(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64,
                         const int32_t *colidx, const int32_t *new_id,
                         uint64_t *bw_sum, void *ws, size_t ws_bytes, void *stream);

/*
 * The graph rewritten under new vertex ids (Sec. "Extension to Graph Reordering": the id of a
 * vertex is its position in memory, and vertices of one partition get consecutive ids): row
 * new_id[v] of the result holds the neighbours of v under their new ids, in ascending order
 * (parallel edges stay, side by side).  Metrics of (graph, pi) equal those of the result under
 * the identity.
 *   rowptr, colidx   the graph as for partition_quality
 *   new_id, order    n int32 each, inverse permutations of [0, n) as partition_permutation
 *                    writes them: new_id[v] = pi(v), order[pi(v)] = v
 *   new_rowptr       n + 1 offsets, written, same width as rowptr (8-byte aligned)
 *   new_colidx       nnz int32, written; must not overlap colidx
 *   ws               graph_reorder_workspace_bytes(n, nnz) bytes
 * If `order` is not a permutation (an entry out of range, or the degrees met through it do not
 * add up to nnz) new_colidx is left unwritten; column indices outside [0, n) are carried over as
 * they are.  No access leaves the buffers in either case.  EP_EINVAL also for nnz >= 2^31 with
 * 32-bit offsets.  Integer work only: the result is bit-reproducible.
 */
int graph_reorder_workspace_bytes(int64_t n, int64_t nnz, size_t *bytes_host);
int graph_reorder(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64,
                  const int32_t *colidx, const int32_t *new_id, const int32_t *order,
                  void *new_rowptr, int32_t *new_colidx, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EMBEDPART_H */
