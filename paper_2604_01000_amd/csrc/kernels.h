// Host-side launchers of the HIP kernels; each enqueues on `s` and returns an EP_* code.
#pragma once

#include "common.h"

namespace ep {

// ---- K-Means, shape-generic kernels (kmeans_generic.hip) ----------------------
constexpr int kObjBlocksMax = 2048;   // partial objectives per assignment launch
constexpr int kUpdBlocksMax = 1024;   // partial sums per small-k update launch
constexpr int kSmallKElems = 8192;    // k*d at or below this: per-workgroup LDS partial sums
constexpr int kSegWavesTarget = 16384; // sorted update: waves to spread k segments over when k is small

// Which centroid update a problem outside the fused small-k kernels takes: per-workgroup partial sums
// for small k * d, otherwise (and for k > 64 at d = 64 or 128, where it is several times faster)
// rows sorted by label + segment means.  The workspace is carved accordingly.
inline bool update_by_sorted_rows(const ep_problem &p) {
    return (int64_t)p.k * p.d > kSmallKElems || (p.k > 64 && (p.d == 64 || p.d == 128));
}

// Chunked centroid update (the flags of kmeans_update): running sums and counts kept in the workspace
// between the calls of one update, at a place that depends on k and d only.
struct UpdateAcc {
    double *sum;         // [k*d] sums of the chunks seen so far
    int64_t *cnt;        // [k]   their counts
    int64_t *chunk_cnt;  // [k]   counts of the current call (added to cnt after a call that does not finalize)
    int flags;           // EP_UPDATE_ACCUMULATE | EP_UPDATE_FINALIZE | kUpdateKeep
};
constexpr int kUpdateKeep = 4;   // internal: a finalizing call also leaves the sums and counts (bounded rounds)
inline UpdateAcc whole_update() { return UpdateAcc{nullptr, nullptr, nullptr, EP_UPDATE_FINALIZE}; }

#ifdef __HIPCC__
// Workgroups of the bounded search (4 waves, 16 rows per wave and step, steps dealt to the waves in order) that
// get any row of a list of `len` rows (clamped to [0, n]) on a grid of `parts`: the first so many.
__device__ __forceinline__ int list_parts(int64_t len, int64_t n, int parts) {
    len = len < 0 ? 0 : (len > n ? n : len);
    const int64_t with_rows = (len + 63) / 64;
    return with_rows < parts ? (int)with_rows : parts;
}

// Last step of every update kernel for element `at` = j * d + column of centroid j, given this call's
// sum `tot` and count `cnt` for it: add what earlier chunks left, then either form the mean (an empty
// cluster keeps its previous centroid) or leave the running sum for the next chunk.  Every element is
// owned by one thread; the running counts are only read here and are brought up to date by a later
// launch (launch_accumulate_counts, or the tail kernel of a bounded round), so no thread reads what
// another writes.
__device__ __forceinline__ void finish_centroid_element(const UpdateAcc &a, int64_t at, int32_t j, bool first_column,
                                                        double tot, int64_t cnt, const float *__restrict__ C_prev,
                                                        float *__restrict__ C_out, int64_t *__restrict__ counts) {
    if (a.flags & EP_UPDATE_ACCUMULATE) tot += a.sum[at];
    if (a.flags & EP_UPDATE_FINALIZE) {
        const int64_t all = (a.flags & EP_UPDATE_ACCUMULATE) ? cnt + a.cnt[j] : cnt;
        C_out[at] = all > 0 ? (float)(tot / (double)all) : C_prev[at];
        if (first_column) counts[j] = all;
    }
    if (!(a.flags & EP_UPDATE_FINALIZE) || (a.flags & kUpdateKeep)) {
        a.sum[at] = tot;
        if (first_column) a.chunk_cnt[j] = cnt;
    }
}
#endif

struct KmeansWs {
    double *obj_part;     // [kObjBlocksMax]
    double *acc_sum;      // [k*d]  running sums of a chunked update
    int64_t *acc_cnt;     // [k]    running counts of a chunked update
    int64_t *chunk_cnt;   // [k]    counts of the chunk in hand
    float *cnorm;         // [k]   generic path: ||c_j||^2; bf16 matrix-core path: -||c_j||^2 / 2 (of the rounded centroids)
    float *cq;            // [k*d] bf16-rounded centroids as fp32 (EP_BF16 only, else unused)
    bf16_t *cq16;         // [k*d] the same as bf16 (EP_BF16 only)
    float *psum;          // [kUpdBlocksMax * k * d]   (small k)
    int32_t *pcnt;        // [kUpdBlocksMax * k]       (small k)
    int64_t *idx;         // [k] init row indices
    float *best_score;    // [n] best score over the centroid slices seen so far (fp32, d in {64,128}, k > 64)
    int32_t *order;       // [n]  rows sorted by label           (large k)
    int32_t *order_tmp;   // [n]
    int64_t *seg;         // [k+1] segment offsets               (large k)
    double *seg_part;     // [kSegWavesTarget * d] sums of the parts of long segments (large k, d = 64 or 128)
    int32_t *sort_hist;   // radix-sort block histograms
    unsigned char *records;  // centroid tile records of the large-k matrix-core path
    int32_t *best_tile;   // [n] code of the 4 candidate centroid rows per point (large-k path)
    size_t bytes;
};
KmeansWs carve_kmeans_ws(const ep_problem &p, void *ws);

int launch_gather_rows(const ep_problem &p, const void *X, const int64_t *idx_dev, float *C, hipStream_t s);
// S[i,:] = X[rows_dev[i],:] for i < m, element type of X, row stride ld_s.
int launch_sample_rows(const ep_problem &p, const void *X, int64_t m, int64_t ld_s, const int64_t *rows_dev, void *S,
                       hipStream_t s);
int launch_prep_centroids(const ep_problem &p, const float *C, const KmeansWs &w, hipStream_t s);
int launch_assign_generic(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                          float *min_d2, double *objective, hipStream_t s);
int launch_update_small(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                        float *C_out, int64_t *counts, const KmeansWs &w, const UpdateAcc &acc, hipStream_t s);
int launch_update_sorted(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                         float *C_out, int64_t *counts, const KmeansWs &w, const UpdateAcc &acc, hipStream_t s);
// After an update call that does not finalize: cnt[j] = (accumulate ? cnt[j] : 0) + chunk_cnt[j].
int launch_accumulate_counts(int32_t k, const UpdateAcc &acc, hipStream_t s);
// result[0] = number of labels outside [0, k), result[1] = index of the first one (n if none).
int launch_validate_labels(int64_t n, int32_t k, const int32_t *labels, int64_t *result, hipStream_t s);

// ---- K-Means, k <= 64, d in {64,128}, fp32: fused matrix-core kernels (kmeans_small.hip) --------
constexpr int kSmallMaxBlocks = 512;  // workgroups (= partial sums) per launch; <= kUpdBlocksMax
// Column count the fused small-k kernels are instantiated for (64, 128: k <= 64; 256: k <= 16): d rounded up;
// rows with fewer columns are padded with zeros as they are read.  0: not a shape of these kernels.
inline int small_padded_d(const ep_problem &p) {
    if (p.d < 4 || p.d > 256 || p.d % 4 != 0) return 0;
    const int dpad = p.d <= 64 ? 64 : p.d <= 128 ? 128 : 256;
    return p.k <= (dpad == 256 ? 16 : 64) ? dpad : 0;
}
bool small_path_supported(const ep_problem &p);
int launch_small_assign(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                        float *min_d2, double *objective, hipStream_t s);
int launch_small_update(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                        float *C_out, int64_t *counts, const KmeansWs &w, const UpdateAcc &acc, hipStream_t s);
// fp32, d in {64,128}, k > 64: the same assignment kernel over slices of 64 centroids (k / 64 passes).
bool small_sliced_supported(const ep_problem &p);
int launch_small_assign_sliced(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                               float *min_d2, double *objective, hipStream_t s);
// One fused round: assign against C, sums, then C <- means (in place), *objective <- this
// round's objective.
// first_round: the data-only term of the objective (sum ||x||^2) is computed and kept in the
// workspace; later rounds of the same kmeans_run reuse it.
// ub, lb (both or neither; d = 64 or 128 exactly, not the first round): the round also leaves every point's
// distance bounds against the centroids it was assigned with, which is what the bounded rounds start from.
int launch_small_round(const ep_problem &p, const void *X, float *C, const KmeansWs &w, int32_t *labels,
                       int64_t *counts, double *objective, bool first_round, hipStream_t s,
                       const UpdateAcc &acc = whole_update(), float *ub = nullptr, float *lb = nullptr);
// Second pass over `parts` per-workgroup partials that another kernel left in w.psum / w.pcnt (the bounded
// rounds): C <- means in place, no objective.  With list_len (device), only the first
// list_parts(*list_len, p.n, parts) partials were written and are read.
int launch_small_finalize_parts(const ep_problem &p, int parts, const int64_t *list_len, float *C, int64_t *counts,
                                const KmeansWs &w, const UpdateAcc &acc, hipStream_t s);
// Where the fused rounds keep sum ||x||^2 between the rounds of a run.
double *small_xsq_total(const KmeansWs &w);

// ---- K-Means, k <= 64: rounds with distance bounds and incremental sums (kmeans_bounds.hip) ---------
struct BoundsWs {
    float *ub;               // [n] upper bound on the distance to the own centroid
    float *lb;               // [n] lower bound on the distance to every other centroid
    int32_t *active_idx;     // [n] rows to search this round, ascending
    int32_t *block_counts;   // per-workgroup counts of the bounds pass
    int64_t *n_active;       // [1] rows to search this round
    int64_t *searched;       // [iters] rows searched per round of the run
    float *delta;            // [k] centroid movement of the last update
    unsigned char *top;      // its two largest values, the centroid that moved most, max ||c||^2
    float *C_old;            // [k*d] the centroids the round's assignment used
    int32_t *scrap;          // four words per thread of the search grid: where lanes without a point store
    size_t bytes;
};
bool bounds_path_supported(const ep_problem &p);
BoundsWs carve_bounds_ws(const ep_problem &p, int32_t iters, void *ws);
int bounds_round_parts(const ep_problem &p);
int launch_record_searched(int64_t value, int64_t *slot, hipStream_t s);
int launch_copy_searched(int32_t iters, const BoundsWs &w, int64_t *out, hipStream_t s);
int launch_keep_centroids(const ep_problem &p, const float *C, const BoundsWs &w, hipStream_t s);
// After the means of a round whose assignment used w.C_old: with add_counts the kept counts take the round's
// changes, the round's objective is formed from the kept sums (objective may be null), and with want_drift the
// centroid movements are left for the next round's bounds pass and w.C_old becomes C_new.
int launch_bounds_tail(const ep_problem &p, const float *C_new, const KmeansWs &kw, const BoundsWs &w,
                       bool add_counts, const double *xsq_total, double *objective, bool want_drift, hipStream_t s);
// Applies the last drift to every point's bounds and lists the rows whose bounds no longer separate.
int launch_bounds_pass(const ep_problem &p, const int32_t *labels, const BoundsWs &w, int64_t *searched_slot,
                       hipStream_t s);
// Searches the listed rows, renews their bounds, updates labels in place and leaves per-workgroup partial sums
// of the rows that changed label in kw.psum / kw.pcnt.
int launch_bounds_round(const ep_problem &p, const void *X, const float *C, const KmeansWs &kw, const BoundsWs &w,
                        int32_t *labels, hipStream_t s);

// ---- K-Means, k > 64, bf16, d in {64,128}: bf16 matrix-core assignment (kmeans_large.hip) -------
bool large_path_supported(const ep_problem &p);
size_t large_record_bytes(const ep_problem &p);
// Rounds C to bf16 (w.cq16), leaves -||c||^2/2 in w.cnorm, then labels / min_d2 / objective.
int launch_large_assign(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                        float *min_d2, double *objective, hipStream_t s);
// Benchmark aid (bench_probe.hip): `parts` workgroups write `elems` partials each; mode 0 nothing more, 1 the last
// workgroup to arrive adds them up behind a ticket, 2 a second launch adds them up.
int launch_bench_fold(float *partials, int32_t parts, int32_t elems, int mode, unsigned *ticket, float *out,
                      hipStream_t s);
// Benchmark aid: 512 workgroups x 4 waves x 16 * iters v_mfma_f32_32x32x16_bf16 on 65,536 bytes of operands.
int launch_bench_mfma(const void *operands, int32_t iters, float *sink, hipStream_t s);

// ---- graph kernels (graph.hip) ---------------------------------------------------
constexpr int kSortBlocksMax = 1024;  // workgroups of one radix-sort pass
// Cut count through buckets of destination ranges (graph_bucket.hip): used when the byte labels are far
// beyond the caches.  shift == 0: not used for this graph.
constexpr int kBucketsMax = 512;
constexpr int64_t kBucketMinVertices = 6 * 1024 * 1024;
struct BucketPlan {
    int shift;   // a bucket holds the entries whose column lies in [b << shift, (b + 1) << shift)
    int nb;      // number of buckets, <= kBucketsMax
};
BucketPlan bucket_plan(int64_t n, int64_t nnz, int32_t k);
size_t bucket_record_slots(int64_t nnz, const BucketPlan &pl);

struct GraphWs {
    int64_t *partial;     // [kGraphBlocksMax] per-workgroup partial counts / sums
    int32_t *sort_hist;   // [kSortBlocksMax * 256]
    int32_t *order_tmp;   // [n]
    int32_t *order_tmp2;  // [n]
    uint8_t *label8;      // [n] byte copy of the labels for the cut sweep (k <= 255)
    // bucketed cut count only (carved last, so that the layout before them is the same for every graph call)
    int64_t *bucket_hist;     // [kBucketsMax] entries per bucket
    int64_t *bucket_base;     // [kBucketsMax + 1] bucket starts in bucket_records
    int64_t *bucket_cursor;   // [kBucketsMax * 16] next free slot per bucket, one 128-byte line each
    int64_t *bucket_items;    // [kBucketsMax + 1] work items of the last pass before each bucket
    int64_t *bucket_dropped;  // [1] records that found no room (0 for a well-formed graph)
    uint32_t *bucket_records; // [nnz + padding] one 32-bit record per entry, grouped by bucket
    size_t bytes;
};
constexpr int kGraphBlocksMax = 8192;
// with_buckets: also the buffers of the bucketed cut count, if bucket_plan(n, nnz, k) uses it.
GraphWs carve_graph_ws(int64_t n, int64_t nnz, int32_t k, void *ws, bool with_buckets = false);
int launch_cut_bucketed(int64_t n, int64_t nnz, const BucketPlan &pl, const void *rowptr, bool i64,
                        const int32_t *colidx, const GraphWs &w, unsigned long long *cut, hipStream_t s);
size_t sort_hist_elems();

int launch_partition_quality(int64_t n, int64_t nnz, int32_t k, const void *rowptr, bool i64, const int32_t *colidx,
                             const int32_t *labels, int64_t *cut, int64_t *sizes, const GraphWs &w, hipStream_t s);
// Stable sort of vertex ids by label: order (sorted position -> vertex) and, if non-null, new_id (its inverse).
int launch_sort_by_label(int64_t n, int32_t k, const int32_t *labels, int32_t *new_id, int32_t *order,
                         int32_t *tmp, int32_t *hist, hipStream_t s);
// Stable LSD radix sort of vertex ids by the low 8 * passes bits of keys[v].  enable: nullptr, or a
// device flag read by every kernel of the sort; 0 turns the whole sort into a no-op.
int launch_sort_by_key(int64_t n, int passes, const int32_t *keys, int32_t *new_id, int32_t *order, int32_t *tmp,
                       int32_t *hist, const int *enable, hipStream_t s);
int launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
enum class EdgeReduce { GapSum, BandwidthSum };
int launch_edge_gap(int64_t n, int64_t nnz, const void *rowptr, bool i64, const int32_t *colidx,
                    const int32_t *new_id, uint64_t *out, EdgeReduce what, const GraphWs &w, hipStream_t s);

// ---- balancing (balance.hip) -------------------------------------------------------
struct BalanceWs {
    unsigned char *plan;  // per-round plan (loads, moves, free capacities, threshold degrees)
    uint32_t *degree_hist;   // [k * bins] class members per partition and degree
    int32_t *tie;            // per vertex range and partition: members at the threshold degree
    size_t bytes;
};
BalanceWs carve_balance_ws(int64_t n, void *ws);
// Up to max_rounds migration rounds of one vertex class; k <= 255.
int launch_balance(int64_t n, int32_t k, const void *rowptr, bool i64, const uint8_t *vclass, int32_t class_id,
                   double beta, uint64_t seed, int32_t max_rounds, int32_t *labels, int64_t *stats,
                   const BalanceWs &w, hipStream_t s);

// ---- the graph under new vertex ids (reorder.hip) ----------------------------------------
struct ReorderWs {
    int64_t *block_sums;   // [ceil(n / 2048)] degree sums per workgroup, then their exclusive scan
    int64_t *total;        // [1] sum of the degrees met through `order` (== nnz for a permutation)
    int64_t *window_rows;  // [ceil(nnz / 4096) + 1] first row starting at or after every window boundary
    size_t bytes;
};
ReorderWs carve_reorder_ws(int64_t n, int64_t nnz, void *ws);
// new_rowptr / new_colidx: the CSR with row new_id[v] = neighbours of v under their new ids, ascending.
int launch_reorder(int64_t n, int64_t nnz, const void *rowptr, bool i64, const int32_t *colidx, const int32_t *new_id,
                   const int32_t *order, void *new_rowptr, int32_t *new_colidx, const ReorderWs &w, hipStream_t s);

}  // namespace ep
