// C-ABI entry points of libembedpart: argument checks on the host, then kernel launches.
// See include/embedpart.h for the contract of every call.
#include <algorithm>
#include <atomic>
#include <mutex>

#include "kernels.h"

namespace ep {

static std::atomic<int> g_last_hip_error{0};
void note_hip_error(hipError_t e) { g_last_hip_error.store((int)e); }

static void **g_prof_events = nullptr;
static int g_prof_capacity = 0, g_prof_class = 0, g_prof_count = 0;

ProfScope::ProfScope(int kernel_class, hipStream_t s, bool kernel_events)
    : start_(nullptr), stop_(nullptr), s_(s), kernel_events_(kernel_events) {
    if (!g_prof_events || kernel_class != g_prof_class) return;
    const int i = g_prof_count++;
    if (2 * i + 1 >= g_prof_capacity) return;
    start_ = static_cast<hipEvent_t>(g_prof_events[2 * i]);
    stop_ = static_cast<hipEvent_t>(g_prof_events[2 * i + 1]);
    if (!kernel_events_) (void)hipEventRecord(start_, s);
}
ProfScope::~ProfScope() {
    if (stop_ && !kernel_events_) (void)hipEventRecord(stop_, s_);
}

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_problem(const ep_problem *p) {
    if (!p) return EP_EINVAL;
    if (p->n < 1 || p->n >= EP_MAX_N || p->d < 1 || p->k < 1 || (int64_t)p->k > p->n || p->ld < p->d) return EP_EINVAL;
    if (p->reserved != 0) return EP_EINVAL;
    if (p->dtype != EP_F32 && p->dtype != EP_BF16 && p->dtype != EP_F16) return EP_EUNSUPPORTED;
    if (p->d > EP_MAX_D || p->k > EP_MAX_K) return EP_EUNSUPPORTED;
    if (p->ld % (p->dtype == EP_F32 ? 4 : 8) != 0) return EP_EINVAL;
    return EP_OK;
}

// The same for a call that works on a row range of a larger matrix (kmeans_assign, kmeans_update): a
// chunk may hold fewer rows than there are clusters.
int check_problem_rows(const ep_problem *p) {
    if (!p) return EP_EINVAL;
    ep_problem q = *p;
    if (q.n >= 1 && (int64_t)q.k > q.n && q.k <= EP_MAX_K) q.n = q.k;   // k > n is not an error here
    return check_problem(&q);
}

int check_x(const ep_problem *p, const void *X) {
    if (!X || !aligned(X, 16)) return EP_EINVAL;
    (void)p;
    return EP_OK;
}

int check_ws(const void *ws, size_t have, size_t need) {
    if (!ws || !aligned(ws, 256) || have < need) return EP_EWORKSPACE;
    return EP_OK;
}

uint64_t splitmix64(uint64_t &state) {
    uint64_t z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int do_assign(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
              float *min_d2, double *objective, hipStream_t s) {
    if (small_path_supported(p)) return launch_small_assign(p, X, C, w, labels, min_d2, objective, s);
    if (small_sliced_supported(p)) return launch_small_assign_sliced(p, X, C, w, labels, min_d2, objective, s);
    if (large_path_supported(p)) return launch_large_assign(p, X, C, w, labels, min_d2, objective, s);
    int rc = launch_prep_centroids(p, C, w, s);
    if (rc != EP_OK) return rc;
    return launch_assign_generic(p, X, C, w, labels, min_d2, objective, s);
}

int do_update(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev, float *C_out,
              int64_t *counts, const KmeansWs &w, int flags, hipStream_t s) {
    const UpdateAcc acc{w.acc_sum, w.acc_cnt, w.chunk_cnt, flags};
    int rc = small_path_supported(p)    ? launch_small_update(p, X, labels, C_prev, C_out, counts, w, acc, s)
             : update_by_sorted_rows(p) ? launch_update_sorted(p, X, labels, C_prev, C_out, counts, w, acc, s)
                                        : launch_update_small(p, X, labels, C_prev, C_out, counts, w, acc, s);
    if (rc != EP_OK || (flags & EP_UPDATE_FINALIZE)) return rc;
    return launch_accumulate_counts(p.k, acc, s);   // the running counts take this chunk's
}

int check_graph(int64_t n, int64_t nnz, const void *rowptr, const int32_t *colidx) {
    if (n < 1 || n >= EP_MAX_N || nnz < 0 || !rowptr || (nnz > 0 && !colidx)) return EP_EINVAL;
    if (!aligned(rowptr, 8) || !aligned(colidx, 16)) return EP_EINVAL;
    return EP_OK;
}

// Full rounds before the first bounded one: while the centroids still move far, no bound survives a round.
// The last of them also takes the first bounds.
constexpr int32_t kBoundsWarmRounds = 3;

bool bounds_in_use(const ep_problem &p, int32_t iters, int flags) {
    return (flags & EP_RUN_BOUNDS) && bounds_path_supported(p) && iters > kBoundsWarmRounds;
}

// Layout of a kmeans_run workspace: the K-Means workspace, then (EP_RUN_BOUNDS) the bounds and the lists.
size_t run_ws_bytes(const ep_problem &p, int32_t iters, int flags) {
    size_t bytes = align_up(carve_kmeans_ws(p, nullptr).bytes, 256);
    if ((flags & EP_RUN_BOUNDS) && bounds_path_supported(p)) bytes += carve_bounds_ws(p, iters, nullptr).bytes;
    return bytes;
}
BoundsWs bounds_ws_of(const ep_problem &p, int32_t iters, void *ws) {
    return carve_bounds_ws(p, iters, static_cast<char *>(ws) + align_up(carve_kmeans_ws(p, nullptr).bytes, 256));
}

// `iters` rounds with EP_RUN_BOUNDS: kBoundsWarmRounds full rounds, the last of which keeps its sums in fp64
// and leaves every point's bounds, then rounds that search only what the bounds let through.
int run_rounds_bounded(const ep_problem &p, const void *X, int32_t iters, float *C, int32_t *labels, int64_t *counts,
                       double *objective_hist, const KmeansWs &w, const BoundsWs &b, hipStream_t s) {
    int rc = EP_OK;
    const UpdateAcc keep{w.acc_sum, w.acc_cnt, w.chunk_cnt, EP_UPDATE_FINALIZE | kUpdateKeep};
    const UpdateAcc add{w.acc_sum, w.acc_cnt, w.chunk_cnt, EP_UPDATE_ACCUMULATE | EP_UPDATE_FINALIZE | kUpdateKeep};
    for (int32_t t = 0; t < kBoundsWarmRounds; ++t) {
        const bool last_full = t == kBoundsWarmRounds - 1;
        double *obj = objective_hist ? objective_hist + t : nullptr;   // round 1 also forms sum ||x||^2, kept for later
        if (last_full && (rc = launch_keep_centroids(p, C, b, s)) != EP_OK) return rc;   // what the bounds refer to
        if ((rc = launch_small_round(p, X, C, w, labels, counts, obj, t == 0, s, last_full ? keep : whole_update(),
                                     last_full ? b.ub : nullptr, last_full ? b.lb : nullptr)) != EP_OK)
            return rc;
        if (last_full) {   // the kept counts are this round's; then the centroids' movement for the first bounds pass
            if ((rc = launch_accumulate_counts(p.k, keep, s)) != EP_OK) return rc;
            if ((rc = launch_bounds_tail(p, C, w, b, false, nullptr, nullptr, true, s)) != EP_OK) return rc;
        }
        if ((rc = launch_record_searched(p.n, b.searched + t, s)) != EP_OK) return rc;
    }
    for (int32_t t = kBoundsWarmRounds; t < iters; ++t) {
        if ((rc = launch_bounds_pass(p, labels, b, b.searched + t, s)) != EP_OK) return rc;
        if ((rc = launch_bounds_round(p, X, C, w, b, labels, s)) != EP_OK) return rc;
        if ((rc = launch_small_finalize_parts(p, bounds_round_parts(p), b.n_active, C, counts, w, add, s)) != EP_OK)
            return rc;
        if ((rc = launch_bounds_tail(p, C, w, b, true, small_xsq_total(w), objective_hist ? objective_hist + t : nullptr,
                                     t + 1 < iters, s)) != EP_OK)
            return rc;
    }
    return EP_OK;
}

// `iters` Lloyd rounds from the centroids in C (see kmeans_run in the header).
int run_rounds(const ep_problem &p, const void *X, int32_t iters, float *C, int32_t *labels, int64_t *counts,
               double *objective_hist, int flags, const KmeansWs &w, hipStream_t s, void *ws_base = nullptr) {
    int rc = EP_OK;
    if (ws_base && bounds_in_use(p, iters, flags)) {
        rc = run_rounds_bounded(p, X, iters, C, labels, counts, objective_hist, w, bounds_ws_of(p, iters, ws_base), s);
        if (rc == EP_OK && (flags & EP_RUN_FINAL_REASSIGN))
            rc = do_assign(p, X, C, w, labels, nullptr, objective_hist ? objective_hist + iters : nullptr, s);
        return rc;
    }
    if (small_path_supported(p)) {  // fused rounds: X is read once per round
        for (int32_t t = 0; t < iters; ++t)
            if ((rc = launch_small_round(p, X, C, w, labels, counts, objective_hist ? objective_hist + t : nullptr,
                                         t == 0, s)) != EP_OK)
                return rc;
        if (flags & EP_RUN_FINAL_REASSIGN)
            rc = do_assign(p, X, C, w, labels, nullptr, objective_hist ? objective_hist + iters : nullptr, s);
        return rc;
    }
    for (int32_t t = 0; t < iters; ++t) {
        if ((rc = do_assign(p, X, C, w, labels, nullptr, objective_hist ? objective_hist + t : nullptr, s)) != EP_OK)
            return rc;
        if ((rc = do_update(p, X, labels, C, C, counts, w, EP_UPDATE_FINALIZE, s)) != EP_OK) return rc;
    }
    if (flags & EP_RUN_FINAL_REASSIGN)
        rc = do_assign(p, X, C, w, labels, nullptr, objective_hist ? objective_hist + iters : nullptr, s);
    return rc;
}

// Workspace of kmeans_run_sampled: the dense sample, its row indices, its labels, and one K-Means
// workspace sized for the full problem (used for the sample's rounds, then for the full assignment).
struct SampledWs {
    void *S;
    int64_t *rows;
    int32_t *labels;
    void *km;
    int64_t ld_s;
    size_t bytes;
};
SampledWs carve_sampled_ws(const ep_problem &p, int64_t m, void *ws) {
    Carver c(ws);
    SampledWs w{};
    const int64_t unit = 16 / elem_bytes(p.dtype);   // rows stay 16-byte aligned
    w.ld_s = (p.d + unit - 1) / unit * unit;
    w.S = c.take<unsigned char>((size_t)m * (size_t)w.ld_s * (size_t)elem_bytes(p.dtype));
    w.rows = c.take<int64_t>((size_t)m);
    w.labels = c.take<int32_t>((size_t)m);
    // one K-Means workspace serves the sample's rounds (m dense rows of stride ld_s) and then the
    // assignment of all n rows: the two shapes can take different kernels, so it is sized for both
    ep_problem ps = p;
    ps.n = m;
    ps.ld = w.ld_s;
    w.km = c.take<unsigned char>(std::max(carve_kmeans_ws(p, nullptr).bytes, carve_kmeans_ws(ps, nullptr).bytes));
    w.bytes = align_up(c.used, 256);
    return w;
}

// ---- kmeans_run_noalloc: the K-Means workspace as a static device array ---------------------------
// Every GPU the library runs on holds its own copy of this array at its own address.  The array's
// name is only a host-side handle: host code never passes it anywhere but to hipGetSymbolAddress,
// and uses the per-device address that call returns (g_scratch_ptr) for kernel arguments.
static __device__ __align__(256) unsigned char scratch[EP_NOALLOC_SCRATCH_BYTES];
constexpr int kScratchMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kScratchMaxDevices] = {};

// Address of `scratch` on the current device (looked up once per device, with that device current).
int scratch_of_current_device(void **out) {
    int dev = -1;
    EP_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kScratchMaxDevices) return EP_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        EP_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return EP_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return EP_OK;
}

}  // namespace
}  // namespace ep

using namespace ep;

extern "C" {

int ep_version(void) { return 100; }

const char *ep_strerror(int code) {
    switch (code) {
        case EP_OK: return "ok";
        case EP_EINVAL: return "invalid argument (null pointer, size out of range, k > n, ld < d or misaligned buffer)";
        case EP_EUNSUPPORTED: return "shape or dtype not supported by this build";
        case EP_EWORKSPACE: return "workspace missing, misaligned or too small";
        case EP_EHIP: return "a HIP runtime call failed (see ep_last_hip_error)";
        default: return "unknown error code";
    }
}

int ep_last_hip_error(void) { return g_last_hip_error.load(); }

int ep_profile_arm(void **events_host, int capacity, int kernel_class) {
    if (events_host && (capacity < 2 || kernel_class < EP_PROF_LLOYD_MAIN || kernel_class > EP_PROF_EDGE_SWEEP))
        return EP_EINVAL;
    g_prof_events = events_host;
    g_prof_capacity = events_host ? capacity : 0;
    g_prof_class = events_host ? kernel_class : 0;
    g_prof_count = 0;
    return EP_OK;
}

int ep_profile_count(void) { return g_prof_count; }

int ep_bench_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || bytes % 16 != 0 || !aligned(dst, 16) || !aligned(src, 16)) return EP_EINVAL;
    return launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream));
}

int ep_bench_fold(float *partials, int32_t parts, int32_t elems, int mode, uint32_t *ticket, float *out, void *stream) {
    if (!partials || !ticket || !out || !aligned(partials, 4) || !aligned(ticket, 4) || !aligned(out, 4)) return EP_EINVAL;
    if (parts < 1 || parts > 2048 || elems < 8 || elems > 8192 || elems % 8 != 0 || mode < 0 || mode > 2) return EP_EINVAL;
    return launch_bench_fold(partials, parts, elems, mode, ticket, out, static_cast<hipStream_t>(stream));
}

int ep_bench_mfma_bf16(const void *operands, int32_t iters, float *sink, void *stream) {
    if (!operands || !sink || !aligned(operands, 16) || !aligned(sink, 4) || iters < 1 || iters > (1 << 22))
        return EP_EINVAL;
    return launch_bench_mfma(operands, iters, sink, static_cast<hipStream_t>(stream));
}

int kmeans_init_indices(uint64_t seed, int64_t n, int32_t k, int64_t *idx_host) {
    if (!idx_host || n < 1 || k < 1 || (int64_t)k > n) return EP_EINVAL;
    uint64_t state = seed;
    int32_t have = 0;
    while (have < k) {
        const int64_t r = (int64_t)(splitmix64(state) % (uint64_t)n);
        bool seen = false;
        for (int32_t j = 0; j < have && !seen; ++j) seen = idx_host[j] == r;
        if (!seen) idx_host[have++] = r;
    }
    return EP_OK;
}

int kmeans_workspace_bytes(const ep_problem *p, size_t *bytes_host) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if (!bytes_host) return EP_EINVAL;
    *bytes_host = carve_kmeans_ws(*p, nullptr).bytes;
    return EP_OK;
}

int kmeans_init(const ep_problem *p, const void *X, const int64_t *idx_host, float *C, void *ws, size_t ws_bytes,
                void *stream) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if ((rc = check_x(p, X)) != EP_OK) return rc;
    if (!idx_host || !C) return EP_EINVAL;
    for (int32_t j = 0; j < p->k; ++j)
        if (idx_host[j] < 0 || idx_host[j] >= p->n) return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, carve_kmeans_ws(*p, nullptr).bytes)) != EP_OK) return rc;
    const KmeansWs w = carve_kmeans_ws(*p, ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    EP_HIP_TRY(hipMemcpyAsync(w.idx, idx_host, sizeof(int64_t) * p->k, hipMemcpyHostToDevice, s));
    return launch_gather_rows(*p, X, w.idx, C, s);
}

int kmeans_assign(const ep_problem *p, const void *X, const float *C, int32_t *labels, float *min_d2,
                  double *objective, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_problem_rows(p);
    if (rc != EP_OK) return rc;
    if ((rc = check_x(p, X)) != EP_OK) return rc;
    if (!C || !labels || !aligned(labels, 16)) return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, carve_kmeans_ws(*p, nullptr).bytes)) != EP_OK) return rc;
    return do_assign(*p, X, C, carve_kmeans_ws(*p, ws), labels, min_d2, objective, static_cast<hipStream_t>(stream));
}

int kmeans_update(const ep_problem *p, const void *X, const int32_t *labels, const float *C_prev, float *C_out,
                  int64_t *counts, int flags, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_problem_rows(p);
    if (rc != EP_OK) return rc;
    if ((rc = check_x(p, X)) != EP_OK) return rc;
    if (!labels || (flags & ~(EP_UPDATE_ACCUMULATE | EP_UPDATE_FINALIZE))) return EP_EINVAL;
    if ((flags & EP_UPDATE_FINALIZE) && (!C_prev || !C_out || !counts)) return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, carve_kmeans_ws(*p, nullptr).bytes)) != EP_OK) return rc;
    return do_update(*p, X, labels, C_prev, C_out, counts, carve_kmeans_ws(*p, ws), flags,
                     static_cast<hipStream_t>(stream));
}

int ep_validate_labels(int64_t n, int32_t k, const int32_t *labels, int64_t *result, void *stream) {
    if (n < 1 || n >= EP_MAX_N || k < 1 || !labels || !result || !aligned(result, 8)) return EP_EINVAL;
    return launch_validate_labels(n, k, labels, result, static_cast<hipStream_t>(stream));
}

int kmeans_run_workspace_bytes(const ep_problem *p, int32_t iters, int flags, size_t *bytes_host) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if (!bytes_host || iters < 0 || (flags & ~(EP_RUN_FINAL_REASSIGN | EP_RUN_BOUNDS))) return EP_EINVAL;
    *bytes_host = run_ws_bytes(*p, iters, flags);
    return EP_OK;
}

int kmeans_run(const ep_problem *p, const void *X, int32_t iters, float *C, int32_t *labels, int64_t *counts,
               double *objective_hist, int flags, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if ((rc = check_x(p, X)) != EP_OK) return rc;
    if (!C || !labels || !aligned(labels, 16) || !counts || iters < 0 ||
        (flags & ~(EP_RUN_FINAL_REASSIGN | EP_RUN_BOUNDS)))
        return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, run_ws_bytes(*p, iters, flags))) != EP_OK) return rc;
    const KmeansWs w = carve_kmeans_ws(*p, ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    return run_rounds(*p, X, iters, C, labels, counts, objective_hist, flags, w, s, ws);
}

int kmeans_run_searched(const ep_problem *p, int32_t iters, int flags, const void *ws, size_t ws_bytes,
                        int64_t *searched, void *stream) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if (!searched || !aligned(searched, 8) || iters < 1 || !(flags & EP_RUN_BOUNDS) ||
        (flags & ~(EP_RUN_FINAL_REASSIGN | EP_RUN_BOUNDS)))
        return EP_EINVAL;
    if (!bounds_in_use(*p, iters, flags)) return EP_EUNSUPPORTED;
    if ((rc = check_ws(ws, ws_bytes, run_ws_bytes(*p, iters, flags))) != EP_OK) return rc;
    return launch_copy_searched(iters, bounds_ws_of(*p, iters, const_cast<void *>(ws)), searched,
                                static_cast<hipStream_t>(stream));
}

int kmeans_run_noalloc(const ep_problem *p, const void *X, int32_t iters, float *C, int32_t *labels, int64_t *counts,
                       double *objective_hist, int flags, void *stream) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if ((rc = check_x(p, X)) != EP_OK) return rc;
    if (!C || !labels || !aligned(labels, 16) || !counts || iters < 0 || (flags & ~EP_RUN_FINAL_REASSIGN))
        return EP_EINVAL;
    // the problem must fit the static array: nothing is allocated to make room
    if (carve_kmeans_ws(*p, nullptr).bytes > (size_t)EP_NOALLOC_SCRATCH_BYTES) return EP_EWORKSPACE;
    void *ws = nullptr;
    if ((rc = scratch_of_current_device(&ws)) != EP_OK) return rc;
    // no part of the workspace has to start at zero: every kernel of a round writes what the next reads
    return run_rounds(*p, X, iters, C, labels, counts, objective_hist, flags, carve_kmeans_ws(*p, ws),
                      static_cast<hipStream_t>(stream));
}

int kmeans_sampled_workspace_bytes(const ep_problem *p, int64_t m, size_t *bytes_host) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if (!bytes_host || m < p->k || m > p->n) return EP_EINVAL;
    *bytes_host = carve_sampled_ws(*p, m, nullptr).bytes;
    return EP_OK;
}

int kmeans_run_sampled(const ep_problem *p, const void *X, int64_t m, const int64_t *sample_rows_host, int32_t iters,
                       float *C, int32_t *labels, int64_t *counts, double *objective_hist, void *ws,
                       size_t ws_bytes, void *stream) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if ((rc = check_x(p, X)) != EP_OK) return rc;
    if (!sample_rows_host || m < p->k || m > p->n || !C || !labels || !aligned(labels, 16) || !counts || iters < 0)
        return EP_EINVAL;
    for (int64_t i = 0; i < m; ++i)
        if (sample_rows_host[i] < 0 || sample_rows_host[i] >= p->n) return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, carve_sampled_ws(*p, m, nullptr).bytes)) != EP_OK) return rc;
    const SampledWs sw = carve_sampled_ws(*p, m, ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ep_problem ps = *p;   // the sample as a problem of its own: m dense rows
    ps.n = m;
    ps.ld = sw.ld_s;
    EP_HIP_TRY(hipMemcpyAsync(sw.rows, sample_rows_host, sizeof(int64_t) * (size_t)m, hipMemcpyHostToDevice, s));
    if ((rc = launch_sample_rows(*p, X, m, sw.ld_s, sw.rows, sw.S, s)) != EP_OK) return rc;
    // initial centroids: the first k rows of the sample (= rows sample_rows[0..k) of X)
    if ((rc = launch_gather_rows(*p, X, sw.rows, C, s)) != EP_OK) return rc;
    if ((rc = run_rounds(ps, sw.S, iters, C, sw.labels, counts, objective_hist, 0, carve_kmeans_ws(ps, sw.km), s)) !=
        EP_OK)
        return rc;
    return do_assign(*p, X, C, carve_kmeans_ws(*p, sw.km), labels, nullptr,
                     objective_hist ? objective_hist + iters : nullptr, s);
}

int graph_workspace_bytes(int64_t n, int64_t nnz, int32_t k, size_t *bytes_host) {
    if (n < 1 || n >= EP_MAX_N || nnz < 0 || k < 1 || !bytes_host) return EP_EINVAL;
    if (k > EP_MAX_K) return EP_EUNSUPPORTED;
    *bytes_host = carve_graph_ws(n, nnz, k, nullptr, true).bytes;
    return EP_OK;
}

int partition_quality(int64_t n, int64_t nnz, int32_t k, const void *rowptr, int rowptr_is_i64, const int32_t *colidx,
                      const int32_t *labels, int64_t *cut, int64_t *sizes, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_graph(n, nnz, rowptr, colidx);
    if (rc != EP_OK) return rc;
    if (k < 1 || !labels || !cut || !sizes) return EP_EINVAL;
    if (k > EP_MAX_K) return EP_EUNSUPPORTED;
    if ((rc = check_ws(ws, ws_bytes, carve_graph_ws(n, nnz, k, nullptr, true).bytes)) != EP_OK) return rc;
    return launch_partition_quality(n, nnz, k, rowptr, rowptr_is_i64 != 0, colidx, labels, cut, sizes,
                                    carve_graph_ws(n, nnz, k, ws, true), static_cast<hipStream_t>(stream));
}

int partition_permutation(int64_t n, int32_t k, const int32_t *labels, int32_t *new_id, int32_t *order, void *ws,
                          size_t ws_bytes, void *stream) {
    if (n < 1 || n >= EP_MAX_N || k < 1 || !labels || !new_id || !order) return EP_EINVAL;
    if (k > EP_MAX_K) return EP_EUNSUPPORTED;
    int rc = check_ws(ws, ws_bytes, carve_graph_ws(n, 0, k, nullptr).bytes);
    if (rc != EP_OK) return rc;
    const GraphWs w = carve_graph_ws(n, 0, k, ws);
    return launch_sort_by_label(n, k, labels, new_id, order, w.order_tmp, w.sort_hist,
                                static_cast<hipStream_t>(stream));
}

int balance_workspace_bytes(int64_t n, size_t *bytes_host) {
    if (n < 1 || n >= EP_MAX_N || !bytes_host) return EP_EINVAL;
    *bytes_host = carve_balance_ws(n, nullptr).bytes;
    return EP_OK;
}

int partition_balance(int64_t n, int32_t k, const void *rowptr, int rowptr_is_i64, const uint8_t *vclass,
                      int32_t class_id, double beta, uint64_t seed, int32_t max_rounds, int32_t *labels,
                      int64_t *stats, void *ws, size_t ws_bytes, void *stream) {
    if (n < 1 || n >= EP_MAX_N || k < 1 || !rowptr || !aligned(rowptr, 8) || !labels || !stats || !aligned(stats, 8))
        return EP_EINVAL;
    if (!(beta >= 1.0) || !(beta < 1.0e6) || max_rounds < 0 || max_rounds > EP_BALANCE_MAX_ROUNDS || class_id < 0 ||
        class_id > 255)
        return EP_EINVAL;
    if (k > EP_BALANCE_MAX_K) return EP_EUNSUPPORTED;
    int rc = check_ws(ws, ws_bytes, carve_balance_ws(n, nullptr).bytes);
    if (rc != EP_OK) return rc;
    return launch_balance(n, k, rowptr, rowptr_is_i64 != 0, vclass, class_id, beta, seed, max_rounds, labels, stats,
                          carve_balance_ws(n, ws), static_cast<hipStream_t>(stream));
}

static int gap_call(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64, const int32_t *colidx,
                    const int32_t *new_id, uint64_t *out, EdgeReduce what, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_graph(n, nnz, rowptr, colidx);
    if (rc != EP_OK) return rc;
    if (!out) return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, carve_graph_ws(n, nnz, 1, nullptr).bytes)) != EP_OK) return rc;
    return launch_edge_gap(n, nnz, rowptr, rowptr_is_i64 != 0, colidx, new_id, out, what,
                           carve_graph_ws(n, nnz, 1, ws), static_cast<hipStream_t>(stream));
}

int edge_gap_sum(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64, const int32_t *colidx,
                 const int32_t *new_id, uint64_t *gap_sum, void *ws, size_t ws_bytes, void *stream) {
    return gap_call(n, nnz, rowptr, rowptr_is_i64, colidx, new_id, gap_sum, EdgeReduce::GapSum, ws, ws_bytes, stream);
}

int vertex_bandwidth_sum(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64, const int32_t *colidx,
                         const int32_t *new_id, uint64_t *bw_sum, void *ws, size_t ws_bytes, void *stream) {
    return gap_call(n, nnz, rowptr, rowptr_is_i64, colidx, new_id, bw_sum, EdgeReduce::BandwidthSum, ws, ws_bytes,
                    stream);
}

int graph_reorder_workspace_bytes(int64_t n, int64_t nnz, size_t *bytes_host) {
    if (n < 1 || n >= EP_MAX_N || nnz < 0 || !bytes_host) return EP_EINVAL;
    *bytes_host = carve_reorder_ws(n, nnz, nullptr).bytes;
    return EP_OK;
}

int graph_reorder(int64_t n, int64_t nnz, const void *rowptr, int rowptr_is_i64, const int32_t *colidx,
                  const int32_t *new_id, const int32_t *order, void *new_rowptr, int32_t *new_colidx, void *ws,
                  size_t ws_bytes, void *stream) {
    int rc = check_graph(n, nnz, rowptr, colidx);
    if (rc != EP_OK) return rc;
    if (!new_id || !order || !new_rowptr || !aligned(new_rowptr, 8) || (nnz > 0 && !new_colidx)) return EP_EINVAL;
    if (!rowptr_is_i64 && nnz >= ((int64_t)1 << 31)) return EP_EINVAL;
    if (new_rowptr == rowptr || (nnz > 0 && new_colidx == colidx)) return EP_EINVAL;
    if ((rc = check_ws(ws, ws_bytes, carve_reorder_ws(n, nnz, nullptr).bytes)) != EP_OK) return rc;
    return launch_reorder(n, nnz, rowptr, rowptr_is_i64 != 0, colidx, new_id, order, new_rowptr, new_colidx,
                          carve_reorder_ws(n, nnz, ws), static_cast<hipStream_t>(stream));
}

static size_t phase2_kmeans_bytes(const ep_problem &p, int64_t m) {
    return align_up(m > 0 ? carve_sampled_ws(p, m, nullptr).bytes : carve_kmeans_ws(p, nullptr).bytes, 256);
}

int cluster_and_balance_workspace_bytes(const ep_problem *p, int64_t sample_rows, size_t *bytes_host) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if (!bytes_host || sample_rows < 0 || (sample_rows > 0 && (sample_rows < p->k || sample_rows > p->n)))
        return EP_EINVAL;
    *bytes_host = phase2_kmeans_bytes(*p, sample_rows) + carve_balance_ws(p->n, nullptr).bytes;
    return EP_OK;
}

int cluster_and_balance(const ep_problem *p, const void *X, const void *rowptr, int rowptr_is_i64,
                        const uint8_t *vclass, const ep_phase2 *opt, const int64_t *rows_host, float *C,
                        int32_t *labels, int64_t *counts, int64_t *stats, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_problem(p);
    if (rc != EP_OK) return rc;
    if (!opt || !stats || !aligned(stats, 8) || opt->sample_rows < 0) return EP_EINVAL;
    if (p->k > EP_BALANCE_MAX_K) return EP_EUNSUPPORTED;
    const int64_t m = opt->sample_rows;
    if (m > 0 && (m < p->k || m > p->n)) return EP_EINVAL;
    const size_t km_bytes = phase2_kmeans_bytes(*p, m), bal_bytes = carve_balance_ws(p->n, nullptr).bytes;
    if ((rc = check_ws(ws, ws_bytes, km_bytes + bal_bytes)) != EP_OK) return rc;
    void *bal_ws = static_cast<char *>(ws) + km_bytes;
    // every argument is validated by the calls themselves before anything is enqueued; the balancing
    // arguments are checked first so that a bad one does not leave a finished clustering behind
    for (int c = 0; c < 3; ++c)
        if (!(opt->beta[c] >= 1.0) || !(opt->beta[c] < 1.0e6)) return EP_EINVAL;
    if (opt->max_rounds < 0 || opt->max_rounds > EP_BALANCE_MAX_ROUNDS || !rowptr || !aligned(rowptr, 8))
        return EP_EINVAL;
    if (m > 0) {
        rc = kmeans_run_sampled(p, X, m, rows_host, opt->iters, C, labels, counts, nullptr, ws, km_bytes, stream);
    } else {
        if ((rc = kmeans_init(p, X, rows_host, C, ws, km_bytes, stream)) != EP_OK) return rc;
        rc = kmeans_run(p, X, opt->iters, C, labels, counts, nullptr, 0, ws, km_bytes, stream);
    }
    if (rc != EP_OK) return rc;
    for (int c = vclass ? 0 : 2; c < 3; ++c) {
        rc = partition_balance(p->n, p->k, rowptr, rowptr_is_i64, vclass, c, opt->beta[c], opt->seed + (uint64_t)c,
                               opt->max_rounds, labels, stats + 3 * c, bal_ws, bal_bytes, stream);
        if (rc != EP_OK) return rc;
    }
    return EP_OK;
}

}  // extern "C"
