// Balancing of a partition: one of the three while-loops of the EmbedPart paper's Alg. 3 with the
// migration policy of Alg. 4 (movers leave overloaded partitions smallest degree first and land in
// underloaded ones in proportion to free capacity), for one vertex class, entirely on the device
// and in integers.
//
// A migration round:
//   1. loads L_i of the class per partition (LDS histogram, integer atomics);
//   2. plan (one thread; k <= 255): capacity C = max(floor(beta |S| / k), ceil(|S| / k)),
//      m_i = L_i - C on the overloaded partitions, the running sum of the free capacities C - L_i
//      of the underloaded ones, their total F;
//   3. key per vertex: (partition << 24) | min(degree, 2^24 - 1) for class members of overloaded
//      partitions, all ones for everyone else;
//   4. stable radix sort of the vertex ids by key (4 passes): inside a partition the members come
//      by ascending degree, equal degrees by ascending id;
//   5. the first m_i vertices of partition i's run move; the destination of vertex v is the
//      partition whose interval of the running sum holds (mix(seed, round, v) mod F).
// The draw is a function of (seed, round, v) only, so the result does not depend on the order in
// which threads get to the vertices.  Rounds whose plan finds nothing overloaded do nothing (every
// kernel after the plan reads its `active` flag and returns): the host enqueues max_rounds rounds
// without ever reading anything back.
#include <algorithm>

#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
constexpr int kPartMax = 255;                 // partition ids fit the top byte of a key, 255 = "stays"
constexpr uint32_t kStay = 0xFFFFFFFFu;
constexpr uint32_t kDegreeMask = 0x00FFFFFFu;

struct BalPlan {
    unsigned long long L[256];    // loads of the class per partition (this round)
    long long m[256];             // vertices to move out (0 unless overloaded)
    long long cumf[256];          // running sum of the free capacities, partitions in index order
    long long seg[257];           // first sorted position of every partition's run
    long long F;                  // total free capacity
    int active;                   // this round moves vertices
    int round;                    // rounds completed before this one (enters the draw)
};

__global__ void bal_reset_kernel(BalPlan *plan, int64_t *stats, int first) {
    const int t = threadIdx.x;
    plan->L[t] = 0;
    if (first && t < 3) stats[t] = 0;
    if (first && t == 0) plan->round = 0;
}

__global__ __launch_bounds__(kBlock) void bal_count_kernel(int64_t n, int32_t k, const uint8_t *__restrict__ vclass,
                                                            int32_t class_id, const int32_t *__restrict__ labels,
                                                            BalPlan *plan) {
    __shared__ unsigned int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x; v < n; v += (int64_t)gridDim.x * kBlock) {
        if (vclass && vclass[v] != class_id) continue;
        const int32_t l = labels[v];
        if (l >= 0 && l < k) atomicAdd(&h[l], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&plan->L[threadIdx.x], (unsigned long long)h[threadIdx.x]);
}

// One thread: k <= 255 partitions.  `allow` is 0 for the closing evaluation after the last round.
__global__ void bal_plan_kernel(int32_t k, double beta, int allow, BalPlan *plan, int64_t *stats) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    long long total = 0;
    for (int i = 0; i < k; ++i) total += (long long)plan->L[i];
    long long cap = (long long)floor(beta * (double)total / (double)k);
    const long long reach = (total + k - 1) / k;
    if (cap < reach) cap = reach;
    long long F = 0, over = 0;
    for (int i = 0; i < k; ++i) {
        const long long L = (long long)plan->L[i];
        if (L < cap) F += cap - L;
        plan->cumf[i] = F;
        plan->m[i] = L > cap ? L - cap : 0;
        if (L > cap) ++over;
    }
    plan->F = F;
    stats[2] = over;
    const int active = allow && over > 0;
    plan->active = active;
    plan->round = (int)stats[0];
    if (active) stats[0] += 1;
}

template <typename RowT>
__global__ __launch_bounds__(kBlock) void bal_keys_kernel(int64_t n, int32_t k, const RowT *__restrict__ rowptr,
                                                           const uint8_t *__restrict__ vclass, int32_t class_id,
                                                           const int32_t *__restrict__ labels,
                                                           const BalPlan *__restrict__ plan,
                                                           int32_t *__restrict__ keys) {
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= n || !plan->active) return;
    uint32_t key = kStay;
    if (!vclass || vclass[v] == class_id) {
        const int32_t l = labels[v];
        if (l >= 0 && l < k && plan->m[l] > 0) {
            const int64_t deg = (int64_t)(rowptr[v + 1] - rowptr[v]);
            key = ((uint32_t)l << 24) | (uint32_t)std::min<int64_t>(deg, (int64_t)kDegreeMask);
        }
    }
    keys[v] = (int32_t)key;
}

// seg[j] = first sorted position whose partition byte is >= j (j = 0 .. 256).
__global__ void bal_segments_kernel(int64_t n, const int32_t *__restrict__ keys, const int32_t *__restrict__ order,
                                    BalPlan *plan) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n || !plan->active) return;
    const int prev = i == 0 ? -1 : (int)((uint32_t)keys[order[i - 1]] >> 24);
    const int cur = i == n ? 256 : (int)((uint32_t)keys[order[i]] >> 24);
    for (int j = prev + 1; j <= cur; ++j) plan->seg[j] = i;
}

__device__ __forceinline__ uint64_t draw64(uint64_t seed, uint32_t round, int64_t v) {
    uint64_t z = seed + (((uint64_t)round << 32) + (uint64_t)v + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(kBlock) void bal_move_kernel(int64_t n, int32_t k, uint64_t seed,
                                                           const int32_t *__restrict__ keys,
                                                           const int32_t *__restrict__ order,
                                                           const BalPlan *__restrict__ plan, int32_t *__restrict__ labels,
                                                           int64_t *__restrict__ stats) {
    if (!plan->active) return;   // uniform over the grid
    __shared__ long long cumf[256];
    cumf[threadIdx.x] = (int)threadIdx.x < k ? plan->cumf[threadIdx.x] : plan->F;
    __syncthreads();
    const int64_t pos = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int moved = 0;
    if (pos < n) {
        const int32_t v = order[pos];
        const uint32_t part = (uint32_t)keys[v] >> 24;
        if (part < (uint32_t)k && pos - plan->seg[part] < plan->m[part]) {
            const uint64_t r = draw64(seed, (uint32_t)plan->round, v) % (uint64_t)plan->F;
            int lo = 0, hi = k - 1;               // first partition whose running sum exceeds r
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if ((uint64_t)cumf[mid] > r) hi = mid; else lo = mid + 1;
            }
            labels[v] = lo;
            moved = 1;
        }
    }
    const unsigned long long b = __ballot(moved);
    if ((threadIdx.x & 63) == 0 && b) atomicAdd(reinterpret_cast<unsigned long long *>(stats + 1), (unsigned long long)__popcll(b));
}

}  // namespace

BalanceWs carve_balance_ws(int64_t n, void *ws) {
    Carver c(ws);
    BalanceWs w{};
    w.plan = c.take<unsigned char>(sizeof(BalPlan));
    w.keys = c.take<int32_t>((size_t)n);
    w.order = c.take<int32_t>((size_t)n);
    w.tmp = c.take<int32_t>((size_t)n);
    w.sort_hist = c.take<int32_t>(sort_hist_elems());
    w.bytes = align_up(c.used, 256);
    return w;
}

int launch_balance(int64_t n, int32_t k, const void *rowptr, bool i64, const uint8_t *vclass, int32_t class_id,
                   double beta, uint64_t seed, int32_t max_rounds, int32_t *labels, int64_t *stats,
                   const BalanceWs &w, hipStream_t s) {
    if (k > kPartMax) return EP_EUNSUPPORTED;
    BalPlan *plan = reinterpret_cast<BalPlan *>(w.plan);
    const unsigned per_vertex = (unsigned)ceil_div(n, kBlock);
    const unsigned count_blocks = (unsigned)std::min<int64_t>(2048, ceil_div(n, kBlock * 8));
    for (int32_t r = 0; r <= max_rounds; ++r) {
        bal_reset_kernel<<<1, 256, 0, s>>>(plan, stats, r == 0);
        EP_LAUNCH_CHECK();
        bal_count_kernel<<<count_blocks, kBlock, 0, s>>>(n, k, vclass, class_id, labels, plan);
        EP_LAUNCH_CHECK();
        bal_plan_kernel<<<1, 64, 0, s>>>(k, beta, r < max_rounds, plan, stats);
        EP_LAUNCH_CHECK();
        if (r == max_rounds) break;   // the closing evaluation only reports what is still overloaded
        if (i64)
            bal_keys_kernel<int64_t><<<per_vertex, kBlock, 0, s>>>(n, k, static_cast<const int64_t *>(rowptr), vclass,
                                                                   class_id, labels, plan, w.keys);
        else
            bal_keys_kernel<int32_t><<<per_vertex, kBlock, 0, s>>>(n, k, static_cast<const int32_t *>(rowptr), vclass,
                                                                   class_id, labels, plan, w.keys);
        EP_LAUNCH_CHECK();
        int rc = launch_sort_by_key(n, 4, w.keys, nullptr, w.order, w.tmp, w.sort_hist, &plan->active, s);
        if (rc != EP_OK) return rc;
        bal_segments_kernel<<<(unsigned)ceil_div(n + 1, kBlock), kBlock, 0, s>>>(n, w.keys, w.order, plan);
        EP_LAUNCH_CHECK();
        bal_move_kernel<<<per_vertex, kBlock, 0, s>>>(n, k, seed, w.keys, w.order, plan, labels, stats);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

}  // namespace ep
