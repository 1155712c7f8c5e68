// Balancing of a partition: one of the three while-loops of the EmbedPart paper's Alg. 3 with the
// migration policy of Alg. 4 (movers leave overloaded partitions smallest degree first and land in
// underloaded ones in proportion to free capacity), for one vertex class, entirely on the device
// and in integers.
//
// A migration round:
//   1. per partition, the number of class members of every degree 0 .. B-2 and of degree >= B-1 (LDS
//      histogram, integer atomics); the loads L_i are the row sums;
//   2. plan (one workgroup; k <= 255): capacity C = max(floor(beta |S| / k), ceil(|S| / k)),
//      m_i = L_i - C on the overloaded partitions, the running sum of the free capacities C - L_i
//      of the underloaded ones, their total F; and, from the degree counts, the degree t_i at which
//      the m_i-th smallest member of partition i sits and how many members of exactly that degree
//      still have to go (need_i);
//   3. selection instead of a sort: the movers of partition i are its members of degree < t_i and,
//      among those of degree t_i, the need_i with the smallest ids.  Their rank by id comes from
//      per-workgroup counts of the degree-t_i members (vertex ranges in order), a scan over the
//      workgroups and an ordered count inside the workgroup;
//   4. the destination of a mover v is the partition whose interval of the running sum holds
//      (mix(seed, round, v) mod F).
//   If some t_i falls into the last histogram bin (more movers than members below degree B-1), the range that
//   holds it is counted again with B bins of equal width and narrowed to the bin with the need_i-th member, level
//   by level until the bins are one degree wide (two or three more counting passes; degrees enter as
//   min(degree, 2^24 - 1)); then step 3 runs as always.  Nothing is sorted; the movers are the first m_i members
//   by ascending degree, equal degrees by ascending id.
// The draw is a function of (seed, round, v) only, so the result does not depend on the order in
// which threads get to the vertices.  Rounds whose plan finds nothing overloaded do nothing (every
// kernel after the plan reads its flags and returns, and once a plan has found nothing overloaded even
// the counting passes of the later rounds return at once): the host enqueues max_rounds rounds without
// ever reading anything back.
#include <algorithm>

#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
constexpr int kPartMax = 255;                 // partition ids fit the top byte of a key, 255 = "stays"
constexpr uint32_t kDegreeMask = 0x00FFFFFFu;

struct BalPlan {
    unsigned long long L[256];    // loads of the class per partition (this round)
    long long m[256];             // vertices to move out (0 unless overloaded)
    long long cumf[256];          // running sum of the free capacities, partitions in index order
    int ref_lo[256];              // refinement: first degree of the range a partition's threshold is known to lie in
    int refining[256];            // refinement: the partition's threshold degree is not yet pinned to one degree
    long long F;                  // total free capacity
    int active;                   // this round moves vertices
    int round;                    // rounds completed before this one (enters the draw)
    int refine;                   // a threshold degree fell into the last histogram bin: the refinement passes run
    int by_select;                // this round moves vertices (selection of the smallest (degree, id) members)
    int finished;                 // a plan found nothing overloaded: later rounds do nothing
    int tdeg[256];                // threshold degree t_i of the overloaded partitions
    long long need[256];          // members of degree t_i that move (the smallest ids)
};

constexpr int kHistCounters = 16384;   // LDS counters of the degree histogram (64 KB)
constexpr int kBinsMax = 256;
constexpr int kSelBlocksMax = 1024;    // vertex ranges of the selection passes
inline int degree_bins(int32_t k) { return std::min(kBinsMax, kHistCounters / k); }   // >= 64 for k <= 255

__global__ __launch_bounds__(kBlock) void bal_reset_kernel(BalPlan *plan, int64_t *stats, int first, int cells,
                                                            unsigned int *__restrict__ dhist) {
    const int t = blockIdx.x * kBlock + threadIdx.x;
    if (first && t == 0) {
        plan->round = 0;
        plan->finished = 0;
    }
    if (first && t < 3) stats[t] = 0;
    if (t < cells) dhist[t] = 0;   // (later rounds: the plan clears the rows it has read)
}

// dhist[l * bins + min(degree, bins - 1)] += 1 for every class member v of partition l.
template <typename RowT>
__global__ __launch_bounds__(kBlock) void bal_count_kernel(int64_t n, int32_t k, int bins,
                                                            const RowT *__restrict__ rowptr,
                                                            const uint8_t *__restrict__ vclass, int32_t class_id,
                                                            const int32_t *__restrict__ labels,
                                                            const BalPlan *__restrict__ plan,
                                                            unsigned int *__restrict__ dhist) {
    if (plan->finished) return;   // uniform over the grid
    __shared__ unsigned int h[kHistCounters];
    const int cells = k * bins;
    for (int i = threadIdx.x; i < cells; i += kBlock) h[i] = 0;
    __syncthreads();
    // Class, label and the two offsets of four vertices per thread are loaded at once and unconditionally (a vertex
    // past the end reads the last one and is ignored): tested one after the other, each under the branch of the test
    // before, they were three memory latencies in a row per vertex, at two workgroups per compute unit.
    constexpr int kPer = 4;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const uint8_t *cls = vclass ? vclass : reinterpret_cast<const uint8_t *>(labels);   // without classes: read, not used
    for (int64_t v0 = (int64_t)blockIdx.x * kBlock + threadIdx.x; v0 < n; v0 += kPer * stride) {
        uint8_t c[kPer];
        int32_t l[kPer];
        RowT lo[kPer], hi[kPer];
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const int64_t v = std::min<int64_t>(v0 + q * stride, n - 1);
            c[q] = cls[v];
            l[q] = labels[v];
            lo[q] = rowptr[v];
            hi[q] = rowptr[v + 1];
        }
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const bool mine = v0 + q * stride < n && (!vclass || c[q] == class_id) && l[q] >= 0 && l[q] < k;
            const int64_t deg = (int64_t)(hi[q] - lo[q]);
            if (mine) atomicAdd(&h[l[q] * bins + (int)std::min<int64_t>(std::max<int64_t>(deg, 0), bins - 1)], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cells; i += kBlock)
        if (h[i]) atomicAdd(&dhist[i], h[i]);   // integers: the order does not matter
}

// One workgroup of 256 threads, thread i = partition i (k <= 255).  `allow` is 0 for the closing evaluation
// after the last round.
__global__ __launch_bounds__(256) void bal_plan_kernel(int32_t k, int bins, double beta, int allow, BalPlan *plan,
                                                        unsigned int *__restrict__ dhist, int64_t *stats) {
    if (plan->finished) return;
    __shared__ long long load_lds[256];
    __shared__ long long cap_lds;
    __shared__ int refine_lds;
    const int i = threadIdx.x;
    long long L = 0;
    if (i < k)
        for (int b = 0; b < bins; ++b) L += dhist[i * bins + b];
    load_lds[i] = L;
    if (i == 0) refine_lds = 0;
    __syncthreads();
    if (i == 0) {
        long long total = 0;
        for (int j = 0; j < k; ++j) total += load_lds[j];
        long long cap = (long long)floor(beta * (double)total / (double)k);
        const long long reach = (total + k - 1) / k;
        if (cap < reach) cap = reach;
        cap_lds = cap;
        long long F = 0, over = 0;
        for (int j = 0; j < k; ++j) {
            const long long Lj = load_lds[j];
            if (Lj < cap) F += cap - Lj;
            plan->cumf[j] = F;
            if (Lj > cap) ++over;
        }
        plan->F = F;
        stats[2] = over;
        const int active = allow && over > 0;
        plan->active = active;
        plan->round = (int)stats[0];
        if (active) stats[0] += 1;
        if (over == 0) plan->finished = 1;
    }
    __syncthreads();
    const long long cap = cap_lds;
    long long m = 0, need = 0;
    int tdeg = 0, refining = 0;
    if (i < k) {
        plan->L[i] = (unsigned long long)L;
        m = L > cap ? L - cap : 0;
        if (m > 0) {   // the degree of the m-th smallest member: the first bin at which the running count reaches m
            long long below = 0;
            int b = 0;
            for (; b < bins - 1; ++b) {
                const long long c = dhist[i * bins + b];
                if (below + c >= m) break;
                below += c;
            }
            tdeg = b;
            need = m - below;
            if (b == bins - 1) {   // the last bin holds every degree from bins - 1 up: narrowed down by the refinement
                refine_lds = 1;
                refining = 1;
            }
        }
        plan->m[i] = m;
        plan->tdeg[i] = tdeg;
        plan->need[i] = need;
        plan->ref_lo[i] = bins - 1;
        plan->refining[i] = refining;
    }
    __syncthreads();
    if (i == 0) {
        plan->refine = plan->active && refine_lds;
        plan->by_select = plan->active;
    }
    if (i < k)   // the next round's count starts from zero
        for (int b = 0; b < bins; ++b) dhist[i * bins + b] = 0;
}

// ---- refinement of a threshold degree that fell into the last bin ------------------------------------------
// The last bin of the first histogram holds every degree from bins - 1 up (degrees enter at most as
// kDegreeMask).  A partition whose threshold lies there is counted again over the range it is known to lie in,
// ref_lo .. ref_lo + bins * width, with `bins` bins of `width` degrees, and the range is narrowed to the bin that
// holds the need-th member; the widths of the levels (a function of `bins` only, so the host launches a fixed
// number of them) end at 1, where the threshold degree and the number of members to take at it are known.
// Nothing is sorted.  Without a refining partition the kernels return at once.
__host__ __device__ inline int64_t refine_width(int bins, int level) {   // level 1, 2, ...: bins of this many degrees
    int64_t w = ((int64_t)kDegreeMask + 1 - (bins - 1) + bins - 1) / bins;
    for (int j = 1; j < level; ++j) w = (w + bins - 1) / bins;
    return w;
}
inline int refine_levels(int bins) {
    int level = 1;
    while (refine_width(bins, level) > 1) ++level;
    return level;
}

template <typename RowT>
__global__ __launch_bounds__(kBlock) void bal_refine_count_kernel(int64_t n, int32_t k, int bins, int64_t width,
                                                                   const RowT *__restrict__ rowptr,
                                                                   const uint8_t *__restrict__ vclass, int32_t class_id,
                                                                   const int32_t *__restrict__ labels,
                                                                   const BalPlan *__restrict__ plan,
                                                                   unsigned int *__restrict__ dhist) {
    if (!plan->refine) return;   // uniform over the grid
    __shared__ unsigned int h[kHistCounters];
    __shared__ int lo_lds[256];
    const int cells = k * bins;
    for (int i = threadIdx.x; i < cells; i += kBlock) h[i] = 0;
    lo_lds[threadIdx.x] = (int)threadIdx.x < k && plan->refining[threadIdx.x] ? plan->ref_lo[threadIdx.x] : -1;
    __syncthreads();
    constexpr int kPer = 4;   // as in bal_count_kernel
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const uint8_t *cls = vclass ? vclass : reinterpret_cast<const uint8_t *>(labels);
    for (int64_t v0 = (int64_t)blockIdx.x * kBlock + threadIdx.x; v0 < n; v0 += kPer * stride) {
        uint8_t c[kPer];
        int32_t l[kPer];
        RowT lo[kPer], hi[kPer];
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const int64_t v = std::min<int64_t>(v0 + q * stride, n - 1);
            c[q] = cls[v];
            l[q] = labels[v];
            lo[q] = rowptr[v];
            hi[q] = rowptr[v + 1];
        }
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const bool mine = v0 + q * stride < n && (!vclass || c[q] == class_id) && l[q] >= 0 && l[q] < k;
            if (!mine) continue;
            const int first = lo_lds[l[q]];
            if (first < 0) continue;
            const int64_t deg = std::min<int64_t>(std::max<int64_t>((int64_t)(hi[q] - lo[q]), 0), (int64_t)kDegreeMask);
            const int64_t off = deg - first;
            if (off >= 0 && off < (int64_t)bins * width) atomicAdd(&h[l[q] * bins + (int)(off / width)], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cells; i += kBlock)
        if (h[i]) atomicAdd(&dhist[i], h[i]);   // integers: the order does not matter
}

// Thread i = partition i: the bin that holds its need-th member becomes its range; at width 1 that is the threshold.
__global__ __launch_bounds__(256) void bal_refine_plan_kernel(int32_t k, int bins, int64_t width, BalPlan *plan,
                                                               unsigned int *__restrict__ dhist) {
    if (!plan->refine) return;
    const int i = threadIdx.x;
    if (i >= k) return;
    if (plan->refining[i]) {
        long long below = 0;
        const long long need = plan->need[i];
        int b = 0;
        for (; b < bins - 1; ++b) {
            const long long c = dhist[i * bins + b];
            if (below + c >= need) break;
            below += c;
        }
        const int first = plan->ref_lo[i] + (int)(b * width);
        plan->ref_lo[i] = first;
        plan->need[i] = need - below;
        if (width == 1) {
            plan->tdeg[i] = first;
            plan->refining[i] = 0;
        }
    }
    for (int b = 0; b < bins; ++b) dhist[i * bins + b] = 0;   // the next count starts from zero
}

// ---- selection: the movers are the members below the threshold degree and the first need_i (by id) at it ----
// Vertex ranges of rows_per_block vertices, one per workgroup, in order.
// Pass 1: tie[b * k + l] = members of partition l with degree exactly t_l in range b.
template <typename RowT>
__global__ __launch_bounds__(kBlock) void bal_tie_count_kernel(int64_t n, int32_t k, int64_t rows_per_block,
                                                                const RowT *__restrict__ rowptr,
                                                                const uint8_t *__restrict__ vclass, int32_t class_id,
                                                                const int32_t *__restrict__ labels,
                                                                const BalPlan *__restrict__ plan,
                                                                int32_t *__restrict__ tie) {
    if (!plan->by_select) return;   // uniform over the grid
    __shared__ int32_t cnt[256];
    __shared__ int32_t tdeg[256];
    cnt[threadIdx.x] = 0;
    tdeg[threadIdx.x] = (int)threadIdx.x < k && plan->m[threadIdx.x] > 0 ? plan->tdeg[threadIdx.x] : -1;
    __syncthreads();
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    constexpr int kPer = 4;   // loads of four vertices per thread at once, unconditionally (as in bal_count_kernel)
    const uint8_t *cls = vclass ? vclass : reinterpret_cast<const uint8_t *>(labels);
    for (int64_t v0 = b + threadIdx.x; v0 < e; v0 += kPer * kBlock) {
        uint8_t c[kPer];
        int32_t l[kPer];
        RowT lo[kPer], hi[kPer];
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const int64_t v = std::min<int64_t>(v0 + q * kBlock, n - 1);
            c[q] = cls[v];
            l[q] = labels[v];
            lo[q] = rowptr[v];
            hi[q] = rowptr[v + 1];
        }
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const bool mine = v0 + q * kBlock < e && (!vclass || c[q] == class_id) && l[q] >= 0 && l[q] < k;
            const int64_t deg = std::min<int64_t>((int64_t)(hi[q] - lo[q]), (int64_t)kDegreeMask);
            if (mine && deg == (int64_t)tdeg[l[q]]) atomicAdd(&cnt[l[q]], 1);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < k) tie[(int64_t)blockIdx.x * k + threadIdx.x] = cnt[threadIdx.x];
}

// Pass 2: per partition, exclusive scan of the counts over the ranges (thread l = partition l).
__global__ __launch_bounds__(256) void bal_tie_scan_kernel(int32_t k, int blocks, const BalPlan *__restrict__ plan,
                                                            int32_t *__restrict__ tie) {
    if (!plan->by_select) return;
    const int l = threadIdx.x;
    if (l >= k) return;
    int32_t run = 0;
    constexpr int kBatch = 16;   // loads in flight per thread (one at a time, each waited for, before)
    for (int b0 = 0; b0 < blocks; b0 += kBatch) {
        int32_t c[kBatch];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) c[q] = tie[(int64_t)std::min(b0 + q, blocks - 1) * k + l];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            if (b0 + q < blocks) {
                tie[(int64_t)(b0 + q) * k + l] = run;
                run += c[q];
            }
        }
    }
}

__device__ __forceinline__ uint64_t draw64(uint64_t seed, uint32_t round, int64_t v) {
    uint64_t z = seed + (((uint64_t)round << 32) + (uint64_t)v + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// x mod F without a 64-bit division per draw: with magic = floor((2^64 - 1) / F), q = high half of x * magic
// is the quotient or up to two less, so at most two subtractions finish the remainder (exact for every x).
__device__ __forceinline__ uint64_t magic_of(uint64_t F) { return F ? ~0ull / F : 0; }
__device__ __forceinline__ uint64_t mod_by(uint64_t x, uint64_t F, uint64_t magic) {
    uint64_t r = x - __umul64hi(x, magic) * F;
    if (r >= F) r -= F;
    if (r >= F) r -= F;
    return r;
}


// Pass 3: the move.  A member of degree t_l moves iff fewer than need_l such members of its partition come
// before it by id: the count before its range, plus the ordered count inside the range (tiles of 256 vertices:
// lanes of a wave with the same partition are matched with ballots, waves and tiles are added up in order).
template <typename RowT>
__global__ __launch_bounds__(kBlock) void bal_select_move_kernel(int64_t n, int32_t k, int64_t rows_per_block,
                                                                  uint64_t seed, const RowT *__restrict__ rowptr,
                                                                  const uint8_t *__restrict__ vclass, int32_t class_id,
                                                                  const BalPlan *__restrict__ plan,
                                                                  const int32_t *__restrict__ tie,
                                                                  int32_t *__restrict__ labels,
                                                                  int64_t *__restrict__ stats) {
    if (!plan->by_select) return;   // uniform over the grid
    constexpr int kWavesPerBlock = kBlock / 64;
    __shared__ long long cumf[256];
    __shared__ long long need[256];
    __shared__ int32_t tdeg[256];
    __shared__ int32_t running[256];                 // degree-t members of every partition met so far (by id)
    __shared__ int32_t wcnt[kWavesPerBlock][256];
    const int t = threadIdx.x, wave = t >> 6;
    const bool over = t < k && plan->m[t] > 0;
    cumf[t] = t < k ? plan->cumf[t] : plan->F;
    need[t] = over ? plan->need[t] : 0;
    tdeg[t] = over ? plan->tdeg[t] : -1;
    running[t] = t < k ? tie[(int64_t)blockIdx.x * k + t] : 0;
    for (int w = 0; w < kWavesPerBlock; ++w) wcnt[w][t] = 0;
    __syncthreads();
    const uint64_t F = (uint64_t)plan->F, magic = magic_of(F);
    const uint32_t round = (uint32_t)plan->round;
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    unsigned long long moved_total = 0;
    const uint8_t *cls = vclass ? vclass : reinterpret_cast<const uint8_t *>(labels);
    // The four values of a vertex are loaded together and unconditionally, one tile ahead: the tile's three
    // barriers pass while the next tile's loads are in flight.  (A tile only writes the labels of its own vertices,
    // so the labels read ahead are not changed by it.)
    uint8_t cq;
    int32_t lab;
    RowT lo, hi;
    auto fetch = [&](int64_t v) {
        const int64_t vq = std::min<int64_t>(v, n - 1);
        cq = cls[vq];
        lab = labels[vq];
        lo = rowptr[vq];
        hi = rowptr[vq + 1];
    };
    fetch(b + t);
    for (int64_t tile = b; tile < e; tile += kBlock) {
        const int64_t v = tile + t;
        int32_t l = -1;
        int64_t deg = 0;
        if (v < e && (!vclass || cq == class_id) && lab >= 0 && lab < k && tdeg[lab] >= 0) {
            l = lab;
            deg = std::min<int64_t>((int64_t)(hi - lo), (int64_t)kDegreeMask);
        }
        fetch(v + kBlock);
        const bool at_threshold = l >= 0 && deg == (int64_t)tdeg[l];
        // lanes of this wave at the threshold of the same partition
        const int key = at_threshold ? l : 0;
        uint64_t peers = __ballot(at_threshold);
        for (int bit = 0; bit < 8; ++bit) {
            const uint64_t m = __ballot((key >> bit) & 1);
            peers &= ((key >> bit) & 1) ? m : ~m;
        }
        const unsigned lane = t & 63;
        const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
        const int rank_in_wave = __popcll(peers & below);
        if (at_threshold && rank_in_wave == 0) wcnt[wave][key] = __popcll(peers);
        __syncthreads();
        bool move = l >= 0 && deg < (int64_t)tdeg[l];
        if (at_threshold) {
            long long before = running[l] + rank_in_wave;
            for (int w = 0; w < wave; ++w) before += wcnt[w][l];
            move = before < need[l];
        }
        if (move) {
            const uint64_t r = mod_by(draw64(seed, round, v), F, magic);
            int lo = 0, hi = k - 1;               // first partition whose running sum exceeds r
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if ((uint64_t)cumf[mid] > r) hi = mid; else lo = mid + 1;
            }
            labels[v] = lo;
        }
        const unsigned long long mb = __ballot(move);
        if (lane == 0) moved_total += (unsigned long long)__popcll(mb);
        __syncthreads();
        int32_t add = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) { add += wcnt[w][t]; wcnt[w][t] = 0; }
        running[t] += add;
        __syncthreads();
    }
    if ((t & 63) == 0 && moved_total) atomicAdd(reinterpret_cast<unsigned long long *>(stats + 1), moved_total);
}


// ---- small graphs: all rounds of a call in one launch ---------------------------------------------
// Up to kSmallN vertices the work of a round is microseconds and the ~20 launches per round of the chain
// above are all the time there is (about 1,000 launches for three classes and 16 rounds each).  One
// workgroup of 1,024 threads then runs the whole call: per round the loads and degree counts, the plan,
// the threshold degree of every overloaded partition, the ordered selection of its movers (every wave
// over a contiguous range of vertices, the members at the threshold before its range counted first) and
// their moves, and it stops at the first round that finds nothing overloaded.  The threshold degree is found by
// selection at any size: if it lies beyond the exact bins, the range that holds it is counted again with
// narrower bins until the bins are one degree wide (at most five passes up to degree 2^24 - 1, the value
// degrees are clamped to, as in the chain above).  Same movers and same draws as the chain above.
__device__ __forceinline__ void wave_lds_fence_() {   // orders a wave's own LDS accesses
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
constexpr int kSmallN = 1 << 18;
constexpr int kSmBlock = 1024;
constexpr int kSmWaves = kSmBlock / 64;
constexpr int kSmPer = 8;             // vertices per thread and turn: their loads are in flight together
constexpr int kSmCounters = 8192;      // LDS counters of the degree histogram (32 KB)
constexpr int kDegreeLimit = 1 << 24;  // degrees are clamped to kDegreeLimit - 1

template <typename RowT>
__global__ __launch_bounds__(kSmBlock) void bal_small_kernel(int32_t n, int32_t k, const RowT *__restrict__ rowptr,
                                                              const uint8_t *__restrict__ vclass, int32_t class_id,
                                                              double beta, uint64_t seed, int32_t max_rounds,
                                                              int32_t *__restrict__ labels, int64_t *__restrict__ stats) {
    // n <= 2^18, so every count fits 32 bits
    __shared__ unsigned int hist[kSmCounters];
    __shared__ int32_t running[kSmWaves][256];   // degree-t members of a partition before a wave's place (by id)
    __shared__ int32_t load_of[256], m_of[256], cumf[256], need[256], below[256];
    __shared__ int32_t lo[256], hi[256], width[256], tdeg[256], refining[256];
    __shared__ int32_t arrived[256];             // movers that landed in a partition this round
    __shared__ int32_t cap_s, F_s, over_s, refine_any;
    __shared__ unsigned int moved_s;
    const int t = threadIdx.x, wave = t >> 6;
    const unsigned lane = t & 63;
    const int bins = min(256, kSmCounters / k), cells = k * bins;
    if (t == 0) moved_s = 0;
    int32_t rounds_run = 0;
    // every wave owns a contiguous range of vertices (a multiple of 64 long), the ranges in wave order
    const int per_wave = (n + 64 * kSmWaves - 1) / (64 * kSmWaves) * 64;
    const int wave_begin = min(n, wave * per_wave), wave_end = min(n, wave_begin + per_wave);

    // Partition and clamped degree of kSmPer vertices v0 + stride q; -1 for a vertex that is not a member of the
    // class (or past the end).  All loads are issued before anything is looked at: one memory round trip.
    auto fetch = [&](int v0, int stride, int end, int32_t(&l)[kSmPer], int32_t(&deg)[kSmPer]) {
        int32_t cls[kSmPer], lab[kSmPer];
        RowT r0[kSmPer], r1[kSmPer];
#pragma unroll
        for (int q = 0; q < kSmPer; ++q) {
            const int v = v0 + q * stride;
            const bool in = v < end;
            const unsigned vs = in ? (unsigned)v : 0u;   // unsigned 32-bit offsets from a uniform base
            cls[q] = vclass ? (int32_t)vclass[vs] : class_id;
            lab[q] = labels[vs];
            r0[q] = rowptr[vs];
            r1[q] = rowptr[vs + 1];
            if (!in) cls[q] = class_id + 1;
        }
#pragma unroll
        for (int q = 0; q < kSmPer; ++q) {
            const bool member = cls[q] == class_id && lab[q] >= 0 && lab[q] < k;
            l[q] = member ? lab[q] : -1;
            const int64_t d = (int64_t)(r1[q] - r0[q]);
            deg[q] = (int32_t)min(max(d, (int64_t)0), (int64_t)kDegreeLimit - 1);
        }
    };

    for (int32_t round = 0;; ++round) {
        // ---- loads of the class per partition and the exact degree bins 0 .. bins - 2 (+ "bins - 1 or more") ----
        for (int i = t; i < cells; i += kSmBlock) hist[i] = 0;
        __syncthreads();
        for (int v0 = t; v0 < n; v0 += kSmPer * kSmBlock) {
            int32_t l[kSmPer], deg[kSmPer];
            fetch(v0, kSmBlock, n, l, deg);
#pragma unroll
            for (int q = 0; q < kSmPer; ++q)
                if (l[q] >= 0) atomicAdd(&hist[l[q] * bins + min(deg[q], bins - 1)], 1u);
        }
        __syncthreads();
        if (t < 256) {
            int32_t L = 0;
            if (t < k)
                for (int b = 0; b < bins; ++b) L += (int32_t)hist[t * bins + b];
            load_of[t] = L;
        }
        __syncthreads();
        if (t == 0) {
            long long total = 0;
            for (int j = 0; j < k; ++j) total += load_of[j];
            long long cap = (long long)floor(beta * (double)total / (double)k);
            const long long reach = (total + k - 1) / k;
            if (cap < reach) cap = reach;
            long long F = 0;
            int32_t over = 0;
            for (int j = 0; j < k; ++j) {
                const long long Lj = load_of[j];
                if (Lj < cap) F += cap - Lj;
                cumf[j] = (int32_t)min(F, (long long)0x7fffffff);   // with something overloaded, F <= k n < 2^26
                if (Lj > cap) ++over;
            }
            cap_s = (int32_t)min(cap, (long long)0x7fffffff);   // a capacity beyond n is never reached
            F_s = (int32_t)min(F, (long long)0x7fffffff);
            over_s = over;
            refine_any = 0;
        }
        __syncthreads();
        if (over_s == 0 || round >= max_rounds) {   // uniform: balanced, or the closing evaluation
            if (t == 0) {
                stats[0] = rounds_run;
                stats[1] = (int64_t)moved_s;
                stats[2] = over_s;
            }
            return;
        }
        rounds_run = round + 1;

        // ---- threshold degree t_i of every overloaded partition: where its m_i-th smallest member sits ----
        if (t < 256) {
            const int32_t m = t < k && load_of[t] > cap_s ? load_of[t] - cap_s : 0;
            m_of[t] = m;
            tdeg[t] = -1;
            need[t] = 0;
            refining[t] = 0;
            if (m > 0) {
                int32_t seen = 0;
                int b = 0;
                for (; b < bins - 1; ++b) {
                    const int32_t c = (int32_t)hist[t * bins + b];
                    if (seen + c >= m) break;
                    seen += c;
                }
                if (b < bins - 1) {
                    tdeg[t] = b;
                    need[t] = m - seen;
                } else {   // beyond the exact bins: narrow the range [bins - 1, 2^24) down
                    below[t] = seen;
                    lo[t] = bins - 1;
                    hi[t] = kDegreeLimit;
                    refining[t] = 1;
                    refine_any = 1;
                }
            }
        }
        __syncthreads();
        int again = refine_any;
        __syncthreads();
        while (again) {   // uniform
            for (int i = t; i < cells; i += kSmBlock) hist[i] = 0;
            if (t < 256 && refining[t]) width[t] = (hi[t] - lo[t] + bins - 1) / bins;
            if (t == 0) refine_any = 0;
            __syncthreads();
            for (int v0 = t; v0 < n; v0 += kSmPer * kSmBlock) {
                int32_t l[kSmPer], deg[kSmPer];
                fetch(v0, kSmBlock, n, l, deg);
#pragma unroll
                for (int q = 0; q < kSmPer; ++q)
                    if (l[q] >= 0 && refining[l[q]] && deg[q] >= lo[l[q]] && deg[q] < hi[l[q]])
                        atomicAdd(&hist[l[q] * bins + (deg[q] - lo[l[q]]) / width[l[q]]], 1u);
            }
            __syncthreads();
            if (t < 256 && refining[t]) {
                int32_t seen = below[t];
                int b = 0;
                for (; b < bins - 1; ++b) {   // the m-th smallest lies in the range, so the last bin ends the search
                    const int32_t c = (int32_t)hist[t * bins + b];
                    if (seen + c >= m_of[t]) break;
                    seen += c;
                }
                below[t] = seen;
                lo[t] += b * width[t];
                hi[t] = min(hi[t], lo[t] + width[t]);
                if (width[t] == 1) {
                    tdeg[t] = lo[t];
                    need[t] = m_of[t] - seen;
                    refining[t] = 0;
                } else {
                    refine_any = 1;
                }
            }
            __syncthreads();
            again = refine_any;
            __syncthreads();
        }

        // ---- members at the threshold before every wave's range: counts per range, then a scan over the ranges ----
        for (int w = 0; w < kSmWaves; ++w)
            if (t < 256) running[w][t] = 0;
        if (t < 256) arrived[t] = 0;
        __syncthreads();
        for (int v0 = wave_begin + (int)lane; v0 < wave_end; v0 += kSmPer * 64) {
            int32_t l[kSmPer], deg[kSmPer];
            fetch(v0, 64, wave_end, l, deg);
#pragma unroll
            for (int q = 0; q < kSmPer; ++q)
                if (l[q] >= 0 && m_of[l[q]] > 0 && deg[q] == tdeg[l[q]]) atomicAdd(&running[wave][l[q]], 1);
        }
        __syncthreads();
        if (t < 256) {
            int32_t run = 0;
            for (int w = 0; w < kSmWaves; ++w) {
                const int32_t c = running[w][t];
                running[w][t] = run;
                run += c;
            }
        }
        __syncthreads();

        // ---- the movers, every wave over its range in id order: below the threshold, or at it among the first need_i ----
        const uint64_t F = (uint64_t)F_s, magic = magic_of(F);
        unsigned int moved_here = 0;
        for (int base = wave_begin; base < wave_end; base += kSmPer * 64) {   // uniform in the wave
            const int v0 = base + (int)lane;
            int32_t l[kSmPer], deg[kSmPer];
            fetch(v0, 64, wave_end, l, deg);
#pragma unroll
            for (int q = 0; q < kSmPer; ++q) {
                const int v = v0 + 64 * q;
                const bool cand = l[q] >= 0 && m_of[l[q]] > 0;
                const bool at_threshold = cand && deg[q] == tdeg[l[q]];
                const int key = at_threshold ? l[q] : 0;
                uint64_t peers = __ballot(at_threshold);   // lanes at the threshold of the same partition
                for (int bit = 0; bit < 8; ++bit) {
                    const uint64_t mb = __ballot((key >> bit) & 1);
                    peers &= ((key >> bit) & 1) ? mb : ~mb;
                }
                const uint64_t lanes_before = lane == 0 ? 0ull : (~0ull >> (64 - lane));
                const int rank_in_wave = __popcll(peers & lanes_before);
                bool move = cand && deg[q] < tdeg[l[q]];
                if (at_threshold) {
                    move = running[wave][key] + rank_in_wave < need[key];
                }
                wave_lds_fence_();
                if (at_threshold && rank_in_wave == 0) running[wave][key] += __popcll(peers);
                wave_lds_fence_();
                if (move) {
                    const uint64_t r = mod_by(draw64(seed, (uint32_t)round, v), F, magic);
                    int a = 0, b = k - 1;               // first partition whose running sum exceeds r
                    while (a < b) {
                        const int mid = (a + b) >> 1;
                        if ((uint64_t)cumf[mid] > r) b = mid; else a = mid + 1;
                    }
                    labels[v] = a;
                    atomicAdd(&arrived[a], 1);   // integer: order does not matter
                }
                moved_here += (unsigned int)__popcll(__ballot(move));
            }
        }
        if (lane == 0 && moved_here) atomicAdd(&moved_s, moved_here);
        __syncthreads();   // the labels written above are read by the next round's count
        // The loads after this round are known without counting again: every overloaded partition is down to the
        // capacity and the others got their arrivals; the capacity itself (a function of the class size) stays.
        // If nothing exceeds it, the next round's evaluation would find the same and end the call.
        if (t == 0) {
            int over = 0;
            for (int j = 0; j < k; ++j) over += load_of[j] - m_of[j] + arrived[j] > cap_s;
            over_s = over;
        }
        __syncthreads();
        if (over_s == 0) {   // uniform
            if (t == 0) {
                stats[0] = rounds_run;
                stats[1] = (int64_t)moved_s;
                stats[2] = 0;
            }
            return;
        }
    }
}

}  // namespace

BalanceWs carve_balance_ws(int64_t n, void *ws) {
    Carver c(ws);
    BalanceWs w{};
    w.plan = c.take<unsigned char>(sizeof(BalPlan));
    w.degree_hist = c.take<uint32_t>(kHistCounters);
    w.tie = c.take<int32_t>((size_t)kSelBlocksMax * 256);
    w.bytes = align_up(c.used, 256);
    return w;
}

int launch_balance(int64_t n, int32_t k, const void *rowptr, bool i64, const uint8_t *vclass, int32_t class_id,
                   double beta, uint64_t seed, int32_t max_rounds, int32_t *labels, int64_t *stats,
                   const BalanceWs &w, hipStream_t s) {
    if (k > kPartMax) return EP_EUNSUPPORTED;
    if (n <= kSmallN) {   // small graph: the whole call in one launch
        if (i64)
            bal_small_kernel<<<1, kSmBlock, 0, s>>>((int32_t)n, k, static_cast<const int64_t *>(rowptr), vclass, class_id, beta, seed,
                                                    max_rounds, labels, stats);
        else
            bal_small_kernel<<<1, kSmBlock, 0, s>>>((int32_t)n, k, static_cast<const int32_t *>(rowptr), vclass, class_id, beta, seed,
                                                    max_rounds, labels, stats);
        EP_LAUNCH_CHECK();
        return EP_OK;
    }
    BalPlan *plan = reinterpret_cast<BalPlan *>(w.plan);
    const unsigned count_blocks = (unsigned)std::min<int64_t>(2048, ceil_div(n, kBlock * 8));
    const int bins = degree_bins(k), cells = k * bins, levels = refine_levels(bins);
    int64_t rows_per_block = std::max<int64_t>(ceil_div(n, kSelBlocksMax), 4 * kBlock);
    rows_per_block = ceil_div(rows_per_block, kBlock) * kBlock;
    const int sel_blocks = (int)ceil_div(n, rows_per_block);
    auto by_width = [&](auto &&f) {
        return i64 ? f(static_cast<const int64_t *>(rowptr)) : f(static_cast<const int32_t *>(rowptr));
    };
    for (int32_t r = 0; r <= max_rounds; ++r) {
        if (r == 0) {
            bal_reset_kernel<<<(unsigned)ceil_div(std::max(cells, 256), kBlock), kBlock, 0, s>>>(plan, stats, 1, cells,
                                                                                              w.degree_hist);
            EP_LAUNCH_CHECK();
        }
        by_width([&](auto *rp) {
            bal_count_kernel<<<count_blocks, kBlock, 0, s>>>(n, k, bins, rp, vclass, class_id, labels, plan, w.degree_hist);
            return 0;
        });
        EP_LAUNCH_CHECK();
        bal_plan_kernel<<<1, 256, 0, s>>>(k, bins, beta, r < max_rounds, plan, w.degree_hist, stats);
        EP_LAUNCH_CHECK();
        if (r == max_rounds) break;   // the closing evaluation only reports what is still overloaded
        // a threshold degree in the last histogram bin is narrowed down first (no-ops otherwise)
        for (int level = 1; level <= levels; ++level) {
            const int64_t width = refine_width(bins, level);
            by_width([&](auto *rp) {
                bal_refine_count_kernel<<<count_blocks, kBlock, 0, s>>>(n, k, bins, width, rp, vclass, class_id, labels, plan,
                                                                        w.degree_hist);
                return 0;
            });
            EP_LAUNCH_CHECK();
            bal_refine_plan_kernel<<<1, 256, 0, s>>>(k, bins, width, plan, w.degree_hist);
            EP_LAUNCH_CHECK();
        }
        // selection: members below the threshold degree move, and the first need_i (by id) at it
        by_width([&](auto *rp) {
            bal_tie_count_kernel<<<sel_blocks, kBlock, 0, s>>>(n, k, rows_per_block, rp, vclass, class_id, labels, plan, w.tie);
            return 0;
        });
        EP_LAUNCH_CHECK();
        bal_tie_scan_kernel<<<1, 256, 0, s>>>(k, sel_blocks, plan, w.tie);
        EP_LAUNCH_CHECK();
        by_width([&](auto *rp) {
            bal_select_move_kernel<<<sel_blocks, kBlock, 0, s>>>(n, k, rows_per_block, seed, rp, vclass, class_id, plan,
                                                                 w.tie, labels, stats);
            return 0;
        });
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

}  // namespace ep
