// Integer kernels over a CSR graph and a label vector: partition sizes, edge cut, the
// partition-sorted relabelling and the gap sums of the reordering metrics.
//
// What they compute (EmbedPart paper): an entry (u,v) is cut iff pid(u) != pid(v) and
// |P_p| is the number of vertices with pid = p (Sec. "Partitioning quality metrics");
// the reordering gives vertices of one partition consecutive ids (Sec. "Adapting
// EmbedPart for Reordering"); gap xi_pi(u,v) = |pi(u) - pi(v)| and the vertex bandwidth
// is its maximum over a vertex's neighbours (Eq. gap, Eq. vertex bandwidth).
// Everything here is integer arithmetic, so results do not depend on execution order.
#include <algorithm>

#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;

__device__ __forceinline__ uint64_t lanemask_lt() {
    const unsigned lane = __lane_id();
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// Sum a per-thread uint64 over the workgroup; the result is valid in thread 0.
__device__ __forceinline__ uint64_t block_sum_u64(uint64_t v, uint64_t *lds /* kBlock/64 */) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    uint64_t total = 0;
    if (threadIdx.x == 0)
        for (int w = 0; w < kBlock / 64; ++w) total += lds[w];
    return total;
}

__global__ void fill_i64_kernel(int64_t *a, int64_t na, int64_t *b, int64_t nb) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < na) a[i] = 0;
    if (b && i < nb) b[i] = 0;
}

// ---- partition sizes ---------------------------------------------------------------
constexpr int kLdsHistMax = 8192;

__global__ __launch_bounds__(kBlock) void label_hist_kernel(int64_t n, int32_t k, const int32_t *__restrict__ labels,
                                                             int64_t *__restrict__ sizes) {
    __shared__ int32_t hist[kLdsHistMax];
    const bool in_lds = k <= kLdsHistMax;
    if (in_lds) {
        for (int j = threadIdx.x; j < k; j += kBlock) hist[j] = 0;
        __syncthreads();
    }
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const int32_t l = labels[i];
        if (l < 0 || l >= k) continue;
        if (in_lds) atomicAdd(&hist[l], 1);
        else atomicAdd(reinterpret_cast<unsigned long long *>(&sizes[l]), 1ull);
    }
    if (in_lds) {
        __syncthreads();
        for (int j = threadIdx.x; j < k; j += kBlock)
            if (hist[j]) atomicAdd(reinterpret_cast<unsigned long long *>(&sizes[j]), (unsigned long long)hist[j]);
    }
}

// ---- edge sweeps ---------------------------------------------------------------------
// Largest r in [0, n) with rowptr[r] <= e, given rowptr[0] <= e < rowptr[n].
template <typename RowT>
__device__ __forceinline__ int64_t find_row(const RowT *__restrict__ rowptr, int64_t n, int64_t e) {
    int64_t lo = 0, hi = n;  // invariant: rowptr[lo] <= e < rowptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if ((int64_t)rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

constexpr int kEdgesPerThread = 4;

// Each thread takes kEdgesPerThread consecutive stored entries, finds the row of the first by
// bisection of rowptr and walks forward.  kCut: counts entries whose end points carry different
// attributes (labels in [0,k), others skipped); otherwise sums |attr(u) - attr(v)| with
// attr = identity when attr == nullptr.
template <typename RowT, bool kCut>
__global__ __launch_bounds__(kBlock) void edge_sweep_kernel(int64_t n, int64_t nnz, int32_t k,
                                                             const RowT *__restrict__ rowptr,
                                                             const int32_t *__restrict__ colidx,
                                                             const int32_t *__restrict__ attr,
                                                             unsigned long long *__restrict__ out) {
    __shared__ uint64_t red[kBlock / 64];
    const int64_t e0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kEdgesPerThread;
    const int64_t end = min(nnz, (int64_t)rowptr[n]);
    uint64_t acc = 0;
    if (e0 < end && e0 >= (int64_t)rowptr[0]) {
        int64_t r = find_row(rowptr, n, e0);
        int64_t row_end = (int64_t)rowptr[r + 1];
        int64_t au = attr ? (int64_t)attr[r] : r;
        const int64_t e1 = min(e0 + kEdgesPerThread, end);
        for (int64_t e = e0; e < e1; ++e) {
            while (e >= row_end) {  // ends because e < rowptr[n]
                ++r;
                row_end = (int64_t)rowptr[r + 1];
                au = attr ? (int64_t)attr[r] : r;
            }
            const int32_t v = colidx[e];
            if (v < 0 || v >= n) continue;
            const int64_t av = attr ? (int64_t)attr[v] : (int64_t)v;
            if (kCut) {
                if (au >= 0 && au < k && av >= 0 && av < k && au != av) acc += 1;
            } else {
                acc += (uint64_t)(au > av ? au - av : av - au);
            }
        }
    }
    const uint64_t total = block_sum_u64(acc, red);
    if (threadIdx.x == 0 && total) atomicAdd(out, (unsigned long long)total);
}

// One thread per vertex: widest gap to a neighbour, summed over vertices.
template <typename RowT>
__global__ __launch_bounds__(kBlock) void bandwidth_kernel(int64_t n, int64_t nnz, const RowT *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            const int32_t *__restrict__ attr,
                                                            unsigned long long *__restrict__ out) {
    __shared__ uint64_t red[kBlock / 64];
    const int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    uint64_t widest = 0;
    if (u < n) {
        const int64_t au = attr ? (int64_t)attr[u] : u;
        const int64_t b = max((int64_t)rowptr[u], (int64_t)0), e = min((int64_t)rowptr[u + 1], nnz);
        for (int64_t t = b; t < e; ++t) {
            const int32_t v = colidx[t];
            if (v < 0 || v >= n) continue;
            const int64_t av = attr ? (int64_t)attr[v] : (int64_t)v;
            const uint64_t gap = (uint64_t)(au > av ? au - av : av - au);
            widest = gap > widest ? gap : widest;
        }
    }
    const uint64_t total = block_sum_u64(widest, red);
    if (threadIdx.x == 0 && total) atomicAdd(out, (unsigned long long)total);
}

// ---- stable LSD radix sort of vertex ids by label, 8 bits per pass ----------------------
constexpr int kRadix = 256;
constexpr int kSortWaves = kBlock / 64;

__device__ __forceinline__ int32_t sort_key(const int32_t *__restrict__ labels, const int32_t *__restrict__ order_in,
                                            int64_t i, int shift, int32_t *vertex) {
    const int32_t v = order_in ? order_in[i] : (int32_t)i;
    *vertex = v;
    return (int32_t)(((uint32_t)labels[v] >> shift) & (kRadix - 1));
}

__global__ __launch_bounds__(kBlock) void sort_hist_kernel(int64_t n, int64_t rows_per_block,
                                                            const int32_t *__restrict__ labels,
                                                            const int32_t *__restrict__ order_in, int shift,
                                                            int32_t *__restrict__ hist) {
    __shared__ int32_t h[kRadix];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    for (int64_t i = b + threadIdx.x; i < e; i += kBlock) {
        int32_t v;
        atomicAdd(&h[sort_key(labels, order_in, i, shift, &v)], 1);
    }
    __syncthreads();
    hist[(int64_t)blockIdx.x * kRadix + threadIdx.x] = h[threadIdx.x];
}

// Exclusive scan of hist[blocks][256] in (digit, block) order, in place.  One workgroup.
__global__ __launch_bounds__(kRadix) void sort_scan_kernel(int32_t *__restrict__ hist, int blocks) {
    __shared__ int32_t total[kRadix];
    const int t = threadIdx.x;
    int32_t run = 0;
    for (int b = 0; b < blocks; ++b) {
        const int32_t c = hist[(int64_t)b * kRadix + t];
        hist[(int64_t)b * kRadix + t] = run;
        run += c;
    }
    total[t] = run;
    __syncthreads();
    if (t == 0) {
        int32_t acc = 0;
        for (int j = 0; j < kRadix; ++j) { const int32_t c = total[j]; total[j] = acc; acc += c; }
    }
    __syncthreads();
    const int32_t base = total[t];
    for (int b = 0; b < blocks; ++b) hist[(int64_t)b * kRadix + t] += base;
}

__global__ __launch_bounds__(kBlock) void sort_scatter_kernel(int64_t n, int64_t rows_per_block,
                                                               const int32_t *__restrict__ labels,
                                                               const int32_t *__restrict__ order_in, int shift,
                                                               const int32_t *__restrict__ offsets,
                                                               int32_t *__restrict__ order_out,
                                                               int32_t *__restrict__ new_id) {
    __shared__ int32_t running[kRadix];
    __shared__ int32_t wcnt[kSortWaves][kRadix];
    const int t = threadIdx.x, wave = t >> 6;
    running[t] = offsets[(int64_t)blockIdx.x * kRadix + t];
    for (int w = 0; w < kSortWaves; ++w) wcnt[w][t] = 0;
    __syncthreads();
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    for (int64_t tile = b; tile < e; tile += kBlock) {
        const int64_t i = tile + t;
        const bool valid = i < e;
        int32_t v = 0;
        const int32_t key = valid ? sort_key(labels, order_in, i, shift, &v) : 0;
        // lanes of this wave that hold the same digit
        uint64_t peers = __ballot(valid);
        for (int bit = 0; bit < 8; ++bit) {
            const uint64_t m = __ballot((key >> bit) & 1);
            peers &= ((key >> bit) & 1) ? m : ~m;
        }
        const int rank = __popcll(peers & lanemask_lt());
        if (valid && rank == 0) wcnt[wave][key] = __popcll(peers);
        __syncthreads();
        if (valid) {
            int32_t pos = running[key] + rank;
            for (int w = 0; w < wave; ++w) pos += wcnt[w][key];
            order_out[pos] = v;
            if (new_id) new_id[v] = pos;
        }
        __syncthreads();
        int32_t add = 0;
        for (int w = 0; w < kSortWaves; ++w) { add += wcnt[w][t]; wcnt[w][t] = 0; }
        running[t] += add;
        __syncthreads();
    }
}

}  // namespace

size_t sort_hist_elems() { return (size_t)kSortBlocksMax * kRadix; }

GraphWs carve_graph_ws(int64_t n, int64_t nnz, int32_t k, void *ws) {
    (void)nnz; (void)k;
    Carver c(ws);
    GraphWs w{};
    w.partial = c.take<int64_t>(kGraphBlocksMax);
    w.sort_hist = c.take<int32_t>(sort_hist_elems());
    w.order_tmp = c.take<int32_t>((size_t)n);
    w.order_tmp2 = c.take<int32_t>((size_t)n);
    w.bytes = align_up(c.used, 256);
    return w;
}

int launch_partition_quality(int64_t n, int64_t nnz, int32_t k, const void *rowptr, bool i64, const int32_t *colidx,
                             const int32_t *labels, int64_t *cut, int64_t *sizes, const GraphWs &w, hipStream_t s) {
    (void)w;
    fill_i64_kernel<<<(unsigned)ceil_div(k, kBlock), kBlock, 0, s>>>(sizes, k, cut, 1);
    EP_LAUNCH_CHECK();
    const int hist_blocks = (int)std::min<int64_t>(2048, ceil_div(n, kBlock * 8));
    label_hist_kernel<<<hist_blocks, kBlock, 0, s>>>(n, k, labels, sizes);
    EP_LAUNCH_CHECK();
    if (nnz > 0) {
        const int64_t blocks = ceil_div(nnz, (int64_t)kBlock * kEdgesPerThread);
        auto out = reinterpret_cast<unsigned long long *>(cut);
        ProfScope prof(EP_PROF_EDGE_SWEEP, s);
        if (i64)
            edge_sweep_kernel<int64_t, true><<<(unsigned)blocks, kBlock, 0, s>>>(
                n, nnz, k, static_cast<const int64_t *>(rowptr), colidx, labels, out);
        else
            edge_sweep_kernel<int32_t, true><<<(unsigned)blocks, kBlock, 0, s>>>(
                n, nnz, k, static_cast<const int32_t *>(rowptr), colidx, labels, out);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

int launch_edge_gap(int64_t n, int64_t nnz, const void *rowptr, bool i64, const int32_t *colidx,
                    const int32_t *new_id, uint64_t *out64, EdgeReduce what, const GraphWs &w, hipStream_t s) {
    (void)w;
    fill_i64_kernel<<<1, kBlock, 0, s>>>(reinterpret_cast<int64_t *>(out64), 1, nullptr, 0);
    EP_LAUNCH_CHECK();
    if (nnz <= 0) return EP_OK;
    auto out = reinterpret_cast<unsigned long long *>(out64);
    ProfScope prof(EP_PROF_EDGE_SWEEP, s);
    if (what == EdgeReduce::GapSum) {
        const int64_t blocks = ceil_div(nnz, (int64_t)kBlock * kEdgesPerThread);
        if (i64)
            edge_sweep_kernel<int64_t, false><<<(unsigned)blocks, kBlock, 0, s>>>(
                n, nnz, 0, static_cast<const int64_t *>(rowptr), colidx, new_id, out);
        else
            edge_sweep_kernel<int32_t, false><<<(unsigned)blocks, kBlock, 0, s>>>(
                n, nnz, 0, static_cast<const int32_t *>(rowptr), colidx, new_id, out);
    } else {
        const int64_t blocks = ceil_div(n, kBlock);
        if (i64)
            bandwidth_kernel<int64_t><<<(unsigned)blocks, kBlock, 0, s>>>(
                n, nnz, static_cast<const int64_t *>(rowptr), colidx, new_id, out);
        else
            bandwidth_kernel<int32_t><<<(unsigned)blocks, kBlock, 0, s>>>(
                n, nnz, static_cast<const int32_t *>(rowptr), colidx, new_id, out);
    }
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_sort_by_label(int64_t n, int32_t k, const int32_t *labels, int32_t *new_id, int32_t *order,
                         int32_t *tmp, int32_t *hist, hipStream_t s) {
    const int passes = k <= kRadix ? 1 : 2;          // k <= 65536
    int64_t rows_per_block = ceil_div(n, kSortBlocksMax);
    rows_per_block = ceil_div(rows_per_block, kBlock) * kBlock;
    const int blocks = (int)ceil_div(n, rows_per_block);
    // ping-pong so that the last pass writes `order`
    const int32_t *src = nullptr;                      // identity
    for (int pass = 0; pass < passes; ++pass) {
        int32_t *dst = (passes - pass) % 2 == 1 ? order : tmp;
        const bool last = pass == passes - 1;
        sort_hist_kernel<<<blocks, kBlock, 0, s>>>(n, rows_per_block, labels, src, 8 * pass, hist);
        EP_LAUNCH_CHECK();
        sort_scan_kernel<<<1, kRadix, 0, s>>>(hist, blocks);
        EP_LAUNCH_CHECK();
        sort_scatter_kernel<<<blocks, kBlock, 0, s>>>(n, rows_per_block, labels, src, 8 * pass, hist, dst,
                                                      last ? new_id : nullptr);
        EP_LAUNCH_CHECK();
        src = dst;
    }
    return EP_OK;
}

}  // namespace ep
