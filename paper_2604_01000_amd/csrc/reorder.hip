// The graph rewritten under the new vertex ids of the EmbedPart paper's Sec. "Extension to Graph
// Reordering": the id of a vertex is its position in memory, so giving the vertices of one
// partition consecutive ids means moving the rows of the CSR.  Row pi(v) of the result holds the
// neighbours of v under their new ids, ascending.
//
//   1. Row starts: the degree of new row r is the degree of old row order[r]; an exclusive scan in
//      three kernels (sums per 2,048 rows, one workgroup scanning those sums, the rows again).
//   2. Entries: the new column array is cut into windows of 4,096 positions (the first row starting
//      at or after every window boundary is found by one binary search per window, all in
//      parallel).  A workgroup owns the rows that START in its window.  Every non-empty owned row
//      marks its first position in LDS, a propagation of the marks (wave scans, no search) tells
//      every position its row, and the entries are gathered position by position (reads of an old
//      row stay coalesced) and relabelled through new_id.  Every row is then sorted by a bitonic
//      network of its own in a padded power-of-two region of LDS, all rows of the window in the
//      same sequence of steps (see "all short rows of a window sorted at once" below), and the
//      columns go back coalesced.  Rows of at most 4,096 entries end at most 4,096 positions past
//      the window, so 8,192 positions and fewer than 16,384 padded slots (64 KB) always hold them.
//   3. A row longer than a window is necessarily the last row starting in its window (the next row
//      starts past the window's end).  Its workgroup sorts it afterwards in place in global
//      memory: tiles of 16,384 entries are sorted in LDS, merge steps whose partners are 16,384 or
//      more apart run on global memory, the rest of every merge again tile by tile in LDS.
// The bitonic network is the one that compares i with its mirror image in the first step of every
// merge, so every compare puts the smaller key at the lower index and positions past the end of
// the data behave as +infinity without ever being touched: any length works, not only powers of 2.
// Everything is integer and the sorted order of a row is unique: the result is bit-reproducible.
#include <algorithm>

#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
constexpr int kScanPer = 8;                     // consecutive rows per thread in the scan kernels
constexpr int kScanTile = kBlock * kScanPer;    // rows per workgroup
constexpr int kScanTop = 1024;                  // threads of the kernel that scans the workgroup sums
constexpr int kWin = 4096;                      // positions of new_colidx per window
constexpr int kCap = 2 * kWin;                  // positions held in LDS
constexpr int kTile32 = 2 * kCap;               // entries of a long row sorted in the same LDS at once

template <typename RowT>
__device__ __forceinline__ int64_t new_row_degree(int64_t n, const RowT *__restrict__ rowptr,
                                                  const int32_t *__restrict__ order, int64_t r) {
    if (r >= n) return 0;
    const int32_t v = order[r];
    if ((uint32_t)v >= (uint64_t)n) return 0;
    return (int64_t)rowptr[v + 1] - (int64_t)rowptr[v];
}

// Exclusive prefix of one value per thread over the workgroup (NT threads); *total gets the sum.
template <int NT>
__device__ __forceinline__ int64_t block_exclusive_scan(int64_t mine, int64_t *sh, int64_t *total) {
    const int t = threadIdx.x;
    sh[t] = mine;
    __syncthreads();
    for (int step = 1; step < NT; step <<= 1) {
        const int64_t add = t >= step ? sh[t - step] : 0;
        __syncthreads();
        sh[t] += add;
        __syncthreads();
    }
    const int64_t incl = sh[t];
    *total = sh[NT - 1];
    __syncthreads();
    return incl - mine;
}

template <typename RowT>
__global__ __launch_bounds__(kBlock) void reorder_degree_sums_kernel(int64_t n, const RowT *__restrict__ rowptr,
                                                                      const int32_t *__restrict__ order,
                                                                      int64_t *__restrict__ block_sums) {
    __shared__ int64_t sh[kBlock];
    const int64_t first = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPer;
    int64_t mine = 0;
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) mine += new_row_degree(n, rowptr, order, first + i);
    int64_t total;
    block_exclusive_scan<kBlock>(mine, sh, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// One workgroup: block_sums[b] becomes the sum of the workgroups before b; *total the sum of all.
__global__ __launch_bounds__(kScanTop) void reorder_scan_sums_kernel(int64_t blocks, int64_t *__restrict__ block_sums,
                                                                      int64_t *__restrict__ total_out) {
    __shared__ int64_t sh[kScanTop];
    const int64_t per = (blocks + kScanTop - 1) / kScanTop;
    const int64_t lo = std::min<int64_t>(blocks, (int64_t)threadIdx.x * per), hi = std::min<int64_t>(blocks, lo + per);
    int64_t mine = 0;
    for (int64_t b = lo; b < hi; ++b) mine += block_sums[b];
    int64_t total;
    int64_t run = block_exclusive_scan<kScanTop>(mine, sh, &total);
    for (int64_t b = lo; b < hi; ++b) {
        const int64_t v = block_sums[b];
        block_sums[b] = run;
        run += v;
    }
    if (threadIdx.x == 0) *total_out = total;
}

template <typename RowT>
__global__ __launch_bounds__(kBlock) void reorder_row_starts_kernel(int64_t n, const RowT *__restrict__ rowptr,
                                                                     const int32_t *__restrict__ order,
                                                                     const int64_t *__restrict__ block_sums,
                                                                     RowT *__restrict__ new_rowptr) {
    __shared__ int64_t sh[kBlock];
    const int64_t first = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPer;
    int64_t deg[kScanPer], mine = 0;
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) {
        deg[i] = new_row_degree(n, rowptr, order, first + i);
        mine += deg[i];
    }
    int64_t total;
    int64_t run = block_sums[blockIdx.x] + block_exclusive_scan<kBlock>(mine, sh, &total);
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) {
        const int64_t r = first + i;
        if (r < n) new_rowptr[r] = (RowT)run;
        run += deg[i];
        if (r == n - 1) new_rowptr[n] = (RowT)run;
    }
}

// First r in [0, n] with rp[r] >= pos (rp[n] >= pos is the caller's business).
template <typename RowT>
__device__ __forceinline__ int64_t first_row_at_or_after(const RowT *__restrict__ rp, int64_t n, int64_t pos) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)rp[mid] >= pos) hi = mid; else lo = mid + 1;
    }
    return lo;
}

template <typename K>
__device__ __forceinline__ void lds_order_pair(K *a, int lo, int hi) {
    const K x = a[lo], y = a[hi];
    if (y < x) { a[lo] = y; a[hi] = x; }
}

// The second and later steps of a merge: partners `stride` apart, strides from_stride, .., 2, 1.
template <typename K>
__device__ __forceinline__ void lds_merge_tail(K *a, int cnt, int from_stride) {
    for (int stride = from_stride; stride >= 1; stride >>= 1) {
        for (int i = threadIdx.x;; i += kBlock) {
            const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
            if (lo + stride >= cnt) break;          // lo grows with i
            lds_order_pair(a, lo, lo + stride);
        }
        __syncthreads();
    }
}

// Sorts a[0 .. cnt) ascending; every thread of the workgroup calls it with the same cnt.
template <typename K>
__device__ __forceinline__ void lds_bitonic_sort(K *a, int cnt) {
    for (int lg = 0; (1 << lg) < cnt; ++lg) {       // merges of 2 * half
        const int half = 1 << lg;
        for (int i = threadIdx.x;; i += kBlock) {
            const int blk = i >> lg, off = i & (half - 1);
            const int lo = (blk << (lg + 1)) + off, hi = (blk << (lg + 1)) + 2 * half - 1 - off;
            if (lo >= cnt) break;                   // lo grows with i
            if (hi < cnt) lds_order_pair(a, lo, hi);
        }
        __syncthreads();
        lds_merge_tail(a, cnt, half >> 1);
    }
}

__device__ __forceinline__ void global_order_pair(uint32_t *d, int64_t lo, int64_t hi) {
    const uint32_t x = d[lo], y = d[hi];
    if (y < x) { d[lo] = y; d[hi] = x; }
}

// A row of len > kWin entries, already relabelled in d[0 .. len): sorted in place by one workgroup.
__device__ void sort_long_row(uint32_t *__restrict__ d, int64_t len, uint32_t *tile) {
    for (int64_t base = 0; base < len; base += kTile32) {
        const int cnt = (int)std::min<int64_t>(kTile32, len - base);
        for (int i = threadIdx.x; i < cnt; i += kBlock) tile[i] = d[base + i];
        __syncthreads();
        lds_bitonic_sort(tile, cnt);
        for (int i = threadIdx.x; i < cnt; i += kBlock) d[base + i] = tile[i];
        __syncthreads();
    }
    for (int lg = __builtin_ctz(kTile32); ((int64_t)1 << lg) < len; ++lg) {     // merges of 2 * half entries
        const int64_t half = (int64_t)1 << lg;
        for (int64_t i = threadIdx.x;; i += kBlock) {
            const int64_t blk = i >> lg, off = i & (half - 1);
            const int64_t lo = (blk << (lg + 1)) + off, hi = (blk << (lg + 1)) + 2 * half - 1 - off;
            if (lo >= len) break;
            if (hi < len) global_order_pair(d, lo, hi);
        }
        __syncthreads();
        for (int64_t stride = half >> 1; stride >= kTile32; stride >>= 1) {
            for (int64_t i = threadIdx.x;; i += kBlock) {
                const int64_t lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
                if (lo + stride >= len) break;
                global_order_pair(d, lo, lo + stride);
            }
            __syncthreads();
        }
        for (int64_t base = 0; base < len; base += kTile32) {
            const int cnt = (int)std::min<int64_t>(kTile32, len - base);
            for (int i = threadIdx.x; i < cnt; i += kBlock) tile[i] = d[base + i];
            __syncthreads();
            lds_merge_tail(tile, cnt, kTile32 / 2);
            for (int i = threadIdx.x; i < cnt; i += kBlock) d[base + i] = tile[i];
            __syncthreads();
        }
    }
}

// window_rows[b] = the first row that starts at or after position b * kWin (n past the last entry).
template <typename RowT>
__global__ __launch_bounds__(kBlock) void reorder_window_rows_kernel(int64_t n, int64_t nnz, int64_t windows,
                                                                      const RowT *__restrict__ new_rowptr,
                                                                      const int64_t *__restrict__ total,
                                                                      int64_t *__restrict__ window_rows) {
    const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (b > windows || *total != nnz) return;
    const int64_t pos = b * kWin;
    window_rows[b] = pos >= nnz ? n : first_row_at_or_after(new_rowptr, n, pos);
}

// ---- all short rows of a window sorted at once -------------------------------------------------
// Every row gets a region of 2^p slots, p = ceil(log2(length)), filled up with +infinity.  The
// regions are laid out by descending p, so every region is aligned to its own size and the slots
// that still take part in the merges of 2^(lg+1) entries are a prefix: bound = first slot of the
// classes p <= lg.  The network is then purely positional (no test per entry, no idle thread but in
// the last iteration), LDS traffic follows sum 2^p p^2 over the rows, and the last three steps of
// every merge (partners 4, 2, 1 apart) run in registers on 8 consecutive slots per thread.
constexpr int kClasses = 13;                    // p = 0 .. 12 (rows of up to kWin = 2^12 entries)
constexpr uint32_t kPadding = 0xFFFFFFFFu;

__device__ __forceinline__ void order_if(bool on, uint32_t &a, uint32_t &b) {
    const uint32_t lo = a < b ? a : b, hi = a < b ? b : a;
    a = on ? lo : a;
    b = on ? hi : b;
}

// Merges of 2, 4 and 8 entries, whole, on 8 consecutive slots per thread.  end0 / end1 / end2: first
// slot that takes no part in the merges of 2 / 4 / 8 (multiples of 2 / 4 / 8).
__device__ __forceinline__ void sort_groups_of_8(uint32_t *pad, int end0, int end1, int end2) {
    for (int g = threadIdx.x; 8 * g < end0; g += kBlock) {
        uint4 a = reinterpret_cast<uint4 *>(pad)[2 * g], b = reinterpret_cast<uint4 *>(pad)[2 * g + 1];
        const int at = 8 * g;
        order_if(at + 2 <= end0, a.x, a.y); order_if(at + 4 <= end0, a.z, a.w);
        order_if(at + 6 <= end0, b.x, b.y); order_if(at + 8 <= end0, b.z, b.w);
        const bool a1 = at + 4 <= end1, b1 = at + 8 <= end1;
        order_if(a1, a.x, a.w); order_if(a1, a.y, a.z); order_if(b1, b.x, b.w); order_if(b1, b.y, b.z);
        order_if(a1, a.x, a.y); order_if(a1, a.z, a.w); order_if(b1, b.x, b.y); order_if(b1, b.z, b.w);
        const bool c2 = at + 8 <= end2;
        order_if(c2, a.x, b.w); order_if(c2, a.y, b.z); order_if(c2, a.z, b.y); order_if(c2, a.w, b.x);
        order_if(c2, a.x, a.z); order_if(c2, a.y, a.w); order_if(c2, b.x, b.z); order_if(c2, b.y, b.w);
        order_if(c2, a.x, a.y); order_if(c2, a.z, a.w); order_if(c2, b.x, b.y); order_if(c2, b.z, b.w);
        reinterpret_cast<uint4 *>(pad)[2 * g] = a;
        reinterpret_cast<uint4 *>(pad)[2 * g + 1] = b;
    }
    __syncthreads();
}

// Partners 4, 2 and 1 apart over the slots below `bound` (a multiple of 8).
__device__ __forceinline__ void merge_tail_of_8(uint32_t *pad, int bound) {
    for (int g = threadIdx.x; 8 * g < bound; g += kBlock) {
        uint4 a = reinterpret_cast<uint4 *>(pad)[2 * g], b = reinterpret_cast<uint4 *>(pad)[2 * g + 1];
        order_if(true, a.x, b.x); order_if(true, a.y, b.y); order_if(true, a.z, b.z); order_if(true, a.w, b.w);
        order_if(true, a.x, a.z); order_if(true, a.y, a.w); order_if(true, b.x, b.z); order_if(true, b.y, b.w);
        order_if(true, a.x, a.y); order_if(true, a.z, a.w); order_if(true, b.x, b.y); order_if(true, b.z, b.w);
        reinterpret_cast<uint4 *>(pad)[2 * g] = a;
        reinterpret_cast<uint4 *>(pad)[2 * g + 1] = b;
    }
    __syncthreads();
}

// One positional step over the pairs below bound / 2; four pairs of a thread are read before the
// first is written.  mirror: the step that opens a merge of 2 * half entries (partner = mirror
// image); otherwise partners are `stride` apart.
template <bool MIRROR>
__device__ __forceinline__ void positional_step(uint32_t *pad, int bound, int lg, int stride) {
    constexpr int kAtOnce = 4;
    const int pairs = bound >> 1;
    for (int t0 = threadIdx.x; t0 < pairs; t0 += kAtOnce * kBlock) {
        int lo[kAtOnce], hi[kAtOnce];
        uint32_t x[kAtOnce], y[kAtOnce];
#pragma unroll
        for (int e = 0; e < kAtOnce; ++e) {
            const int t = min(t0 + e * kBlock, pairs - 1);          // a repeated pair is harmless: same values
            if (MIRROR) {
                const int half = 1 << lg, blk = t >> lg, off = t & (half - 1);
                lo[e] = (blk << (lg + 1)) + off;
                hi[e] = (blk << (lg + 1)) + 2 * half - 1 - off;
            } else {
                lo[e] = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                hi[e] = lo[e] + stride;
            }
            x[e] = pad[lo[e]];
            y[e] = pad[hi[e]];
        }
#pragma unroll
        for (int e = 0; e < kAtOnce; ++e)
            if (y[e] < x[e]) { pad[lo[e]] = y[e]; pad[hi[e]] = x[e]; }
    }
    __syncthreads();
}

// class_base[p]: first slot of the rows of class p (classes laid out from kClasses - 1 down to 0);
// classes: the number of classes in use (largest p + 1).
__device__ __forceinline__ void sort_regions(uint32_t *pad, const int *class_base, int classes) {
    sort_groups_of_8(pad, class_base[0], classes > 1 ? class_base[1] : 0, classes > 2 ? class_base[2] : 0);
    for (int lg = 3; lg < classes - 1; ++lg) {          // merges of 2^(lg+1) entries: classes above lg
        const int bound = class_base[lg];
        positional_step<true>(pad, bound, lg, 0);
        for (int stride = (1 << lg) >> 1; stride >= 8; stride >>= 1) positional_step<false>(pad, bound, lg, stride);
        merge_tail_of_8(pad, bound);
    }
}

template <typename RowT>
__global__ __launch_bounds__(kBlock) void reorder_rows_kernel(int64_t n, int64_t nnz, const RowT *__restrict__ rowptr,
                                                               const int32_t *__restrict__ colidx,
                                                               const int32_t *__restrict__ new_id,
                                                               const int32_t *__restrict__ order,
                                                               const RowT *__restrict__ new_rowptr,
                                                               const int64_t *__restrict__ total,
                                                               const int64_t *__restrict__ window_rows,
                                                               int32_t *__restrict__ new_colidx) {
    constexpr int kChunks = kCap / kWave, kPer = kCap / kBlock, kWaves = kBlock / kWave, kGroup = 32;
    __shared__ __attribute__((aligned(16))) uint32_t lds[2 * kCap];   // marks | regions of the rows, then the padded slots
    __shared__ uint32_t chunk_mark[kChunks];       // largest mark of a chunk of 64 positions, then the carry into it
    __shared__ int64_t plan[2];
    __shared__ int class_count[kClasses], class_base[kClasses + 1];
    // `order` was not a permutation of the rows: the row starts do not add up, nothing is written.
    if (*total != nnz) return;
    uint32_t *mark = lds, *region = lds + kCap;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t r0 = window_rows[blockIdx.x], r1 = window_rows[blockIdx.x + 1];
    const int64_t s0 = (int64_t)new_rowptr[r0], s1 = (int64_t)new_rowptr[r1];
    if (s1 == s0) return;                                        // no entry starts here (uniform)
    auto relabel = [&](int32_t col) -> uint32_t {
        return (uint32_t)col < (uint64_t)n ? (uint32_t)new_id[col] : (uint32_t)col;
    };

    // Marks: the first position of every owned row of at most kWin entries gets (row - r0 + 1), and
    // the row takes the next region of its class.  A longer row can only be the last owned one; it
    // is set aside.
    const int span = (int)std::min<int64_t>(kCap, s1 - s0);
    for (int i = threadIdx.x; i < span; i += kBlock) mark[i] = 0;
    if (threadIdx.x < kClasses) class_count[threadIdx.x] = 0;
    if (threadIdx.x == 0) { plan[0] = s1; plan[1] = -1; }
    __syncthreads();
    for (int64_t r = r0 + threadIdx.x; r < r1; r += kBlock) {
        const int64_t st = (int64_t)new_rowptr[r], en = (int64_t)new_rowptr[r + 1];
        if (en - st > kWin) { plan[0] = st; plan[1] = r; }
        else if (en > st && st - s0 < span) {
            const int len = (int)(en - st), p = len <= 1 ? 0 : 32 - __builtin_clz(len - 1);
            mark[st - s0] = (uint32_t)(r - r0 + 1);
            region[st - s0] = (uint32_t)p << 16 | (uint32_t)atomicAdd(&class_count[p], 1);
        }
    }
    __syncthreads();
    const int64_t short_end = plan[0], long_row = plan[1];
    const int64_t cnt64 = short_end - s0;
    if (cnt64 > span) return;                       // cannot happen with monotone row starts
    const int cnt = (int)cnt64;
    if (cnt > 0) {
        if (threadIdx.x == 0) {
            int at = 0;
            for (int p = kClasses - 1; p >= 0; --p) { class_base[p] = at; at += class_count[p] << p; }
            class_base[kClasses] = at;               // slots in use: less than 2 * cnt
        }
        // Every position learns its row: the marks are propagated forward (they grow with the position).
        // Position i = threadIdx.x + kBlock * j lies in chunk wave + kWaves * j of 64 positions.
        const int chunks = (cnt + kWave - 1) / kWave;
        uint32_t own[kPer];                          // running maximum inside the chunk
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int c = wave + kWaves * j, i = c * kWave + lane;
            own[j] = 0;
            if (c < chunks) {                        // uniform over the wave
                own[j] = wave_inclusive_max(i < cnt ? mark[i] : 0u);
                if (lane == kWave - 1) chunk_mark[c] = own[j];
            }
        }
        __syncthreads();
        if (wave == 0) {                            // carry into chunk c = the largest mark before it
            uint32_t carry = 0;
            for (int c0 = 0; c0 < chunks; c0 += kWave) {
                const int c = c0 + lane;
                const uint32_t mine = c < chunks ? chunk_mark[c] : 0u;
                const uint32_t incl = wave_inclusive_max(mine);
                const uint32_t before = (uint32_t)__shfl_up((int)incl, 1, kWave);
                const uint32_t excl = lane == 0 ? 0u : before;
                if (c < chunks) chunk_mark[c] = excl > carry ? excl : carry;
                const uint32_t all = (uint32_t)__shfl((int)incl, kWave - 1, kWave);
                carry = all > carry ? all : carry;
            }
        }
        __syncthreads();
        // Gather.  The chain position -> row -> old row -> old entry -> new id is four dependent loads;
        // each link is issued for kGroup positions of the thread at once so that their latencies overlap.
        uint32_t renamed[kPer];
        int slot[kPer];                              // where the entry waits in the padded layout, -1: none
#pragma unroll
        for (int g = 0; g < kPer; g += kGroup) {
            uint32_t m[kGroup];
#pragma unroll
            for (int e = 0; e < kGroup; ++e) {
                const int c = wave + kWaves * (g + e), i = c * kWave + lane;
                m[e] = 0;
                if (i < cnt) m[e] = own[g + e] > chunk_mark[c] ? own[g + e] : chunk_mark[c];
            }
            int32_t v[kGroup];
            int64_t first[kGroup];
#pragma unroll
            for (int e = 0; e < kGroup; ++e) {       // m > 0 wherever i < cnt: position 0 is the start of a row
                const int64_t r = r0 + (m[e] > 0 ? (int64_t)m[e] - 1 : 0);
                v[e] = order[r];
                first[e] = (int64_t)new_rowptr[r];
            }
            int64_t from[kGroup];
#pragma unroll
            for (int e = 0; e < kGroup; ++e) {
                const int i = threadIdx.x + kBlock * (g + e);
                from[e] = m[e] > 0 ? (int64_t)rowptr[v[e]] + (s0 + i - first[e]) : 0;
            }
            int32_t col[kGroup];
#pragma unroll
            for (int e = 0; e < kGroup; ++e) col[e] = colidx[from[e]];
#pragma unroll
            for (int e = 0; e < kGroup; ++e) {
                const int i = threadIdx.x + kBlock * (g + e);
                renamed[g + e] = relabel(col[e]);
                slot[g + e] = -1;
                if (m[e] > 0) {
                    const int start = (int)(first[e] - s0);
                    const uint32_t reg = region[start];
                    const int p = (int)(reg >> 16);
                    slot[g + e] = class_base[p] + ((int)(reg & 0xFFFF) << p) + (i - start);
                }
            }
        }
        __syncthreads();                             // marks and regions are not read any more
        uint32_t *pad = lds;
        const int slots = class_base[kClasses];
        int classes = kClasses;
        while (classes > 1 && class_count[classes - 1] == 0) --classes;   // uniform
        for (int i = threadIdx.x; i < (slots + 7) / 8 * 8; i += kBlock) pad[i] = kPadding;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (slot[j] >= 0) pad[slot[j]] = renamed[j];
        __syncthreads();
        sort_regions(pad, class_base, classes);
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (slot[j] >= 0) new_colidx[s0 + threadIdx.x + kBlock * j] = (int32_t)pad[slot[j]];
    }
    if (long_row >= 0) {                             // uniform over the workgroup
        __syncthreads();
        const int32_t v = order[long_row];
        const int64_t len = s1 - short_end;
        const int32_t *src = colidx + (int64_t)rowptr[v];
        uint32_t *dst = reinterpret_cast<uint32_t *>(new_colidx + short_end);
        for (int64_t j = threadIdx.x; j < len; j += kBlock) dst[j] = relabel(src[j]);
        __syncthreads();
        sort_long_row(dst, len, lds);
    }
}

}  // namespace

ReorderWs carve_reorder_ws(int64_t n, int64_t nnz, void *ws) {
    Carver c(ws);
    ReorderWs w{};
    w.block_sums = c.take<int64_t>((size_t)ceil_div(n, kScanTile));
    w.total = c.take<int64_t>(1);
    w.window_rows = c.take<int64_t>((size_t)ceil_div(nnz, kWin) + 1);
    w.bytes = align_up(c.used, 256);
    return w;
}

template <typename RowT>
static int launch_reorder_t(int64_t n, int64_t nnz, const RowT *rowptr, const int32_t *colidx, const int32_t *new_id,
                            const int32_t *order, RowT *new_rowptr, int32_t *new_colidx, const ReorderWs &w,
                            hipStream_t s) {
    const int64_t blocks = ceil_div(n, kScanTile);
    reorder_degree_sums_kernel<RowT><<<(unsigned)blocks, kBlock, 0, s>>>(n, rowptr, order, w.block_sums);
    EP_LAUNCH_CHECK();
    reorder_scan_sums_kernel<<<1, kScanTop, 0, s>>>(blocks, w.block_sums, w.total);
    EP_LAUNCH_CHECK();
    reorder_row_starts_kernel<RowT><<<(unsigned)blocks, kBlock, 0, s>>>(n, rowptr, order, w.block_sums, new_rowptr);
    EP_LAUNCH_CHECK();
    if (nnz <= 0) return EP_OK;
    const int64_t windows = ceil_div(nnz, kWin);
    reorder_window_rows_kernel<RowT><<<(unsigned)ceil_div(windows + 1, kBlock), kBlock, 0, s>>>(
        n, nnz, windows, new_rowptr, w.total, w.window_rows);
    EP_LAUNCH_CHECK();
    reorder_rows_kernel<RowT><<<(unsigned)windows, kBlock, 0, s>>>(n, nnz, rowptr, colidx, new_id, order, new_rowptr,
                                                                   w.total, w.window_rows, new_colidx);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_reorder(int64_t n, int64_t nnz, const void *rowptr, bool i64, const int32_t *colidx, const int32_t *new_id,
                   const int32_t *order, void *new_rowptr, int32_t *new_colidx, const ReorderWs &w, hipStream_t s) {
    if (ceil_div(nnz, kWin) >= ((int64_t)1 << 31)) return EP_EUNSUPPORTED;
    return i64 ? launch_reorder_t<int64_t>(n, nnz, static_cast<const int64_t *>(rowptr), colidx, new_id, order,
                                           static_cast<int64_t *>(new_rowptr), new_colidx, w, s)
               : launch_reorder_t<int32_t>(n, nnz, static_cast<const int32_t *>(rowptr), colidx, new_id, order,
                                           static_cast<int32_t *>(new_rowptr), new_colidx, w, s);
}

}  // namespace ep
