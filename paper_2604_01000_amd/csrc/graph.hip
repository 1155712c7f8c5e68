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

__global__ __launch_bounds__(kBlock) void ep_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                          int64_t count) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += stride) dst[i] = src[i];
}

__global__ void fill_i64_kernel(int64_t *a, int64_t na, int64_t *b, int64_t nb) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < na) a[i] = 0;
    if (b && i < nb) b[i] = 0;
}

// ---- partition sizes (and the compact label copy the sweep gathers from) -------------------
constexpr int kLdsHistMax = 16384;  // 64 KB of LDS
constexpr int kByteLabelMaxK = 255;   // labels fit a byte with 255 left over as "out of range"

// sizes[p] += #{v : labels[v] == p}; with label8 != nullptr also label8[v] = labels[v] (255 when
// out of range).  Gathering bytes instead of words keeps the label vector of a large graph in
// cache (2.4 MB instead of 9.8 MB at 2.45 M vertices, 111 MB instead of 444 MB at 111 M).
__global__ __launch_bounds__(kBlock) void label_prep_kernel(int64_t n, int32_t k, const int32_t *__restrict__ labels,
                                                             uint8_t *__restrict__ label8,
                                                             int64_t *__restrict__ sizes) {
    __shared__ int32_t hist[kLdsHistMax];
    const bool in_lds = k <= kLdsHistMax;
    if (in_lds) {
        for (int j = threadIdx.x; j < k; j += kBlock) hist[j] = 0;
        __syncthreads();
    }
    // four consecutive labels per thread: one 16-byte load and one 4-byte store of the byte copy (both arrays are
    // 16-byte aligned allocations; the last, partial group goes element by element)
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int64_t groups = n / 4;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const bool vec = (reinterpret_cast<uintptr_t>(labels) & 15) == 0 && (reinterpret_cast<uintptr_t>(label8) & 3) == 0;
    auto count = [&](int32_t l) {
        if (in_lds) atomicAdd(&hist[l], 1);
        else atomicAdd(reinterpret_cast<unsigned long long *>(&sizes[l]), 1ull);
    };
    const int64_t first_single = vec ? 4 * groups : 0;
    if (vec) {
        for (int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x; g < groups; g += stride) {
            const i32x4 l4 = *reinterpret_cast<const i32x4 *>(labels + 4 * g);
            uint32_t packed = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool ok = l4[q] >= 0 && l4[q] < k;
                packed |= (ok ? (uint32_t)l4[q] & 0xffu : 255u) << (8 * q);
                if (ok) count(l4[q]);
            }
            if (label8) *reinterpret_cast<uint32_t *>(label8 + 4 * g) = packed;
        }
    }
    for (int64_t i = first_single + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const int32_t l = labels[i];
        const bool ok = l >= 0 && l < k;
        if (label8) label8[i] = ok ? (uint8_t)l : (uint8_t)255;
        if (ok) count(l);
    }
    if (in_lds) {
        __syncthreads();
        for (int j = threadIdx.x; j < k; j += kBlock)
            if (hist[j]) atomicAdd(reinterpret_cast<unsigned long long *>(&sizes[j]), (unsigned long long)hist[j]);
    }
}

// ---- CSR sweeps -------------------------------------------------------------------------
// L consecutive lanes own one row and stride over its entries, so rows are read as contiguous
// runs and a wave covers 64 / L neighbouring rows per step; L follows the mean row length.
// Workgroups take blocks of rows round-robin, which spreads heavy rows of a skewed degree
// distribution over the grid.
enum SweepOp { kCut = 0, kGapSum = 1, kBandwidth = 2 };

template <typename RowT, typename AttrT, int L, int OP>
__global__ __launch_bounds__(kBlock) void csr_sweep_kernel(int64_t n, int64_t nnz, int32_t k,
                                                            const RowT *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            const AttrT *__restrict__ attr,
                                                            unsigned long long *__restrict__ out) {
    __shared__ uint64_t red[kBlock / 64];
    constexpr int kRowsPerBlock = kBlock / L;
    const int sub = threadIdx.x % L;
    const int64_t row_in_block = threadIdx.x / L;
    const int64_t blocks_of_rows = (n + kRowsPerBlock - 1) / kRowsPerBlock;
    uint64_t acc = 0;        // per-lane sum (gap, bandwidth)
    uint32_t wave_cut = 0;   // per-wave count (cut), identical in every lane
    for (int64_t rb = blockIdx.x; rb < blocks_of_rows; rb += gridDim.x) {
        const int64_t u = rb * kRowsPerBlock + row_in_block;
        int64_t b = 0, e = 0, au = 0;
        bool u_ok = false;
        if (u < n) {
            b = max((int64_t)rowptr[u], (int64_t)0);
            e = min((int64_t)rowptr[u + 1], nnz);
            au = attr ? (int64_t)attr[u] : u;
            if (OP == kCut) u_ok = sizeof(AttrT) == 1 ? au != 255 : (au >= 0 && au < k);
        }
        uint64_t widest = 0;
        // All lanes of the wave run the same number of steps (until the longest row of the wave is
        // done), so the ballot that counts cut entries is taken with every lane present.
        const int64_t len = e - b;
        for (int64_t t = sub; __ballot(t < len) != 0; t += L) {
            const int64_t p = b + t;
            bool hit = false;
            if (p < e) {
                const int32_t v = colidx[p];
                if (v >= 0 && v < n) {
                    const int64_t av = attr ? (int64_t)attr[v] : (int64_t)v;
                    if (OP == kCut) {
                        const bool v_ok = sizeof(AttrT) == 1 ? av != 255 : (av >= 0 && av < k);
                        hit = u_ok && v_ok && au != av;
                    } else {
                        const uint64_t gap = (uint64_t)(au > av ? au - av : av - au);
                        if (OP == kGapSum) acc += gap; else widest = gap > widest ? gap : widest;
                    }
                }
            }
            if (OP == kCut) wave_cut += (uint32_t)__popcll(__ballot(hit));
        }
        if (OP == kBandwidth) {
            for (int off = L / 2; off > 0; off >>= 1) {
                const uint64_t o = __shfl_xor(widest, off, 64);
                widest = o > widest ? o : widest;
            }
            if (sub == 0) acc += widest;
        }
    }
    if (OP == kCut) acc = (threadIdx.x & 63) == 0 ? wave_cut : 0;
    const uint64_t total = block_sum_u64(acc, red);
    if (threadIdx.x == 0 && total) atomicAdd(out, (unsigned long long)total);
}

// Edge-parallel sweep for sums over entries (cut count, gap sum).  A wave takes 64 consecutive
// rows: their offsets (one coalesced load) and their attributes go to a wave-private LDS window,
// and the rows' entries, which are one contiguous run of colidx, are streamed 256 at a time with
// 16-byte loads, the next step's loads in flight while the current one is worked on.  A lane finds
// the row of its first entry by bisecting the 64 row ends in LDS and walks forward from there,
// so row length (empty rows, hubs) does not change the access pattern.
template <typename RowT, typename AttrT, int OP>
__global__ __launch_bounds__(kBlock) void edge_block_sweep_kernel(int64_t n, int64_t nnz, int32_t k,
                                                                   const RowT *__restrict__ rowptr,
                                                                   const int32_t *__restrict__ colidx,
                                                                   const AttrT *__restrict__ attr,
                                                                   unsigned long long *__restrict__ out) {
    constexpr int kWavesPerBlock = kBlock / 64;
    __shared__ int64_t rp_lds[kWavesPerBlock][66];
    __shared__ int32_t au_lds[kWavesPerBlock][64];
    __shared__ uint64_t red[kWavesPerBlock];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int64_t *rp = rp_lds[wave];
    int32_t *aus = au_lds[wave];
    const int64_t row_blocks = (n + 63) / 64;
    uint64_t acc = 0;
    uint32_t wave_cut = 0;
    for (int64_t rb = (int64_t)blockIdx.x * kWavesPerBlock + wave; rb < row_blocks;
         rb += (int64_t)gridDim.x * kWavesPerBlock) {
        const int64_t r0 = rb * 64;
        {   // window: rp[i] = offset of row r0 + i (clamped into [0, nnz], rows past n are empty)
            const int64_t r = min(r0 + lane, n);
            const int64_t v = min(max((int64_t)rowptr[r], (int64_t)0), nnz);
            rp[lane] = v;
            if (lane == 0) {
                const int64_t rl = min(r0 + 64, n);
                rp[64] = min(max((int64_t)rowptr[rl], (int64_t)0), nnz);
            }
            int32_t a = 0;
            if (r0 + lane < n) a = attr ? (int32_t)attr[r0 + lane] : (int32_t)(r0 + lane);
            aus[lane] = a;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int64_t e_begin = rp[0];
        const int64_t e_end = rp[64];
        const int64_t start = e_begin & ~(int64_t)3;  // 16-byte aligned
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        auto load4 = [&](int64_t p) {
            i32x4 c = {0, 0, 0, 0};
            if (p < e_end) {
                if (p + 3 < nnz) c = *reinterpret_cast<const i32x4 *>(colidx + p);
                else for (int t = 0; t < 4; ++t) if (p + t < nnz) c[t] = colidx[p + t];
            }
            return c;
        };
        // The attribute of an entry's column is a random gather: the gathers of step s + 1 are issued (all
        // four of a lane at once, unconditionally, with the index clamped into range) before step s
        // is worked on, and the entries of step s + 2 are loaded, so a lane has 8 gathers and one
        // 16-byte load in flight instead of one gather at a time.
        struct Gathered {
            int32_t a[4];
        };
        auto gather4 = [&](const i32x4 &c) {
            Gathered gt;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int32_t v = c[t];
                const int32_t vi = (v >= 0 && v < n) ? v : 0;
                gt.a[t] = attr ? (int32_t)attr[vi] : vi;
            }
            return gt;
        };
        i32x4 cur = load4(start + 4 * lane);
        i32x4 nxt = load4(start + 256 + 4 * lane);
        Gathered gcur = gather4(cur);
        for (int64_t p0 = start; p0 < e_end; p0 += 256) {
            const int64_t p = p0 + 4 * lane;
            const i32x4 nn = load4(p + 512);
            const Gathered gnxt = gather4(nxt);
            // j = row (relative to r0) of entry max(p, e_begin): the number of row ends <= it
            int j = 0;
            {
                const int64_t q = max(p, e_begin);
#pragma unroll
                for (int step = 32; step > 0; step >>= 1)
                    if (rp[j + step] <= q) j += step;   // rp[j + step] is the end of row j + step - 1
            }
            int64_t row_end = rp[min(j + 1, 64)];
            int64_t au = aus[min(j, 63)];
            uint32_t hits = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t pe = p + t;
                const bool live = pe >= e_begin && pe < e_end;
                if (live) {
                    while (pe >= row_end) {  // ends: pe < e_end = rp[64]
                        ++j;
                        row_end = rp[j + 1];
                        au = aus[j];
                    }
                    const int32_t v = cur[t];
                    if (v >= 0 && v < n) {
                        const int64_t av = (int64_t)gcur.a[t];
                        if (OP == kCut) {
                            const bool ok = sizeof(AttrT) == 1 ? (au != 255 && av != 255)
                                                               : (au >= 0 && au < k && av >= 0 && av < k);
                            hits += (ok && au != av) ? 1u : 0u;
                        } else {
                            acc += (uint64_t)(au > av ? au - av : av - au);
                        }
                    }
                }
            }
            if (OP == kCut) wave_cut += hits;
            cur = nxt;
            gcur = gnxt;
            nxt = nn;
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (OP == kCut) acc = wave_cut;
    const uint64_t total = block_sum_u64(acc, red);
    if (threadIdx.x == 0 && total) atomicAdd(out, (unsigned long long)total);
}

template <typename RowT, typename AttrT, int OP>
int launch_edge_blocks(int64_t n, int64_t nnz, int32_t k, const RowT *rowptr, const int32_t *colidx,
                       const AttrT *attr, unsigned long long *out, hipStream_t s) {
    const int64_t row_blocks = ceil_div(n, 64);
    const unsigned grid = (unsigned)std::min<int64_t>(ceil_div(row_blocks, kBlock / 64), 256 * 8);
    edge_block_sweep_kernel<RowT, AttrT, OP><<<grid, kBlock, 0, s>>>(n, nnz, k, rowptr, colidx, attr, out);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

template <typename RowT, typename AttrT, int OP>
int launch_sweep(int64_t n, int64_t nnz, int32_t k, const RowT *rowptr, const int32_t *colidx, const AttrT *attr,
                 unsigned long long *out, hipStream_t s) {
    const double mean = (double)nnz / (double)n;
    const int lanes = mean <= 6 ? 4 : mean <= 12 ? 8 : mean <= 24 ? 16 : mean <= 48 ? 32 : 64;
    const int64_t blocks_of_rows = ceil_div(n, kBlock / lanes);
    const unsigned grid = (unsigned)std::min<int64_t>(blocks_of_rows, 256 * 16);
#define EP_SWEEP(L_) csr_sweep_kernel<RowT, AttrT, L_, OP><<<grid, kBlock, 0, s>>>(n, nnz, k, rowptr, colidx, attr, out)
    switch (lanes) {
        case 4: EP_SWEEP(4); break;
        case 8: EP_SWEEP(8); break;
        case 16: EP_SWEEP(16); break;
        case 32: EP_SWEEP(32); break;
        default: EP_SWEEP(64); break;
    }
#undef EP_SWEEP
    EP_LAUNCH_CHECK();
    return EP_OK;
}

template <typename AttrT, int OP>
int launch_sweep_rows(int64_t n, int64_t nnz, int32_t k, const void *rowptr, bool i64, const int32_t *colidx,
                      const AttrT *attr, unsigned long long *out, hipStream_t s) {
    if (OP != kBandwidth)
        return i64 ? launch_edge_blocks<int64_t, AttrT, OP>(n, nnz, k, static_cast<const int64_t *>(rowptr), colidx,
                                                            attr, out, s)
                   : launch_edge_blocks<int32_t, AttrT, OP>(n, nnz, k, static_cast<const int32_t *>(rowptr), colidx,
                                                            attr, out, s);
    return i64 ? launch_sweep<int64_t, AttrT, OP>(n, nnz, k, static_cast<const int64_t *>(rowptr), colidx, attr, out, s)
               : launch_sweep<int32_t, AttrT, OP>(n, nnz, k, static_cast<const int32_t *>(rowptr), colidx, attr, out, s);
}

// ---- stable LSD radix sort of vertex ids by label, 8 bits per pass ----------------------
constexpr int kRadix = 256;
constexpr int kSortWaves = kBlock / 64;

// clamp_k > 0: the keys are labels, and a label outside [0, clamp_k) sorts as clamp_k, behind every valid one.
__device__ __forceinline__ int32_t sort_key(const int32_t *__restrict__ labels, const int32_t *__restrict__ order_in,
                                            int64_t i, int shift, uint32_t clamp_k, int32_t *vertex) {
    const int32_t v = order_in ? order_in[i] : (int32_t)i;
    *vertex = v;
    uint32_t key = (uint32_t)labels[v];
    if (clamp_k) key = min(key, clamp_k);   // a negative label is a large unsigned one
    return (int32_t)((key >> shift) & (kRadix - 1));
}

__global__ __launch_bounds__(kBlock) void sort_hist_kernel(int64_t n, int64_t rows_per_block,
                                                            const int32_t *__restrict__ labels,
                                                            const int32_t *__restrict__ order_in, int shift,
                                                            uint32_t clamp_k, int32_t *__restrict__ hist,
                                                            const int *__restrict__ enable) {
    if (enable && !*enable) return;   // uniform over the grid: a sort whose result nobody will use
    __shared__ int32_t h[kRadix];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    for (int64_t i = b + threadIdx.x; i < e; i += kBlock) {
        int32_t v;
        atomicAdd(&h[sort_key(labels, order_in, i, shift, clamp_k, &v)], 1);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = h[threadIdx.x];  // digit-major
}

// hist is [256][blocks] (digit-major).  Workgroup d scans row d in place (exclusive) and writes the
// row total; the scatter kernel adds the totals of the lower digits itself.
__global__ __launch_bounds__(kRadix) void sort_scan_kernel(int32_t *__restrict__ hist, int blocks,
                                                            int32_t *__restrict__ digit_total,
                                                            const int *__restrict__ enable) {
    if (enable && !*enable) return;
    __shared__ int32_t part[kRadix];
    const int t = threadIdx.x;
    int32_t *row = hist + (int64_t)blockIdx.x * blocks;
    const int chunk = (blocks + kRadix - 1) / kRadix;
    const int b = min(t * chunk, blocks), e = min(b + chunk, blocks);
    int32_t sum = 0;
    for (int i = b; i < e; ++i) sum += row[i];
    part[t] = sum;
    __syncthreads();
    for (int off = 1; off < kRadix; off <<= 1) {  // inclusive scan of the chunk sums
        const int32_t add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    int32_t run = part[t] - sum;
    for (int i = b; i < e; ++i) {
        const int32_t c = row[i];
        row[i] = run;
        run += c;
    }
    if (t == kRadix - 1) digit_total[blockIdx.x] = part[t];
}

__global__ __launch_bounds__(kBlock) void sort_scatter_kernel(int64_t n, int64_t rows_per_block,
                                                               const int32_t *__restrict__ labels,
                                                               const int32_t *__restrict__ order_in, int shift,
                                                               uint32_t clamp_k,
                                                               const int32_t *__restrict__ offsets,
                                                               const int32_t *__restrict__ digit_total,
                                                               int32_t *__restrict__ order_out,
                                                               int32_t *__restrict__ new_id,
                                                               const int *__restrict__ enable) {
    if (enable && !*enable) return;
    __shared__ int32_t running[kRadix];
    __shared__ int32_t wcnt[kSortWaves][kRadix];
    const int t = threadIdx.x, wave = t >> 6;
    {   // first output position of digit t: the totals of the digits below it (exclusive scan in LDS)
        const int32_t mine = digit_total[t];
        running[t] = mine;
        __syncthreads();
        for (int off = 1; off < kRadix; off <<= 1) {
            const int32_t add = t >= off ? running[t - off] : 0;
            __syncthreads();
            running[t] += add;
            __syncthreads();
        }
        const int32_t base = running[t] - mine;
        __syncthreads();
        running[t] = base + offsets[(int64_t)t * gridDim.x + blockIdx.x];
    }
    for (int w = 0; w < kSortWaves; ++w) wcnt[w][t] = 0;
    __syncthreads();
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    for (int64_t tile = b; tile < e; tile += kBlock) {
        const int64_t i = tile + t;
        const bool valid = i < e;
        int32_t v = 0;
        const int32_t key = valid ? sort_key(labels, order_in, i, shift, clamp_k, &v) : 0;
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

int launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
    const int64_t count = (int64_t)(bytes / 16);
    if (count == 0) return EP_OK;
    const unsigned grid = (unsigned)std::min<int64_t>(ceil_div(count, kBlock), 256 * 16);
    ep_copy_kernel<<<grid, kBlock, 0, s>>>(static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), count);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

size_t sort_hist_elems() { return (size_t)kSortBlocksMax * kRadix + kRadix; }  // histograms + digit totals

GraphWs carve_graph_ws(int64_t n, int64_t nnz, int32_t k, void *ws, bool with_buckets) {
    Carver c(ws);
    GraphWs w{};
    w.partial = c.take<int64_t>(kGraphBlocksMax);
    w.sort_hist = c.take<int32_t>(sort_hist_elems());
    w.order_tmp = c.take<int32_t>((size_t)n);
    w.order_tmp2 = c.take<int32_t>((size_t)n);
    w.label8 = c.take<uint8_t>((size_t)n);
    const BucketPlan pl = with_buckets ? bucket_plan(n, nnz, k) : BucketPlan{0, 0};
    if (pl.shift) {
        w.bucket_hist = c.take<int64_t>(kBucketsMax);
        w.bucket_base = c.take<int64_t>(kBucketsMax + 1);
        w.bucket_cursor = c.take<int64_t>((size_t)kBucketsMax * 16);   // one 128-byte line per cursor
        w.bucket_items = c.take<int64_t>(kBucketsMax + 1);
        w.bucket_dropped = c.take<int64_t>(1);
        w.bucket_records = c.take<uint32_t>(bucket_record_slots(nnz, pl));
    }
    w.bytes = align_up(c.used, 256);
    return w;
}

int launch_partition_quality(int64_t n, int64_t nnz, int32_t k, const void *rowptr, bool i64, const int32_t *colidx,
                             const int32_t *labels, int64_t *cut, int64_t *sizes, const GraphWs &w, hipStream_t s) {
    fill_i64_kernel<<<(unsigned)ceil_div(k, kBlock), kBlock, 0, s>>>(sizes, k, cut, 1);
    EP_LAUNCH_CHECK();
    const bool bytes = k <= kByteLabelMaxK;
    const int prep_blocks = (int)std::min<int64_t>(2048, ceil_div(n, kBlock * 8));
    label_prep_kernel<<<prep_blocks, kBlock, 0, s>>>(n, k, labels, bytes ? w.label8 : nullptr, sizes);
    EP_LAUNCH_CHECK();
    if (nnz <= 0) return EP_OK;
    auto out = reinterpret_cast<unsigned long long *>(cut);
    const BucketPlan pl = bucket_plan(n, nnz, k);
    if (pl.shift && w.bucket_records) return launch_cut_bucketed(n, nnz, pl, rowptr, i64, colidx, w, out, s);
    ProfScope prof(EP_PROF_EDGE_SWEEP, s);
    return bytes ? launch_sweep_rows<uint8_t, kCut>(n, nnz, k, rowptr, i64, colidx, w.label8, out, s)
                 : launch_sweep_rows<int32_t, kCut>(n, nnz, k, rowptr, i64, colidx, labels, out, s);
}

int launch_edge_gap(int64_t n, int64_t nnz, const void *rowptr, bool i64, const int32_t *colidx,
                    const int32_t *new_id, uint64_t *out64, EdgeReduce what, const GraphWs &w, hipStream_t s) {
    (void)w;
    fill_i64_kernel<<<1, kBlock, 0, s>>>(reinterpret_cast<int64_t *>(out64), 1, nullptr, 0);
    EP_LAUNCH_CHECK();
    if (nnz <= 0) return EP_OK;
    auto out = reinterpret_cast<unsigned long long *>(out64);
    ProfScope prof(EP_PROF_EDGE_SWEEP, s);
    return what == EdgeReduce::GapSum
               ? launch_sweep_rows<int32_t, kGapSum>(n, nnz, 0, rowptr, i64, colidx, new_id, out, s)
               : launch_sweep_rows<int32_t, kBandwidth>(n, nnz, 0, rowptr, i64, colidx, new_id, out, s);
}

static int sort_passes(int64_t n, int passes, uint32_t clamp_k, const int32_t *keys, int32_t *new_id, int32_t *order,
                       int32_t *tmp, int32_t *hist, const int *enable, hipStream_t s) {
    int64_t rows_per_block = std::max<int64_t>(ceil_div(n, kSortBlocksMax), 2048);
    rows_per_block = ceil_div(rows_per_block, kBlock) * kBlock;
    const int blocks = (int)ceil_div(n, rows_per_block);
    // ping-pong so that the last pass writes `order`
    const int32_t *src = nullptr;                      // identity
    for (int pass = 0; pass < passes; ++pass) {
        int32_t *dst = (passes - pass) % 2 == 1 ? order : tmp;
        const bool last = pass == passes - 1;
        sort_hist_kernel<<<blocks, kBlock, 0, s>>>(n, rows_per_block, keys, src, 8 * pass, clamp_k, hist, enable);
        EP_LAUNCH_CHECK();
        sort_scan_kernel<<<kRadix, kRadix, 0, s>>>(hist, blocks, hist + (size_t)kSortBlocksMax * kRadix, enable);
        EP_LAUNCH_CHECK();
        sort_scatter_kernel<<<blocks, kBlock, 0, s>>>(n, rows_per_block, keys, src, 8 * pass, clamp_k, hist,
                                                      hist + (size_t)kSortBlocksMax * kRadix, dst,
                                                      last ? new_id : nullptr, enable);
        EP_LAUNCH_CHECK();
        src = dst;
    }
    return EP_OK;
}

int launch_sort_by_key(int64_t n, int passes, const int32_t *keys, int32_t *new_id, int32_t *order, int32_t *tmp,
                       int32_t *hist, const int *enable, hipStream_t s) {
    return sort_passes(n, passes, 0, keys, new_id, order, tmp, hist, enable, s);
}

int launch_sort_by_label(int64_t n, int32_t k, const int32_t *labels, int32_t *new_id, int32_t *order,
                         int32_t *tmp, int32_t *hist, hipStream_t s) {
    // keys 0 .. k (k = "outside [0, k)", sorted behind the valid labels); k <= 65536
    const int passes = k < kRadix ? 1 : k < kRadix * kRadix ? 2 : 3;
    return sort_passes(n, passes, (uint32_t)k, labels, new_id, order, tmp, hist, nullptr, s);
}

}  // namespace ep
