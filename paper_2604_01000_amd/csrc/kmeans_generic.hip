// Shape-generic K-Means kernels: any d, any k, fp32 or bf16 embeddings.  They are the
// reference-shaped fallbacks of the library; the shapes the benchmark runs have tuned
// kernels elsewhere and share these kernels' reductions and second passes.
//
// What they compute (EmbedPart paper, Alg. 3, step P <- KMeans(E, k)): one Lloyd round =
// assign every embedding to its nearest centroid (squared Euclidean, evaluated as
// ||c||^2 - 2 x.c, lowest index on ties), then move every centroid to the mean of its
// embeddings (an empty cluster keeps its centroid).
#include <algorithm>
#include <type_traits>

#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;

// ---- init: C[j,:] = X[idx[j],:] ------------------------------------------------------------
template <typename XT>
__global__ void gather_rows_kernel(int32_t d, int32_t k, int64_t ld, const XT *__restrict__ X,
                                   const int64_t *__restrict__ idx, float *__restrict__ C) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)k * d) return;
    const int32_t j = (int32_t)(t / d), m = (int32_t)(t % d);
    C[t] = load_elem(X + idx[j] * ld + m);
}

// ---- sample: S[i,:] = X[rows[i],:] in the element type of X, row stride ld_s >= d -----------------
// (the columns d .. ld_s - 1 of S are zeroed; no kernel reads them)
template <typename XT>
__global__ void sample_rows_kernel(int32_t d, int64_t m, int64_t ld, int64_t ld_s, const XT *__restrict__ X,
                                   const int64_t *__restrict__ rows, XT *__restrict__ S) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= m * ld_s) return;
    const int64_t i = t / ld_s, c = t % ld_s;
    S[t] = c < d ? X[rows[i] * ld + c] : XT(0);
}

// ---- centroid preparation: squared norms (and bf16-rounded copies) -------------------------
// One wave per centroid; the norm is accumulated in fp64 and rounded once.
__global__ __launch_bounds__(kBlock) void prep_centroids_kernel(int32_t d, int32_t k, int round_bf16,
                                                                 const float *__restrict__ C,
                                                                 float *__restrict__ cnorm, float *__restrict__ cq,
                                                                 bf16_t *__restrict__ cq16) {
    const int j = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (j >= k) return;
    const int lane = threadIdx.x & 63;
    double acc = 0.0;
    for (int m = lane; m < d; m += 64) {
        float c = C[(int64_t)j * d + m];
        if (round_bf16) {
            const bf16_t q = f32_to_bf16_rne(c);
            c = bf16_to_f32(q);
            cq[(int64_t)j * d + m] = c;
            cq16[(int64_t)j * d + m] = q;
        }
        acc += (double)c * (double)c;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) cnorm[j] = (float)acc;
}

// ---- assignment ------------------------------------------------------------------------------
// One point per lane.  Centroids pass through LDS in chunks of kChunk; each lane keeps kChunk
// running dot products and folds them into its best (score, index) pair with a strict <, so
// the lowest index wins ties.
constexpr int kChunk = 16;
constexpr int kChunkLdsFloats = 8192;  // 32 KB

template <typename XT>
__global__ __launch_bounds__(kBlock) void assign_generic_kernel(int64_t n, int32_t d, int32_t k, int64_t ld,
                                                                 const XT *__restrict__ X,
                                                                 const float *__restrict__ C,
                                                                 const float *__restrict__ cnorm,
                                                                 int32_t *__restrict__ labels,
                                                                 float *__restrict__ min_d2,
                                                                 double *__restrict__ obj_part) {
    __shared__ float cs[kChunkLdsFloats];
    __shared__ double red[kBlock / 64];
    const int dseg = min(d, kChunkLdsFloats / kChunk);  // columns of a chunk held in LDS at once
    double obj = 0.0;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int64_t rounds = (n + stride - 1) / stride;
    for (int64_t it = 0; it < rounds; ++it) {
        const int64_t i = it * stride + (int64_t)blockIdx.x * kBlock + threadIdx.x;
        const bool valid = i < n;
        const XT *x = X + (valid ? i : 0) * ld;
        float best = 3.0e38f;
        int32_t best_j = 0;
        float xnorm = 0.f;
        for (int32_t j0 = 0; j0 < k; j0 += kChunk) {
            const int kc = min(kChunk, k - j0);
            float acc[kChunk];
#pragma unroll
            for (int j = 0; j < kChunk; ++j) acc[j] = 0.f;
            for (int32_t m0 = 0; m0 < d; m0 += dseg) {
                const int dm = min(dseg, d - m0);
                __syncthreads();
                for (int t = threadIdx.x; t < kc * dm; t += kBlock) {
                    const int j = t / dm, m = t % dm;
                    cs[j * dseg + m] = C[(int64_t)(j0 + j) * d + m0 + m];
                }
                for (int t = threadIdx.x + kc * dseg; t < kChunk * dseg; t += kBlock) cs[t] = 0.f;  // unused slots
                __syncthreads();
                if (valid) {
                    const int dm4 = dm & ~3;
                    for (int m = 0; m < dm4; m += 4) {
                        const float4 xv = load4(x + m0 + m);
                        if (j0 == 0) xnorm += xv.x * xv.x + xv.y * xv.y + xv.z * xv.z + xv.w * xv.w;
#pragma unroll
                        for (int j = 0; j < kChunk; ++j) {
                            const float *c = cs + j * dseg + m;
                            acc[j] += xv.x * c[0] + xv.y * c[1] + xv.z * c[2] + xv.w * c[3];
                        }
                    }
                    for (int m = dm4; m < dm; ++m) {
                        const float xv = load_elem(x + m0 + m);
                        if (j0 == 0) xnorm += xv * xv;
#pragma unroll
                        for (int j = 0; j < kChunk; ++j) acc[j] += xv * cs[j * dseg + m];
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < kChunk; ++j) {
                if (j < kc) {
                    const float score = cnorm[j0 + j] - 2.f * acc[j];
                    if (score < best) { best = score; best_j = j0 + j; }
                }
            }
        }
        if (valid) {
            labels[i] = best_j;
            const float d2 = fmaxf(xnorm + best, 0.f);
            if (min_d2) min_d2[i] = d2;
            obj += (double)d2;
        }
    }
    if (obj_part) {
        for (int off = 32; off > 0; off >>= 1) obj += __shfl_down(obj, off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = obj;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int w = 0; w < kBlock / 64; ++w) t += red[w];
            obj_part[blockIdx.x] = t;
        }
    }
}

__global__ void sum_partials_kernel(const double *__restrict__ part, int count, double *__restrict__ out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double t = 0.0;
        for (int b = 0; b < count; ++b) t += part[b];
        *out = t;
    }
}

// ---- update, small k: per-workgroup LDS partial sums + fixed-order second pass -----------------
// Workgroup b owns rows [b*R, (b+1)*R).  Thread t owns column t % dpad of the rows with
// (row - b*R) % rpp == t / dpad, and adds them into its own LDS copy, so no two threads ever
// touch the same LDS word and the order of additions is fixed.
template <typename XT>
__global__ __launch_bounds__(kBlock) void update_partial_kernel(int64_t n, int32_t d, int32_t k, int64_t ld,
                                                                 int64_t rows_per_block, int dpad, int rpp,
                                                                 const XT *__restrict__ X,
                                                                 const int32_t *__restrict__ labels,
                                                                 float *__restrict__ psum,
                                                                 int32_t *__restrict__ pcnt) {
    extern __shared__ float lds[];  // rpp * k * d floats, then rpp * k ints
    float *sums = lds;
    int32_t *cnts = reinterpret_cast<int32_t *>(lds + (size_t)rpp * k * d);
    const int kd = k * d;
    for (int t = threadIdx.x; t < rpp * kd; t += kBlock) sums[t] = 0.f;
    for (int t = threadIdx.x; t < rpp * k; t += kBlock) cnts[t] = 0;
    __syncthreads();
    const int sub = threadIdx.x / dpad, col0 = threadIdx.x % dpad;
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    if (sub < rpp) {
        float *mine = sums + (size_t)sub * kd;
        for (int64_t i = b + sub; i < e; i += rpp) {
            const int32_t l = labels[i];
            if (l < 0 || l >= k) continue;
            for (int m = col0; m < d; m += dpad) mine[l * d + m] += load_elem(X + i * ld + m);
            if (col0 == 0) cnts[sub * k + l] += 1;
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kd; t += kBlock) {
        float s = sums[t];
        for (int r = 1; r < rpp; ++r) s += sums[(size_t)r * kd + t];
        psum[(int64_t)blockIdx.x * kd + t] = s;
    }
    for (int t = threadIdx.x; t < k; t += kBlock) {
        int32_t c = cnts[t];
        for (int r = 1; r < rpp; ++r) c += cnts[r * k + t];
        pcnt[(int64_t)blockIdx.x * k + t] = c;
    }
}

}  // namespace

// Second pass shared with the fused kernels: fp64 sum of the per-workgroup partials in
// workgroup order, divide, round to fp32; empty clusters keep C_prev.
__global__ __launch_bounds__(kBlock) void update_finalize_kernel(int32_t d, int32_t k, int blocks,
                                                                  const float *__restrict__ psum,
                                                                  const int32_t *__restrict__ pcnt,
                                                                  const float *__restrict__ C_prev,
                                                                  float *__restrict__ C_out,
                                                                  int64_t *__restrict__ counts, UpdateAcc acc) {
    const int t = blockIdx.x * kBlock + threadIdx.x;
    const int kd = k * d;
    if (t >= kd) return;
    const int j = t / d;
    double s = 0.0;
    int64_t c = 0;
    for (int b = 0; b < blocks; ++b) {
        s += (double)psum[(int64_t)b * kd + t];
        c += pcnt[(int64_t)b * k + j];
    }
    finish_centroid_element(acc, t, j, t % d == 0, s, c, C_prev, C_out, counts);
}

__global__ void accumulate_counts_kernel(int32_t k, UpdateAcc acc) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < k) acc.cnt[j] = ((acc.flags & EP_UPDATE_ACCUMULATE) ? acc.cnt[j] : 0) + acc.chunk_cnt[j];
}

// result[0] += labels outside [0, k) among this workgroup's, result[1] = min(result[1], first such index).
__global__ __launch_bounds__(kBlock) void validate_labels_kernel(int64_t n, int32_t k,
                                                                  const int32_t *__restrict__ labels,
                                                                  unsigned long long *__restrict__ result) {
    __shared__ unsigned long long bad_lds[kBlock / 64], first_lds[kBlock / 64];
    unsigned long long bad = 0, first = (unsigned long long)n;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        if ((uint32_t)labels[i] >= (uint32_t)k) {   // a negative label is a large unsigned one
            ++bad;
            first = min(first, (unsigned long long)i);
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        bad += __shfl_down(bad, off, 64);
        first = min(first, (unsigned long long)__shfl_down(first, off, 64));
    }
    if ((threadIdx.x & 63) == 0) {
        bad_lds[threadIdx.x >> 6] = bad;
        first_lds[threadIdx.x >> 6] = first;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / 64; ++w) {
            bad += bad_lds[w];
            first = min(first, first_lds[w]);
        }
        if (bad) {   // integers: the order of the atomics does not matter
            atomicAdd(&result[0], bad);
            atomicMin(&result[1], first);
        }
    }
}

__global__ void validate_labels_init_kernel(int64_t n, unsigned long long *__restrict__ result) {
    result[0] = 0;
    result[1] = (unsigned long long)n;
}

namespace {

// ---- update, large k: rows sorted by label, one wave per cluster --------------------------------
// seg[j] = first sorted position whose key is >= j, for j = 0 .. k.  The key is the one the sort used:
// the label, or k for a label outside [0, k); such rows sit behind seg[k] and belong to no cluster.
// The keys are monotone along `order`, so every seg entry is written exactly once.
__global__ void segment_offsets_kernel(int64_t n, int32_t k, const int32_t *__restrict__ labels,
                                       const int32_t *__restrict__ order, int64_t *__restrict__ seg) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    const int32_t prev = i == 0 ? -1 : (int32_t)min((uint32_t)labels[order[i - 1]], (uint32_t)k);
    const int32_t cur = i == n ? k : (int32_t)min((uint32_t)labels[order[i]], (uint32_t)k);
    for (int32_t j = prev + 1; j <= cur; ++j) seg[j] = i;
}

// One wave per cluster.  kLanes = d / 8 lanes share a row (8 consecutive columns each, one or two
// 16-byte loads), so a wave reads 64 / kLanes rows per step; sums are fp64 from the start.  The row
// groups are added in a fixed order at the end.  kLanes == 0 selects a shape-generic variant.
template <typename XT>
__device__ __forceinline__ void load8(const XT *p, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float *p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<f16_t>(const f16_t *p, float (&v)[8]) {
    const float4 a = load4(p), b = load4(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t *p, float (&v)[8]) {
    const uint4 r = *reinterpret_cast<const uint4 *>(p);
    v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xFFFF0000u);
    v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xFFFF0000u);
    v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xFFFF0000u);
    v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xFFFF0000u);
}

// Sum of the rows order[b .. e) in fp64 by one wave, for d = 8 * kLanes: lane = (sub, chunk) adds the
// rows b + sub, b + sub + 64 / kLanes, ... in 8 columns, then the sub-lanes are added in a fixed
// butterfly.  Every lane ends with the totals of its 8 columns.
template <typename XT, int kLanes>
__device__ __forceinline__ void sum_sorted_rows(const XT *__restrict__ X, int64_t ld, const int32_t *__restrict__ order,
                                                int64_t b, int64_t e, int lane, double (&acc)[8]) {
    constexpr int kL = kLanes > 0 ? kLanes : 1, kRows = 64 / kL;
    const int chunk = lane % kL, sub = lane / kL;
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.0;
    // Four rows in flight per lane, and the row indices of the next four loaded (unconditionally, from positions
    // clamped into the segment) before these rows are waited for: one exposed latency per four rows instead of an
    // index latency and a row latency per two.  Every lane still adds its rows in ascending order.
    constexpr int kAhead = 4;
    int64_t t = b + sub;
    if (e > b) {
        auto index_at = [&](int64_t pos) { return (int64_t)order[pos < e ? pos : e - 1]; };
        int64_t a[kAhead];
#pragma unroll
        for (int r = 0; r < kAhead; ++r) a[r] = index_at(t + r * kRows);
        for (; t + (kAhead - 1) * kRows < e; t += kAhead * kRows) {
            int64_t nx[kAhead];
#pragma unroll
            for (int r = 0; r < kAhead; ++r) nx[r] = index_at(t + (kAhead + r) * kRows);
            float v[kAhead][8];
#pragma unroll
            for (int r = 0; r < kAhead; ++r) load8(X + a[r] * ld + 8 * chunk, v[r]);
#pragma unroll
            for (int r = 0; r < kAhead; ++r)
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] += (double)v[r][q];
#pragma unroll
            for (int r = 0; r < kAhead; ++r) a[r] = nx[r];
        }
#pragma unroll
        for (int r = 0; r < kAhead - 1; ++r) {   // what is left of this lane's rows, one by one (their indices are loaded)
            if (t + r * kRows < e) {
                float v0[8];
                load8(X + a[r] * ld + 8 * chunk, v0);
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] += (double)v0[q];
            }
        }
    }
#pragma unroll
    for (int off = kL; off < 64; off <<= 1)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] += __shfl_xor(acc[q], off, 64);
}

// Few, long segments (k well below the number of waves the chip runs): every segment is cut into
// `pieces` contiguous parts, one wave each; the parts' sums go to the workspace in fp64 and
// segment_combine_kernel adds them in order.  The cut depends on (n, k) only: reproducible.
template <typename XT, int kLanes>
__global__ __launch_bounds__(kBlock) void segment_partial_kernel(int32_t d, int32_t k, int32_t pieces, int64_t ld,
                                                                  const XT *__restrict__ X,
                                                                  const int32_t *__restrict__ order,
                                                                  const int64_t *__restrict__ seg,
                                                                  double *__restrict__ part) {
    const int64_t w = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (w >= (int64_t)k * pieces) return;
    const int j = (int)(w / pieces), piece = (int)(w % pieces), lane = threadIdx.x & 63;
    const int64_t b = seg[j], cnt = seg[j + 1] - b;
    double acc[8];
    sum_sorted_rows<XT, kLanes>(X, ld, order, b + cnt * piece / pieces, b + cnt * (piece + 1) / pieces, lane, acc);
    if (lane < kLanes) {
#pragma unroll
        for (int q = 0; q < 8; ++q) part[w * d + 8 * lane + q] = acc[q];
    }
}

__global__ __launch_bounds__(kBlock) void segment_combine_kernel(int32_t d, int32_t k, int32_t pieces,
                                                                  const int64_t *__restrict__ seg,
                                                                  const double *__restrict__ part,
                                                                  const float *__restrict__ C_prev,
                                                                  float *__restrict__ C_out,
                                                                  int64_t *__restrict__ counts, UpdateAcc acc) {
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t >= (int64_t)k * d) return;
    const int j = (int)(t / d), col = (int)(t % d);
    const int64_t cnt = seg[j + 1] - seg[j];
    double tot = 0.0;
    for (int piece = 0; piece < pieces; ++piece) tot += part[((int64_t)j * pieces + piece) * d + col];
    finish_centroid_element(acc, t, j, col == 0, tot, cnt, C_prev, C_out, counts);
}

template <typename XT, int kLanes>
__global__ __launch_bounds__(kBlock) void segment_mean_kernel(int32_t d, int32_t k, int64_t ld,
                                                               const XT *__restrict__ X,
                                                               const int32_t *__restrict__ order,
                                                               const int64_t *__restrict__ seg,
                                                               const float *__restrict__ C_prev,
                                                               float *__restrict__ C_out,
                                                               int64_t *__restrict__ counts, UpdateAcc upd) {
    const int j = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (j >= k) return;
    const int lane = threadIdx.x & 63;
    const int64_t b = seg[j], e = seg[j + 1];
    const int64_t cnt = e - b;
    if (kLanes > 0) {
        const int chunk = lane % (kLanes > 0 ? kLanes : 1), sub = lane / (kLanes > 0 ? kLanes : 1);
        double acc[8];
        sum_sorted_rows<XT, kLanes>(X, ld, order, b, e, lane, acc);
        if (sub == 0) {
#pragma unroll
            for (int q = 0; q < 8; ++q)
                finish_centroid_element(upd, (int64_t)j * d + 8 * chunk + q, j, chunk == 0 && q == 0, acc[q], cnt, C_prev,
                                        C_out, counts);
        }
        return;
    }
    for (int m0 = 0; m0 < d; m0 += 128) {  // shape-generic: two columns per lane per sweep
        const int m = m0 + 2 * lane;
        double s0 = 0.0, s1 = 0.0;
        if (m < d) {
            for (int64_t t = b; t < e; ++t) {
                const XT *x = X + (int64_t)order[t] * ld + m;
                s0 += (double)load_elem(x);
                if (m + 1 < d) s1 += (double)load_elem(x + 1);
            }
            finish_centroid_element(upd, (int64_t)j * d + m, j, m == 0, s0, cnt, C_prev, C_out, counts);
            if (m + 1 < d) finish_centroid_element(upd, (int64_t)j * d + m + 1, j, false, s1, cnt, C_prev, C_out, counts);
        }
    }
}

template <typename F>
int by_dtype(const ep_problem &p, F &&f) {
    if (p.dtype == EP_F32) return f(static_cast<const float *>(nullptr));
    if (p.dtype == EP_F16) return f(static_cast<const f16_t *>(nullptr));
    return f(static_cast<const bf16_t *>(nullptr));
}

}  // namespace

KmeansWs carve_kmeans_ws(const ep_problem &p, void *ws) {
    Carver c(ws);
    KmeansWs w{};
    const size_t kd = (size_t)p.k * p.d;
    w.obj_part = c.take<double>(kObjBlocksMax);
    // the running sums of a chunked update come first: their place must not depend on n, because the
    // chunks of one update may differ in size
    w.acc_sum = c.take<double>(kd);
    w.acc_cnt = c.take<int64_t>(p.k);
    w.chunk_cnt = c.take<int64_t>(p.k);
    w.cnorm = c.take<float>(p.k);
    w.idx = c.take<int64_t>(p.k);
    if (p.dtype == EP_BF16) {
        w.cq = c.take<float>(kd);
        w.cq16 = c.take<bf16_t>(kd);
    }
    if (small_sliced_supported(p)) w.best_score = c.take<float>((size_t)p.n);
    if (!update_by_sorted_rows(p)) {
        w.psum = c.take<float>((size_t)kUpdBlocksMax * std::max(kd, (size_t)p.k * (size_t)small_padded_d(p)));
        w.pcnt = c.take<int32_t>((size_t)kUpdBlocksMax * p.k);
    } else {
        w.order = c.take<int32_t>((size_t)p.n);
        w.order_tmp = c.take<int32_t>((size_t)p.n);
        w.seg = c.take<int64_t>((size_t)p.k + 1);
        if (p.d == 64 || p.d == 128) w.seg_part = c.take<double>((size_t)kSegWavesTarget * p.d);
        w.sort_hist = c.take<int32_t>(sort_hist_elems());
    }
    if (large_path_supported(p)) {
        w.records = c.take<unsigned char>(large_record_bytes(p));
        w.best_tile = c.take<int32_t>((size_t)p.n);
    }
    w.bytes = align_up(c.used, 256);
    return w;
}

int launch_gather_rows(const ep_problem &p, const void *X, const int64_t *idx_dev, float *C, hipStream_t s) {
    const int64_t total = (int64_t)p.k * p.d;
    return by_dtype(p, [&](auto *tag) {
        using XT = std::remove_cv_t<std::remove_pointer_t<decltype(tag)>>;
        gather_rows_kernel<XT><<<(unsigned)ceil_div(total, kBlock), kBlock, 0, s>>>(
            p.d, p.k, p.ld, static_cast<const XT *>(X), idx_dev, C);
        EP_LAUNCH_CHECK();
        return EP_OK;
    });
}

int launch_sample_rows(const ep_problem &p, const void *X, int64_t m, int64_t ld_s, const int64_t *rows_dev, void *S,
                       hipStream_t s) {
    const int64_t total = m * ld_s;
    return by_dtype(p, [&](auto *tag) {
        using XT = std::remove_cv_t<std::remove_pointer_t<decltype(tag)>>;
        sample_rows_kernel<XT><<<(unsigned)ceil_div(total, kBlock), kBlock, 0, s>>>(
            p.d, m, p.ld, ld_s, static_cast<const XT *>(X), rows_dev, static_cast<XT *>(S));
        EP_LAUNCH_CHECK();
        return EP_OK;
    });
}

int launch_prep_centroids(const ep_problem &p, const float *C, const KmeansWs &w, hipStream_t s) {
    prep_centroids_kernel<<<(unsigned)ceil_div(p.k, kBlock / 64), kBlock, 0, s>>>(
        p.d, p.k, p.dtype == EP_BF16, C, w.cnorm, w.cq, w.cq16);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_assign_generic(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                          float *min_d2, double *objective, hipStream_t s) {
    const int blocks = (int)std::min<int64_t>(kObjBlocksMax, ceil_div(p.n, kBlock));
    const float *Cuse = p.dtype == EP_BF16 ? w.cq : C;
    int rc = by_dtype(p, [&](auto *tag) {
        using XT = std::remove_cv_t<std::remove_pointer_t<decltype(tag)>>;
        ProfScope prof(EP_PROF_LLOYD_MAIN, s);
        assign_generic_kernel<XT><<<blocks, kBlock, 0, s>>>(p.n, p.d, p.k, p.ld, static_cast<const XT *>(X), Cuse,
                                                            w.cnorm, labels, min_d2,
                                                            objective ? w.obj_part : nullptr);
        EP_LAUNCH_CHECK();
        return EP_OK;
    });
    if (rc != EP_OK) return rc;
    if (objective) {
        sum_partials_kernel<<<1, 64, 0, s>>>(w.obj_part, blocks, objective);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

int launch_accumulate_counts(int32_t k, const UpdateAcc &acc, hipStream_t s) {
    accumulate_counts_kernel<<<(unsigned)ceil_div(k, kBlock), kBlock, 0, s>>>(k, acc);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_validate_labels(int64_t n, int32_t k, const int32_t *labels, int64_t *result, hipStream_t s) {
    auto out = reinterpret_cast<unsigned long long *>(result);
    validate_labels_init_kernel<<<1, 1, 0, s>>>(n, out);
    EP_LAUNCH_CHECK();
    const unsigned grid = (unsigned)std::min<int64_t>(ceil_div(n, kBlock * 4), 2048);
    validate_labels_kernel<<<grid, kBlock, 0, s>>>(n, k, labels, out);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_update_small(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                        float *C_out, int64_t *counts, const KmeansWs &w, const UpdateAcc &acc, hipStream_t s) {
    const int kd = p.k * p.d;
    int dpad = 1;
    while (dpad < p.d && dpad < kBlock) dpad <<= 1;
    int rpp = kBlock / dpad;
    while (rpp > 1 && (size_t)rpp * (kd + p.k) * 4 > 64 * 1024) rpp >>= 1;
    const size_t lds = (size_t)rpp * (kd + p.k) * 4;
    int64_t rows_per_block = std::max<int64_t>(ceil_div(p.n, kUpdBlocksMax), 64);
    const int blocks = (int)ceil_div(p.n, rows_per_block);
    int rc = by_dtype(p, [&](auto *tag) {
        using XT = std::remove_cv_t<std::remove_pointer_t<decltype(tag)>>;
        ProfScope prof(EP_PROF_UPDATE_SUMS, s);
        update_partial_kernel<XT><<<blocks, kBlock, lds, s>>>(p.n, p.d, p.k, p.ld, rows_per_block, dpad, rpp,
                                                              static_cast<const XT *>(X), labels, w.psum, w.pcnt);
        EP_LAUNCH_CHECK();
        return EP_OK;
    });
    if (rc != EP_OK) return rc;
    update_finalize_kernel<<<(unsigned)ceil_div(kd, kBlock), kBlock, 0, s>>>(p.d, p.k, blocks, w.psum, w.pcnt, C_prev,
                                                                             C_out, counts, acc);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_update_sorted(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                         float *C_out, int64_t *counts, const KmeansWs &w, const UpdateAcc &acc, hipStream_t s) {
    int rc = launch_sort_by_label(p.n, p.k, labels, nullptr, w.order, w.order_tmp, w.sort_hist, s);
    if (rc != EP_OK) return rc;
    segment_offsets_kernel<<<(unsigned)ceil_div(p.n + 1, kBlock), kBlock, 0, s>>>(p.n, p.k, labels, w.order, w.seg);
    EP_LAUNCH_CHECK();
    return by_dtype(p, [&](auto *tag) {
        using XT = std::remove_cv_t<std::remove_pointer_t<decltype(tag)>>;
        ProfScope prof(EP_PROF_UPDATE_SUMS, s);
        const unsigned grid = (unsigned)ceil_div(p.k, kBlock / 64);
        const XT *Xt = static_cast<const XT *>(X);
        const int pieces = kSegWavesTarget / p.k;   // waves per segment; k * pieces <= kSegWavesTarget
        if (pieces >= 2 && w.seg_part) {
            const unsigned pgrid = (unsigned)ceil_div((int64_t)p.k * pieces, kBlock / 64);
            if (p.d == 128)
                segment_partial_kernel<XT, 16><<<pgrid, kBlock, 0, s>>>(p.d, p.k, pieces, p.ld, Xt, w.order, w.seg, w.seg_part);
            else
                segment_partial_kernel<XT, 8><<<pgrid, kBlock, 0, s>>>(p.d, p.k, pieces, p.ld, Xt, w.order, w.seg, w.seg_part);
            EP_LAUNCH_CHECK();
            segment_combine_kernel<<<(unsigned)ceil_div((int64_t)p.k * p.d, kBlock), kBlock, 0, s>>>(
                p.d, p.k, pieces, w.seg, w.seg_part, C_prev, C_out, counts, acc);
            EP_LAUNCH_CHECK();
            return EP_OK;
        }
        if (p.d == 128)
            segment_mean_kernel<XT, 16><<<grid, kBlock, 0, s>>>(p.d, p.k, p.ld, Xt, w.order, w.seg, C_prev, C_out, counts, acc);
        else if (p.d == 64)
            segment_mean_kernel<XT, 8><<<grid, kBlock, 0, s>>>(p.d, p.k, p.ld, Xt, w.order, w.seg, C_prev, C_out, counts, acc);
        else
            segment_mean_kernel<XT, 0><<<grid, kBlock, 0, s>>>(p.d, p.k, p.ld, Xt, w.order, w.seg, C_prev, C_out, counts, acc);
        EP_LAUNCH_CHECK();
        return EP_OK;
    });
}

}  // namespace ep
