// Lloyd rounds with distance bounds and incremental sums for partition-scale k (k <= 64, d = 64 or
// 128, fp32 or bfloat16 rows): the same rounds as the fused kernels of kmeans_small.hip, reached with
// less work once the centroids have settled.
//
// What it computes (EmbedPart paper, Alg. 3, step P <- KMeans(E, k); the contribution list leaves the
// clustering algorithm of Phase 2 open to more advanced ones): the published bound scheme of Hamerly
// ("Making k-means even faster", SDM 2010).  Every point keeps u >= its distance to its own centroid
// and l <= its distance to every other centroid.  When the centroids move by delta_j, u grows by the
// own delta and l shrinks by the largest delta among the others; a point whose bounds still separate
// cannot change its label and is not even read.  The other points are gathered by index, scored with
// exactly the arithmetic of the fused kernels (so the labels are the same bits), get fresh bounds
// from their best and second-best score, and only those that change their label touch the sums: their
// row leaves one sum and joins another.  The sums live in fp64 between the rounds.
//
// All bounds are kept on the safe side of fp32 rounding: an upper bound is rounded up, a lower bound
// down, and the test leaves room for the rounding of the scores themselves, so a skipped point is one
// whose scores, had they been computed, would have named the same centroid.
//
// The first bounds come from the last full round: the fused kernel of kmeans_small.hip, built with its bounds
// option, also tracks every point's second-best score and stores u and l next to the label.
//
// Kernels of one bounded round:
//   bounds_update_kernel    streams (label, u, l), 12 bytes per point, applies the drift, marks and counts
//                           the points that must be searched (per workgroup)
//   bounds_compact_kernel   writes the indices of the points to search, in ascending order (a workgroup adds
//                           up the counts of the workgroups before it)
//   bounds_round_kernel     the search of those points (matrix cores), new bounds, label changes, and
//                           per-workgroup partial sums of the rows that changed side (+x new, -x old)
//   lloyd_small_finalize_kernel (kmeans_small.hip) adds the partials to the kept sums and forms the means
//   bounds_tail_kernel      one workgroup: brings the kept counts up to date, forms the round's objective from
//                           the sums (sum ||x||^2 - 2 sum_j c_j.s_j + sum_j n_j ||c_j||^2), then delta_j, its two
//                           largest values and max ||c||^2, and keeps the new centroids for the next round
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "kernels.h"
#include "small_common.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kSub = 16;              // points per sub-tile of the search
constexpr int kBoundsBlocksMax = 2048;   // workgroups of the bounds pass (each a contiguous chunk of rows)

// room the test leaves for the rounding of the two scores it stands in for
constexpr float kTestSlack = 0x1p-12f;

// Written by bounds_tail_kernel, read by the bounds pass of the next round.
struct DriftTop {
    float first, second;   // largest and second-largest centroid movement (rounded up)
    float cmax2;           // max_j ||c_j||^2 of the new centroids (rounded up)
    int32_t jfirst;        // the centroid that moved most
};

// The bounds of a point still separate its own centroid from all others, with room for the scores' rounding:
// ||x|| <= ||c_own|| + u, so the products behind the two scores are at most (cmax + u)^2 + cmax^2 in size.
__device__ __forceinline__ bool bounds_hold(float u, float l, float cmax, float cmax2) {
    const float r = cmax + u;
    return l > u && (l - u) * (l + u) > kTestSlack * (r * r + cmax2);
}

__device__ __forceinline__ uint64_t lanes_below() {
    const unsigned lane = __lane_id();
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// ---- the bounds pass ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void bounds_update_kernel(int64_t n, int64_t rows_per_block, int32_t k,
                                                                const int32_t *__restrict__ labels,
                                                                float *__restrict__ ub, float *__restrict__ lb,
                                                                const float *__restrict__ delta,
                                                                const DriftTop *__restrict__ top,
                                                                int32_t *__restrict__ block_counts) {
    __shared__ int32_t wave_cnt[kWaves];
    const DriftTop t = *top;
    const float cmax = sqrtf(t.cmax2) * kUp;
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    int32_t mine = 0;
    for (int64_t i = b + threadIdx.x; i < e; i += kBlock) {
        const int32_t a = labels[i];
        const float da = (uint32_t)a < (uint32_t)k ? delta[a] : t.first;
        const float u = (ub[i] + da) * kUp;
        float l = lb[i] - (a == t.jfirst ? t.second : t.first);
        l = l > 0.f ? l * kDown : l * kUp;   // down in either case
        // the decision is taken once, here: a point that must be searched carries it in the sign of its upper
        // bound (the search writes a fresh, positive one), and the compaction reads nothing else
        const bool hold = bounds_hold(u, l, cmax, t.cmax2);
        ub[i] = hold ? u : -u;
        lb[i] = l;
        mine += hold ? 0 : 1;
    }
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off, 64);
    if ((threadIdx.x & 63) == 0) wave_cnt[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) block_counts[blockIdx.x] = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
}

// Writes the indices of the marked points in ascending order.  A workgroup's first position is the sum of the
// counts of the workgroups before it (at most kBoundsBlocksMax of them, added up here in integers); the last
// workgroup also records the total.
__global__ __launch_bounds__(kBlock) void bounds_compact_kernel(int64_t n, int64_t rows_per_block,
                                                                 const float *__restrict__ ub,
                                                                 const int32_t *__restrict__ block_counts,
                                                                 int32_t *__restrict__ active_idx,
                                                                 int64_t *__restrict__ n_active,
                                                                 int64_t *__restrict__ searched_slot) {
    __shared__ int32_t wave_cnt[kWaves];
    __shared__ int64_t wave_before[kWaves];
    const int64_t b = (int64_t)blockIdx.x * rows_per_block, e = min(n, b + rows_per_block);
    const int wave = threadIdx.x >> 6;
    int64_t before = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kBlock) before += block_counts[i];
    for (int off = 32; off > 0; off >>= 1) before += __shfl_down(before, off, 64);
    if ((threadIdx.x & 63) == 0) wave_before[wave] = before;
    __syncthreads();
    int64_t running = wave_before[0] + wave_before[1] + wave_before[2] + wave_before[3];
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const int64_t total = running + block_counts[blockIdx.x];
        *n_active = total;
        *searched_slot = total;
    }
    // Four consecutive points per thread (one 16-byte load; the range starts on a multiple of 256 points, and what
    // a load reads past the last point lies inside the workspace and is not looked at): a quarter of the barriers.
    for (int64_t tile = b; tile < e; tile += 4 * kBlock) {
        const int64_t i0 = tile + 4 * threadIdx.x;
        const u32x4 u4 = *reinterpret_cast<const u32x4 *>(ub + (i0 < e ? i0 : b));   // always a position of the range
        bool active[4];
        uint64_t mask[4];
        int before_lanes = 0, mine = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            active[q] = i0 + q < e && (u4[q] >> 31) != 0;   // marked by bounds_update_kernel
            mask[q] = __ballot(active[q]);
            before_lanes += __popcll(mask[q] & lanes_below());
        }
        if ((threadIdx.x & 63) == 0)
            wave_cnt[wave] = __popcll(mask[0]) + __popcll(mask[1]) + __popcll(mask[2]) + __popcll(mask[3]);
        __syncthreads();
        int64_t pos = running + before_lanes;
        for (int w = 0; w < wave; ++w) pos += wave_cnt[w];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (active[q]) active_idx[pos + mine] = (int32_t)(i0 + q);
            mine += active[q] ? 1 : 0;
        }
        running += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
        __syncthreads();
    }
}

__global__ void record_searched_kernel(int64_t value, int64_t *__restrict__ slot) { *slot = value; }

__global__ __launch_bounds__(kBlock) void copy_floats_kernel(int64_t count, const float *__restrict__ src,
                                                              float *__restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < count) dst[i] = src[i];
}

__global__ __launch_bounds__(kBlock) void copy_i64_kernel(int64_t count, const int64_t *__restrict__ src,
                                                           int64_t *__restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < count) dst[i] = src[i];
}

// The centroid as the distances use it: rounded to bfloat16 for bfloat16 rows.
template <bool BF16>
__device__ __forceinline__ double centroid_used(float c) {
    return BF16 ? (double)bf16_to_f32(f32_to_bf16_rne(c)) : (double)c;
}

// What follows the means of a bounded round, in one workgroup:
//   the kept counts take the round's changes (cnt += chunk_cnt; not after a full round, whose counts are whole);
//   objective (if asked for) of the round whose assignment used C_old (as the distances use it) and left the sums
//   and counts: sum ||x||^2 - 2 sum_j c_j . s_j + sum_j n_j ||c_j||^2, in fp64 and a fixed order;
//   drift (if another round follows): delta_j = ||c_new_j - c_old_j|| of the centroids as the distances use them,
//   its two largest values and max_j ||c_new_j||^2 (wave w takes the centroids w, w + 4, ...), after which C_old
//   becomes C_new for that round.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void bounds_tail_kernel(int32_t k, int32_t d, const float *__restrict__ C_new,
                                                              float *__restrict__ C_old,
                                                              const double *__restrict__ sum, int64_t *__restrict__ cnt,
                                                              const int64_t *__restrict__ chunk_cnt, int add_counts,
                                                              const double *__restrict__ xsq_total,
                                                              double *__restrict__ objective, int want_drift,
                                                              float *__restrict__ delta, DriftTop *__restrict__ top) {
    __shared__ double wave_part[kWaves];
    __shared__ int64_t cnt_lds[64];
    __shared__ float delta_lds[64], norm_lds[64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)threadIdx.x < k) {
        int64_t all = cnt[threadIdx.x];
        if (add_counts) {
            all += chunk_cnt[threadIdx.x];
            cnt[threadIdx.x] = all;
        }
        cnt_lds[threadIdx.x] = all;
    }
    __syncthreads();
    if (objective) {
        double part = 0.0;
        for (int e = threadIdx.x; e < k * d; e += kBlock) {
            const double c = centroid_used<BF16>(C_old[e]);
            part += c * ((double)cnt_lds[e / d] * c - 2.0 * sum[e]);
        }
        for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
        if (lane == 0) wave_part[wave] = part;
        __syncthreads();
        if (threadIdx.x == 0) *objective = *xsq_total + (wave_part[0] + wave_part[1] + wave_part[2] + wave_part[3]);
    }
    if (!want_drift) return;
    for (int j = wave; j < k; j += kWaves) {
        double moved = 0.0, norm = 0.0;
        for (int m = lane; m < d; m += 64) {
            const double a = centroid_used<BF16>(C_new[(int64_t)j * d + m]);
            const double diff = a - centroid_used<BF16>(C_old[(int64_t)j * d + m]);
            moved += diff * diff;
            norm += a * a;
        }
        for (int off = 32; off > 0; off >>= 1) {
            moved += __shfl_down(moved, off, 64);
            norm += __shfl_down(norm, off, 64);
        }
        if (lane == 0) {
            delta_lds[j] = (float)sqrt(moved) * kUp;
            norm_lds[j] = (float)norm * kUp;
        }
    }
    __syncthreads();   // every read of C_old is done
    for (int e = threadIdx.x; e < k * d; e += kBlock) C_old[e] = C_new[e];
    if ((int)threadIdx.x < k) delta[threadIdx.x] = delta_lds[threadIdx.x];
    if (threadIdx.x == 0) {
        DriftTop t{0.f, 0.f, 0.f, -1};
        for (int j = 0; j < k; ++j) {
            const float dj = delta_lds[j];
            if (dj > t.first) { t.second = t.first; t.first = dj; t.jfirst = j; }
            else if (dj > t.second) { t.second = dj; }
            t.cmax2 = fmaxf(t.cmax2, norm_lds[j]);
        }
        *top = t;
    }
}

// ---- the search of the points whose bounds no longer separate ------------------------------------
// Lane layout, centroid operand, score arithmetic and arg-max are those of lloyd_small_kernel (lane = 16 g + c
// holds columns 16 j + 4 g .. + 3 of point c; scores of points 4 g .. 4 g + 3 against centroid 16 mt + c come back
// in the lane's four accumulator words), so a searched point gets the label the fused kernel would give it.
template <int D, int KT>
struct BoundsLds {
    static constexpr int kStride = D + 4;
    static constexpr int kBytes = kWaves * (16 * KT + 1) * kStride * 4;
};

template <int D, int KT, typename XT>
__global__ __launch_bounds__(kBlock, KT <= 2 ? 2 : 1) void bounds_round_kernel(
    int64_t n, int64_t ld, int32_t k, const XT *__restrict__ X, const float *__restrict__ C,
    const int32_t *__restrict__ active_idx, const int64_t *__restrict__ n_active_ptr, int32_t *__restrict__ labels,
    float *__restrict__ ub, float *__restrict__ lb, float *__restrict__ psum, int32_t *__restrict__ pcnt,
    int32_t *__restrict__ scrap) {
    constexpr int NJ = D / 16;
    constexpr int NX = NJ;
    constexpr int STRIDE = D + 4;
    constexpr bool kBf16 = std::is_same<XT, bf16_t>::value;
    constexpr bool kHalf = std::is_same<XT, f16_t>::value;
    constexpr bool kSplit = KT >= 2 || kBf16;
    constexpr bool kThreeTerms = kSplit && !kBf16;
    constexpr int KS = D / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];
    float *lds = reinterpret_cast<float *>(dyn_lds);
    __shared__ int32_t cnt_lds[16 * KT];

    // a workgroup that gets no row of the list leaves no partial (the second pass knows which ones do)
    static_assert(kSub * kWaves == 64, "list_parts counts workgroups of 64 rows per step");
    if ((int)blockIdx.x >= list_parts(*n_active_ptr, n, (int)gridDim.x)) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, c = lane & 15;
    float *wsums = lds + wave * (16 * KT + 1) * STRIDE;
    for (int i = lane; i < (16 * KT + 1) * STRIDE; i += 64) wsums[i] = 0.f;
    if (threadIdx.x < 16 * KT) cnt_lds[threadIdx.x] = 0;
    __syncthreads();

    // this wave's share of the sub-tiles of the list (a fixed function of the list's length and the grid)
    const int64_t n_act = min(max(*n_active_ptr, (int64_t)0), n);
    const int64_t total_sub = (n_act + kSub - 1) / kSub;
    const int64_t waves = (int64_t)gridDim.x * kWaves, wave_id = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t per = total_sub / waves, extra = total_sub % waves;
    const int64_t first = wave_id * per + min(wave_id, extra);
    const int64_t last = first + per + (wave_id < extra ? 1 : 0);

    // Row of this lane's point in sub-tile st, in two steps.  The list entry is loaded unconditionally (from a
    // position clamped into the list) and not looked at; it is checked one sub-tile later, where it is used.
    // A value that is tested right after its load makes the wave wait for that load, and on this chip that wait
    // is for every older and, when a branch stands in between, every younger access too: the row loads of the
    // next sub-tile, issued just before, would be waited for at once.  The same holds for the old labels and is
    // why the stores below have no branch.
    auto fetch_raw = [&](int64_t st) -> int32_t {
        const int64_t pos = st * kSub + c;
        return active_idx[pos < n_act ? pos : n_act - 1];   // n_act >= 1: a workgroup without rows has left
    };
    auto resolve_row = [&](int32_t raw, int64_t st) -> int64_t {   // -1: none
        const int64_t pos = st * kSub + c;
        return (st < last && pos < n_act && raw >= 0 && (int64_t)raw < n) ? (int64_t)raw : -1;
    };
    auto load_x = [&](int64_t row, f32x4(&dst)[NX]) {
        const XT *ptr = X + (row < 0 ? 0 : row) * ld + 4 * g;
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            if constexpr (kBf16) {
                const u32x2 raw = *reinterpret_cast<const u32x2 *>(ptr + 16 * q);
                dst[q] = f32x4{__uint_as_float(raw[0] << 16), __uint_as_float(raw[0] & 0xffff0000u),
                               __uint_as_float(raw[1] << 16), __uint_as_float(raw[1] & 0xffff0000u)};
            } else if constexpr (kHalf) {
                dst[q] = __builtin_convertvector(*reinterpret_cast<const f16x4_t *>(ptr + 16 * q), f32x4);
            } else {
                dst[q] = *reinterpret_cast<const f32x4 *>(ptr + 16 * q);
            }
        }
    };
    auto load_old_raw = [&](int64_t row) -> int32_t { return labels[row < 0 ? 0 : row]; };   // checked in process()

    // ---- centroid operand (as in lloyd_small_kernel) ----
    f32x4 creg[kSplit ? 1 : KT][kSplit ? 1 : NJ];
    u32x4 ch[kSplit ? KT : 1][kSplit ? KS : 1], cm[kThreeTerms ? KT : 1][kThreeTerms ? KS : 1],
        cl[kThreeTerms ? KT : 1][kThreeTerms ? KS : 1];
    float hn[KT];
    float cmax2 = 0.f;   // max ||c||^2 over the centroids, the same in every lane after the loop below
    auto load_centroids = [&]() {
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const int cent = 16 * mt + c;
            const bool real = cent < k;
            double nacc = 0.0;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (real) v = *reinterpret_cast<const f32x4 *>(C + (int64_t)cent * D + 16 * j + 4 * g);
                if constexpr (kBf16) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = bf16_to_f32(f32_to_bf16_rne(v[e]));
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) nacc = fma((double)v[e], (double)v[e], nacc);
                if constexpr (kSplit) {
                    const int s = j >> 1, w = 2 * (j & 1);
                    const Split3 lo = split3_pair(v[0], v[1]), hi = split3_pair(v[2], v[3]);
                    ch[mt][s][w] = lo.h, ch[mt][s][w + 1] = hi.h;
                    if constexpr (kThreeTerms) {
                        cm[mt][s][w] = lo.m, cl[mt][s][w] = lo.l;
                        cm[mt][s][w + 1] = hi.m, cl[mt][s][w + 1] = hi.l;
                    }
                } else {
                    creg[mt][j] = v;
                }
            }
            nacc += __shfl_xor(nacc, 16, 64);
            nacc += __shfl_xor(nacc, 32, 64);
            hn[mt] = real ? (float)(-0.5 * nacc) : -3.0e38f;
            if (real) cmax2 = fmaxf(cmax2, (float)nacc * kUp);
        }
        cmax2 = key_float(row16_max(float_key(cmax2)));
        if constexpr (kSplit) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    asm volatile("" : "+a"(ch[mt][s]));
                    if constexpr (kThreeTerms) {
                        asm volatile("" : "+a"(cm[mt][s]));
                        asm volatile("" : "+a"(cl[mt][s]));
                    }
                }
        }
    };

    // ---- scores of a sub-tile: the instruction sequence of lloyd_small_kernel, term by term ----
    auto scores = [&](const f32x4(&x)[NX], f32x4(&acc)[KT]) {
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) acc[mt] = f32x4{hn[mt], hn[mt], hn[mt], hn[mt]};
        if constexpr (!kSplit) {
            f32x4 acc1[KT];
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) acc1[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) {
                        if (j & 1)
                            acc1[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j][e], creg[mt][j][e], acc1[mt], 0, 0, 0);
                        else
                            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j][e], creg[mt][j][e], acc[mt], 0, 0, 0);
                    }
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) acc[mt] += acc1[mt];
        } else if constexpr (!kThreeTerms) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                u32x4 a;
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    const f32x4 &v = x[2 * s + (pr >> 1)];
                    a[pr] = (__float_as_uint(v[2 * (pr & 1) + 1]) & 0xffff0000u) | (__float_as_uint(v[2 * (pr & 1)]) >> 16);
                }
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) acc[mt] = mfma_bf16_k32(a, ch[mt][s], acc[mt]);
            }
        } else {
            // The operands of K-step s + 1 are split between the instruction groups of K-step s (as in
            // lloyd_small_kernel): a wave cannot issue past a matrix instruction that waits for the pipe, so 24
            // of them back to back would leave the vector pipe idle for as long as the matrix pipe is busy.
            u32x4 xh[2], xm[2], xl[2];
            auto split_pair = [&](int s, int pr) {
                const f32x4 &v = x[2 * s + (pr >> 1)];
                const Split3 t = split3_pair(v[2 * (pr & 1)], v[2 * (pr & 1) + 1]);
                xh[s & 1][pr] = t.h, xm[s & 1][pr] = t.m, xl[s & 1][pr] = t.l;
            };
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) split_pair(0, pr);
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int pp = 0; pp < 6; ++pp) {   // xh.cl, xl.ch, xm.cm, xh.cm, xm.ch, xh.ch
                    const u32x4 &a = pp == 1 ? xl[s & 1] : (pp == 2 || pp == 4) ? xm[s & 1] : xh[s & 1];
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) {
                        const u32x4 &b = pp == 0 ? cl[mt][s] : (pp == 2 || pp == 3) ? cm[mt][s] : ch[mt][s];
                        acc[mt] = mfma_bf16_k32(a, b, acc[mt]);
                    }
                    if (pp < 4 && s + 1 < KS) split_pair(s + 1, pp);
                    __builtin_amdgcn_sched_barrier(0);   // pin the interleaving
                }
            }
        }
    };

    auto process = [&](int64_t st, const f32x4(&x)[NX], int64_t row_c, int32_t old_raw) {
        const int rows_here = (int)min((int64_t)kSub, n_act - st * kSub);   // uniform, >= 1
        const int32_t old_c = (row_c >= 0 && (uint32_t)old_raw < (uint32_t)k) ? old_raw : -1;
        f32x4 acc[KT];
        scores(x, acc);

        float xpart = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            xpart += x[j][0] * x[j][0] + x[j][1] * x[j][1] + x[j][2] * x[j][2] + x[j][3] * x[j][3];
        xpart += __shfl_xor(xpart, 16, 64);
        xpart += __shfl_xor(xpart, 32, 64);   // ||x||^2 of point c, in all four lanes that hold a quarter of it

        // best (as in lloyd_small_kernel: strict > over ascending tiles in the lane, then the maximum and the
        // lowest index among the lanes that hold it) and second-best score of the points 4 g + v
        int bkey[4], skey[4];
        int32_t lab[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float sc = acc[0][v];
            int idx = c;
            float m1 = acc[0][v], m2 = -3.4e38f;   // the lane's largest and second-largest (equal values count twice)
#pragma unroll
            for (int mt = 1; mt < KT; ++mt) {
                const float s2 = acc[mt][v];
                if (s2 > sc) { sc = s2; idx = 16 * mt + c; }
                if (s2 > m1) { m2 = m1; m1 = s2; }
                else if (s2 > m2) { m2 = s2; }
            }
            const int key = float_key(sc);
            bkey[v] = row16_max(key);
            const int win = row16_min(key == bkey[v] ? idx : 0x7fffffff);
            lab[v] = (4 * g + v < rows_here) ? win : -1;
            // every lane offers its best, the winner's lane what is left without the winning entry
            skey[v] = row16_max(float_key(c == (win & 15) ? m2 : m1));
        }

        // lane c < 4 of every 16-lane row owns point 4 g + c: new bounds, label
        const int sel = c & 3;
        const float s_best = key_float(sel == 0 ? bkey[0] : sel == 1 ? bkey[1] : sel == 2 ? bkey[2] : bkey[3]);
        const float s_second = key_float(sel == 0 ? skey[0] : sel == 1 ? skey[1] : sel == 2 ? skey[2] : skey[3]);
        const int32_t my_l = sel == 0 ? lab[0] : sel == 1 ? lab[1] : sel == 2 ? lab[2] : lab[3];
        const int src = 4 * g + sel;   // a lane that holds point 4 g + c's row index, old label and norm
        const int64_t own_row = __shfl(row_c, src, 64);
        const float own_xn = __shfl(xpart, src, 64);
        {   // every lane stores, without a branch: a lane that owns no point writes its three scrap words, and an
            // owner writes its label whether it changed or not
            const bool owner = c < 4 && 4 * g + c < rows_here && own_row >= 0;
            float u, l;
            fresh_bounds(own_xn, s_best, s_second, cmax2, u, l);
            int32_t *mine = scrap + ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
            float *pu = owner ? ub + own_row : reinterpret_cast<float *>(mine);
            float *pl = owner ? lb + own_row : reinterpret_cast<float *>(mine + 1);
            int32_t *pa = owner ? labels + own_row : mine + 2;
            *pu = u;
            *pl = l;
            *pa = my_l;
        }

        // the rows that change side: + x into the new label's sum, - x out of the old one's
        const int32_t new_c = __shfl(my_l, 16 * (c >> 2) + (c & 3), 64);   // label of this lane's point
        const bool mover = row_c >= 0 && c < rows_here && new_c != old_c;
        if (__ballot(mover) != 0) {
            add_rows_to_lds_sums<NJ, STRIDE>(x, mover ? new_c : -1, g, wsums, cnt_lds);
            f32x4 neg[NX];
#pragma unroll
            for (int q = 0; q < NX; ++q) neg[q] = -x[q];
            add_rows_to_lds_sums<NJ, STRIDE, -1>(neg, mover ? old_c : -1, g, wsums, cnt_lds);
        }
    };

    // Two register sets in ping-pong; the row indices run one sub-tile further ahead than the rows.
    f32x4 xa[NX], xb[NX];
    int64_t st = first;
    int64_t row_a = resolve_row(fetch_raw(st), st), row_b;
    int32_t raw_n = fetch_raw(st + 1);   // the list entry of the sub-tile after the one whose rows are in flight
    int32_t old_a = load_old_raw(row_a), old_b;
    load_x(row_a, xa);
    __builtin_amdgcn_sched_barrier(0);
    load_centroids();
    while (st < last) {
        row_b = resolve_row(raw_n, st + 1);
        load_x(row_b, xb);
        old_b = load_old_raw(row_b);
        raw_n = fetch_raw(st + 2);
        __builtin_amdgcn_sched_barrier(0);
        process(st, xa, row_a, old_a);
        ++st;
        if (st >= last) break;
        row_a = resolve_row(raw_n, st + 1);
        load_x(row_a, xa);
        old_a = load_old_raw(row_a);
        raw_n = fetch_raw(st + 2);
        __builtin_amdgcn_sched_barrier(0);
        process(st, xb, row_b, old_b);
        ++st;
    }

    // ---- partial sums of this workgroup: the waves' tables added in wave order ----
    __syncthreads();
    for (int i = threadIdx.x; i < k * D; i += kBlock) {
        const int at = (i / D) * STRIDE + (i % D);
        float v = lds[at];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) v += lds[w * (16 * KT + 1) * STRIDE + at];
        psum[(int64_t)blockIdx.x * k * D + i] = v;
    }
    if ((int)threadIdx.x < k) pcnt[(int64_t)blockIdx.x * k + threadIdx.x] = cnt_lds[threadIdx.x];
}

constexpr int kBoundsGridMax = 512;
int bounds_grid(const ep_problem &p) { return p.k <= 32 ? kBoundsGridMax : 256; }

struct PassGeometry {
    int blocks;
    int64_t rows_per_block;
};
PassGeometry pass_geometry(int64_t n) {
    int64_t rows = std::max<int64_t>(ceil_div(n, kBoundsBlocksMax), 4 * kBlock);
    rows = ceil_div(rows, kBlock) * kBlock;
    return PassGeometry{(int)ceil_div(n, rows), rows};
}

}  // namespace

bool bounds_path_supported(const ep_problem &p) {
    return small_path_supported(p) && (p.d == 64 || p.d == 128) && p.k <= 64 && p.k >= 2;
}

BoundsWs carve_bounds_ws(const ep_problem &p, int32_t iters, void *ws) {
    Carver c(ws);
    BoundsWs w{};
    w.ub = c.take<float>((size_t)p.n);
    w.lb = c.take<float>((size_t)p.n);
    w.active_idx = c.take<int32_t>((size_t)p.n);
    w.block_counts = c.take<int32_t>(kBoundsBlocksMax);
    w.n_active = c.take<int64_t>(1);
    w.searched = c.take<int64_t>((size_t)std::max(iters, 1));
    w.delta = c.take<float>((size_t)p.k);
    w.top = c.take<unsigned char>(sizeof(DriftTop));
    w.C_old = c.take<float>((size_t)p.k * p.d);
    w.scrap = c.take<int32_t>((size_t)kBoundsGridMax * kBlock * 4);
    w.bytes = align_up(c.used, 256);
    return w;
}

int launch_record_searched(int64_t value, int64_t *slot, hipStream_t s) {
    record_searched_kernel<<<1, 1, 0, s>>>(value, slot);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_copy_searched(int32_t iters, const BoundsWs &w, int64_t *out, hipStream_t s) {
    copy_i64_kernel<<<(unsigned)ceil_div(iters, kBlock), kBlock, 0, s>>>(iters, w.searched, out);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_keep_centroids(const ep_problem &p, const float *C, const BoundsWs &w, hipStream_t s) {
    const int64_t count = (int64_t)p.k * p.d;
    copy_floats_kernel<<<(unsigned)ceil_div(count, kBlock), kBlock, 0, s>>>(count, C, w.C_old);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_bounds_tail(const ep_problem &p, const float *C_new, const KmeansWs &kw, const BoundsWs &w,
                       bool add_counts, const double *xsq_total, double *objective, bool want_drift, hipStream_t s) {
    DriftTop *top = reinterpret_cast<DriftTop *>(w.top);
    if (p.dtype == EP_BF16)
        bounds_tail_kernel<true><<<1, kBlock, 0, s>>>(p.k, p.d, C_new, w.C_old, kw.acc_sum, kw.acc_cnt, kw.chunk_cnt,
                                                      add_counts ? 1 : 0, xsq_total, objective, want_drift ? 1 : 0,
                                                      w.delta, top);
    else
        bounds_tail_kernel<false><<<1, kBlock, 0, s>>>(p.k, p.d, C_new, w.C_old, kw.acc_sum, kw.acc_cnt, kw.chunk_cnt,
                                                       add_counts ? 1 : 0, xsq_total, objective, want_drift ? 1 : 0,
                                                       w.delta, top);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_bounds_pass(const ep_problem &p, const int32_t *labels, const BoundsWs &w, int64_t *searched_slot,
                       hipStream_t s) {
    const PassGeometry geo = pass_geometry(p.n);
    const DriftTop *top = reinterpret_cast<const DriftTop *>(w.top);
    bounds_update_kernel<<<geo.blocks, kBlock, 0, s>>>(p.n, geo.rows_per_block, p.k, labels, w.ub, w.lb, w.delta, top,
                                                       w.block_counts);
    EP_LAUNCH_CHECK();
    bounds_compact_kernel<<<geo.blocks, kBlock, 0, s>>>(p.n, geo.rows_per_block, w.ub, w.block_counts, w.active_idx,
                                                        w.n_active, searched_slot);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int bounds_round_parts(const ep_problem &p) { return bounds_grid(p); }

int launch_bounds_round(const ep_problem &p, const void *X, const float *C, const KmeansWs &kw, const BoundsWs &w,
                        int32_t *labels, hipStream_t s) {
    const int grid = bounds_grid(p);
    const int kt = p.k <= 16 ? 1 : p.k <= 32 ? 2 : 4;
    const int32_t *idx = w.active_idx;
    const int64_t *n_act = w.n_active;
    ProfScope prof(EP_PROF_LLOYD_MAIN, s);
#define EP_BOUNDS_LAUNCH(D_, KT_, XT_)                                                                          \
    do {                                                                                                        \
        constexpr int lds_bytes = BoundsLds<D_, KT_>::kBytes;                                                   \
        auto kern = bounds_round_kernel<D_, KT_, XT_>;                                                          \
        if (lds_bytes > 64 * 1024) {   /* once per kernel variant and device */                                \
            static std::atomic<uint64_t> attr_set{0};                                                           \
            int dev_ = 0;                                                                                       \
            EP_HIP_TRY(hipGetDevice(&dev_));                                                                    \
            const uint64_t bit_ = 1ull << (dev_ & 63);                                                          \
            if (!(attr_set.load(std::memory_order_acquire) & bit_)) {                                           \
                EP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                            \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));        \
                attr_set.fetch_or(bit_, std::memory_order_release);                                             \
            }                                                                                                   \
        }                                                                                                       \
        kern<<<grid, kBlock, lds_bytes, s>>>(p.n, p.ld, p.k, static_cast<const XT_ *>(X), C, idx, n_act, labels, \
                                             w.ub, w.lb, kw.psum, kw.pcnt, w.scrap);                            \
    } while (0)
#define EP_BOUNDS_LAUNCH_T(D_, KT_)                                                                             \
    do {                                                                                                        \
        if (p.dtype == EP_BF16) EP_BOUNDS_LAUNCH(D_, KT_, bf16_t);                                              \
        else if (p.dtype == EP_F16) EP_BOUNDS_LAUNCH(D_, KT_, f16_t);                                           \
        else EP_BOUNDS_LAUNCH(D_, KT_, float);                                                                  \
    } while (0)
    if (p.d == 128) {
        if (kt == 1) EP_BOUNDS_LAUNCH_T(128, 1); else if (kt == 2) EP_BOUNDS_LAUNCH_T(128, 2); else EP_BOUNDS_LAUNCH_T(128, 4);
    } else {
        if (kt == 1) EP_BOUNDS_LAUNCH_T(64, 1); else if (kt == 2) EP_BOUNDS_LAUNCH_T(64, 2); else EP_BOUNDS_LAUNCH_T(64, 4);
    }
#undef EP_BOUNDS_LAUNCH
#undef EP_BOUNDS_LAUNCH_T
    EP_LAUNCH_CHECK();
    return EP_OK;
}

}  // namespace ep
