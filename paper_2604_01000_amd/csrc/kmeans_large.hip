// Assignment step for reordering-scale k (hundreds to 65,536 clusters), bf16 embeddings, d in
// {64, 128}: x.c on the bf16 matrix cores with the arg-max folded into the product's epilogue,
// so the n x k score matrix (160 GB at n = 2.45 M, k = 16,384) never exists.
//
// What it computes (EmbedPart paper, Alg. 3, step P <- KMeans(E, k), used at large k for the
// reordering of Sec. "Adapting EmbedPart for Reordering"): labels[i] = argmin_j ||x_i - c_j||^2
// = argmax_j (x_i.c_j - ||c_j||^2 / 2), lowest j on ties, with the centroids rounded to bf16 for
// the products and fp32 accumulation.
//
// Three kernels:
//  1. large_prep_kernel: rounds the centroids to bf16, forms -||c||^2/2 from the rounded values
//     (fp64 accumulation) and writes one "tile record" per 32 centroids: the 32 x d block already
//     in the lane order of the matrix instruction's operand (so staging is a straight copy and LDS
//     reads are conflict-free) followed by the 32 biases.
//  2. large_assign_kernel: a wave keeps 128 points (4 operand tiles of 32) in registers and walks
//     all centroid tiles; records are staged through a 3-deep LDS ring shared by the 4 waves of a
//     workgroup, with LDS-direct loads (no staging registers).  v_mfma_f32_32x32x16_bf16 with
//     centroids as rows and points as columns leaves 16 centroids of one point in each lane, as
//     4 groups of 4 consecutive rows.  Per tile and point the fold takes the 4 group maxima and
//     their maximum and keeps (best score, 8 tile + 2 group) with one compare and two selects:
//     under one VALU operation per score, no per-score index bookkeeping.  One accumulation
//     chain per point tile, preset with the bias from LDS; the fold of the previous chain's
//     result is issued between the matrix instructions of the running chain.
//  3. large_refine_kernel: the sweep names, per point, 4 consecutive centroid rows that hold the
//     winner; they are evaluated again on the vector unit (v_dot2_f32_bf16) to name the winner
//     itself (lowest index on ties) and to produce ||x - c||^2 for the objective: 1/4096 of the
//     work of step 2, and 1 KB of centroid data per point instead of the whole tile.
#include <hip/hip_ext.h>

#include <algorithm>

#include "kernels.h"

namespace ep {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr int kWaves = 4;
constexpr int kTile = 32;            // centroids per tile record, points per operand tile
constexpr int kMainPointTiles = 4;   // operand tiles of points a wave keeps in registers
constexpr int kMainOccupancy = 2;    // workgroups per compute unit of the sweep kernel
constexpr float kNever = -3.0e38f;   // bias of a padding centroid

template <int D> constexpr int record_bytes() { return (D / 16) * 1024 + kTile * 4; }

// ---- 1. tile records ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBlock) void large_prep_kernel(int32_t k, const float *__restrict__ C,
                                                             bf16_t *__restrict__ cq16, float *__restrict__ hneg,
                                                             unsigned char *__restrict__ records) {
    constexpr int NS = D / 16;
    __shared__ bf16_t rows[kTile][D + 8];
    __shared__ float bias[kTile];
    const int t = threadIdx.x, tile = blockIdx.x;
    {   // 8 threads per centroid row, D/8 columns each; the norm is summed in fp64 in a fixed order
        const int r = t >> 3, part = t & 7;
        const int cent = tile * kTile + r;
        double acc = 0.0;
        for (int m = part * (D / 8); m < (part + 1) * (D / 8); ++m) {
            bf16_t q = 0;
            if (cent < k) {
                q = f32_to_bf16_rne(C[(int64_t)cent * D + m]);
                cq16[(int64_t)cent * D + m] = q;
            }
            rows[r][m] = q;
            const double v = (double)bf16_to_f32(q);
            acc += v * v;
        }
        acc += __shfl_xor(acc, 1, 64);
        acc += __shfl_xor(acc, 2, 64);
        acc += __shfl_xor(acc, 4, 64);
        if (part == 0) {
            const float h = cent < k ? (float)(-0.5 * acc) : kNever;
            bias[r] = h;
            if (cent < k) hneg[cent] = h;
        }
    }
    __syncthreads();
    unsigned char *rec = records + (int64_t)tile * record_bytes<D>();
    // operand order: piece (s, L) = row L % 32, columns 16 s + 8 (L / 32) .. + 7, at byte (64 s + L) * 16
    for (int piece = t; piece < NS * 64; piece += kBlock) {
        const int s = piece >> 6, L = piece & 63;
        const bf16_t *src = &rows[L & 31][16 * s + 8 * (L >> 5)];
        uint4 v;
        v.x = src[0] | ((uint32_t)src[1] << 16);
        v.y = src[2] | ((uint32_t)src[3] << 16);
        v.z = src[4] | ((uint32_t)src[5] << 16);
        v.w = src[6] | ((uint32_t)src[7] << 16);
        *reinterpret_cast<uint4 *>(rec + (int64_t)piece * 16) = v;
    }
    if (t < kTile) reinterpret_cast<float *>(rec + NS * 1024)[t] = bias[t];
}

// ---- 2. matrix-core sweep ------------------------------------------------------------------------
// Rows [row_begin, n) in blocks of PT * 32 rows per wave, PT even.
template <int D, int PT>
__global__ __launch_bounds__(kBlock, kMainOccupancy) void large_assign_kernel(int64_t row_begin, int64_t n, int64_t ld,
                                                                  int32_t tiles, const bf16_t *__restrict__ X,
                                                                  const unsigned char *__restrict__ records,
                                                                  int32_t *__restrict__ best_code) {
    constexpr int kPointTiles = PT;
    constexpr int kPointsPerWave = kTile * kPointTiles;
    static_assert(kPointTiles % 2 == 0, "two accumulators alternate over the point tiles");
    constexpr int NS = D / 16;
    constexpr int REC = record_bytes<D>();
    constexpr int REC16 = REC / 16;                    // 16-byte pieces per record
    constexpr int STAGE = (REC16 + kBlock - 1) / kBlock;  // pieces per thread
    __shared__ __attribute__((aligned(16))) unsigned char ring[3][REC];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, half = lane >> 5;
    float pos_inf = __builtin_inff();
    asm volatile("" : "+s"(pos_inf));

    const int64_t wave_blocks = (n - row_begin + kPointsPerWave - 1) / kPointsPerWave;
    const int64_t wg_blocks = (wave_blocks + kWaves - 1) / kWaves;

    // A record travels from global memory straight into its ring slot (LDS-direct loads: lane l of a
    // wave delivers its 16 bytes to the wave's LDS base + 16 l), STAGE pieces per thread; no
    // staging registers.  The loads count in vmcnt; the compiler waits for them before a barrier.
    typedef __attribute__((address_space(3))) void *lds_ptr;
    auto stage = [&](int tile, int slot) {
        const uint4 *src = reinterpret_cast<const uint4 *>(records + (int64_t)tile * REC);
#pragma unroll
        for (int q = 0; q < STAGE; ++q) {
            const int wave_piece = q * kBlock + wave * 64;   // uniform
            if (wave_piece + lane < REC16)
                __builtin_amdgcn_global_load_lds(src + wave_piece + lane, (lds_ptr)(ring[slot] + wave_piece * 16), 16, 0, 0);
        }
    };

    for (int64_t wb = blockIdx.x; wb < wg_blocks; wb += gridDim.x) {
        const int64_t row0 = row_begin + (wb * kWaves + wave) * kPointsPerWave;
        // Point operand: piece (p, s) of lane (half, col) = row row0 + 32 p + col, columns 16 s + 8 half .. + 7.
        // Buffer loads with a descriptor that ends at the last valid row: rows past n read as zeros.
        bf16x8 xb[kPointTiles][NS];
        {
            const int64_t rows_here = min((int64_t)kPointsPerWave, n - row0);
            const bool any = rows_here > 0;
            const int bytes = any ? (int)(((rows_here - 1) * ld + D) * 2) : 0;
            __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<bf16_t *>(X + (any ? row0 : 0) * ld), 0, bytes, 0x00020000);
#pragma unroll
            for (int p = 0; p < kPointTiles; ++p) {
                const int voff = (int)(((32 * p + col) * ld + 8 * half) * 2);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const u32x4 raw = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, 32 * s, 0);
                    xb[p][s] = __builtin_bit_cast(bf16x8, raw);
                }
            }
        }
        // Per point tile: the best score so far and the code of the group of 4 consecutive centroid
        // rows it came from, code = 8 tile + 2 group (+ half, added at the end).
        float best[kPointTiles];
        int32_t bcode[kPointTiles];
#pragma unroll
        for (int p = 0; p < kPointTiles; ++p) {
            best[p] = kNever;
            bcode[p] = 0;
        }

        // ring prologue: records 0 and 1
        __syncthreads();  // the previous block's readers are done with the ring
        {
            stage(0, 0);
            if (tiles > 1) stage(1, 1);
        }
        __syncthreads();

        // Epilogue of one 32 x 32 product: this lane holds 16 centroid rows of one point as 4 groups of
        // 4 consecutive rows.  Group maxima, their maximum, one compare, two selects.  Ties keep
        // the earlier tile (strict >) and, inside a tile, the lower group.
        // Maxima of 4 values in two instructions: a 3-input maximum, then the median of (that, the
        // fourth, +infinity), which is their maximum for ordered inputs.  A plain 2-input maximum of
        // matrix-instruction results costs three instructions (the compiler first quiets both
        // inputs); the median is a target operation it leaves alone.  +infinity is kept opaque in a
        // scalar register so that the median is not folded back into a maximum.
        float qm[4];
        auto max4 = [&](float v0, float v1, float v2, float v3) {
            return __builtin_amdgcn_fmed3f(fmaxf(fmaxf(v0, v1), v2), v3, pos_inf);
        };
        auto fold = [&](int piece, const f32x16 &acc, int p, int t) {   // pieces 0 .. 4, in order
            if (piece < 4) {
                const int j = piece;
                qm[j] = max4(acc[4 * j], acc[4 * j + 1], acc[4 * j + 2], acc[4 * j + 3]);
            } else {
                const float m = max4(qm[0], qm[1], qm[2], qm[3]);
                // lowest group that holds the maximum, as 0/1 arithmetic (a chain of selects here is
                // turned into branches by the compiler, which would split the instruction stream)
                const int e0 = qm[0] == m, e1 = qm[1] == m, e2 = qm[2] == m;
                const int grp = (1 - e0) * (1 + (1 - e1) * (2 - e2));
                const bool better = m > best[p];
                best[p] = better ? m : best[p];
                bcode[p] = better ? 8 * t + 2 * grp : bcode[p];
            }
        };

        // One accumulation chain per point tile (a chain of dependent matrix instructions runs at
        // the full rate), two accumulators in alternation: while the chain of point tile p runs, the
        // finished accumulator of the previous point tile is folded on the vector unit, so a wave
        // keeps the matrix pipe fed by itself instead of relying on the other wave of its SIMD
        // being out of phase.
        f32x16 acc[2];
        // bias of the 16 centroid rows this lane's accumulators stand for (rows 8 (v/4) + 4 half + v%4),
        // read from the record straight into the accumulator that the next chain starts from
        auto load_bias = [&](const unsigned char *rec) {
            f32x16 b;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 b4 = *reinterpret_cast<const f32x4 *>(rec + NS * 1024 + (8 * q + 4 * half) * 4);
                b[4 * q + 0] = b4[0];
                b[4 * q + 1] = b4[1];
                b[4 * q + 2] = b4[2];
                b[4 * q + 3] = b4[3];
            }
            return b;
        };
        for (int t = 0; t < tiles; ++t) {
            if (t + 2 < tiles) stage(t + 2, (t + 2) % 3);   // that slot's readers passed the last barrier

            const unsigned char *rec = ring[t % 3];
            bf16x8 a[NS];
#pragma unroll
            for (int s = 0; s < NS; ++s) a[s] = *reinterpret_cast<const bf16x8 *>(rec + (64 * s + lane) * 16);
            if (t == 0) acc[0] = load_bias(rec);
#pragma unroll
            for (int p = 0; p < kPointTiles; ++p) {
                // acc[p & 1] holds the bias; the other accumulator holds the previous chain's scores,
                // which are folded piece by piece behind the matrix instructions of this chain (the
                // scheduling barriers keep the pieces there: left alone, the compiler issues the chain
                // first, and a wave cannot issue past a matrix instruction that waits for the pipe)
                const bool have_prev = p > 0 || t > 0;
                const int pp = p > 0 ? p - 1 : kPointTiles - 1, pt = p > 0 ? t : t - 1;
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    acc[p & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], xb[p][s], acc[p & 1], 0, 0, 0);
                    constexpr int NF = NS - 1 < 5 ? NS - 1 : 5;   // chain slots that carry fold pieces
                    if (have_prev && s < NF) {
#pragma unroll
                        for (int piece = s * 5 / NF; piece < (s + 1) * 5 / NF; ++piece)
                            fold(piece, acc[(p + 1) & 1], pp, pt);
                    }
                    // the folded accumulator is free: preset it for the next chain while this one runs
                    if (s == NF && p + 1 < kPointTiles) acc[(p + 1) & 1] = load_bias(rec);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __syncthreads();
            // first chain of the next tile starts from that tile's bias (its record is published by the barrier)
            if (t + 1 < tiles) acc[0] = load_bias(ring[(t + 1) % 3]);
        }
#pragma unroll
        for (int piece = 0; piece < 5; ++piece) fold(piece, acc[(kPointTiles - 1) & 1], kPointTiles - 1, tiles - 1);

        // The code names the group of 4 consecutive centroid rows that holds the winner (rows
        // 8 group + 4 half .. + 3 of the tile).  Codes ascend with the centroid index, so the smaller
        // code wins a tie between the two halves of a column.
#pragma unroll
        for (int p = 0; p < kPointTiles; ++p) {
            int32_t code = bcode[p] + half;
            const float ob = __shfl_xor(best[p], 32, 64);
            const int32_t oc = __shfl_xor(code, 32, 64);
            if (ob > best[p] || (ob == best[p] && oc < code)) { best[p] = ob; code = oc; }
            const int64_t row = row0 + 32 * p + col;
            if (half == 0 && row < n) best_code[row] = code;
        }
    }
}

// ---- 3. winner inside the winning tile, distance, objective -------------------------------------
// 32 lanes per point.  The sweep names 4 consecutive centroid rows (4 * d contiguous bf16 values);
// they are read 512 bytes at a time across the 32 lanes, and the d/8 lanes that hold one
// centroid's pieces add their partial products with DPP row operations.  Rows come by in
// ascending order for every lane, so a strict > keeps the lowest index inside a lane group; the
// groups are merged with the same rule.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int LANES>  // sum over aligned groups of LANES (<= 16) consecutive lanes
__device__ __forceinline__ float group_sum(float v) {
    if (LANES >= 2) v = dpp_add<0xB1>(v);    // xor 1
    if (LANES >= 4) v = dpp_add<0x4E>(v);    // xor 2
    if (LANES >= 8) v = dpp_add<0x141>(v);   // mirror within 8
    if (LANES >= 16) v = dpp_add<0x140>(v);  // mirror within 16
    return v;
}
__device__ __forceinline__ float dot8(const uint4 &a, const uint4 &b, float acc) {
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.x), __builtin_bit_cast(bf16x2, b.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.y), __builtin_bit_cast(bf16x2, b.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.z), __builtin_bit_cast(bf16x2, b.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.w), __builtin_bit_cast(bf16x2, b.w), acc, false);
    return acc;
}

template <int D>
__global__ __launch_bounds__(kBlock) void large_refine_kernel(int64_t n, int64_t ld, int32_t k,
                                                               const bf16_t *__restrict__ X,
                                                               const bf16_t *__restrict__ cq16,
                                                               const float *__restrict__ hneg,
                                                               const int32_t *__restrict__ best_code,
                                                               int32_t *__restrict__ labels,
                                                               float *__restrict__ min_d2,
                                                               double *__restrict__ obj_part) {
    constexpr int CH = D / 8;          // 16-byte pieces per row = lanes per centroid
    constexpr int ROWS = 32 / CH;      // centroid rows covered by one 512-byte read
    constexpr int CAND = 4;            // candidate rows named by the sweep
    __shared__ double red[kBlock / 64];
    const int r = threadIdx.x & 31;
    const int chunk = r % CH, sub = r / CH;
    const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 5;
    const int64_t groups = ((int64_t)gridDim.x * kBlock) >> 5;
    double obj = 0.0;
    // The code and the row piece of the next point are loaded (unconditionally, from a clamped index) before this
    // point's candidate rows are waited for, and no load of the loop stands under a branch, so the compiler's wait
    // counts stay exact: the loop exposes one memory latency per point instead of two.
    int64_t i = group;
    int code_raw = best_code[i < n ? i : 0];
    uint4 xc = *reinterpret_cast<const uint4 *>(X + (i < n ? i : 0) * ld + 8 * chunk);
    for (int64_t i0 = 0; i0 < n; i0 += groups) {   // uniform trip count: the lane exchanges need every lane
        const bool valid = i < n;
        const int64_t i_next = i + groups;
        const int code_next = best_code[i_next < n ? i_next : 0];
        const uint4 xc_next = *reinterpret_cast<const uint4 *>(X + (i_next < n ? i_next : 0) * ld + 8 * chunk);
        const int code = valid ? code_raw : 0;
        // candidates: rows 8 group + 4 half .. + 3 of tile code / 8
        const int64_t first_row = (int64_t)(code >> 3) * kTile + 8 * ((code >> 1) & 3) + 4 * (code & 1);
        float best = kNever;
        int bidx = 0x7fffffff;
#pragma unroll
        for (int q = 0; q < (CAND + ROWS - 1) / ROWS; ++q) {
            const int row = q * ROWS + sub;
            const bool real = row < CAND && first_row + row < k;   // rows of the padded last tile are never read
            const int64_t at = real ? first_row + row : 0;          // (a lane without a row reads row 0 and ignores it)
            const uint4 cc = *reinterpret_cast<const uint4 *>(cq16 + at * D + 8 * chunk);
            const float bias = hneg[at];
            const float dot = group_sum<CH>(dot8(xc, cc, 0.f));
            const float score = real ? dot + bias : kNever;
            if (score > best) { best = score; bidx = (int)(first_row + row); }
        }
#pragma unroll
        for (int off = CH; off < 32; off <<= 1) {   // merge the lane groups (different rows)
            const float os = __shfl_xor(best, off, 64);
            const int oi = __shfl_xor(bidx, off, 64);
            if (os > best || (os == best && oi < bidx)) { best = os; bidx = oi; }
        }
        const float xx = group_sum<CH>(dot8(xc, xc, 0.f));
        if (valid && r == 0) {
            labels[i] = bidx;
            const float d2 = fmaxf(xx - 2.f * best, 0.f);
            if (min_d2) min_d2[i] = d2;
            obj += (double)d2;
        }
        i = i_next;
        code_raw = code_next;
        xc = xc_next;
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

__global__ __launch_bounds__(64) void large_sum_obj_kernel(const double *__restrict__ part, int count,
                                                            double *__restrict__ out) {
    const int l = threadIdx.x;
    double o = 0.0;
    for (int q = l; q < count; q += 64) o += part[q];
    for (int off = 32; off > 0; off >>= 1) o += __shfl_down(o, off, 64);
    if (l == 0) *out = o;
}

template <int D>
int launch_large(const ep_problem &p, const bf16_t *X, const float *C, const KmeansWs &w, int32_t *labels,
                 float *min_d2, double *objective, hipStream_t s) {
    const int tiles = (int)ceil_div(p.k, kTile);
    large_prep_kernel<D><<<tiles, kBlock, 0, s>>>(p.k, C, w.cq16, w.cnorm, w.records);
    EP_LAUNCH_CHECK();
    {
        // A grid of resident workgroups loops over the workgroup-blocks of 512 rows.  (Splitting off
        // the last, partly filled round into a launch of its own with half-size blocks was measured
        // and is slower: the chip is power-limited in this kernel, and the clock rises while the
        // last round drains.)
        const int64_t wg_blocks = ceil_div(ceil_div(p.n, (int64_t)kTile * kMainPointTiles), kWaves);
        const int grid = (int)std::min<int64_t>(wg_blocks, 256 * kMainOccupancy);
        ProfScope prof(EP_PROF_LLOYD_MAIN, s, true);
        if (prof.start_)   // timed launch: the events get the kernel's own begin and end
            hipExtLaunchKernelGGL((large_assign_kernel<D, kMainPointTiles>), dim3(grid), dim3(kBlock), 0, s, prof.start_,
                                  prof.stop_, 0, (int64_t)0, p.n, p.ld, tiles, X, w.records, w.best_tile);
        else
            large_assign_kernel<D, kMainPointTiles><<<grid, kBlock, 0, s>>>(0, p.n, p.ld, tiles, X, w.records, w.best_tile);
        EP_LAUNCH_CHECK();
    }
    const int blocks = (int)std::min<int64_t>(kObjBlocksMax, ceil_div(p.n, kBlock / 32));
    large_refine_kernel<D><<<blocks, kBlock, 0, s>>>(p.n, p.ld, p.k, X, w.cq16, w.cnorm, w.best_tile, labels, min_d2,
                                                     objective ? w.obj_part : nullptr);
    EP_LAUNCH_CHECK();
    if (objective) {
        large_sum_obj_kernel<<<1, 64, 0, s>>>(w.obj_part, blocks, objective);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

// ---- benchmark aid: the matrix instruction alone -------------------------------------------------
// 16 operand registers per lane from memory, then 16 * iters dependent-chain matrix instructions in two
// accumulation chains and nothing else: what the pipe sustains on these operand values.
constexpr int kMfmaBenchGrid = 512;
__global__ __launch_bounds__(kBlock, 2) void mfma_rate_kernel(const u32x4 *__restrict__ operands, int32_t iters,
                                                               float *__restrict__ sink) {
    bf16x8 a[8], b[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        a[s] = __builtin_bit_cast(bf16x8, operands[s * kBlock + threadIdx.x]);
        b[s] = __builtin_bit_cast(bf16x8, operands[(8 + s) * kBlock + threadIdx.x]);
    }
    f32x16 c0 = {}, c1 = {};
#pragma unroll 1
    for (int32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int s = 0; s < 8; ++s) c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], b[s], c0, 0, 0, 0);
#pragma unroll
        for (int s = 0; s < 8; ++s) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], b[7 - s], c1, 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) r += c0[q] + c1[q];
    if (r == 123.456f) *sink = r;   // keeps the chains alive
}

}  // namespace

int launch_bench_mfma(const void *operands, int32_t iters, float *sink, hipStream_t s) {
    mfma_rate_kernel<<<kMfmaBenchGrid, kBlock, 0, s>>>(static_cast<const u32x4 *>(operands), iters, sink);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

bool large_path_supported(const ep_problem &p) {
    return p.dtype == EP_BF16 && (p.d == 64 || p.d == 128) && p.k > 64 && p.ld < ((int64_t)1 << 23);
}

size_t large_record_bytes(const ep_problem &p) {
    return (size_t)ceil_div(p.k, kTile) * (p.d == 128 ? record_bytes<128>() : record_bytes<64>());
}

int launch_large_assign(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                        float *min_d2, double *objective, hipStream_t s) {
    const bf16_t *Xb = static_cast<const bf16_t *>(X);
    return p.d == 128 ? launch_large<128>(p, Xb, C, w, labels, min_d2, objective, s)
                      : launch_large<64>(p, Xb, C, w, labels, min_d2, objective, s);
}

}  // namespace ep
