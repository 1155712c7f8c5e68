// Lloyd round for partition-scale k: one kernel reads every embedding once, finds its nearest
// centroid and adds it to that centroid's sum.  Instantiated for 64 and 128 columns (k <= 64) and
// 256 columns (k <= 16), fp32 or bfloat16 rows; d below the instantiated width (a multiple of 4) is
// padded with zeros as the rows are read.  The assignment-only mode also serves fp32 rows with
// k > 64, one slice of 64 centroids per launch (launch_small_assign_sliced).
//
// What it computes (EmbedPart paper, Alg. 3, step P <- KMeans(E, k)): the assignment
// argmin_j ||x - c_j||^2 = argmax_j (x.c_j - ||c_j||^2 / 2), lowest j on ties, and the per-cluster
// sums and counts from which the second pass forms the means.
//
// Mapping to the hardware (one wave = 64 lanes, lane = 16 * g + c):
//   * A wave owns a contiguous range of 16-point sub-tiles.  A sub-tile is read with buffer loads
//     in the layout the score product wants (lane (g, c): point c, columns 16 j + 4 g .. + 3),
//     one or two sub-tiles ahead of the arithmetic.
//   * Scores on the matrix cores, points as rows and 16 centroids per tile as columns, the
//     accumulators preset to -||c||^2 / 2 (formed by the wave itself in its prologue):
//       k <= 16: v_mfma_f32_16x16x4_f32;
//       k >  16: six bf16 products of an exact three-way bf16 split of x and c
//                (v_mfma_f32_16x16x32_bf16), as accurate as the fp32 instruction at a third of
//                its time.
//   * The result holds, in lane (g, c), the scores of points 4g .. 4g + 3 against centroid c; the
//     arg-max is a 16-lane DPP butterfly on an order-preserving integer key (maximum first, then
//     the lowest index among the lanes that hold it).  Labels are buffered in LDS and written
//     out in bursts.
//   * Sums without atomics and in a fixed order:
//       k <= 16: sums[centroid][column] += onehot[centroid][point] * x[point][column] on the fp32
//                matrix cores (multiplying by exact 0/1 keeps every addition an ordinary fp32
//                addition), accumulators in registers for the whole life of the wave; the operand
//                needs the transposed layout, which costs one trip through a padded LDS tile;
//       k >  16: a k x d table of sums per wave in LDS; the points of a sub-tile are ranked among
//                the earlier points with the same label, and round r adds the rows of rank r.
//   * k <= 32 runs two waves per SIMD; 32 < k <= 64 leaves room for one, and its fused loop is
//     software-pipelined by hand (the previous sub-tile's vector work sits between the matrix
//     instructions of the current one).
//   * bfloat16 rows are widened to fp32 on arrival; the centroids are rounded to bfloat16 for the
//     scores, so for k > 16 one of the six split products is left.
//   * At the end the four waves of a workgroup add their sums in wave order through LDS and store
//     one partial per workgroup; lloyd_small_finalize_kernel reduces those in fp64.
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "kernels.h"
#include "small_common.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kSub = 16;  // points per sub-tile
constexpr double kLastLevelCacheBytes = 256.0 * 1024 * 1024;   // MI355X: 256 MB memory-side cache
constexpr int kLabelFlush = 64;                  // sub-tiles whose labels are written out together (4 KB)

enum Mode { kAssignOnly = 0, kUpdateOnly = 1, kFused = 2 };


// Dynamic LDS of lloyd_small_kernel: floats (transposition tiles, or per-wave tables of sums for
// k > 16) followed by the per-wave label buffers.
template <int D, int KT>
struct SmallLds {
    static constexpr int kStride = D + 4;
    static constexpr int kFlush = KT >= 2 ? 16 : kLabelFlush;   // sub-tiles per label flush
    static constexpr int kFloatBytes = (KT >= 2 ? kWaves * (16 * KT + 1) * kStride : kWaves * kSub * kStride) * 4;
    static constexpr int kBytes = kFloatBytes + kWaves * kFlush * kSub * 4;
};

// XSQ: also accumulate sum ||x||^2 (needed once per data set for the objective).
// XT: element type of X.  bfloat16 rows are widened to fp32 as they arrive (exact) and the centroids
// are rounded to bfloat16 for the scores (the reading taken for bfloat16 embeddings: see
// large_assign_kernel); sums and means use the data in full precision.
// PAD: the rows have d < D columns (d a multiple of 4, passed at run time); columns d .. D - 1 are
// read as zeros (their loads are sent out of the buffer's range), which changes neither scores nor
// sums, and only the first d columns of the centroids exist in memory.
// BND (fused rounds only): also leave, per point, the distance bounds that the bounded rounds start from
// (upper bound on the distance to the own centroid from the best score, lower bound on the distance to all
// others from the second-best score; see kmeans_bounds.hip) in ub / lb.
template <int D, int KT, int MODE, bool XSQ, bool STREAM, typename XT, bool PAD, bool BND = false>
__global__ __launch_bounds__(kBlock, (KT <= 2 && D <= 128) ? 2 : 1) void lloyd_small_kernel(
    int64_t n, int64_t ld, int32_t d, int32_t k, int64_t subtiles_per_wave, int64_t waves_with_one_more,
    const XT *__restrict__ X,
    const float *__restrict__ C, int32_t *__restrict__ labels_out,
    const int32_t *__restrict__ labels_in, float *__restrict__ min_d2, float *__restrict__ psum,
    int32_t *__restrict__ pcnt, double *__restrict__ s_part, double *__restrict__ xsq_part,
    int32_t label_base, float *__restrict__ best_score, float *__restrict__ ub = nullptr,
    float *__restrict__ lb = nullptr) {
    static_assert(!BND || MODE == kFused, "bounds are taken in a fused round");
    constexpr int NJ = D / 16;       // 16-byte pieces per lane in the transposed layout; also column tiles
    constexpr int NH = D / 64;       // 16-byte pieces per lane and point in the load layout
    constexpr int STRIDE = D + 4;    // padded LDS row: consecutive rows start 4 banks apart
    // k <= 16: sums on the matrix cores (register accumulators).  Larger k: the matrix cores would
    // spend k/16 times the work of the scores on mostly-zero one-hot products, so every wave keeps
    // its own padded k x d table of sums in LDS and adds rows to it (see add_rows_to_lds_sums).
    constexpr bool kLdsSums = KT >= 2;
    constexpr bool kBf16 = std::is_same<XT, bf16_t>::value;
    constexpr bool kHalf = std::is_same<XT, f16_t>::value;   // widened on arrival, then handled as fp32 rows
    constexpr int kElem = (int)sizeof(XT);
    const int dr = PAD ? d : D;                  // columns that exist in memory
    constexpr int kOutOfRange = 0x7f000000;      // a byte offset beyond any sub-tile: the load returns zeros
    constexpr int kFlush = SmallLds<D, KT>::kFlush;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];
    float *lds = reinterpret_cast<float *>(dyn_lds);                       // transposition tiles | per-wave sums
    int32_t *label_lds = reinterpret_cast<int32_t *>(dyn_lds + SmallLds<D, KT>::kFloatBytes);
    __shared__ float xn_lds[kWaves][kSub];
    __shared__ double red[2][kWaves];
    __shared__ int32_t cnt_lds[16 * KT];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: keeps the loop scalar
    const int g = lane >> 4, c = lane & 15;
    float *tile = lds + wave * kSub * STRIDE;                // !kLdsSums
    float *wsums = lds + wave * (16 * KT + 1) * STRIDE;       // kLdsSums: this wave's sums (+ one idle row), row stride STRIDE
    if (kLdsSums && MODE != kAssignOnly) {
        for (int i = lane; i < (16 * KT + 1) * STRIDE; i += 64) wsums[i] = 0.f;
        if (threadIdx.x < 16 * KT) cnt_lds[threadIdx.x] = 0;
        __syncthreads();
    }

    // Centroid operand of the assignment product: lane (g, c) holds, for centroid 16*mt + c,
    // columns 16j + 4g .. 16j + 4g + 3 for every j.  Padding centroids can never win.
    //
    // k > 16 (kSplit): the fp32 matrix instructions would bound the kernel (2 k d flop per point at a
    // sixteenth of the bf16 rate), so x and c are each written as an exact sum of three bf16 terms
    // h + m + l and x.c is taken as the six bf16 products hh + hm + mh + hl + lh + mm with fp32
    // accumulation.  The dropped products (ml, lm, ll) are below 2^-23 |x_i c_i|, the size of fp32
    // rounding itself.  One bf16 instruction covers 32 columns: columns 16(2s) + 4g .. + 3 and
    // 16(2s+1) + 4g .. + 3 for K-step s, the same for both operands (the reduction index is free).
    constexpr bool kSplit = KT >= 2 || kBf16;   // scores on the bf16 instructions (bfloat16 rows: at any k)
    constexpr int KS = D / 32;       // K-steps of the bf16 instruction
    f32x4 creg[kSplit ? 1 : KT][kSplit ? 1 : NJ];
    // bfloat16 data: x is its own high term and the rounded centroid has no lower terms either, so of
    // the six products only xh.ch is left and cm, cl are not kept.
    constexpr bool kThreeTerms = kSplit && !kBf16;
    u32x4 ch[kSplit ? KT : 1][kSplit ? KS : 1], cm[kThreeTerms ? KT : 1][kThreeTerms ? KS : 1],
        cl[kThreeTerms ? KT : 1][kThreeTerms ? KS : 1];
    float hn[KT];   // -||c||^2 / 2 of centroid 16*mt + c: the value the score accumulators start from
    float cmax2 = 0.f;   // BND: max ||c||^2 over the centroids (rounded up), the same in every lane
    // Called after the first sub-tile's loads have been issued, so that the two latencies overlap.
    auto load_centroids = [&]() {
        if (MODE != kUpdateOnly) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const int cent = 16 * mt + c;
                const bool real = cent < k;
                double nacc = 0.0;   // this lane's quarter of ||c||^2, in fp64, columns in ascending order
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    f32x4 v = {0.f, 0.f, 0.f, 0.f};
                    if (real && (!PAD || 16 * j + 4 * g < dr))
                        v = *reinterpret_cast<const f32x4 *>(C + (int64_t)cent * dr + 16 * j + 4 * g);
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
                // the four lanes (g = 0..3) that hold the centroid add their quarters pairwise; the two
                // additions commute, so all four get the same bits
                nacc += __shfl_xor(nacc, 16, 64);
                nacc += __shfl_xor(nacc, 32, 64);
                hn[mt] = real ? (float)(-0.5 * nacc) : -3.0e38f;
                if (BND && real) cmax2 = fmaxf(cmax2, (float)nacc * kUp);
            }
            if constexpr (BND) cmax2 = key_float(row16_max(float_key(cmax2)));
            if constexpr (kSplit) {
                // The 3 * KT * KS operands are only ever read by matrix instructions: pin them to the
                // accumulation registers, which those instructions read directly.  Left to itself the
                // register allocator parks them there as spilled vector registers and copies four
                // words back before every instruction.
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
        }
    };

    f32x4 accu[KT][NJ];  // sums: lane (g, c), register v <-> centroid 16*mt + 4g + v, column col(t, c)
    int32_t cnt[KT];
#pragma unroll
    for (int mt = 0; mt < KT; ++mt) {
        cnt[mt] = 0;
#pragma unroll
        for (int t = 0; t < NJ; ++t) accu[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    double obj_x = 0.0, obj_s = 0.0;

    // Every wave owns a contiguous range of sub-tiles (a fixed function of n and the grid).
    const int64_t total_sub = (n + kSub - 1) / kSub;
    // (the first waves_with_one_more waves of the grid take one sub-tile more than the others)
    const int64_t wave_id = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t first = wave_id * subtiles_per_wave + min(wave_id, waves_with_one_more);
    const int64_t last = min(total_sub, first + subtiles_per_wave + (wave_id < waves_with_one_more ? 1 : 0));

    // Rows are read with buffer loads: the descriptor is rebuilt per sub-tile from a scalar base
    // and covers exactly the sub-tile's valid bytes, so lanes that would read past the last row
    // get zeros from the hardware bounds check and the loop needs no ragged special case.
    // Two lane layouts (16 * ld * 4 < 2^31 is checked on the host):
    //   point-per-lane (assignment operand): lane (g, c), piece j = row c, columns 16j + 4g .. + 3;
    //     each 4-lane group reads one aligned 64-byte segment, pieces j, j + 1 share a cache line.
    //   row-per-group (sum operand): lane (g, c), piece (r, h) = row 4g + r, columns 64h + 4c .. + 3.
    constexpr int NX = NJ;  // 16-byte pieces per lane and sub-tile (NJ == 4 * NH)
    constexpr bool kPointPerLane = MODE != kUpdateOnly || KT >= 2;
    int voff[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) voff[r] = (int)(((4 * g + r) * ld + 4 * c) * kElem);
    const int voff_a = (int)((c * ld + 4 * g) * kElem);

    auto load_subtile = [&](int64_t st, f32x4(&dst)[NX]) {
        // A sub-tile past this workgroup's range gets an empty descriptor: the loads are still
        // issued (so that the number of loads in flight is the same on every path and the waits
        // before the first use stay exact) but touch no memory and return zeros.
        const bool live = st < last;
        const int64_t row0 = live ? st * kSub : 0;
        const int rows_here = (int)min((int64_t)kSub, n - row0);
        const int bytes = live ? (int)(((rows_here - 1) * ld + dr) * kElem) : 0;
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<XT *>(X + row0 * ld), 0, bytes, 0x00020000);
        // STREAM: a matrix larger than the last-level cache is read with the non-temporal hint (it
        // cannot be there again next round, and the hint buys ~2% of stream rate); a smaller one is
        // left to the caches, which serve it in the later rounds.
        constexpr int kAux = STREAM ? 2 : 0;
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            int va = voff_a, vr = voff[q / NH];
            if constexpr (PAD) {   // pieces whose columns do not exist
                va = 16 * q + 4 * g < dr ? va : kOutOfRange;
                vr = 64 * (q % NH) + 4 * c < dr ? vr : kOutOfRange;
            }
            if constexpr (kBf16) {   // the same four columns per piece, 8 bytes of them
                const u32x2 raw = kPointPerLane
                                      ? __builtin_amdgcn_raw_buffer_load_b64(rsrc, va, 32 * q, kAux)
                                      : __builtin_amdgcn_raw_buffer_load_b64(rsrc, vr, 128 * (q % NH), kAux);
                dst[q] = f32x4{__uint_as_float(raw[0] << 16), __uint_as_float(raw[0] & 0xffff0000u),
                               __uint_as_float(raw[1] << 16), __uint_as_float(raw[1] & 0xffff0000u)};
            } else if constexpr (kHalf) {
                const u32x2 raw = kPointPerLane
                                      ? __builtin_amdgcn_raw_buffer_load_b64(rsrc, va, 32 * q, kAux)
                                      : __builtin_amdgcn_raw_buffer_load_b64(rsrc, vr, 128 * (q % NH), kAux);
                dst[q] = __builtin_convertvector(__builtin_bit_cast(f16x4_t, raw), f32x4);
            } else {
                const u32x4 raw = kPointPerLane
                                      ? __builtin_amdgcn_raw_buffer_load_b128(rsrc, va, 64 * q, kAux)
                                      : __builtin_amdgcn_raw_buffer_load_b128(rsrc, vr, 256 * (q % NH), kAux);
                dst[q] = __builtin_bit_cast(f32x4, raw);
            }
        }
    };

    // Labels are collected in a wave-private LDS buffer and written kLabelFlush sub-tiles at a
    // time as whole, consecutive cache lines.  Single 64-byte label writes scattered through the
    // read stream cost about a tenth of the kernel's time in DRAM read/write turnarounds; bursts
    // of 4 KB cost almost nothing.
    int32_t *lbuf = label_lds + wave * kFlush * kSub;
    int buffered = 0;  // sub-tiles in the buffer (uniform)
    auto flush_labels = [&](int64_t next_st) {
        if (MODE == kUpdateOnly || buffered == 0) return;
        wave_lds_fence();
        const int64_t base_row = (next_st - buffered) * kSub;
        for (int q = lane; q < buffered * 4; q += 64) {
            const i32x4 v = *reinterpret_cast<const i32x4 *>(lbuf + 4 * q);
            const int64_t row = base_row + 4 * q;
            if (row + 3 < n) {
                *reinterpret_cast<i32x4 *>(labels_out + row) = v;
            } else {
                for (int e = 0; e < 4; ++e)
                    if (row + e < n) labels_out[row + e] = (int32_t)v[e];
            }
        }
        wave_lds_fence();
        buffered = 0;
    };

    // Scores of a sub-tile on the bf16 instructions (kSplit): acc[mt] += x . c over all columns, small
    // products first.  The operands of K-step s + 1 are split while the products of K-step s are
    // issued; after_group(i) is called after each of the 6 * KS groups of KT instructions.
    u32x4 xh[2], xm[2], xl[2];
    auto split_x = [&](const f32x4(&x)[NX], int s, int pr) {   // pair pr (0..3) of K-step s
        const f32x4 &v = x[2 * s + (pr >> 1)];
        const Split3 t = split3_pair(v[2 * (pr & 1)], v[2 * (pr & 1) + 1]);
        xh[s & 1][pr] = t.h, xm[s & 1][pr] = t.m, xl[s & 1][pr] = t.l;
    };
    constexpr int kScoreGroups = kThreeTerms ? 6 * KS : KS;   // groups of KT matrix instructions per sub-tile
    auto split_scores = [&](const f32x4(&x)[NX], f32x4(&acc)[KT], auto &&after_group) {
        if constexpr (!kThreeTerms) {   // widened bfloat16: the operand is the upper halves, packed again
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
                after_group(s);
            }
            return;
        }
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) split_x(x, 0, pr);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int pp = 0; pp < 6; ++pp) {   // xh.cl, xl.ch, xm.cm, xh.cm, xm.ch, xh.ch
                const u32x4 &a = pp == 1 ? xl[s & 1] : (pp == 2 || pp == 4) ? xm[s & 1] : xh[s & 1];
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) {
                    const u32x4 &b = pp == 0 ? cl[mt][s] : (pp == 2 || pp == 3) ? cm[mt][s] : ch[mt][s];
                    acc[mt] = mfma_bf16_k32(a, b, acc[mt]);
                }
                if (pp < 4 && s + 1 < KS) split_x(x, s + 1, pp);
                after_group(s * 6 + pp);
            }
    };

    // BND: bounds of the 16 points of a sub-tile from the row maxima of their best (bk) and second-best (sk)
    // scores and this lane's quarter of ||x_c||^2; lane c < 4 of every 16-lane row owns point 4 g + c.
    auto store_bounds = [&](int bk0, int bk1, int bk2, int bk3, int sk0, int sk1, int sk2, int sk3, float xpart,
                            int64_t row0, int rows) __attribute__((always_inline)) {
        float xn = xpart;
        xn += __shfl_xor(xn, 16, 64);
        xn += __shfl_xor(xn, 32, 64);   // ||x||^2 of point c, in all four lanes that hold a quarter of it
        const int sel = c & 3;
        const float s_best = key_float(sel == 0 ? bk0 : sel == 1 ? bk1 : sel == 2 ? bk2 : bk3);
        const float s_second = key_float(sel == 0 ? sk0 : sel == 1 ? sk1 : sel == 2 ? sk2 : sk3);
        const float own_xn = __shfl(xn, 4 * g + sel, 64);
        float u, l;
        fresh_bounds(own_xn, s_best, s_second, cmax2, u, l);
        if (c < 4 && 4 * g + c < rows) {
            ub[row0 + 4 * g + c] = u;
            lb[row0 + 4 * g + c] = l;
        }
    };

    auto process = [&](int64_t st, const f32x4(&x)[NX]) {
        const int64_t row0 = st * kSub;
        const int rows_here = (int)min((int64_t)kSub, n - row0);  // uniform
        int32_t lab[4];
        f32x4 bt[NX];  // sum operand: piece r * NH + h
        // Assignment over a slice of the centroids (best_score != nullptr, assignment mode only): the
        // best score of the earlier slices is fetched now and met at the end of the sub-tile.
        float earlier_best = -3.4e38f;
        if (MODE == kAssignOnly && best_score && label_base > 0 && c < 4 && 4 * g + c < rows_here)
            earlier_best = best_score[row0 + 4 * g + c];
        if (MODE != kUpdateOnly) {
            // The sum product needs the other layout: the sub-tile goes through the wave's LDS tile
            // (written point-per-lane, read row-per-group) in the shadow of the score product.
            if (MODE == kFused && !kLdsSums) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) *reinterpret_cast<f32x4 *>(tile + c * STRIDE + 16 * j + 4 * g) = x[j];
            }

            // scores.  k <= 16: fp32 matrix instructions, two accumulation chains per centroid tile
            // (even / odd j), added at the end.  k > 16: bf16 split products (the same arithmetic as the
            // pipelined loop below: both give the same scores bit for bit)
            f32x4 acc0[KT], acc1[KT];
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                acc0[mt] = f32x4{hn[mt], hn[mt], hn[mt], hn[mt]};
                acc1[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            if constexpr (kSplit) {
                split_scores(x, acc0, [](int) {});
            } else {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int mt = 0; mt < KT; ++mt) {
                            if (j & 1)
                                acc1[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j][e], creg[mt][j][e], acc1[mt], 0, 0, 0);
                            else
                                acc0[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j][e], creg[mt][j][e], acc0[mt], 0, 0, 0);
                        }
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) acc0[mt] += acc1[mt];
            }

            if (MODE == kFused && !kLdsSums) {
                wave_lds_fence();
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int h = 0; h < NH; ++h)
                        bt[r * NH + h] =
                            *reinterpret_cast<const f32x4 *>(tile + (4 * g + r) * STRIDE + 64 * h + 4 * c);
                wave_lds_fence();  // the tile is overwritten by the next sub-tile
            }

            float xpart = 0.f;
            if (XSQ || BND || min_d2) {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    xpart += x[j][0] * x[j][0] + x[j][1] * x[j][1] + x[j][2] * x[j][2] + x[j][3] * x[j][3];
            }

            // argmax over centroids: inside the lane over tiles (ascending index, strict >), then a
            // 16-lane butterfly on an order-preserving integer key: the maximum first, then the
            // lowest index among the lanes that hold it.
            int bkey[4], skey[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float sc = acc0[0][v];
                int idx = c;
                float m1 = acc0[0][v], m2 = -3.4e38f;   // BND: the lane's largest and second-largest (equal values count twice)
#pragma unroll
                for (int mt = 1; mt < KT; ++mt) {
                    const float s2 = acc0[mt][v];
                    if (s2 > sc) { sc = s2; idx = 16 * mt + c; }
                    if constexpr (BND) {
                        if (s2 > m1) { m2 = m1; m1 = s2; }
                        else if (s2 > m2) { m2 = s2; }
                    }
                }
                const int key = float_key(sc);
                bkey[v] = row16_max(key);
                const int win = row16_min(key == bkey[v] ? idx : 0x7fffffff);
                lab[v] = (4 * g + v < rows_here) ? win : -1;
                // every lane offers its best, the winner's lane what is left without the winning entry
                if constexpr (BND) skey[v] = row16_max(float_key(c == (win & 15) ? m2 : m1));
            }
            if constexpr (BND)
                store_bounds(bkey[0], bkey[1], bkey[2], bkey[3], skey[0], skey[1], skey[2], skey[3], xpart, row0, rows_here);

            // lane c < 4 of every group owns point 4g + c for the stores and the objective
            const int sel = c & 3;
            const float my_s = key_float(sel == 0 ? bkey[0] : sel == 1 ? bkey[1] : sel == 2 ? bkey[2] : bkey[3]);
            const int32_t my_l = sel == 0 ? lab[0] : sel == 1 ? lab[1] : sel == 2 ? lab[2] : lab[3];
            const bool owner = c < 4 && 4 * g + c < rows_here;
            bool sliced = false;
            if constexpr (MODE == kAssignOnly) sliced = best_score != nullptr;   // uniform
            float fin_s = my_s;   // the point's best score over this and the earlier slices
            if (sliced) {   // strict >: on equal scores the earlier slice (lower index) keeps the point
                const bool better = my_s > earlier_best;
                fin_s = better ? my_s : earlier_best;
                if (owner) {
                    if (better) labels_out[row0 + 4 * g + c] = my_l + label_base;
                    best_score[row0 + 4 * g + c] = fin_s;
                }
            } else {
                if (c < 4) lbuf[buffered * kSub + 4 * g + c] = my_l;
                ++buffered;
            }
            if (kLdsSums && !sliced) {   // every lane of a 16-lane row keeps the row's sum; lane c == 0's is used
#pragma unroll
                for (int v = 0; v < 4; ++v) obj_s += (double)(4 * g + v < rows_here ? key_float(bkey[v]) : 0.f);
            } else if (owner) {
                obj_s += (double)fin_s;
            }
            if (XSQ && c < rows_here) obj_x += (double)xpart;
            if (min_d2) {  // uniform branch
                float xn = xpart;
                xn += __shfl_xor(xn, 16, 64);
                xn += __shfl_xor(xn, 32, 64);
                if (g == 0) xn_lds[wave][c] = xn;
                wave_lds_fence();
                if (owner) min_d2[row0 + 4 * g + c] = fmaxf(xn_lds[wave][4 * g + c] - 2.f * fin_s, 0.f);
                wave_lds_fence();
            }
        } else if (!kLdsSums) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int32_t l = (4 * g + v < rows_here) ? labels_in[row0 + 4 * g + v] : -1;
                lab[v] = (l >= 0 && l < k) ? l : -1;
            }
#pragma unroll
            for (int q = 0; q < NX; ++q) bt[q] = x[q];
        }

        if (MODE != kAssignOnly && kLdsSums) {
            // label of point c (this lane's point in the point-per-lane layout)
            int32_t lab_c;
            if (MODE == kFused) {
                wave_lds_fence();
                lab_c = lbuf[(buffered - 1) * kSub + c];
            } else {
                const int32_t l = c < rows_here ? labels_in[row0 + c] : -1;
                lab_c = (l >= 0 && l < k) ? l : -1;
            }
            add_rows_to_lds_sums<NJ, STRIDE>(x, lab_c, g, wsums, cnt_lds);
        }

        if (MODE != kAssignOnly && !kLdsSums) {
            if constexpr (kBf16 && KT == 1) {
                // bfloat16 rows: one bf16 instruction takes all four points a lane holds (K = 16 points);
                // the one-hot operand and the rows are exact in bfloat16.  (For fp32 rows the same with
                // an exact three-term split of the rows was measured: no faster than the fp32 products.)
                u32x2 a;
                a[0] = (lab[0] == c ? 0x3F80u : 0u) | (lab[1] == c ? 0x3F800000u : 0u);
                a[1] = (lab[2] == c ? 0x3F80u : 0u) | (lab[3] == c ? 0x3F800000u : 0u);
                cnt[0] += (lab[0] == c) + (lab[1] == c) + (lab[2] == c) + (lab[3] == c);
#pragma unroll
                for (int t = 0; t < NJ; ++t) {
                    const int h = t >> 2, e = t & 3;
                    u32x2 b;
                    b[0] = (__float_as_uint(bt[1 * NH + h][e]) & 0xffff0000u) | (__float_as_uint(bt[0 * NH + h][e]) >> 16);
                    b[1] = (__float_as_uint(bt[3 * NH + h][e]) & 0xffff0000u) | (__float_as_uint(bt[2 * NH + h][e]) >> 16);
                    accu[0][t] = mfma_bf16_k16(a, b, accu[0][t]);
                }
            } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) {
                    const bool hit = lab[r] == 16 * mt + c;
                    const float a = hit ? 1.f : 0.f;
                    cnt[mt] += hit ? 1 : 0;
#pragma unroll
                    for (int t = 0; t < NJ; ++t)
                        accu[mt][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bt[r * NH + (t >> 2)][t & 3], accu[mt][t],
                                                                           0, 0, 0);
                }
            }
        }
    };

    // (with the bounds option at d = 128 the pipeline's three register sets no longer fit: that one round runs the
    // plain loop)
    if constexpr (kLdsSums && MODE == kFused && KT >= 4 && !(BND && D == 128)) {
        // k > 32, fused round.  With four centroid tiles the split centroid operand (192 registers) and
        // the sum tables (137 KB) leave room for one wave per SIMD only, so nothing else hides a wave's
        // latencies.  (Two tiles fit two waves per SIMD and run the plain loop below: measured
        // 304 us against 385 us for this pipeline at one wave, n = 2.45 M, k = 32.)
        // Everything that is not part of the score product
        // (arg-max, labels, ranks, the row adds into the LDS sums) is done one sub-tile late, in the
        // issue slots between the matrix instructions of the next sub-tile.  The deferred work of the
        // previous sub-tile is a list of items (4 arg-max, label store, 2 rank halves, one per 16-byte
        // piece of the fixed row-add rounds) spread evenly, in program order, over the 6 * KS groups of
        // matrix instructions.  The items hold no branch (lanes with nothing to do write to scrap
        // words instead), so the whole step is one basic block whose order the scheduling barriers fix.
        // Ranks 0 and 1 without branches, higher ranks (a tenth of the sub-tiles at k = 64) in a loop.  A
        // third fixed round was measured: its 8 row-add pieces per sub-tile cost more than the branches
        // they save (16.6 -> 15.95 ms per round on 111 M points).
        constexpr int kFixedRounds = 2;
        constexpr int kFirstAdd = 7;                       // items 0 .. 6: arg-max (4), labels, rank (2)
        constexpr int kItems = kFirstAdd + kFixedRounds * NJ;
        constexpr int kGroups = kScoreGroups;
        __shared__ __attribute__((aligned(16))) int32_t scrap[4 * kBlock];   // 16 bytes per lane, written by idle lanes, never read
        float *dummy = wsums + 16 * KT * STRIDE + 4 * g;   // the extra row idle lanes add to; never read
        f32x4 scp[KT];         // previous sub-tile: scores
        int prev_rows = 0;     // rows of the previous sub-tile
        int bkeyp[4], skeyp[4];
        int64_t prev_st = 0;   // the previous sub-tile
        int32_t labp[4];
        int32_t lab_c = -1;
        int rank = -1;
        float *rowp = dummy;
        f32x4 pending = {0.f, 0.f, 0.f, 0.f};   // LDS read of the next row-add piece, in flight

        auto item = [&](int b, const f32x4(&xp)[NX]) {   // b = 0 .. kItems - 1, uniform
            if (b < 4) {   // arg-max of point group v = b
                const int v = b;
                float sc = scp[0][v];
                int idx = c;
                float m1 = scp[0][v], m2 = -3.4e38f;   // BND: as in process()
#pragma unroll
                for (int mt = 1; mt < KT; ++mt) {
                    const float s2 = scp[mt][v];
                    if (s2 > sc) { sc = s2; idx = 16 * mt + c; }
                    if constexpr (BND) {
                        if (s2 > m1) { m2 = m1; m1 = s2; }
                        else if (s2 > m2) { m2 = s2; }
                    }
                }
                const int key = float_key(sc);
                bkeyp[v] = row16_max(key);
                const int win = row16_min(key == bkeyp[v] ? idx : 0x7fffffff);
                labp[v] = (4 * g + v < prev_rows) ? win : -1;
                if constexpr (BND) skeyp[v] = row16_max(float_key(c == (win & 15) ? m2 : m1));
            } else if (b == 4) {   // labels to the LDS buffer, objective terms
                // every lane of a 16-lane row holds the row's four results: lane c == 0 stores them,
                // and every lane keeps the running sum of best scores (only lane c == 0's is used)
                i32x4 *dst = reinterpret_cast<i32x4 *>(c == 0 ? lbuf + buffered * kSub + 4 * g : scrap + 4 * threadIdx.x);
                *dst = i32x4{labp[0], labp[1], labp[2], labp[3]};
#pragma unroll
                for (int v = 0; v < 4; ++v) obj_s += (double)(4 * g + v < prev_rows ? key_float(bkeyp[v]) : 0.f);
                if (XSQ || BND) {
                    float xpart = 0.f;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        xpart += xp[j][0] * xp[j][0] + xp[j][1] * xp[j][1] + xp[j][2] * xp[j][2] + xp[j][3] * xp[j][3];
                    if (XSQ) obj_x += (double)(c < prev_rows ? xpart : 0.f);
                    if constexpr (BND)
                        store_bounds(bkeyp[0], bkeyp[1], bkeyp[2], bkeyp[3], skeyp[0], skeyp[1], skeyp[2], skeyp[3], xpart,
                                     prev_st * kSub, prev_rows);
                }
                wave_lds_fence();
            } else if (b == 5) {   // label of this lane's point; first half of its rank among earlier equal labels
                lab_c = lbuf[buffered * kSub + c];
                ++buffered;
                rank = same_label_before<1, 8>(lab_c, 0);
                int32_t *cp = (g == 0 && lab_c >= 0) ? cnt_lds + lab_c : scrap + threadIdx.x;
                atomicAdd(cp, 1);   // integer: order does not matter
            } else if (b == 6) {
                rank = same_label_before<9, 15>(lab_c, rank);
                if (lab_c < 0) rank = -1;
                rowp = wsums + (lab_c < 0 ? 0 : lab_c) * STRIDE + 4 * g;
                pending = *reinterpret_cast<const f32x4 *>((rank == 0 ? rowp : dummy));   // read of piece 0
            } else {
                // one 16-byte piece of one round of row adds; its read was issued one item earlier, the
                // next piece's read is issued here (a round never touches a column group twice, and the
                // same column group of the next round comes NJ items later)
                const int q = b - kFirstAdd, r = q / NJ, j = q % NJ;
                f32x4 *p = reinterpret_cast<f32x4 *>((rank == r ? rowp : dummy) + 16 * j);
                const f32x4 sum = pending + xp[j];
                if (q + 1 < kFixedRounds * NJ) {
                    const int r1 = (q + 1) / NJ, j1 = (q + 1) % NJ;
                    pending = *reinterpret_cast<const f32x4 *>((rank == r1 ? rowp : dummy) + 16 * j1);
                }
                *p = sum;
            }
        };
        auto finish_prev = [&](const f32x4(&xp)[NX]) {   // ranks beyond the fixed rounds
            for (int r = kFixedRounds; __ballot(rank >= r) != 0; ++r) {
                if (rank == r) {
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        f32x4 *p = reinterpret_cast<f32x4 *>(rowp + 16 * j);
                        *p = *p + xp[j];
                    }
                }
                wave_lds_fence();
            }
        };

        // scores of sub-tile st (in x); with DEFERRED, the previous sub-tile's (in xp) other work in between
        auto step = [&](int64_t st, const f32x4(&x)[NX], const f32x4(&xp)[NX], auto deferred) {
            constexpr bool DEFERRED = decltype(deferred)::value;
            f32x4 acc[KT];
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) acc[mt] = f32x4{hn[mt], hn[mt], hn[mt], hn[mt]};
            split_scores(x, acc, [&](int grp) {
                if (DEFERRED) {
#pragma unroll
                    for (int b = grp * kItems / kGroups; b < (grp + 1) * kItems / kGroups; ++b) item(b, xp);
                    __builtin_amdgcn_sched_barrier(0);   // pin the interleaving
                }
            });
            // the scores are pinned here, in the block of the matrix instructions, so that no later
            // block is a better place for them in the compiler's eyes
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                scp[mt] = acc[mt];
                asm volatile("" : "+v"(scp[mt]));
            }
            __builtin_amdgcn_sched_barrier(0);
            if (DEFERRED) finish_prev(xp);
            prev_rows = (int)min((int64_t)kSub, n - st * kSub);
            prev_st = st;
        };
        auto drain = [&](const f32x4(&xp)[NX]) {   // the last sub-tile's deferred work, no matrix work to hide in
#pragma unroll
            for (int b = 0; b < kItems; ++b) item(b, xp);
            finish_prev(xp);
        };
        using std::false_type;
        using std::true_type;

        // Three register sets in rotation: current, previous (still needed for its row adds), next (in
        // flight).  A fourth set (two sub-tiles in flight) was measured and bought nothing.
        f32x4 x0[NX], x1[NX], x2[NX];
        int64_t st = first;
        if (first < last) {
            load_subtile(st, x0);
            load_subtile(st + 1, x1);
            __builtin_amdgcn_sched_barrier(0);
            load_centroids();
            step(st, x0, x0, false_type{});
            ++st;
            int phase = 0;   // which set holds the previous sub-tile when the loop ends
#define EP_PIPE_STEP(CUR, PREV, FREE, PHASE)              \
    load_subtile(st + 1, FREE);                           \
    __builtin_amdgcn_sched_barrier(0);                    \
    step(st, CUR, PREV, true_type{});                     \
    ++st;                                                 \
    if (buffered == kFlush) flush_labels(st - 1);         \
    phase = PHASE;
            while (st < last) {
                EP_PIPE_STEP(x1, x0, x2, 1)
                if (st >= last) break;
                EP_PIPE_STEP(x2, x1, x0, 2)
                if (st >= last) break;
                EP_PIPE_STEP(x0, x2, x1, 0)
            }
#undef EP_PIPE_STEP
            if (phase == 0) drain(x0); else if (phase == 1) drain(x1); else drain(x2);
            flush_labels(st);
        }
    } else {
    // Two register sets in ping-pong: while one sub-tile is processed, the next one is in flight.
    f32x4 xa[NX], xb[NX];
    int64_t st = first;
    load_subtile(st, xa);
    __builtin_amdgcn_sched_barrier(0);
    load_centroids();
    while (st < last) {
        load_subtile(st + 1, xb);
        __builtin_amdgcn_sched_barrier(0);  // keep the whole prefetch ahead of the arithmetic
        process(st, xa);
        ++st;
        if (buffered == kFlush) flush_labels(st);
        if (st >= last) break;
        load_subtile(st + 1, xa);
        __builtin_amdgcn_sched_barrier(0);
        process(st, xb);
        ++st;
        if (buffered == kFlush) flush_labels(st);
    }
    flush_labels(st);
    }

    // ---- objective partials of this workgroup (fixed order) ----
    if (MODE != kUpdateOnly && s_part) {
        double os = obj_s, ox = obj_x;
        bool per_row = kLdsSums;            // k > 16: all 16 lanes of a row hold the same sum,
        if constexpr (MODE == kAssignOnly) per_row = per_row && best_score == nullptr;   // except over slices
        if (per_row && c != 0) os = 0.0;
        for (int off = 32; off > 0; off >>= 1) {
            os += __shfl_down(os, off, 64);
            if (XSQ) ox += __shfl_down(ox, off, 64);
        }
        if (lane == 0) {
            red[0][wave] = os;
            red[1][wave] = ox;
        }
    }

    // ---- partial sums of this workgroup: waves add their accumulators in wave order ----
    if (MODE != kAssignOnly && kLdsSums) {
        __syncthreads();  // every wave's table is complete
        for (int i = threadIdx.x; i < k * D; i += kBlock) {
            const int at = (i / D) * STRIDE + (i % D);
            float v = lds[at];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) v += lds[w * (16 * KT + 1) * STRIDE + at];   // wave order
            psum[(int64_t)blockIdx.x * k * D + i] = v;
        }
        if ((int)threadIdx.x < k) pcnt[(int64_t)blockIdx.x * k + threadIdx.x] = cnt_lds[threadIdx.x];
    } else if (MODE != kAssignOnly) {
        // k <= 16: every wave stores its accumulators to its own LDS tile (the transposition tile, no
        // longer needed), then all threads add the four copies in wave order.
        static_assert(kSub * STRIDE >= 16 * D, "a wave's tile holds its 16 x D sums");
        wave_lds_fence();
        float *mine = lds + wave * kSub * STRIDE;
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int h = 0; h < NH; ++h)   // columns 64h + 4c .. + 3 of row 4g + v are tiles t = 4h .. 4h + 3
                *reinterpret_cast<f32x4 *>(mine + (4 * g + v) * D + 64 * h + 4 * c) =
                    f32x4{accu[0][4 * h][v], accu[0][4 * h + 1][v], accu[0][4 * h + 2][v], accu[0][4 * h + 3][v]};
        if (threadIdx.x < 16 * KT) cnt_lds[threadIdx.x] = 0;
        __syncthreads();
        // counts: lanes of a column hold the counts of the 4 groups' points
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            int32_t v = cnt[mt];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (g == 0 && v) atomicAdd(&cnt_lds[16 * mt + c], v);
        }
        for (int i = threadIdx.x; i < k * D / 4; i += kBlock) {
            f32x4 v = *reinterpret_cast<const f32x4 *>(lds + 4 * i);
#pragma unroll
            for (int w = 1; w < kWaves; ++w) v += *reinterpret_cast<const f32x4 *>(lds + w * kSub * STRIDE + 4 * i);
            *reinterpret_cast<f32x4 *>(psum + (int64_t)blockIdx.x * k * D + 4 * i) = v;
        }
        __syncthreads();
        if ((int)threadIdx.x < k) pcnt[(int64_t)blockIdx.x * k + threadIdx.x] = cnt_lds[threadIdx.x];
    } else {
        __syncthreads();
    }
    if (MODE != kUpdateOnly && s_part && threadIdx.x == 0) {
        double ts = 0.0, tx = 0.0;
        for (int w = 0; w < kWaves; ++w) {
            ts += red[0][w];
            tx += red[1][w];
        }
        s_part[blockIdx.x] = ts;
        if (XSQ) xsq_part[blockIdx.x] = tx;
    }
}

// Lane l adds partials l, l + 64, ...; then a fixed shuffle tree.  Called by one full wave.
__device__ __forceinline__ double wave_sum_fixed(const double *__restrict__ part, int count, int l) {
    constexpr int kPerLane = kSmallMaxBlocks / 64;
    double v[kPerLane];
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) v[q] = l + 64 * q < count ? part[l + 64 * q] : 0.0;   // one round trip
    double o = 0.0;
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) o += v[q];
    for (int off = 32; off > 0; off >>= 1) o += __shfl_down(o, off, 64);
    return o;
}

// objective = sum ||x||^2 - 2 * sum best score.  The first term is taken from xsq_part when
// `fresh` (and then stored in *xsq_total), otherwise from *xsq_total.
__device__ __forceinline__ void write_objective(const double *__restrict__ s_part, const double *__restrict__ xsq_part,
                                                int parts, int fresh, double *__restrict__ xsq_total,
                                                double *__restrict__ objective, int l) {
    const double s = wave_sum_fixed(s_part, parts, l);
    double x2 = 0.0;
    if (fresh) x2 = wave_sum_fixed(xsq_part, parts, l);
    if (l == 0) {
        if (fresh) *xsq_total = x2; else x2 = *xsq_total;
        *objective = x2 - 2.0 * s;
    }
}

// Second pass of a round.  Workgroup (j, slice) forms 32 columns of centroid j.  Thread (seg, m4)
// reads columns 4 m4 .. + 3 of the slice from the partials b = seg, seg + 64, ... with 16-byte
// loads, all in flight at once (parts <= 512: at most 8), and adds them in fp64 in ascending
// order; the 64 segment sums are then added in segment order, divided by the count and rounded
// to fp32; an empty cluster keeps its centroid.  Workgroup 0 also forms the round's objective.
constexpr int kFinBlock = 512;
constexpr int kFinCols = 32;                       // columns per workgroup
constexpr int kFinSegs = kFinBlock / (kFinCols / 4);
constexpr int kFinBatch = kSmallMaxBlocks / kFinSegs;
__global__ __launch_bounds__(kFinBlock) void lloyd_small_finalize_kernel(
    int32_t d_pad, int32_t d, int32_t k, int parts, const float *__restrict__ psum, const int32_t *__restrict__ pcnt,
    const double *__restrict__ s_part, const double *__restrict__ xsq_part, int fresh_xsq,
    double *__restrict__ xsq_total, const float *__restrict__ C_prev, float *__restrict__ C_out,
    int64_t *__restrict__ counts, double *__restrict__ objective, UpdateAcc acc, const int64_t *__restrict__ list_len,
    int64_t n) {
    __shared__ double seg_sum[kFinSegs * kFinCols];
    __shared__ unsigned long long total_cnt;
    if (list_len) parts = list_parts(*list_len, n, parts);   // the workgroups beyond wrote no partial
    const int slices = d_pad / kFinCols;   // the partial sums have d_pad columns, the centroids d <= d_pad
    const int j = blockIdx.x / slices, col0 = kFinCols * (blockIdx.x % slices), t = threadIdx.x;
    const int m4 = t % (kFinCols / 4), seg = t / (kFinCols / 4);
    // every load of this thread is issued before anything is waited for
    const int32_t my_cnt = t < parts ? pcnt[(int64_t)t * k + j] : 0;
    const float4 *col = reinterpret_cast<const float4 *>(psum + (int64_t)j * d_pad + col0) + m4;
    const int64_t stride4 = (int64_t)k * d_pad / 4;
    float4 v[kFinBatch];
#pragma unroll
    for (int q = 0; q < kFinBatch; ++q) {
        const int b = seg + q * kFinSegs;
        v[q] = b < parts ? col[(int64_t)b * stride4] : float4{0.f, 0.f, 0.f, 0.f};
    }
    if (t == 0) total_cnt = 0;
    __syncthreads();
    {   // counts: added per wave, then one LDS atomic per wave (integers: order-free)
        int32_t c = my_cnt;
        for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off, 64);
        if ((t & 63) == 0 && c) atomicAdd(&total_cnt, (unsigned long long)c);
    }
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
    for (int q = 0; q < kFinBatch; ++q) {   // ascending workgroup order; missing partials add +0.0
        s0 += (double)v[q].x;
        s1 += (double)v[q].y;
        s2 += (double)v[q].z;
        s3 += (double)v[q].w;
    }
    seg_sum[seg * kFinCols + 4 * m4 + 0] = s0;
    seg_sum[seg * kFinCols + 4 * m4 + 1] = s1;
    seg_sum[seg * kFinCols + 4 * m4 + 2] = s2;
    seg_sum[seg * kFinCols + 4 * m4 + 3] = s3;
    __syncthreads();
    if (t < kFinCols) {
        double tot = seg_sum[t];
        for (int q = 1; q < kFinSegs; ++q) tot += seg_sum[q * kFinCols + t];
        const int64_t cc = (int64_t)total_cnt;
        const int64_t at = (int64_t)j * d + col0 + t;
        if (col0 + t < d) finish_centroid_element(acc, at, j, t == 0 && col0 == 0, tot, cc, C_prev, C_out, counts);
    } else if (t >= 64 && t < 128 && blockIdx.x == 0 && objective) {  // second wave
        write_objective(s_part, xsq_part, parts, fresh_xsq, xsq_total, objective, t - 64);
    }
}

// The objective of a stand-alone assignment: the same additions as in the finalize kernel.
__global__ __launch_bounds__(64) void sum_obj_kernel(const double *__restrict__ s_part,
                                                      const double *__restrict__ xsq_part, int parts,
                                                      double *__restrict__ xsq_total, double *__restrict__ out) {
    write_objective(s_part, xsq_part, parts, 1, xsq_total, out, threadIdx.x);
}

struct Geometry {
    int blocks;
    int64_t subtiles_per_wave;      // every wave takes this many sub-tiles,
    int64_t waves_with_one_more;    // and the first so many waves one more
};

Geometry geometry(int64_t n) {
    const int64_t total_sub = ceil_div(n, kSub);
    const int64_t wgs = std::min<int64_t>(kSmallMaxBlocks, ceil_div(total_sub, kWaves));
    const int64_t waves = wgs * kWaves;
    return Geometry{(int)wgs, total_sub / waves, total_sub % waves};
}

// Workspace slots inside KmeansWs::obj_part (kObjBlocksMax doubles).
double *s_part_of(const KmeansWs &w) { return w.obj_part; }
double *xsq_part_of(const KmeansWs &w) { return w.obj_part + kSmallMaxBlocks; }
double *xsq_total_of(const KmeansWs &w) { return w.obj_part + 2 * kSmallMaxBlocks; }

// label_base / best_score: assignment over one 64-centroid slice of a larger k (see
// launch_small_assign_sliced); 0 / nullptr otherwise.
// BND: the fused round also leaves the distance bounds of every point in ub / lb (exact d = 64 or 128 only).
template <int MODE, bool XSQ, bool BND = false>
int launch_mode(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels_out,
                const int32_t *labels_in, float *min_d2, bool want_obj, hipStream_t s, int32_t label_base = 0,
                float *best_score = nullptr, float *ub = nullptr, float *lb = nullptr) {
    const Geometry geo = geometry(p.n);
    const int kt = p.k <= 16 ? 1 : p.k <= 32 ? 2 : 4;
    const bool stream_x = (double)p.n * (double)p.ld * (double)elem_bytes(p.dtype) > kLastLevelCacheBytes;
    double *sp = want_obj ? s_part_of(w) : nullptr;
    ProfScope prof(MODE == kUpdateOnly ? EP_PROF_UPDATE_SUMS : EP_PROF_LLOYD_MAIN, s, true);
#define EP_SMALL_LAUNCH_P(D_, KT_, XT_, PAD_)                                                                 \
    do {                                                                                                      \
        if constexpr (BND && (PAD_ || D_ == 256)) return EP_EUNSUPPORTED;   /* not instantiated */           \
        else {                                                                                                \
        constexpr int lds_bytes = SmallLds<D_, KT_>::kBytes;                                                  \
        const XT_ *Xt = static_cast<const XT_ *>(X);                                                          \
        auto kern = stream_x ? lloyd_small_kernel<D_, KT_, MODE, XSQ, true, XT_, PAD_, BND>                   \
                             : lloyd_small_kernel<D_, KT_, MODE, XSQ, false, XT_, PAD_, BND>;                 \
        if (lds_bytes > 64 * 1024) {   /* once per kernel variant and device */                              \
            static std::atomic<uint64_t> attr_set[2];   /* one bit per device, per STREAM variant */          \
            int dev_ = 0;                                                                                     \
            EP_HIP_TRY(hipGetDevice(&dev_));                                                                  \
            const uint64_t bit_ = 1ull << (dev_ & 63);                                                        \
            if (!(attr_set[stream_x ? 1 : 0].load(std::memory_order_acquire) & bit_)) {                       \
                EP_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                          \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));      \
                attr_set[stream_x ? 1 : 0].fetch_or(bit_, std::memory_order_release);                         \
            }                                                                                                 \
        }                                                                                                     \
        if (prof.start_)   /* timed launch: the events get the kernel's own begin and end */                \
            hipExtLaunchKernelGGL(kern, dim3(geo.blocks), dim3(kBlock), lds_bytes, s, prof.start_, prof.stop_, 0,  \
                                  p.n, p.ld, p.d, p.k, geo.subtiles_per_wave, geo.waves_with_one_more, Xt, C,  \
                                  labels_out, labels_in, min_d2,                                              \
                                  w.psum, w.pcnt, sp, xsq_part_of(w), label_base, best_score, ub, lb);        \
        else                                                                                                  \
            kern<<<geo.blocks, kBlock, lds_bytes, s>>>(p.n, p.ld, p.d, p.k, geo.subtiles_per_wave,            \
                                                       geo.waves_with_one_more, Xt, C, labels_out, labels_in, \
                                                       min_d2, w.psum, w.pcnt, sp, xsq_part_of(w),            \
                                                       label_base, best_score, ub, lb);                       \
        }                                                                                                     \
    } while (0)
#define EP_SMALL_LAUNCH_T(D_, KT_, XT_)                                                                       \
    do {                                                                                                      \
        if (p.d != D_) EP_SMALL_LAUNCH_P(D_, KT_, XT_, true); else EP_SMALL_LAUNCH_P(D_, KT_, XT_, false);    \
    } while (0)
#define EP_SMALL_LAUNCH(D_, KT_)                                                                              \
    do {                                                                                                      \
        if (p.dtype == EP_BF16) EP_SMALL_LAUNCH_T(D_, KT_, bf16_t);                                           \
        else if (p.dtype == EP_F16) EP_SMALL_LAUNCH_T(D_, KT_, f16_t);                                        \
        else EP_SMALL_LAUNCH_T(D_, KT_, float);                                                               \
    } while (0)
    const int dpad = small_padded_d(p);
    if (dpad == 256) {
        EP_SMALL_LAUNCH(256, 1);
    } else if (dpad == 128) {
        if (kt == 1) EP_SMALL_LAUNCH(128, 1); else if (kt == 2) EP_SMALL_LAUNCH(128, 2); else EP_SMALL_LAUNCH(128, 4);
    } else {
        if (kt == 1) EP_SMALL_LAUNCH(64, 1); else if (kt == 2) EP_SMALL_LAUNCH(64, 2); else EP_SMALL_LAUNCH(64, 4);
    }
#undef EP_SMALL_LAUNCH_P
#undef EP_SMALL_LAUNCH_T
#undef EP_SMALL_LAUNCH
    EP_LAUNCH_CHECK();
    return EP_OK;
}

}  // namespace

bool small_path_supported(const ep_problem &p) {
    return small_padded_d(p) != 0 && p.ld < ((int64_t)1 << 24);
}

int small_blocks(const ep_problem &p) { return geometry(p.n).blocks; }

int launch_small_assign(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                        float *min_d2, double *objective, hipStream_t s) {
    int rc = objective ? launch_mode<kAssignOnly, true>(p, X, C, w, labels, nullptr, min_d2, true, s)
                       : launch_mode<kAssignOnly, false>(p, X, C, w, labels, nullptr, min_d2, false, s);
    if (rc != EP_OK) return rc;
    if (objective) {
        sum_obj_kernel<<<1, 64, 0, s>>>(s_part_of(w), xsq_part_of(w), small_blocks(p), xsq_total_of(w), objective);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

// fp32 rows, d in {64, 128}, k > 64: the assignment kernel runs once per slice of 64 centroids and
// keeps, per point, the best score so far (in the workspace) and its label: k / 64 passes over X
// with the exact arithmetic of the k <= 64 kernel.  Ties go to the lower index: a later slice must
// beat the earlier ones strictly.
bool small_sliced_supported(const ep_problem &p) {
    return (p.dtype == EP_F32 || p.dtype == EP_F16) && (p.d == 64 || p.d == 128) && p.k > 64 && p.ld < ((int64_t)1 << 24);
}

int launch_small_assign_sliced(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                               float *min_d2, double *objective, hipStream_t s) {
    float *best = w.best_score;
    for (int32_t base = 0; base < p.k; base += 64) {
        ep_problem slice = p;
        slice.k = std::min<int32_t>(64, p.k - base);
        const float *Cs = C + (int64_t)base * p.d;
        int rc = objective ? launch_mode<kAssignOnly, true>(slice, X, Cs, w, labels, nullptr, min_d2, true, s, base, best)
                           : launch_mode<kAssignOnly, false>(slice, X, Cs, w, labels, nullptr, min_d2, false, s, base, best);
        if (rc != EP_OK) return rc;
    }
    if (objective) {
        sum_obj_kernel<<<1, 64, 0, s>>>(s_part_of(w), xsq_part_of(w), small_blocks(p), xsq_total_of(w), objective);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

static int launch_small_finalize(const ep_problem &p, const float *C_prev, float *C_out, int64_t *counts,
                                 const KmeansWs &w, double *objective, bool fresh_xsq, const UpdateAcc &acc,
                                 hipStream_t s, int parts = 0, const int64_t *list_len = nullptr) {
    if (parts == 0) parts = small_blocks(p);
    const int dpad = small_padded_d(p);
    lloyd_small_finalize_kernel<<<p.k * (dpad / kFinCols), kFinBlock, 0, s>>>(
        dpad, p.d, p.k, parts, w.psum, w.pcnt, s_part_of(w), xsq_part_of(w), fresh_xsq ? 1 : 0, xsq_total_of(w), C_prev,
        C_out, counts, objective, acc, list_len, p.n);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_small_update(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                        float *C_out, int64_t *counts, const KmeansWs &w, const UpdateAcc &acc, hipStream_t s) {
    int rc = launch_mode<kUpdateOnly, false>(p, X, nullptr, w, nullptr, labels, nullptr, false, s);
    if (rc != EP_OK) return rc;
    return launch_small_finalize(p, C_prev, C_out, counts, w, nullptr, false, acc, s);
}

int launch_small_finalize_parts(const ep_problem &p, int parts, const int64_t *list_len, float *C, int64_t *counts,
                                const KmeansWs &w, const UpdateAcc &acc, hipStream_t s) {
    return launch_small_finalize(p, C, C, counts, w, nullptr, false, acc, s, parts, list_len);
}

double *small_xsq_total(const KmeansWs &w) { return xsq_total_of(w); }

int launch_small_round(const ep_problem &p, const void *X, float *C, const KmeansWs &w, int32_t *labels,
                       int64_t *counts, double *objective, bool first_round, hipStream_t s, const UpdateAcc &acc,
                       float *ub, float *lb) {
    const bool fresh = objective && first_round;  // sum ||x||^2 is computed in the first round and kept
    if (ub && (fresh || !lb)) return EP_EINVAL;   // bounds are taken in a later round
    int rc = ub ? launch_mode<kFused, false, true>(p, X, C, w, labels, nullptr, nullptr, objective != nullptr, s, 0,
                                                   nullptr, ub, lb)
           : fresh ? launch_mode<kFused, true>(p, X, C, w, labels, nullptr, nullptr, true, s)
                   : launch_mode<kFused, false>(p, X, C, w, labels, nullptr, nullptr, objective != nullptr, s);
    if (rc != EP_OK) return rc;
    return launch_small_finalize(p, C, C, counts, w, objective, fresh, acc, s);
}

}  // namespace ep
