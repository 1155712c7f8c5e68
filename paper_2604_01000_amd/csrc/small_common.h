// Device helpers shared by the fused small-k Lloyd kernels (kmeans_small.hip) and the bounded rounds
// (kmeans_bounds.hip): vector types, 16-lane DPP reductions, the order-preserving float key, the exact
// three-way bf16 split, the bf16 matrix-instruction wrappers and the rank-ordered row adds into LDS sums.
#pragma once

#include "common.h"

namespace ep {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Reductions over the 16 lanes of a DPP row; every lane of the row gets the result.
// Steps: xor 1, xor 2 (quad permutes), then mirror within 8 and within 16 lanes.
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ int row16_max(int v) {
    v = max(v, dpp_i<0xB1>(v));   // quad_perm [1,0,3,2]
    v = max(v, dpp_i<0x4E>(v));   // quad_perm [2,3,0,1]
    v = max(v, dpp_i<0x141>(v));  // row_half_mirror
    v = max(v, dpp_i<0x140>(v));  // row_mirror
    return v;
}
__device__ __forceinline__ int row16_min(int v) {
    v = min(v, dpp_i<0xB1>(v));
    v = min(v, dpp_i<0x4E>(v));
    v = min(v, dpp_i<0x141>(v));
    v = min(v, dpp_i<0x140>(v));
    return v;
}
// Order-preserving map between finite floats and signed integers (its own inverse).
__device__ __forceinline__ int float_key(float f) {
    const int b = __float_as_int(f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_float(int key) { return __int_as_float(key ^ ((key >> 31) & 0x7fffffff)); }

// x0 = h0 + m0 + l0 and x1 = h1 + m1 + l1 exactly, every term a bf16: each term is what is left,
// rounded to nearest even (fp32 has 24 significant bits, bf16 has 8, and both remainders are exact
// in fp32).  The results are packed two to a word, x0's in the low half.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
struct Split3 {
    unsigned h, m, l;
};
__device__ __forceinline__ Split3 split3_pair(float x0, float x1) {
    Split3 t;
    t.h = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{x0, x1}, bf16x2_t));
    const float r0 = x0 - __uint_as_float(t.h << 16), r1 = x1 - __uint_as_float(t.h & 0xffff0000u);
    t.m = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{r0, r1}, bf16x2_t));
    const float s0 = r0 - __uint_as_float(t.m << 16), s1 = r1 - __uint_as_float(t.m & 0xffff0000u);
    t.l = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{s0, s1}, bf16x2_t));
    return t;
}
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 mfma_bf16_k16(const u32x2 &a, const u32x2 &b, const f32x4 &acc) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4_t, a), __builtin_bit_cast(bf16x4_t, b),
                                                      acc, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_bf16_k32(const u32x4 &a, const u32x4 &b, const f32x4 &acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   acc, 0, 0, 0);
}

// Distance bounds of the bounded rounds, kept on the safe side of fp32 rounding: an upper bound is rounded up, a
// lower bound down.
constexpr float kUp = 1.0f + 0x1p-21f;      // pushes a non-negative value up past any fp32 rounding of one operation
constexpr float kDown = 1.0f - 0x1p-21f;
// |d^2 as computed from a score - true d^2| <= kEvalSlack * (||x||^2 + max ||c||^2): 768 fp32 additions of a
// six-term split product bound the relative error of a score by 768 * 2^-24 < 2^-14 of |x| |c|; this is twice that.
constexpr float kEvalSlack = 0x1p-13f;
// Fresh bounds of a point from its best and second-best score (score = x.c - ||c||^2 / 2, so
// d^2 = ||x||^2 - 2 score): u >= the distance to the own centroid, l <= the distance to every other one
// (+infinity when there is no other centroid: the padding score is -3e38).
__device__ __forceinline__ void fresh_bounds(float xn, float s_best, float s_second, float cmax2, float &u, float &l) {
    const float slack = kEvalSlack * (xn + cmax2);
    const float d2_best = fmaxf(xn - 2.f * s_best, 0.f) + slack;
    const float d2_second = fmaxf(xn - 2.f * s_second - slack, 0.f);
    u = __fsqrt_rn(d2_best) * kUp;
    l = __fsqrt_rn(d2_second) * kDown;
}

// sums[label of point c][:] += x_c for the 16 points of a sub-tile, in LDS, without atomics and in
// a fixed order.  Lane (g, c) holds a quarter of point c's row (columns 16 j + 4 g .. + 3).  Points
// of the sub-tile that share a label must not update the same row at once, so every point gets
// its rank among the earlier points with the same label (15 DPP row shifts) and round r handles
// the points of rank r: rows touched in one round are distinct, and every row receives its
// points in ascending order.  The padded row stride spreads different labels over the banks.
template <int CTRL>
__device__ __forceinline__ int row_shr(int v) {
    return __builtin_amdgcn_update_dpp(-2, v, CTRL, 0xF, 0xF, false);   // lanes shifted in from outside keep -2
}
template <int R, int R_LAST = 15>
__device__ __forceinline__ int same_label_before(int lab, int acc) {
    if constexpr (R > R_LAST) {
        return acc;
    } else {
        acc += row_shr<0x110 + R>(lab) == lab ? 1 : 0;
        return same_label_before<R + 1, R_LAST>(lab, acc);
    }
}
// COUNT: what a row adds to its label's count (-1 when x is the negated row of a point that leaves the label).
template <int NJ, int STRIDE, int COUNT = 1>
__device__ __forceinline__ void add_rows_to_lds_sums(const f32x4 (&x)[NJ], int32_t lab_c, int g, float *wsums,
                                                     int32_t *cnt_lds) {
    int rank = same_label_before<1>(lab_c, 0);
    if (lab_c < 0) rank = -1;
    if (g == 0 && lab_c >= 0) atomicAdd(&cnt_lds[lab_c], COUNT);   // integer: order does not matter
    float *row = wsums + (lab_c < 0 ? 0 : lab_c) * STRIDE + 4 * g;
    for (int r = 0; __ballot(rank >= r) != 0; ++r) {
        if (rank == r) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                f32x4 *p = reinterpret_cast<f32x4 *>(row + 16 * j);
                *p = *p + x[j];
            }
        }
        wave_lds_fence();
    }
}

}  // namespace
}  // namespace ep
