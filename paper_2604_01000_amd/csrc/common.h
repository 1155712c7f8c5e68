// Internal helpers shared by the HIP translation units of libembedpart (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/embedpart.h"
#include "../../include/embedpart_bench.h"

namespace ep {

// Records the failing hipError_t for ep_last_hip_error().
void note_hip_error(hipError_t e);

#define EP_HIP_TRY(expr)                                  \
    do {                                                  \
        hipError_t _e = (expr);                           \
        if (_e != hipSuccess) {                           \
            ::ep::note_hip_error(_e);                     \
            return EP_EHIP;                               \
        }                                                 \
    } while (0)

#define EP_LAUNCH_CHECK() EP_HIP_TRY(hipGetLastError())

// Times one kernel launch with the caller's events while ep_profile_arm() is in force.
// Default: the two events are recorded on the stream before and after the launch (the interval
// then includes the launch overhead of the bracketing events, a few microseconds).
// kernel_events: nothing is recorded; the launch site passes start_ / stop_ to
// hipExtLaunchKernelGGL, which stamps them with the kernel's own begin and end.
struct ProfScope {
    ProfScope(int kernel_class, hipStream_t s, bool kernel_events = false);
    ~ProfScope();
    hipEvent_t start_, stop_;
    hipStream_t s_;
    bool kernel_events_;
};

constexpr int kWave = 64;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- workspace carving ------------------------------------------------------
struct Carver {
    char *base;
    size_t used;
    explicit Carver(void *p) : base(static_cast<char *>(p)), used(0) {}
    template <typename T> T *take(size_t count) {
        used = align_up(used, 256);
        T *r = base ? reinterpret_cast<T *>(base + used) : nullptr;
        used += count * sizeof(T);
        return r;
    }
};

// ---- device helpers -----------------------------------------------------------
typedef uint16_t bf16_t;  // storage type of bfloat16

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(static_cast<uint32_t>(v) << 16); }

// fp32 -> bf16, round to nearest, ties to even (finite inputs).
__device__ __forceinline__ bf16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

// Inclusive running maximum over the 64 lanes, on the data-parallel-primitive paths (no LDS):
// shifts by 1, 2, 4, 8 inside rows of 16 lanes, then the last lane of row 0 / 2 into rows 1 / 3 and
// the last lane of row 1 into rows 2 and 3.  Lanes without a source see 0 (the values are unsigned).
__device__ __forceinline__ uint32_t wave_inclusive_max(uint32_t v) {
    auto fold = [&](uint32_t other) { v = other > v ? other : v; };
    fold((uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true));    // row_shr:1
    fold((uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true));    // row_shr:2
    fold((uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true));    // row_shr:4
    fold((uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true));    // row_shr:8
    fold((uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false));   // row_bcast:15 into rows 1, 3
    fold((uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false));   // row_bcast:31 into rows 2, 3
    return v;
}

// Inclusive running sum over the 64 lanes, same paths as wave_inclusive_max (lanes without a source add 0).
__device__ __forceinline__ int wave_inclusive_add(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);    // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2, 3
    return v;
}

typedef _Float16 f16_t;   // storage type of IEEE binary16 (widening to fp32 is exact)
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

inline int elem_bytes(int dtype) { return dtype == EP_F32 ? 4 : 2; }

__device__ __forceinline__ float load_elem(const float *p) { return *p; }
__device__ __forceinline__ float load_elem(const f16_t *p) { return (float)*p; }
__device__ __forceinline__ float load_elem(const bf16_t *p) { return bf16_to_f32(*p); }

// Four consecutive elements starting at a 4-element-aligned column.
__device__ __forceinline__ float4 load4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 load4(const f16_t *p) {
    const f32x4_t v = __builtin_convertvector(*reinterpret_cast<const f16x4_t *>(p), f32x4_t);
    return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float4 load4(const bf16_t *p) {
    uint2 r = *reinterpret_cast<const uint2 *>(p);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}

}  // namespace ep
