// Benchmark aid, not part of the method: what it would cost to fold the second pass of a Lloyd round (the
// reduction of the per-workgroup partial sums) into the round's first kernel, "the last workgroup to arrive
// reduces the partials, behind an integer ticket", against the second small launch the library uses.
#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
constexpr int kReduceBlock = 512;

// Every workgroup writes `elems` floats of partials.  FOLD: then a device-scope fence, an integer ticket, and the
// last workgroup to arrive adds all partials in fp64 (16 loads in flight per thread, in workgroup order) and
// resets the ticket.  No workgroup waits for another.
template <bool FOLD>
__global__ __launch_bounds__(kBlock) void fold_producer_kernel(float *__restrict__ part, int elems,
                                                                unsigned *__restrict__ ticket,
                                                                float *__restrict__ out) {
    __shared__ int last;
    const float v = (float)blockIdx.x;
    for (int e = threadIdx.x; e < elems; e += kBlock) part[(size_t)blockIdx.x * elems + e] = v + (float)e;
    if (FOLD) {
        __threadfence();
        __syncthreads();
        if (threadIdx.x == 0) last = atomicAdd(ticket, 1u) == gridDim.x - 1;
        __syncthreads();
        if (last) {
            __threadfence();
            for (int e = threadIdx.x; e < elems; e += kBlock) {
                double s = 0.0;
                unsigned b = 0;
                for (; b + 16 <= gridDim.x; b += 16) {
                    float w[16];
#pragma unroll
                    for (int q = 0; q < 16; ++q) w[q] = part[(size_t)(b + q) * elems + e];
#pragma unroll
                    for (int q = 0; q < 16; ++q) s += (double)w[q];
                }
                for (; b < gridDim.x; ++b) s += (double)part[(size_t)b * elems + e];
                out[e] = (float)s;
            }
            if (threadIdx.x == 0) *ticket = 0;
        }
    }
}

// The separate second pass: one workgroup per 8 elements, 64 partial loads in flight per element.
__global__ __launch_bounds__(kReduceBlock) void fold_reduce_kernel(const float *__restrict__ part, int elems, int parts,
                                                                    float *__restrict__ out) {
    __shared__ double seg[64 * 8];
    const int col = blockIdx.x * 8 + (threadIdx.x & 7), sg = threadIdx.x >> 3;
    double s = 0.0;
    for (int b = sg; b < parts; b += 64) s += (double)part[(size_t)b * elems + col];
    seg[sg * 8 + (threadIdx.x & 7)] = s;
    __syncthreads();
    if (threadIdx.x < 8) {
        double t = 0.0;
        for (int q = 0; q < 64; ++q) t += seg[q * 8 + threadIdx.x];
        out[blockIdx.x * 8 + threadIdx.x] = (float)t;
    }
}

}  // namespace

int launch_bench_fold(float *partials, int32_t parts, int32_t elems, int mode, unsigned *ticket, float *out,
                      hipStream_t s) {
    if (mode == 1) {
        fold_producer_kernel<true><<<parts, kBlock, 0, s>>>(partials, elems, ticket, out);
        EP_LAUNCH_CHECK();
        return EP_OK;
    }
    fold_producer_kernel<false><<<parts, kBlock, 0, s>>>(partials, elems, ticket, out);
    EP_LAUNCH_CHECK();
    if (mode == 2) {
        fold_reduce_kernel<<<elems / 8, kReduceBlock, 0, s>>>(partials, elems, parts, out);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

}  // namespace ep
