/*
 * embedpart_bench.h -- benchmark aids of libembedpart.  NOT part of the method and not needed by
 * any user of embedpart.h: they exist so that a benchmark can time single kernels of the library
 * with events of its own and calibrate hardware counters against a kernel of known traffic.
 */
#ifndef EMBEDPART_BENCH_H
#define EMBEDPART_BENCH_H

#include "embedpart.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Benchmark aid, not part of the method: per-kernel timing with HIP events the caller owns.
 * While armed, launch number i (counted from arming) of a kernel of class `kernel_class` made by
 * any call is bracketed by events_host[2*i] and events_host[2*i+1] on that call's stream, for
 * i < capacity / 2; later launches are not timed.  The tuned Lloyd kernels hand the pair to the
 * launch itself, which stamps them with the kernel's own begin and end; the other kernels record
 * them on the stream just before and just after the launch.
 * events_host: host array of hipEvent_t handles created with timing enabled; it must stay
 * valid until disarmed.  ep_profile_arm(NULL, 0, 0) disarms.  This and the HIP error code are
 * process-global state; arming is not thread-safe.
 * ep_profile_count(): launches of the armed class seen since arming (may exceed capacity / 2).
 */
#define EP_PROF_LLOYD_MAIN  1  /* the kernel that reads X in a Lloyd round (assignment, fused with the sums where fused) */
#define EP_PROF_UPDATE_SUMS 2  /* the separate partial-sum / segment-mean kernel of kmeans_update */
#define EP_PROF_EDGE_SWEEP  3  /* the CSR sweep of partition_quality / edge_gap_sum */
int ep_profile_arm(void **events_host, int capacity, int kernel_class);
int ep_profile_count(void);

/*
 * Benchmark aid: plain streaming copy of `bytes` bytes (a multiple of 16, both pointers 16-byte
 * aligned) with 16-byte loads and stores.  It gives benchmarks a kernel of exactly known traffic
 * (bytes read + bytes written) to calibrate hardware counters and to quote the copy bandwidth of
 * the machine at hand next to the roofline figures.
 */
int ep_bench_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Benchmark aid: the rate of the bf16 matrix instruction alone, on operand values of the caller's choice.
 * 512 workgroups of 4 waves; every lane takes 16 operand registers (16 bytes each) from `operands`
 * (device, 65,536 bytes, 16-byte aligned: piece s of thread t at byte (256 s + t) * 16, s < 16) and the wave
 * issues 16 * iters v_mfma_f32_32x32x16_bf16 in two accumulation chains, nothing else:
 * 512 * 4 * 16 * iters * 32,768 flop per call.  The chip is power-limited in this instruction and the power
 * follows the operand values, so the rate on all-zero operands (the published peak) and the rate on rows of
 * the workload differ; a benchmark quotes both next to the rate of the assignment kernel.
 *   iters in [1, 2^22]; sink: 4 bytes of device memory, 4-byte aligned, written only by a lane whose sums
 *   add up to one particular value (it keeps the arithmetic alive; its content means nothing).  EP_EINVAL
 *   for a null or misaligned pointer or iters out of range.
 */
#define EP_BENCH_MFMA_OPERAND_BYTES 65536
#define EP_BENCH_MFMA_FLOP_PER_ITER (512.0 * 4 * 16 * 32768)
int ep_bench_mfma_bf16(const void *operands, int32_t iters, float *sink, void *stream);

/*
 * Benchmark aid: the price of folding the second pass of a Lloyd round into its first kernel.  `parts`
 * workgroups each write `elems` floats of partial sums to `partials`; then
 *   mode 0  nothing more (the producer alone);
 *   mode 1  every workgroup passes a device-scope fence and takes an integer ticket, and the last one to arrive
 *           adds all partials in fp64 and writes `out` ("the last workgroup reduces": one launch);
 *   mode 2  a second launch of elems / 8 workgroups adds the partials and writes `out` (what the library's
 *           rounds do).
 * No workgroup waits for another in any mode.
 *   partials  parts * elems floats, device, written;  out  elems floats, device, written (modes 1, 2);
 *   ticket    4 bytes, device, zero before the first call (mode 1 leaves it zero again);
 *   parts in [1, 2048], elems a multiple of 8 in [8, 8192]; EP_EINVAL otherwise or for a null pointer.
 */
int ep_bench_fold(float *partials, int32_t parts, int32_t elems, int mode, uint32_t *ticket, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EMBEDPART_BENCH_H */
