/*
 * pc_probe.h - achievable-peak probes for the benchmark.  NOT part of the choreographed-attention
 * library: they live in a library of their own (libpc_probe.so), name no passage of the paper, and
 * no attention call uses them.  They measure what this GPU sustains for the two resources the
 * attention kernels are priced against, the same way the kernels are timed (events on the caller's
 * stream), so that a roofline fraction can be read against the datasheet figure and against what
 * the chip really delivers.
 *
 * Both enqueue one untimed and `reps` timed launches on `stream` (a hipStream_t passed as void*),
 * bracket the timed ones with events, WAIT for them and write the sustained rate to a host double.
 * They allocate no device memory: the caller passes the buffers (device pointers).  Return value:
 * PC_PROBE_OK or a negative PC_PROBE_ERR_* (the numbers are those of pc.h's PC_ERR_*); nothing is
 * enqueued when an argument is rejected.
 *
 *  pc_probe_mfma_bf16: the rate of 32x32x16 bf16 matrix instructions with nothing else in the
 *    loop, on every compute unit with `waves_per_simd` (1 or 2) waves per SIMD, each wave running
 *    iters * 16 of them (iters <= 65536, reps <= 100).  `operands` (operand_bytes >= 16384, 16-byte
 *    aligned) supplies eight sets of bf16 A and B fragments that consecutive instructions cycle
 *    through; the clock the chip holds depends on how many operand bits toggle, so all-zero
 *    operands give the datasheet rate and random ones the rate real data can reach.
 *  pc_probe_hbm_read: the rate of a streaming read of `bytes` (multiple of 16, 16-byte aligned)
 *    with 16-byte loads; use a buffer several times the last-level cache.
 *  sink: one device float the kernels may write (their way of keeping the work observable).
 */
#ifndef PC_PROBE_H_
#define PC_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PC_PROBE_OK               0
#define PC_PROBE_ERR_INVALID_ARG (-1)
#define PC_PROBE_ERR_SHAPE       (-4)
#define PC_PROBE_ERR_HIP         (-5)

int32_t pc_probe_mfma_bf16(const void *operands, int64_t operand_bytes, int32_t iters, int32_t waves_per_simd,
                           int32_t reps, float *sink, double *tflops, void *stream);
int32_t pc_probe_hbm_read(const void *src, int64_t bytes, int32_t reps, float *sink, double *gb_per_s,
                          void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PC_PROBE_H_ */
