/*
 * probes.h - C ABI of libmq_probe.so, a measurement-only library used by bench.py.  It is not part
 * of the product library (libmq.so, include/mq.h) and computes nothing of the method.  Return value:
 * 0 = ok, 1 = NULL pointer, 2 = size out of range, 4 = pointer not 16-byte aligned, 7 = launch failed
 * (the numbering of mq_status).  All pointers are device pointers; `hip_stream` is a hipStream_t.
 */
#ifndef MQ_BENCH_PROBES_H
#define MQ_BENCH_PROBES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement helpers (they compute nothing of the method): ceilings of this GPU as measured by
 * kernels that only multiply or only read, to put next to the published peaks.
 *
 * mq_probe_mfma: 256 workgroups of one wave per SIMD run `iters` rounds of 12 independent
 *   32x32x16 bf16 matrix-core products per wave = 256 * 4 * iters * 12 * 32768 flops.
 *   operands_bf16  device, 32768 bf16 values (64 KB) the products are fed with: their bit patterns
 *                  set the power the loop draws, hence the clock it sustains
 *   sink           device [65536] float, overwritten
 * mq_probe_mfma16: the same loop with 16x16x32 bf16 products, 256 workgroups of two waves per SIMD, 24
 *   independent accumulators per wave = 256 * 8 * iters * 24 * 16384 flops.
 *   operands_bf16  as above;  sink  device [131072] float, overwritten
 * mq_probe_read: reads `bytes` (a multiple of 16) from src once with 16-byte loads.
 *   sink           device [1] uint32, practically never written
 */
int mq_probe_mfma(const uint16_t *operands_bf16, int64_t iters, float *sink, void *hip_stream);
int mq_probe_mfma16(const uint16_t *operands_bf16, int64_t iters, float *sink, void *hip_stream);
int mq_probe_read(const void *src, int64_t bytes, uint32_t *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MQ_BENCH_PROBES_H */
