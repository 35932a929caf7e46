/*
 * Entry points of the same library that serve its benchmarks and tests, not its users: measured
 * ceilings of the device and hooks that pin a kernel configuration.  Nothing in the linear-layer
 * path depends on them.  Conventions (device pointers, status codes, streams) as in fp6.h.
 */
#ifndef FP6_BENCH_H
#define FP6_BENCH_H

#include "fp6.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostics for benchmarks: empirical ceilings of the device, measured with the request
 * patterns of the linear kernels (the paper's Section 7.1 reads the same two utilisations
 * off its profiler: DRAM bandwidth and Tensor-Core use).
 *   fp6_probe_read: `buffer` (device) is cut into pieces of 8 KB; 1024 waves sweep it front to
 *     back, wave w reading pieces w, 1024 + w, 2048 + w, ... with the non-temporal 128-bit loads
 *     of the weight path, sixteen in flight, and XOR the 32-bit words of their pieces together
 *     into sink[w] (device, 1024 x uint32).  fp6_probe_read_bytes(bytes) is the number of bytes
 *     actually read (a whole, even number of pieces per wave).  bytes >= 16 MiB, else FP6_ERR_SHAPE.
 *   fp6_probe_mfma: 4096 waves (four per SIMD) each issue iters x 4 independent
 *     v_mfma_f32_32x32x16_f16 (32768 flop each) on register operands; `sink` (device,
 *     fp6_probe_mfma_sink_bytes() bytes) receives one float per lane.
 */
fp6_status fp6_probe_read(const void *buffer, size_t bytes, void *sink, void *stream);
size_t fp6_probe_read_bytes(size_t bytes);
fp6_status fp6_probe_mfma(int64_t iters, void *sink, void *stream);
size_t fp6_probe_mfma_sink_bytes(void);

/*
 * Tuning hook for benchmarks and tests: force the split-K factor used by fp6_linear, fp5_linear,
 * fp4_linear, fp3_linear and fp16_linear (0 = choose automatically, the default).  Process-wide; affects the
 * workspace size queries as well.  Values the shape cannot honour are clamped.
 */
void fp6_tuning_set_split_k(int split_k);

/*
 * Tuning hook for benchmarks and tests: force the block tile of the kernel used for N > 64:
 * block_rows in {128, 256} output channels x block_tokens in {64, 128} tokens; any
 * other pair restores the automatic choice.  fp16_linear uses 128 rows where 256 is
 * asked for.  Process-wide; affects the workspace size queries as well.
 */
void fp6_tuning_set_tile(int block_rows, int block_tokens);

#ifdef __cplusplus
}
#endif

#endif /* FP6_BENCH_H */
