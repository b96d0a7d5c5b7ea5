/*
 * spiffy_probe.h - C ABI of libspiffy_probe.so: two machine microbenchmarks behind the "measured peaks" of the
 * benchmark's roofline figures.  Not part of the paper's method and not part of libspiffy.so; only bench.py and
 * one GPU test load it.  Status codes are those of spiffy.h.
 *
 * spiffy_probe_mfma: every SIMD of the chip runs iters x 4 dense bf16 matrix instructions (32x32x16, fp32
 * accumulation) on operands held in registers, all zero or (random_operands != 0) pseudo-random in (-1, 1); no
 * memory traffic.  *flop (host) receives the floating-point operations of the launch; sink is device memory
 * for at least 1024 floats (overwritten).  1 <= iters <= 2^24.
 * spiffy_probe_hbm_read: one read-only pass over `bytes` of device memory at src (16-byte aligned); sink is device
 * memory for one uint32.  Time either call with events on the stream (a hipStream_t passed as void*).
 */
#ifndef SPIFFY_PROBE_H
#define SPIFFY_PROBE_H

#include "spiffy.h"

#ifdef __cplusplus
extern "C" {
#endif

int spiffy_probe_mfma(int32_t iters, int32_t random_operands, float *sink, double *flop, void *stream);
int spiffy_probe_hbm_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPIFFY_PROBE_H */
