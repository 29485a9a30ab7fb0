/*
 * ape_probe.h -- C ABI of libape_probe.so: measured ceilings of the GPU the attention library runs
 * on, reported by bench.py next to the published peaks.  Not part of the attention path; nothing
 * else loads it.  Both calls time their own kernel with events on `stream` after `warm_ms`
 * milliseconds of the same kernel untimed, synchronise, and return 0 on success.
 */
#ifndef APE_PROBE_H
#define APE_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Rate of the bf16 matrix-core instruction the flash kernels use (MFMA 32x32x16), issued back to
 * back by one wavefront per SIMD on every CU.
 *   operands      DEVICE, 64 KiB: the 16 operand fragments of every lane, read once (all zeros, random
 *                 bf16, ...: the sustained clock, and with it the rate, depends on the data)
 *   with_softmax  != 0: every MFMA carries half a slice of a flash-attention softmax in its shadow
 *                 (per pair of scores two FMAs, two exponentials, two adds, one packed conversion)
 *   sink          DEVICE, 4 bytes, never written in practice (keeps the arithmetic alive)
 *   tflops        HOST, receives the rate
 */
int ape_probe_mfma(const void *operands, int with_softmax, float *sink, float warm_ms, void *stream, double *tflops);

/*
 * Rate of a kernel that only reads `bytes` of DEVICE memory at `buf` (16 bytes per lane, 2048
 * workgroups): the HBM bandwidth a bandwidth-bound kernel can approach.  Use a buffer well beyond
 * the 256 MB last-level cache.
 */
int ape_probe_hbm_read(const void *buf, size_t bytes, float *sink, float warm_ms, void *stream, double *gbs);

#ifdef __cplusplus
}
#endif
#endif /* APE_PROBE_H */
