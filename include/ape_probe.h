/*
 * ape_probe.h -- C ABI of libape_probe.so: measured ceilings of the GPU the attention library runs
 * on, reported by bench.py next to the published peaks.  Not part of the attention path; nothing
 * else loads it.  Every call times its own kernel with events on `stream` after `warm_ms`
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
 *   level         0: the MFMAs alone.  1: every MFMA carries half a slice of a flash-attention softmax in
 *                 its shadow (per pair of scores two FMAs, two exponentials, two adds, one packed
 *                 conversion).  2: the A operands are also fetched from LDS the way a flash body
 *                 fetches its K and V^T fragments (eight 16-byte and sixteen transposing 8-byte reads per
 *                 32 MFMAs).  3: every 32 MFMAs also load a 16 KB block straight into a ring of LDS
 *                 slots (out of the cache: the 64 KiB of operands), wait for an older block and pass a
 *                 workgroup barrier -- a flash block loop without bookkeeping, masks and HBM traffic.
 *                 4: the same for the narrow tile (a wavefront has 32 rows: 16 MFMAs and half the softmax per
 *                 block next to the same fragment reads and loads, two workgroups per CU).
 *                 Anything else is an error.
 *   sink          DEVICE, 4 bytes, never written in practice (keeps the arithmetic alive)
 *   tflops        HOST, receives the rate
 */
int ape_probe_mfma(const void *operands, int level, float *sink, float warm_ms, void *stream, double *tflops);

/*
 * Issue rate of the softmax's vector instructions alone (per pair of scores two FMAs, two exponentials,
 * two adds, one packed conversion; no MFMA, no memory access), with `waves_per_simd` (1, 2 or 4; anything
 * else is an error) wavefronts on every SIMD of every CU.  ns_per_instruction (HOST) receives the time per
 * instruction as one SIMD sees it: elapsed time / (instructions per wavefront x wavefronts per SIMD).  One
 * wavefront alone gets an instruction out about every 8 cycles; what the block loop of a kernel with one
 * wavefront per SIMD can hide behind its MFMAs follows from that.
 */
int ape_probe_valu_issue(int waves_per_simd, float *sink, float warm_ms, void *stream, double *ns_per_instruction);

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
