// Measured ceilings of the box, for the roofline report (libape_probe.so; loaded by bench.py only --
// nothing of the attention path depends on it).  Three kernels, each timed with events on the
// stream it is launched on:
//   - the bf16 MFMA 32x32x16 issued back to back, one wavefront per SIMD, on operands of the
//     caller's choice (the rate the chip sustains depends on the operand data: it is power-limited);
//   - the same MFMAs with the vector work of a flash-attention softmax in their shadows (per pair
//     of scores: two FMAs, two exponentials, two adds, one packed conversion -- no LDS reads, no
//     loads, no barriers): what the matrix cores deliver next to that arithmetic alone;
//   - a read-only stream over a buffer (16 bytes per lane), the HBM rate a kernel that only
//     reads can reach.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ape_probe.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// 32 MFMAs per iteration on 8 + 2 accumulators (the accumulator pattern of a flash body: 16 into the
// output tile, 16 into two score tiles).  SOFTMAX: half of a softmax slice after every MFMA.
template <bool SOFTMAX>
__global__ __launch_bounds__(256) void mfma_kernel(const uint32_t* __restrict__ operands, float* __restrict__ sink, int iters, float sc) {
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // 16 bytes per lane and fragment, distinct per lane: the caller's data (zeros, random, ...)
        const u32x4 wa = *(const u32x4*)(operands + ((size_t)(i * 256 + threadIdx.x) * 4));
        const u32x4 wb = *(const u32x4*)(operands + ((size_t)((8 + i) * 256 + threadIdx.x) * 4));
        a[i] = __builtin_bit_cast(bf16x8, wa);
        b[i] = __builtin_bit_cast(bf16x8, wb);
    }
    f32x16 o[8], s[2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[i][r] = 0.f;
    float sv[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) sv[i] = threadIdx.x * 1e-3f + i * 0.01f;
    float p0 = 0.f, p1 = 0.f, m = 1.f, e0 = 0.f, e1 = 0.f;
    uint32_t pk[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pk[i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            if (n < 16) o[n & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 7], b[(n >> 3) * 4 + (n & 3)], o[n & 7], 0, 0, 0);
            else s[n & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(n >> 1) & 7], b[n & 7], s[n & 1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (SOFTMAX) {
                const int k = n >> 1;
                if ((n & 1) == 0) {
                    e0 = __builtin_amdgcn_exp2f(fmaf(sv[2 * k], sc, -m));
                    e1 = __builtin_amdgcn_exp2f(fmaf(sv[2 * k + 1], sc, -m));
                } else {
                    p0 += e0; p1 += e1;
                    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk[k]) : "v"(e0), "v"(e1), "v"(p0), "v"(p1));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (SOFTMAX) m += p0 * 1e-30f;
    }
    float r = p0 + p1 + e0 + e1;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) r += o[i][q];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) r += s[i][q];
#pragma unroll
    for (int i = 0; i < 16; ++i) r += (float)pk[i];
    if (r == 1.2345f) sink[0] = r;                       // keeps the work alive; practically never true
}

__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ buf, size_t n_vec, float* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
        const u32x4 w = __builtin_nontemporal_load(buf + i);
        acc[0] ^= w[0]; acc[1] ^= w[1]; acc[2] ^= w[2]; acc[3] ^= w[3];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[0] = 1.f;
}

// Runs `launch` untimed for at least warm_ms of GPU time, then times `reps` launches.
template <typename F>
int timed(F launch, int reps, float warm_ms, hipStream_t s, float* ms_per_launch) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1;
    float spent = 0.f, ms = 0.f;
    int rc = 0;
    while (spent < warm_ms && rc == 0) {
        hipEventRecord(e0, s);
        launch();
        hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = -1;
        spent += ms > 0.f ? ms : 1.f;
    }
    if (rc == 0) {
        hipEventRecord(e0, s);
        for (int i = 0; i < reps; ++i) launch();
        hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess) rc = -1;
        *ms_per_launch = ms / reps;
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return rc;
}

}  // namespace

extern "C" {

int ape_probe_mfma(const void* operands, int with_softmax, float* sink, float warm_ms, void* stream, double* tflops) {
    if (!operands || !sink || !tflops) return -1;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    const int iters = 4000;
    float ms = 0.f;
    auto launch = [&] {
        if (with_softmax) mfma_kernel<true><<<cus, 256, 0, s>>>((const uint32_t*)operands, sink, iters, 1.0001f);
        else mfma_kernel<false><<<cus, 256, 0, s>>>((const uint32_t*)operands, sink, iters, 1.0001f);
    };
    if (timed(launch, 5, warm_ms, s, &ms)) return -1;
    // one workgroup per CU, 4 wavefronts, 32 MFMAs of 32*32*16*2 flop per iteration
    *tflops = (double)cus * 4 * 32 * 32768.0 * iters / (ms * 1e-3) / 1e12;
    return 0;
}

int ape_probe_hbm_read(const void* buf, size_t bytes, float* sink, float warm_ms, void* stream, double* gbs) {
    if (!buf || !sink || !gbs || bytes < 16) return -1;
    hipStream_t s = (hipStream_t)stream;
    float ms = 0.f;
    const size_t n_vec = bytes / 16;
    auto launch = [&] { read_kernel<<<2048, 256, 0, s>>>((const u32x4*)buf, n_vec, sink); };
    if (timed(launch, 10, warm_ms, s, &ms)) return -1;
    *gbs = (double)n_vec * 16 / (ms * 1e-3) / 1e9;
    return 0;
}

}  // extern "C"
