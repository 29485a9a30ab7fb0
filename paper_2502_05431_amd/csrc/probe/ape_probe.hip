// Measured ceilings of the box, for the roofline report (libape_probe.so; loaded by bench.py only --
// nothing of the attention path depends on it).  Four kernels, each timed with events on the
// stream it is launched on:
//   - the bf16 MFMA 32x32x16 issued back to back, one wavefront per SIMD, on operands of the
//     caller's choice (the rate the chip sustains depends on the operand data: it is power-limited);
//   - the same MFMAs with the vector work of a flash-attention softmax in their shadows (per pair
//     of scores: two FMAs, two exponentials, two adds, one packed conversion -- no LDS reads, no
//     loads, no barriers): what the matrix cores deliver next to that arithmetic alone; then also
//     with their operand fragments fetched from LDS, and with a block loaded straight into an LDS
//     ring, a wait and a workgroup barrier per 32 MFMAs (a flash block loop's skeleton);
//   - a read-only stream over a buffer (16 bytes per lane), the HBM rate a kernel that only
//     reads can reach;
//   - the softmax's vector instructions alone (no MFMA), with 1, 2 or 4 wavefronts per SIMD: the
//     rate at which a SIMD issues them depends on how many wavefronts it has to pick from.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ape_probe.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// 32 MFMAs per iteration on 8 + 2 accumulators (the accumulator pattern of a flash body: 16 into the
// output tile, 16 into two score tiles).  LEVEL 1: half of a softmax slice after every MFMA.  LEVEL 2:
// the A operands are fetched from LDS the way a flash body fetches its K and V^T fragments (eight
// 16-byte reads and sixteen transposing 8-byte reads per 32 MFMAs, each some MFMAs ahead of its use).
// LEVEL 3: every iteration also loads a 16 KB block straight into a ring of six LDS slots (four 1 KB
// loads per wavefront, from the 64 KiB of operands, i.e. out of the cache), waits for the block of two
// iterations ago and passes a workgroup barrier: a flash block loop without its bookkeeping and its HBM traffic.
// LEVEL 4: the same for the narrow tile -- a wavefront has 32 rows instead of 64, i.e. 16 MFMAs and half the
// softmax per block next to the same fragment reads and loads, a ring of five slots, two workgroups per CU.
constexpr int kSlotBytes = 16384;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
__device__ __forceinline__ bf16x8 lds_frag_tr(const char* p) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 2048));
    return __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
}
template <int LEVEL>
__global__ __launch_bounds__(256) void mfma_kernel(const uint32_t* __restrict__ operands, float* __restrict__ sink, int iters, float sc) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr bool SOFTMAX = LEVEL >= 1, LDSOPS = LEVEL >= 2, RING = LEVEL >= 3, NARROW = LEVEL == 4;
    constexpr int kRingSlots = NARROW ? 5 : 6;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bf16x8 a[8], b[8], kf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // 16 bytes per lane and fragment, distinct per lane: the caller's data (zeros, random, ...)
        const u32x4 wa = *(const u32x4*)(operands + ((size_t)(i * 256 + threadIdx.x) * 4));
        const u32x4 wb = *(const u32x4*)(operands + ((size_t)((8 + i) * 256 + threadIdx.x) * 4));
        a[i] = __builtin_bit_cast(bf16x8, wa);
        kf[i] = a[i];
        b[i] = __builtin_bit_cast(bf16x8, wb);
    }
    // per-lane LDS offsets of a flash body's fragment reads: K fragment ks at k_off + 512*ks, V^T fragment
    // f = 4*sl + db at v_off[db] + 4096*sl (+2048 for its second half)
    int k_off = 0, v_off[4] = {0, 0, 0, 0};
    if (LDSOPS) {
        const int l32 = lane & 31, hi = lane >> 5, g16 = lane >> 4, s16 = lane & 15;
        k_off = (l32 >> 4) * 4096 + hi * 256 + (l32 & 15) * 16;
        const int row0 = 4 * (g16 >> 1) + (s16 >> 2), chlow = 2 * (g16 & 1) + ((s16 & 3) >> 1);
#pragma unroll
        for (int db = 0; db < 4; ++db) v_off[db] = 8192 + row0 * 256 + (((4 * db + chlow) ^ ((row0 & 3) << 2)) << 4) + (s16 & 1) * 8;
        // every slot starts out holding operand data
        for (int i = threadIdx.x; i < (RING ? kRingSlots : 1) * kSlotBytes / 16; i += 256)
            *(u32x4*)(lds + i * 16) = *(const u32x4*)(operands + (size_t)(i & 4095) * 4);
        __syncthreads();
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
    int slot_rd = 0, slot_wr = (kRingSlots - 2) * kSlotBytes;                 // ring offsets: the block read now, the block whose loads start now
    const uint32_t src_off = (uint32_t)(wave * 4096 + lane * 16);
    for (int it = 0; it < iters; ++it) {
        const char* slot = lds + slot_rd;
        if (RING) {
            // all but the two youngest blocks have landed (4 loads per block), for every wavefront
            __builtin_amdgcn_s_waitcnt(0x0f70 | 8);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            if (NARROW && (n & 1)) {
                // (the narrow tile: every second slot has no MFMA)
            } else if (n < 16) o[n & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 7], b[(n >> 3) * 4 + (n & 3)], o[n & 7], 0, 0, 0);
            else if (NARROW) s[(n >> 1) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[(n >> 1) & 7], b[n & 7], s[(n >> 1) & 1], 0, 0, 0);
            else s[n & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[(n >> 1) & 7], b[n & 7], s[n & 1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (LDSOPS) {
                // the read schedule of the wide flash body: V^T fragments 4..7 and K fragments 0..3 in the
                // first half, V^T fragments 0..3 (for the next iteration) and K fragments 4..7 in the second
                if (n < 2) { a[4 + 2 * n] = lds_frag_tr(slot + v_off[(2 * n) & 3] + 4096); a[5 + 2 * n] = lds_frag_tr(slot + v_off[(2 * n + 1) & 3] + 4096); }
                if (n == 2) { kf[0] = *(const bf16x8*)(slot + k_off); kf[1] = *(const bf16x8*)(slot + k_off + 512); }
                if (n == 3) { kf[2] = *(const bf16x8*)(slot + k_off + 1024); kf[3] = *(const bf16x8*)(slot + k_off + 1536); }
                if (n >= 16 && n < 20) { a[n - 16] = lds_frag_tr(slot + v_off[n - 16]); kf[n - 12] = *(const bf16x8*)(slot + k_off + 512 * (n - 12)); }
            }
            if (RING && n < 4) {
                const uint32_t m0v = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)(lds + slot_wr + wave * 4096 + n * 1024);
                const uint32_t voff = src_off + n * 1024 + ((it & 3) << 14);
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(voff), "s"(operands), "s"(m0v) : "m0", "memory");
            }
            if (SOFTMAX && !(NARROW && (n & 2))) {
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
        if (RING) {
            slot_rd = slot_rd + kSlotBytes == kRingSlots * kSlotBytes ? 0 : slot_rd + kSlotBytes;
            slot_wr = slot_wr + kSlotBytes == kRingSlots * kSlotBytes ? 0 : slot_wr + kSlotBytes;
        }
    }
    if (RING) __builtin_amdgcn_s_waitcnt(0x0f70);              // (no load is in flight when the workgroup ends)
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

// The vector work of eight softmax slices per iteration (per slice two FMAs, two exponentials, two adds,
// one packed conversion), each slice independent of the one before it; the reference m is carried
// around the loop so that nothing can leave it.
constexpr int kValuInstrPerIter = 8 * 7 + 2;
__global__ __launch_bounds__(1024) void valu_kernel(float* __restrict__ sink, int iters, float sc) {
    float sv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) sv[i] = threadIdx.x * 1e-3f + i * 0.01f;
    float p0 = 0.f, p1 = 0.f, m = 1.f;
    uint32_t pk[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pk[i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float e0 = __builtin_amdgcn_exp2f(fmaf(sv[2 * k], sc, -m));
            const float e1 = __builtin_amdgcn_exp2f(fmaf(sv[2 * k + 1], sc, -m));
            p0 += e0; p1 += e1;
            asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk[k]) : "v"(e0), "v"(e1), "v"(p0), "v"(p1));
            __builtin_amdgcn_sched_barrier(0);
        }
        m += p0 * 1e-30f;
    }
    float r = p0 + p1 + m;
#pragma unroll
    for (int i = 0; i < 8; ++i) r += (float)pk[i];
    if (r == 1.2345f) sink[0] = r;
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

int ape_probe_mfma(const void* operands, int level, float* sink, float warm_ms, void* stream, double* tflops) {
    if (!operands || !sink || !tflops || level < 0 || level > 4) return -1;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    const int iters = 4000;
    const int lds_bytes = level == 4 ? 5 * kSlotBytes : level == 3 ? 6 * kSlotBytes : level == 2 ? kSlotBytes : 0;
    if (level == 3 && hipFuncSetAttribute((const void*)mfma_kernel<3>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess) return -1;
    if (level == 4 && hipFuncSetAttribute((const void*)mfma_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess) return -1;
    float ms = 0.f;
    auto launch = [&] {
        const uint32_t* ops = (const uint32_t*)operands;
        if (level == 0) mfma_kernel<0><<<cus, 256, lds_bytes, s>>>(ops, sink, iters, 1.0001f);
        else if (level == 1) mfma_kernel<1><<<cus, 256, lds_bytes, s>>>(ops, sink, iters, 1.0001f);
        else if (level == 2) mfma_kernel<2><<<cus, 256, lds_bytes, s>>>(ops, sink, iters, 1.0001f);
        else if (level == 3) mfma_kernel<3><<<cus, 256, lds_bytes, s>>>(ops, sink, iters, 1.0001f);
        else mfma_kernel<4><<<2 * cus, 256, lds_bytes, s>>>(ops, sink, iters, 1.0001f);
    };
    if (timed(launch, 5, warm_ms, s, &ms)) return -1;
    // levels 0..3: one workgroup per CU, 4 wavefronts, 32 MFMAs of 32*32*16*2 flop per iteration; level 4: two
    // workgroups per CU with 16 MFMAs per wavefront and iteration -- the same number per CU
    *tflops = (double)cus * 4 * 32 * 32768.0 * iters / (ms * 1e-3) / 1e12;
    return 0;
}

int ape_probe_valu_issue(int waves_per_simd, float* sink, float warm_ms, void* stream, double* ns_per_instruction) {
    if (!sink || !ns_per_instruction || (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4)) return -1;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    const int iters = 20000;
    float ms = 0.f;
    // one workgroup per CU: 4 SIMDs x waves_per_simd wavefronts
    auto launch = [&] { valu_kernel<<<cus, 256 * waves_per_simd, 0, s>>>(sink, iters, 1.0001f); };
    if (timed(launch, 5, warm_ms, s, &ms)) return -1;
    *ns_per_instruction = (double)ms * 1e6 / ((double)iters * kValuInstrPerIter * waves_per_simd);
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
