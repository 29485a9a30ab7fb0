// Rotary position embedding with positions re-used across contexts, fused with the write of the
// KV cache: the step in front of the attention kernels (arXiv 2502.05431, Section 1 "Re-using
// Positions": every context occupies the same range of positions).  The rotation is the published
// rotary embedding in half-split pairing: dims (c, c + d/2) turn by pos * base^(-2c/d).
//
// Bandwidth-bound: every element is read once and written once.  One workgroup per token: the
// d/2 angles of the token's position are reduced mod 2 pi in fp64 (an fp32 product pos * freq
// would be off by 1e-4 rad at position 2000), their fp32 sines and cosines are shared through
// LDS by all the token's Q and K heads; V is copied.
#include "ape_internal.h"

#include <math.h>

namespace ape {
namespace {

constexpr int kRopeThreads = 256;

template <typename T> struct Vec16;                       // 16 bytes of T
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<__bf16> { static constexpr int N = 8; };

template <typename T>
__device__ __forceinline__ void load16(const T* p, float (&x)[Vec16<T>::N]) {
    const uint4 w = *(const uint4*)p;
    if constexpr (sizeof(T) == 4) {
        x[0] = __uint_as_float(w.x); x[1] = __uint_as_float(w.y); x[2] = __uint_as_float(w.z); x[3] = __uint_as_float(w.w);
    } else {
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[2 * i] = __uint_as_float(u[i] << 16); x[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u); }
    }
}
template <typename T>
__device__ __forceinline__ void store16(T* p, const float (&x)[Vec16<T>::N]) {
    if constexpr (sizeof(T) == 4) {
        *(uint4*)p = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3]));
    } else {
        uint32_t u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __bf16 lo = (__bf16)x[2 * i], hi = (__bf16)x[2 * i + 1];          // round to nearest even
            u[i] = (uint32_t)__builtin_bit_cast(unsigned short, lo) | ((uint32_t)__builtin_bit_cast(unsigned short, hi) << 16);
        }
        *(uint4*)p = make_uint4(u[0], u[1], u[2], u[3]);
    }
}

// grid: x = packed token.  VEC: d/2 is a multiple of the 16-byte vector width.
template <typename T, bool VEC>
__global__ __launch_bounds__(kRopeThreads) void rope_write_kernel(const RopeArgs a) {
    __shared__ float cs[128], sn[128];
    const int tid = threadIdx.x;
    const long t = blockIdx.x;
    const int d = a.head_dim, half = d / 2, hq = a.n_q_heads, hkv = a.n_kv_heads;

    int lo = 0, hi = a.n_chunks - 1;                     // segment that holds token t
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (scalar_load_i32(a.cu + mid) <= t) lo = mid; else hi = mid - 1;
    }
    const long j = t - scalar_load_i32(a.cu + lo);       // index inside the segment
    if (tid < half) {
        const double ang = (double)(a.position_offset + j) * kernarg<RopeArgs>()->inv_freq[tid];
        const double k = rint(ang * 0.15915494309189535);                       // 1 / (2 pi)
        double r = fma(-k, 6.283185307179586, ang);
        r = fma(-k, 2.4492935982947064e-16, r);                                 // 2 pi = hi + lo
        cs[tid] = cosf((float)r);
        sn[tid] = sinf((float)r);
    }
    __syncthreads();

    const T* q_src = a.q_raw ? (const T*)a.q_raw + t * a.q_stride : nullptr;     // this token's rows
    T* q_dst = (T*)a.q_rot + t * hq * d;
    const T* k_src = a.k_raw ? (const T*)a.k_raw + t * a.k_stride : nullptr;
    T* k_dst = nullptr;
    if (k_src) k_dst = a.k_packed ? (T*)a.k_packed + t * hkv * d : (T*)scalar_load_ptr((const void* const*)a.k_cache + lo) + j * hkv * d;
    const int rows_q = q_src ? hq : 0, rows_k = k_src ? hkv : 0;

    if constexpr (VEC) {
        constexpr int N = Vec16<T>::N;
        const int gpr = half / N;                        // vector pairs per row
        for (int item = tid; item < (rows_q + rows_k) * gpr; item += kRopeThreads) {
            const int row = item / gpr, c = (item - row * gpr) * N;
            const T* src; T* dst;
            if (row < rows_q) { src = q_src + row * d; dst = q_dst + row * d; }
            else { src = k_src + (row - rows_q) * d; dst = k_dst + (row - rows_q) * d; }
            float x1[N], x2[N], y1[N], y2[N];
            load16<T>(src + c, x1);
            load16<T>(src + c + half, x2);
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const float co = cs[c + e], si = sn[c + e];
                y1[e] = x1[e] * co - x2[e] * si;
                y2[e] = x2[e] * co + x1[e] * si;
            }
            store16<T>(dst + c, y1);
            store16<T>(dst + c + half, y2);
        }
    } else {
        for (int item = tid; item < (rows_q + rows_k) * half; item += kRopeThreads) {
            const int row = item / half, c = item - row * half;
            const T* src; T* dst;
            if (row < rows_q) { src = q_src + row * d; dst = q_dst + row * d; }
            else { src = k_src + (row - rows_q) * d; dst = k_dst + (row - rows_q) * d; }
            const float x1 = (float)src[c], x2 = (float)src[c + half];
            dst[c] = (T)(x1 * cs[c] - x2 * sn[c]);
            dst[c + half] = (T)(x2 * cs[c] + x1 * sn[c]);
        }
    }
    if (a.v_raw) {                                        // values: copied unchanged, 16 bytes at a time (d * sizeof(T) is a multiple of 16)
        const uint4* src = (const uint4*)((const T*)a.v_raw + t * a.v_stride);
        uint4* dst = (uint4*)(a.v_packed ? (T*)a.v_packed + t * hkv * d : (T*)scalar_load_ptr((const void* const*)a.v_cache + lo) + j * hkv * d);
        const int n16 = hkv * d * (int)sizeof(T) / 16;
        for (int i = tid; i < n16; i += kRopeThreads) dst[i] = src[i];
    }
}

}  // namespace

hipError_t launch_rope_write(const RopeArgs& a, int dtype, hipStream_t s) {
    if (a.total_rows == 0) return hipSuccess;
    dim3 grid((unsigned)a.total_rows);
    const int half = a.head_dim / 2;
    if (dtype == APE_F32) {
        if (half % 4 == 0) rope_write_kernel<float, true><<<grid, kRopeThreads, 0, s>>>(a);
        else rope_write_kernel<float, false><<<grid, kRopeThreads, 0, s>>>(a);
    } else {
        if (half % 8 == 0) rope_write_kernel<__bf16, true><<<grid, kRopeThreads, 0, s>>>(a);
        else rope_write_kernel<__bf16, false><<<grid, kRopeThreads, 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace ape
