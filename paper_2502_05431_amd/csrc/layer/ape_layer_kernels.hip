// Kernels and the rocBLAS wrapper of the layer library (libape_layer.so): the projections and the
// MLP that turn the attention kernels into a per-layer prefill latency (arXiv 2502.05431, Section
// 5.4 measures whole-model prefill; the layer itself is the published Llama architecture).
// The four matrix products go to rocBLAS (plain GEMMs, fp32 accumulation, the residual added by
// beta = 1); RMSNorm and SiLU(gate) * up are the kernels below; the rotary embedding + cache write
// and the attention are the attention library's (libape_hip.so, which this library links against
// and which itself stays free of rocBLAS and of any state).
#include "ape_layer_internal.h"

#include <rocblas/rocblas.h>

#include <cmath>
#include <mutex>

namespace ape {
namespace {

constexpr int kWave = 64;

template <typename T> struct V16;                        // 16 bytes of T
template <> struct V16<float> { static constexpr int N = 4; };
template <> struct V16<__bf16> { static constexpr int N = 8; };

template <typename T>
__device__ __forceinline__ void ld16(const T* p, float (&x)[V16<T>::N]) {
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
__device__ __forceinline__ void st16(T* p, const float (&x)[V16<T>::N]) {
    if constexpr (sizeof(T) == 4) {
        *(uint4*)p = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3]));
    } else {
        uint32_t u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __bf16 lo = (__bf16)x[2 * i], hi = (__bf16)x[2 * i + 1];
            u[i] = (uint32_t)__builtin_bit_cast(unsigned short, lo) | ((uint32_t)__builtin_bit_cast(unsigned short, hi) << 16);
        }
        *(uint4*)p = make_uint4(u[0], u[1], u[2], u[3]);
    }
}

// RMSNorm: y = x / sqrt(mean(x^2) + eps) * w.  One wavefront per row, four rows per workgroup;
// the row stays in registers between the two passes (up to kMaxVec 16-byte vectors per lane),
// longer rows are read twice.  Bandwidth-bound: the row is read once and written once.
constexpr int kNormRows = 4;
constexpr int kMaxVec = 8;
template <typename T>
__global__ __launch_bounds__(kWave * kNormRows) void rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ w, T* __restrict__ y,
                                                                    long rows, int hidden, float eps) {
    constexpr int N = V16<T>::N;
    const int lane = threadIdx.x & (kWave - 1);
    const long row = (long)blockIdx.x * kNormRows + threadIdx.x / kWave;
    if (row >= rows) return;
    const T* xr = x + row * hidden;
    T* yr = y + row * hidden;
    const int n_vec = hidden / N;                         // hidden is a multiple of N
    float keep[kMaxVec][N];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int v = lane + i * kWave;
        if (v < n_vec) {
            ld16<T>(xr + v * N, keep[i]);
#pragma unroll
            for (int e = 0; e < N; ++e) ss = fmaf(keep[i][e], keep[i][e], ss);
        }
    }
    for (int v = lane + kMaxVec * kWave; v < n_vec; v += kWave) {
        float t[N];
        ld16<T>(xr + v * N, t);
#pragma unroll
        for (int e = 0; e < N; ++e) ss = fmaf(t[e], t[e], ss);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float r = 1.0f / sqrtf(ss / (float)hidden + eps);
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int v = lane + i * kWave;
        if (v < n_vec) {
            float ww[N], o[N];
            ld16<T>(w + v * N, ww);
#pragma unroll
            for (int e = 0; e < N; ++e) o[e] = keep[i][e] * r * ww[e];
            st16<T>(yr + v * N, o);
        }
    }
    for (int v = lane + kMaxVec * kWave; v < n_vec; v += kWave) {
        float t[N], ww[N], o[N];
        ld16<T>(xr + v * N, t);
        ld16<T>(w + v * N, ww);
#pragma unroll
        for (int e = 0; e < N; ++e) o[e] = t[e] * r * ww[e];
        st16<T>(yr + v * N, o);
    }
}

// act[m, i] = SiLU(gate_up[m, i]) * gate_up[m, inter + i].  16 bytes per lane.
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T* __restrict__ gu, T* __restrict__ act, long rows, int inter) {
    constexpr int N = V16<T>::N;
    const long vec_per_row = inter / N;
    const long total = rows * vec_per_row;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const long m = i / vec_per_row, c = (i - m * vec_per_row) * N;
        float g[N], u[N], o[N];
        ld16<T>(gu + m * 2 * inter + c, g);
        ld16<T>(gu + m * 2 * inter + inter + c, u);
#pragma unroll
        for (int e = 0; e < N; ++e) o[e] = g[e] / (1.0f + __expf(-g[e])) * u[e];
        st16<T>(act + m * inter + c, o);
    }
}

// ---- rocBLAS: one handle per device for the life of the process.  The handle carries the stream
// of the call that uses it, so a call holds g_blas_mutex from its first GEMM to its last (taken by
// BlasCall, below): two host threads on one device are serialised instead of racing on the handle.
std::mutex g_handle_mutex;
std::recursive_mutex g_blas_mutex;
rocblas_handle g_handles[64] = {};

rocblas_handle blas_handle() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_handle_mutex);
    if (!g_handles[dev] && rocblas_create_handle(&g_handles[dev]) != rocblas_status_success) g_handles[dev] = nullptr;
    return g_handles[dev];
}

}  // namespace

BlasCall::BlasCall() { g_blas_mutex.lock(); }
BlasCall::~BlasCall() { g_blas_mutex.unlock(); }

// Creating a handle allocates device memory: a caller that captures a HIP graph creates it first,
// outside the capture, with a plain call on the same device.
bool blas_ready_for(hipStream_t s) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) return false;
    if (st == hipStreamCaptureStatusNone) return blas_handle() != nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(g_handle_mutex);
    return g_handles[dev] != nullptr;                 // capturing: only an existing handle will do
}

hipError_t launch_rmsnorm(const void* x, const void* w, void* y, long rows, int hidden, float eps, int dtype, hipStream_t s) {
    if (rows == 0) return hipSuccess;
    const unsigned grid = (unsigned)((rows + kNormRows - 1) / kNormRows);
    if (dtype == APE_F32) rmsnorm_kernel<float><<<grid, kWave * kNormRows, 0, s>>>((const float*)x, (const float*)w, (float*)y, rows, hidden, eps);
    else rmsnorm_kernel<__bf16><<<grid, kWave * kNormRows, 0, s>>>((const __bf16*)x, (const __bf16*)w, (__bf16*)y, rows, hidden, eps);
    return hipGetLastError();
}

hipError_t launch_swiglu(const void* gate_up, void* act, long rows, int inter, int dtype, hipStream_t s) {
    if (rows == 0) return hipSuccess;
    const long vecs = rows * (inter / (dtype == APE_F32 ? 4 : 8));
    const unsigned grid = (unsigned)(vecs / 256 + 1 < 65536 ? vecs / 256 + 1 : 65536);
    if (dtype == APE_F32) swiglu_kernel<float><<<grid, 256, 0, s>>>((const float*)gate_up, (float*)act, rows, inter);
    else swiglu_kernel<__bf16><<<grid, 256, 0, s>>>((const __bf16*)gate_up, (__bf16*)act, rows, inter);
    return hipGetLastError();
}

// y[rows, n] = x[rows, k] W[n, k]^T (+ residual[rows, n]); all row-major, leading dimensions given in
// elements.  In the column-major terms of the library: y^T = W^T(op T) x^T.
int gemm_xwT(const void* x, long ldx, const void* w, const void* residual, void* y, long ldy, long rows, int n, int k,
             int dtype, hipStream_t s) {
    rocblas_handle h = blas_handle();
    if (!h) return -1;
    if (rocblas_set_stream(h, s) != rocblas_status_success) return -1;
    if (rows == 0) return 0;
    const float alpha = 1.f, beta = residual ? 1.f : 0.f;
    const rocblas_datatype t = dtype == APE_F32 ? rocblas_datatype_f32_r : rocblas_datatype_bf16_r;
    const rocblas_status st = rocblas_gemm_ex(h, rocblas_operation_transpose, rocblas_operation_none, n, (rocblas_int)rows, k, &alpha,
                                              w, t, k, x, t, (rocblas_int)ldx, &beta, residual ? residual : y, t, (rocblas_int)ldy,
                                              y, t, (rocblas_int)ldy, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    return st == rocblas_status_success ? 0 : -1;
}

}  // namespace ape
