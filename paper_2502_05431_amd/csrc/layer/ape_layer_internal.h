// Internal declarations of the layer library (libape_layer.so).  Not part of the public ABI (that
// is include/ape_layer.h).
#pragma once

#include "ape_internal.h"
#include "ape_layer.h"

namespace ape {

hipError_t launch_rmsnorm(const void* x, const void* w, void* y, long rows, int hidden, float eps, int dtype, hipStream_t s);
hipError_t launch_swiglu(const void* gate_up, void* act, long rows, int inter, int dtype, hipStream_t s);
// y[rows, n] = x[rows, k] W[n, k]^T (+ residual); 0 on success.  The caller holds a BlasCall.
int gemm_xwT(const void* x, long ldx, const void* w, const void* residual, void* y, long ldy, long rows, int n, int k,
             int dtype, hipStream_t s);
// Holds the process-wide lock of the rocBLAS handles for the duration of one entry-point call.
struct BlasCall {
    BlasCall();
    ~BlasCall();
    BlasCall(const BlasCall&) = delete;
    BlasCall& operator=(const BlasCall&) = delete;
};
// true when the current device has (or, outside a graph capture, can be given) a rocBLAS handle
bool blas_ready_for(hipStream_t s);

}  // namespace ape
