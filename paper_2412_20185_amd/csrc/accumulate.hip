// Step 4 of dynamic error compensation (DecDEC Section 4.1): o = o_b + o_dec.
//
// The paper adds o_dec into o_b with atomics from inside its fused kernel
// (Section 4.3 "Kernel Fusion").  Here both producers leave fp32 partial rows
// (the base GEMV one per K-slice, the residual kernel one per slice of the
// selected channels) and this kernel, enqueued on the caller's stream after
// both, adds them in a fixed order and rounds once to fp16: the result does
// not depend on which kernel finished first.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace decdec {
namespace {

__global__ __launch_bounds__(256) void accumulate_kernel(const float* __restrict__ gpart, int gslices,
                                                        const float* __restrict__ cpart, int cslices, int N,
                                                        _Float16* __restrict__ y) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float ob = 0.f;
#pragma unroll 8
    for (int s = 0; s < gslices; ++s) ob += gpart[(size_t)s * N + n];
    float odec = 0.f;
#pragma unroll 8
    for (int r = 0; r < cslices; ++r) odec += cpart[(size_t)r * N + n];
    y[n] = (_Float16)(ob + odec);
}

}  // namespace

hipError_t launch_accumulate(const float* gpart, int gslices, const float* cpart, int cslices, int N, void* y,
                             hipStream_t stream) {
    accumulate_kernel<<<dim3((N + 255) / 256), dim3(256), 0, stream>>>(gpart, gslices, cpart, cslices, N,
                                                                       static_cast<_Float16*>(y));
    return hipGetLastError();
}

}  // namespace decdec
