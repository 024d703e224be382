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

struct AccJobs {
    _Float16* y[kMaxMulti];
    int col0[kMaxMulti + 1];
    int n;
};

__global__ __launch_bounds__(256) void accumulate_kernel(const AccJobs jobs, const float* __restrict__ gpart,
                                                        int gslices, const float* __restrict__ cpart, int cslices,
                                                        int Ntot) {
    const int c = blockIdx.x * 256 + threadIdx.x;  // concatenated column
    if (c >= Ntot) return;
    float ob = 0.f;
#pragma unroll 8
    for (int s = 0; s < gslices; ++s) ob += gpart[(size_t)s * Ntot + c];
    float odec = 0.f;
#pragma unroll 8
    for (int r = 0; r < cslices; ++r) odec += cpart[(size_t)r * Ntot + c];
    int m = 0;
#pragma unroll
    for (int i = 1; i < kMaxMulti; ++i) m += (i < jobs.n && c >= jobs.col0[i]) ? 1 : 0;
    jobs.y[m][c - jobs.col0[m]] = (_Float16)(ob + odec);
}

__global__ __launch_bounds__(256) void clear_u32_kernel(unsigned* p, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace

hipError_t launch_clear_u32(unsigned* p, int n, hipStream_t stream) {
    clear_u32_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(p, n);
    return hipGetLastError();
}

hipError_t launch_accumulate(const MultiShape& sh, void* const* y, const float* gpart, int gslices,
                             const float* cpart, int cslices, hipStream_t stream, const KernelTimer* tm) {
    AccJobs jobs{};
    jobs.n = sh.n;
    for (int m = 0; m < sh.n; ++m) {
        jobs.y[m] = static_cast<_Float16*>(y[m]);
        jobs.col0[m] = sh.col0[m];
    }
    jobs.col0[sh.n] = sh.col0[sh.n];
    const int Ntot = sh.col0[sh.n];
    return launch_kernel(tm, accumulate_kernel, dim3((Ntot + 255) / 256), dim3(256), 0, stream, jobs, gpart, gslices,
                         cpart, cslices, Ntot);
}

}  // namespace decdec
