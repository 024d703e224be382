// Step 4 of dynamic error compensation (DecDEC Section 4.1): o = o_b + o_dec.
//
// The paper adds o_dec into o_b with atomics from inside its fused kernel
// (Section 4.3 "Kernel Fusion").  Here both producers leave fp32 partial rows
// (the base GEMV one per K-slice, the residual kernel one per slice of the
// selected channels), which are added in a fixed order and rounded once to
// fp16, so that the result does not depend on which producer finished first.
// By default the producers do that themselves (finalize.h: the last workgroup
// of a 64-column tile adds the tile); this kernel is the other way to do it
// (decdec_ws_set_inkernel_accumulate(ws, 0)): enqueued on the caller's stream
// after both producers, same order, same bits.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace decdec {
namespace {

struct AccJobs {
    _Float16* y[kMaxMulti];
    int col0[kMaxMulti + 1];
    int n;
};

// One workgroup = 64 columns x 8 wavefronts.  Wavefront p adds the partial rows s = p, p + 8, ... of both
// producers (all its loads are independent and issued together), the eight part sums are combined as a
// fixed tree: y = ((v0 + v1) + (v2 + v3)) + ((v4 + v5) + (v6 + v7)),  v_p = o_b,p + o_dec,p.
__global__ __launch_bounds__(512) void accumulate_kernel(const AccJobs jobs, const float* __restrict__ gpart,
                                                        int gslices, const float* __restrict__ cpart, int cslices,
                                                        int Ntot) {
    __shared__ float part[8][64];
    const int lane = threadIdx.x & 63, p = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;  // concatenated column; Ntot is a multiple of 64
    float ob = 0.f, odec = 0.f;
#pragma unroll 8
    for (int s = p; s < gslices; s += 8) ob += gpart[(size_t)s * Ntot + c];
#pragma unroll 8
    for (int r = p; r < cslices; r += 8) odec += cpart[(size_t)r * Ntot + c];
    part[p][lane] = ob + odec;
    __syncthreads();
    if (p != 0) return;
    const float v = ((part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane])) +
                    ((part[4][lane] + part[5][lane]) + (part[6][lane] + part[7][lane]));
    int m = 0;
#pragma unroll
    for (int i = 1; i < kMaxMulti; ++i) m += (i < jobs.n && c >= jobs.col0[i]) ? 1 : 0;
    jobs.y[m][c - jobs.col0[m]] = (_Float16)v;
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
    return launch_kernel(tm, accumulate_kernel, dim3(Ntot / 64), dim3(512), 0, stream, jobs, gpart, gslices,
                         cpart, cslices, Ntot);
}

}  // namespace decdec
