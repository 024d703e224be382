// Step 4 of dynamic error compensation (DecDEC Section 4.1): o = o_b + o_dec,
// as a kernel of its own.
//
// By default the producers add their part sums themselves, with one
// fixed-point atomic per output column (finalize.h).  This kernel is the other
// way to do it (decdec_ws_set_inkernel_accumulate(ws, 0)): both producers leave
// fp32 partial rows (the base GEMV one per K-slice, the residual kernel one per
// slice of the selected channels) and this kernel, enqueued on the caller's
// stream after both, converts every entry to the same fixed point, adds the
// integers and rounds once to fp16: the same bits as the atomic path, by a
// mechanism that shares nothing with it but the conversion.
#include <hip/hip_runtime.h>

#include "finalize.h"
#include "kernels.h"

namespace decdec {
namespace {

struct AccJobs {
    _Float16* y[kMaxMulti];
    int col0[kMaxMulti + 1];
    int n;
};

// One workgroup = 64 columns x 8 wavefronts.  Wavefront p adds the partial rows s = p, p + 8, ... of both
// producers in fixed point (all its loads are independent and issued together); the eight integer part sums
// are added through LDS.
__global__ __launch_bounds__(512) void accumulate_kernel(const AccJobs jobs, const float* __restrict__ gpart,
                                                        int gslices, const float* __restrict__ cpart, int cslices,
                                                        int Ntot) {
    __shared__ long long part[8][64];
    const int lane = threadIdx.x & 63, p = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;  // concatenated column; Ntot is a multiple of 64
    long long sum = 0;
#pragma unroll 8
    for (int s = p; s < gslices; s += 8) sum += to_fixed(gpart[(size_t)s * Ntot + c]);
#pragma unroll 8
    for (int r = p; r < cslices; r += 8) sum += to_fixed(cpart[(size_t)r * Ntot + c]);
    part[p][lane] = sum;
    __syncthreads();
    if (p != 0) return;
#pragma unroll
    for (int q = 1; q < 8; ++q) sum += part[q][lane];
    int m = 0;
#pragma unroll
    for (int i = 1; i < kMaxMulti; ++i) m += (i < jobs.n && c >= jobs.col0[i]) ? 1 : 0;
    jobs.y[m][c - jobs.col0[m]] = from_fixed(sum);
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
