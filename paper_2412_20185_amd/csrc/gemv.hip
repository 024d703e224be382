// Base GEMV as a kernel of its own (k = 0, or when the compensation runs in
// separate kernels).  The device code is in gemv_body.h.
#include <hip/hip_runtime.h>

#include "gemv_body.h"

namespace decdec {
namespace {

template <int KIND, int WPB, int NBUF>
__global__ __launch_bounds__(WPB * 64) void gemv_kernel(const GemvJobs jobs, const FinalizeArgs fa,
                                                        const uint32_t* __restrict__ x32, float* __restrict__ part,
                                                        int Ntot, int G, int slices, int gpw) {
    gemv_block<KIND, WPB, NBUF>(jobs, fa, x32, part, Ntot, G, slices, gpw, (int)blockIdx.x);
}

template <int KIND, int WPB>
hipError_t launch_depth(int nbuf, const KernelTimer* tm, dim3 grid, hipStream_t stream, const GemvJobs& jobs,
                        const FinalizeArgs& fa, const uint32_t* x32, float* part, int Ntot, int G, int slices, int gpw) {
    const dim3 block(WPB * 64);
    if (nbuf >= 4)
        return launch_kernel(tm, gemv_kernel<KIND, WPB, 4>, grid, block, 0, stream, jobs, fa, x32, part, Ntot, G, slices,
                             gpw);
    return launch_kernel(tm, gemv_kernel<KIND, WPB, 2>, grid, block, 0, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
}

template <int KIND>
hipError_t launch_waves(int wpb, int nbuf, const KernelTimer* tm, dim3 grid, hipStream_t stream, const GemvJobs& jobs,
                        const FinalizeArgs& fa, const uint32_t* x32, float* part, int Ntot, int G, int slices, int gpw) {
    switch (wpb) {
        case 4: return launch_depth<KIND, 4>(nbuf, tm, grid, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
        case 8: return launch_depth<KIND, 8>(nbuf, tm, grid, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
        case 16: return launch_depth<KIND, 16>(nbuf, tm, grid, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

GemvPlan gemv_plan(long tiles, int G, int gpw_request, int wpb_request) {
    // One group per wavefront, so that a wavefront requests all its weights at once, as long as the chip
    // holds the wavefronts that makes at one time; two groups beyond that.  A K-slice more costs one atomic
    // per column (finalize.h), so the slices are not kept few: small matrices take small workgroups, which
    // start sooner and spread over more compute units; in between, the largest workgroups (a workgroup that
    // walks all of K alone writes y itself); the largest matrices run in several rounds of workgroups,
    // which medium workgroups fill more evenly.  Read from a sweep over the shapes of Llama-3 8B and 70B.
    GemvPlan p;
    const long units = tiles * G;  // (tile, group) pairs = wavefront iterations
    p.wpb = wpb_request > 0 ? wpb_request : units <= 4096 ? 4 : units <= 16384 ? 16 : 8;
    p.gpw = gpw_request > 0 ? gpw_request : units <= 12288 ? 1 : 2;
    int per_block = p.gpw * p.wpb;
    p.slices = (G + per_block - 1) / per_block;
    while (p.slices > kMaxGemvSlices) {
        ++p.gpw;
        per_block = p.gpw * p.wpb;
        p.slices = (G + per_block - 1) / per_block;
    }
    return p;
}

hipError_t launch_gemv(int kind, const MultiShape& sh, const GemvOperands& op, const void* x, float* part,
                       int slices, int gpw, int wpb, const FinalizeArgs& fa, hipStream_t stream, const KernelTimer* tm) {
    const int G = sh.K / kGroup;
    GemvJobs jobs{};
    jobs.n = sh.n;
    int tiles = 0;
    for (int m = 0; m < sh.n; ++m) {
        jobs.Wq[m] = static_cast<const uint4*>(op.Wq[m]);
        jobs.scales[m] = static_cast<const uint16_t*>(op.scales[m]);
        jobs.zeros_or_lut[m] = static_cast<const uint16_t*>(op.zeros_or_lut[m]);
        jobs.N[m] = sh.N[m];
        jobs.col0[m] = sh.col0[m];
        tiles += sh.N[m] / kTileCols;
        jobs.tile_end[m] = tiles;
    }
    const dim3 grid((unsigned)(tiles * slices));
    const uint32_t* x32 = static_cast<const uint32_t*>(x);
    const int Ntot = sh.col0[sh.n];
    const int nbuf = gpw > 2 ? 4 : 2;  // tiles a wave keeps in flight
    switch (kind) {
        case PACK_U4:
            return launch_waves<PACK_U4>(wpb, nbuf, tm, grid, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
        case PACK_U3:
            return launch_waves<PACK_U3>(wpb, nbuf, tm, grid, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
        case PACK_LUT3:
            return launch_waves<PACK_LUT3>(wpb, nbuf, tm, grid, stream, jobs, fa, x32, part, Ntot, G, slices, gpw);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace decdec
