// One launch for a whole compensated GEMV (DecDEC Section 4.1): the first
// `nfetch` workgroups of the grid do steps 1-3 (selection for themselves, then
// zero-copy fetch of the selected residual rows and the residual GEMV), all
// other workgroups do the base GEMV.
//
// Why one grid instead of the paper's two streams (Section 4.1, 4.3): measured
// on MI355X, handing work from one hardware queue to another costs about 10 us
// per join, more than the base GEMV itself for Llama-3-8B shapes, and a GEMV
// kernel that runs beside the fetch kernel from another queue starts late and
// runs 5-7x slower.  Inside one grid the fetch workgroups are dispatched first
// (lowest workgroup ids), the GEMV workgroups fill the rest of the chip and
// finish while the fetch workgroups are still waiting for the host link, and
// every workgroup adds its part sums into the per-column accumulators, the
// last arrival writing y (finalize.h), so nothing has to be joined and nothing
// else has to be launched.  (fp16 and 4-bit residuals; the 2- and 8-bit variants
// of the bit-width study use the separate kernels.)  How many workgroups fetch (the paper's n_tb,
// Section 4.4) follows from the number of wavefronts that share the rows of a
// column segment (decdec_ws_set_fetch_split).
#include <hip/hip_runtime.h>

#include "fetch_body.h"
#include "gemv_body.h"

namespace decdec {
namespace {

template <int KIND, int RBITS, int SELECT_NCH>
__global__ __launch_bounds__(kBlockThreads) void compensated_gemv_kernel(
    const GemvJobs gjobs, const FetchJobs fjobs, const FinalizeArgs fa, const uint16_t* __restrict__ x,
    int32_t* idx_g, uint16_t* xsel_g, int k, int K, int Ntot, float* __restrict__ gpart, float* __restrict__ cpart,
    int G, int gslices, int gpw, int segments, int cslices, int row_waves, int nfetch) {
    const int bid = (int)blockIdx.x;
    if (bid < nfetch) {
        fetch_block<RBITS, SELECT_NCH>(fjobs, fa, x, idx_g, xsel_g, k, K, Ntot, cpart, segments, cslices, row_waves, bid);
    } else {
        gemv_block<KIND, kWavesPerBlock, 2>(gjobs, fa, reinterpret_cast<const uint32_t*>(x), gpart, Ntot, G, gslices,
                                            gpw, bid - nfetch);
    }
}

template <int KIND, int RBITS>
hipError_t launch_nch(int nch, const KernelTimer* tm, dim3 grid, unsigned lds, hipStream_t stream,
                      const GemvJobs& gj, const FetchJobs& fj, const FinalizeArgs& fa, const uint16_t* x, int32_t* idx,
                      uint16_t* xs, int k, int K, int Ntot, float* gpart, float* cpart, int G, int gslices, int gpw,
                      int segments, int cslices, int row_waves, int nfetch) {
    const dim3 block(kBlockThreads);
    switch (nch) {
        case 0:
            return launch_kernel(tm, compensated_gemv_kernel<KIND, RBITS, 0>, grid, block, lds, stream, gj, fj, fa, x, idx,
                                 xs, k, K, Ntot, gpart, cpart, G, gslices, gpw, segments, cslices, row_waves, nfetch);
        case 1:
            return launch_kernel(tm, compensated_gemv_kernel<KIND, RBITS, 1>, grid, block, lds, stream, gj, fj, fa, x, idx,
                                 xs, k, K, Ntot, gpart, cpart, G, gslices, gpw, segments, cslices, row_waves, nfetch);
        case 2:
            return launch_kernel(tm, compensated_gemv_kernel<KIND, RBITS, 2>, grid, block, lds, stream, gj, fj, fa, x, idx,
                                 xs, k, K, Ntot, gpart, cpart, G, gslices, gpw, segments, cslices, row_waves, nfetch);
        case 4:
            return launch_kernel(tm, compensated_gemv_kernel<KIND, RBITS, 4>, grid, block, lds, stream, gj, fj, fa, x, idx,
                                 xs, k, K, Ntot, gpart, cpart, G, gslices, gpw, segments, cslices, row_waves, nfetch);
        case 8:
            return launch_kernel(tm, compensated_gemv_kernel<KIND, RBITS, 8>, grid, block, lds, stream, gj, fj, fa, x, idx,
                                 xs, k, K, Ntot, gpart, cpart, G, gslices, gpw, segments, cslices, row_waves, nfetch);
        default:
            return hipErrorInvalidValue;
    }
}

template <int KIND, typename... A>
hipError_t launch_rfmt(int rfmt, A... a) {
    return rfmt == 0 ? launch_nch<KIND, 16>(a...) : launch_nch<KIND, 4>(a...);
}

}  // namespace

hipError_t launch_compensated_gemv(int kind, int rfmt, const MultiShape& sh, const GemvOperands& gop,
                                   const FetchOperands& fop, const void* x, int select_chunks, int32_t* idx, void* xsel,
                                   int k, float* gpart, int gslices, int gpw, float* cpart, const FetchPlan& plan,
                                   const FinalizeArgs& fa, hipStream_t stream, const KernelTimer* tm) {
    if (rfmt != 0 && rfmt != 1) return hipErrorInvalidValue;  // built for fp16 and 4-bit residuals only
    const int G = sh.K / kGroup;
    GemvJobs gj{};
    const FetchJobs fj = make_fetch_jobs(sh, fop);
    gj.n = sh.n;
    int tiles = 0;
    for (int m = 0; m < sh.n; ++m) {
        gj.Wq[m] = static_cast<const uint4*>(gop.Wq[m]);
        gj.scales[m] = static_cast<const uint16_t*>(gop.scales[m]);
        gj.zeros_or_lut[m] = static_cast<const uint16_t*>(gop.zeros_or_lut[m]);
        gj.N[m] = sh.N[m];
        gj.col0[m] = sh.col0[m];
        tiles += sh.N[m] / kTileCols;
        gj.tile_end[m] = tiles;
    }
    const int nfetch = plan.segments * plan.slices;
    const dim3 grid((unsigned)(nfetch + tiles * gslices));
    const unsigned lds = select_chunks > 0 ? (unsigned)(((size_t)k * 6 + 15) / 16 * 16) : 0u;
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* xs = static_cast<uint16_t*>(xsel);
    const int Ntot = sh.col0[sh.n];
    switch (kind) {
        case PACK_U4:
            return launch_rfmt<PACK_U4>(rfmt, select_chunks, tm, grid, lds, stream, gj, fj, fa, xp, idx, xs, k, sh.K, Ntot,
                                        gpart, cpart, G, gslices, gpw, plan.segments, plan.slices, plan.row_waves, nfetch);
        case PACK_U3:
            return launch_rfmt<PACK_U3>(rfmt, select_chunks, tm, grid, lds, stream, gj, fj, fa, xp, idx, xs, k, sh.K, Ntot,
                                        gpart, cpart, G, gslices, gpw, plan.segments, plan.slices, plan.row_waves, nfetch);
        case PACK_LUT3:
            return launch_rfmt<PACK_LUT3>(rfmt, select_chunks, tm, grid, lds, stream, gj, fj, fa, xp, idx, xs, k, sh.K,
                                          Ntot, gpart, cpart, G, gslices, gpw, plan.segments, plan.slices,
                                          plan.row_waves, nfetch);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace decdec
