// Residual fetch + residual GEMV as a kernel of its own.  The device code is
// in fetch_body.h.
#include <hip/hip_runtime.h>

#include "fetch_body.h"

namespace decdec {
namespace {

template <int BITS, int SELECT_NCH>
__global__ __launch_bounds__(kBlockThreads) void fetch_kernel(const FetchJobs jobs, const FinalizeArgs fa,
                                                             const uint16_t* __restrict__ x, int32_t* idx_g,
                                                             uint16_t* xsel_g, int k, int K, int Ntot,
                                                             float* __restrict__ cpart, int segments, int slices,
                                                             int row_waves) {
    fetch_block<BITS, SELECT_NCH>(jobs, fa, x, idx_g, xsel_g, k, K, Ntot, cpart, segments, slices, row_waves,
                                  (int)blockIdx.x);
}

}  // namespace

FetchPlan fetch_plan(int rfmt, const MultiShape& sh, int k, int row_split, bool in_hbm) {
    FetchPlan p;
    p.segments = 0;
    for (int m = 0; m < sh.n; ++m) p.segments += (sh.N[m] + kFetchSegmentCols - 1) / kFetchSegmentCols;
    // Host link: about 128 wavefronts x 4 KiB of row loads each = 512 KiB of requests in flight saturate it.
    // Rows in device memory: latency bound, so eight times as many wavefronts.
    const int waves = in_hbm ? 1024 : 128;
    // wavefronts that share the rows of one segment
    int per_segment = row_split > 0 ? row_split : (waves + p.segments - 1) / p.segments;
    // fp16 rows: one workgroup per segment is enough once there are eight segments (64 wavefronts already
    // fill the link, and every column has one part sum fewer to add); measured 0.6 % on the Llama-3-8B layer
    if (row_split <= 0 && !in_hbm && rfmt == 0 && p.segments >= 8 && per_segment > kWavesPerBlock)
        per_segment = kWavesPerBlock;
    if (per_segment > kMaxFetchSlices * kWavesPerBlock) per_segment = kMaxFetchSlices * kWavesPerBlock;
    if (per_segment > k) per_segment = k;
    if (per_segment < 1) per_segment = 1;
    p.slices = (per_segment + kWavesPerBlock - 1) / kWavesPerBlock;
    p.row_waves = (per_segment + p.slices - 1) / p.slices;
    return p;
}

int fetch_select_chunks(int K, int k) {
    // In-kernel selection: the keys of a workgroup stay in registers (at most 8 chunks of 8 per thread)
    // and the selection must fit in LDS.
    constexpr int per_chunk_round = 8 * kBlockThreads;  // channels covered by one chunk per thread
    if (k < 1 || k > 4096 || K > 8 * per_chunk_round) return 0;
    return K <= per_chunk_round ? 1 : K <= 2 * per_chunk_round ? 2 : K <= 4 * per_chunk_round ? 4 : 8;
}

template <int NCH>
static hipError_t launch_fetch_nch(int rfmt, const FetchJobs& jobs, const FinalizeArgs& fa, const uint16_t* x,
                                   int32_t* idx, uint16_t* xs, int k, int K, int Ntot, float* cpart,
                                   const FetchPlan& p, hipStream_t stream, const KernelTimer* tm) {
    const unsigned lds = NCH > 0 ? (unsigned)(((size_t)k * 6 + 15) / 16 * 16) : 0u;
    const dim3 grid((unsigned)(p.segments * p.slices)), block(kBlockThreads);
    switch (rfmt) {
        case 0:
            return launch_kernel(tm, fetch_kernel<16, NCH>, grid, block, lds, stream, jobs, fa, x, idx, xs, k, K, Ntot,
                                 cpart, p.segments, p.slices, p.row_waves);
        case 1:
            return launch_kernel(tm, fetch_kernel<4, NCH>, grid, block, lds, stream, jobs, fa, x, idx, xs, k, K, Ntot,
                                 cpart, p.segments, p.slices, p.row_waves);
        case 2:
            return launch_kernel(tm, fetch_kernel<2, NCH>, grid, block, lds, stream, jobs, fa, x, idx, xs, k, K, Ntot,
                                 cpart, p.segments, p.slices, p.row_waves);
        default:
            return launch_kernel(tm, fetch_kernel<8, NCH>, grid, block, lds, stream, jobs, fa, x, idx, xs, k, K, Ntot,
                                 cpart, p.segments, p.slices, p.row_waves);
    }
}

// select_chunks > 0: the kernel selects for itself from x (and writes the selection to idx / xsel);
// 0: idx / xsel hold the selection already.
hipError_t launch_fetch(int rfmt, const MultiShape& sh, const FetchOperands& op, const void* x, int select_chunks,
                        int32_t* idx, void* xsel, int k, float* cpart, const FetchPlan& plan, const FinalizeArgs& fa,
                        hipStream_t stream, const KernelTimer* tm) {
    const FetchJobs jobs = make_fetch_jobs(sh, op);
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* xs = static_cast<uint16_t*>(xsel);
    const int Ntot = sh.col0[sh.n];
    switch (select_chunks) {
        case 0: return launch_fetch_nch<0>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, plan, stream, tm);
        case 1: return launch_fetch_nch<1>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, plan, stream, tm);
        case 2: return launch_fetch_nch<2>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, plan, stream, tm);
        case 4: return launch_fetch_nch<4>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, plan, stream, tm);
        case 8: return launch_fetch_nch<8>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, plan, stream, tm);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace decdec
