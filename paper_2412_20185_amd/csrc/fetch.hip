// Residual fetch + residual GEMV as a kernel of its own.  The device code is
// in fetch_body.h.
#include <hip/hip_runtime.h>

#include "fetch_body.h"

namespace decdec {
namespace {

template <int SELECT_NCH>
__global__ __launch_bounds__(kBlockThreads) void fetch_fp16_kernel(const FetchJobs jobs, const FinalizeArgs fa,
                                                        const uint16_t* __restrict__ x, int32_t* idx_g,
                                                        uint16_t* xsel_g, int k, int K, int Ntot,
                                                        float* __restrict__ cpart, int wavecols, int slices) {
    fetch_fp16_block<SELECT_NCH>(jobs, fa, x, idx_g, xsel_g, k, K, Ntot, cpart, wavecols, slices, (int)blockIdx.x);
}

template <int BITS, int SELECT_NCH>
__global__ __launch_bounds__(kBlockThreads) void fetch_int_kernel(const FetchJobs jobs, const FinalizeArgs fa,
                                                                 const uint16_t* __restrict__ x, int32_t* idx_g,
                                                                 uint16_t* xsel_g, int k, int K, int Ntot,
                                                                 float* __restrict__ cpart, int wavecols,
                                                                 int slices) {
    fetch_int_block<BITS, SELECT_NCH>(jobs, fa, x, idx_g, xsel_g, k, K, Ntot, cpart, wavecols, slices,
                                      (int)blockIdx.x);
}

inline int cols_per_wave(int rfmt) { return fetch_cols_per_wave(rfmt); }

inline int total_wavecols(int rfmt, const MultiShape& sh) {
    int wc = 0;
    for (int m = 0; m < sh.n; ++m) wc += (sh.N[m] + cols_per_wave(rfmt) - 1) / cols_per_wave(rfmt);
    return wc;
}

}  // namespace

int fetch_slices(int rfmt, const MultiShape& sh, int k, int row_split, bool in_hbm) {
    const int wavecols = total_wavecols(rfmt, sh);
    int slices;
    if (row_split > 0) {
        slices = row_split;
    } else {
        // Host link: about 128 wavefronts x kUnroll rows x 1 KiB = 512 KiB of requests in flight saturate
        // it.  Rows in device memory: latency bound, so eight times as many wavefronts.
        const int waves = in_hbm ? 1024 : 128;
        slices = (waves + wavecols - 1) / wavecols;
    }
    if (slices > k) slices = k;
    if (slices > kMaxFetchSlices) slices = kMaxFetchSlices;
    if (slices < 1) slices = 1;
    return slices;
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
                                   int32_t* idx, uint16_t* xs, int k, int K, int Ntot, float* cpart, int wc,
                                   int slices, dim3 grid, hipStream_t stream, const KernelTimer* tm) {
    const unsigned lds = NCH > 0 ? (unsigned)(((size_t)k * 6 + 15) / 16 * 16) : 0u;
    if (rfmt == 0) {
        return launch_kernel(tm, fetch_fp16_kernel<NCH>, grid, dim3(kBlockThreads), lds, stream, jobs, fa, x, idx, xs, k, K,
                             Ntot, cpart, wc, slices);
    }
    if (rfmt == 1) {
        return launch_kernel(tm, fetch_int_kernel<4, NCH>, grid, dim3(kBlockThreads), lds, stream, jobs, fa, x, idx, xs, k,
                             K, Ntot, cpart, wc, slices);
    }
    if (rfmt == 2) {
        return launch_kernel(tm, fetch_int_kernel<2, NCH>, grid, dim3(kBlockThreads), lds, stream, jobs, fa, x, idx, xs, k,
                             K, Ntot, cpart, wc, slices);
    }
    return launch_kernel(tm, fetch_int_kernel<8, NCH>, grid, dim3(kBlockThreads), lds, stream, jobs, fa, x, idx, xs, k, K,
                         Ntot, cpart, wc, slices);
}

// select_chunks > 0: the kernel selects for itself from x (and writes the selection to idx / xsel);
// 0: idx / xsel hold the selection already.
hipError_t launch_fetch(int rfmt, const MultiShape& sh, const FetchOperands& op, const void* x, int select_chunks,
                        int32_t* idx, void* xsel, int k, float* cpart, int slices, const FinalizeArgs& fa,
                        hipStream_t stream, const KernelTimer* tm) {
    FetchJobs jobs{};
    jobs.n = sh.n;
    int wc = 0;
    for (int m = 0; m < sh.n; ++m) {
        jobs.R[m] = static_cast<const uint4*>(op.R[m]);
        jobs.Rs[m] = static_cast<const uint16_t*>(op.R_scales[m]);
        jobs.N[m] = sh.N[m];
        jobs.col0[m] = sh.col0[m];
        wc += (sh.N[m] + cols_per_wave(rfmt) - 1) / cols_per_wave(rfmt);
        jobs.wc_end[m] = wc;
    }
    const int tasks = wc * slices;
    const dim3 grid((unsigned)((tasks + kWavesPerBlock - 1) / kWavesPerBlock));
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint16_t* xs = static_cast<uint16_t*>(xsel);
    const int Ntot = sh.col0[sh.n];
    switch (select_chunks) {
        case 0: return launch_fetch_nch<0>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, wc, slices, grid, stream, tm);
        case 1: return launch_fetch_nch<1>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, wc, slices, grid, stream, tm);
        case 2: return launch_fetch_nch<2>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, wc, slices, grid, stream, tm);
        case 4: return launch_fetch_nch<4>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, wc, slices, grid, stream, tm);
        case 8: return launch_fetch_nch<8>(rfmt, jobs, fa, xp, idx, xs, k, sh.K, Ntot, cpart, wc, slices, grid, stream, tm);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace decdec
