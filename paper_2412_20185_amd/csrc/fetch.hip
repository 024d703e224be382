// Steps 2 and 3 of dynamic error compensation (DecDEC Section 4.1): fetch the
// residual rows of the selected input channels from pinned CPU memory and
// multiply them with x[sc_indices]:  o_dec[n] = sum_j R_hat[s_j][n] * x[s_j].
//
// Zero-copy (Section 4.3): the kernel reads the rows in place over the host
// link with plain 128-bit loads; a wavefront covers 1 KiB of one row per load,
// so requests are cache-line sized and contiguous per row (Section 4.2: each
// input-channel row is contiguous in CPU memory).  As in the paper's kernel
// (Section 4.3 "Kernel Fusion") a wave owns a column segment of the rows it
// handles, so the sum over its rows needs no cross-lane reduction.  Unlike the
// paper's kernel the rows are additionally split into `slices` (the knob that
// plays the role of n_tb in Section 4.4: enough requests in flight to fill
// the link without taking compute units from the base GEMV); each slice
// writes one fp32 partial row and the accumulate kernel adds them.
#include <hip/hip_runtime.h>

#include "finalize.h"
#include "kernels.h"

namespace decdec {
namespace {

constexpr int kUnroll = 4;  // row loads in flight per lane

__device__ __forceinline__ float h2f(uint32_t bits16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

struct FetchJobs {
    const uint4* R[kMaxMulti];
    const uint16_t* Rs[kMaxMulti];
    int N[kMaxMulti];
    int col0[kMaxMulti];
    int wc_end[kMaxMulti];  // cumulative count of wave-wide column segments up to and including matrix m
    int n;
};

struct WaveTask {
    int m, wc, rs;
    bool valid;
};

// Task t of the grid: row slice rs = t / wavecols, column segment t % wavecols
// of the concatenated matrices.
__device__ __forceinline__ WaveTask wave_task(const FetchJobs& jobs, int wavecols, int slices) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int task = blockIdx.x * 4 + wave;
    WaveTask t;
    t.valid = task < wavecols * slices;
    t.rs = task / wavecols;
    const int c = task - t.rs * wavecols;
    int m = 0;
#pragma unroll
    for (int i = 0; i < kMaxMulti - 1; ++i) m += (i + 1 < jobs.n && c >= jobs.wc_end[i]) ? 1 : 0;
    t.m = m;
    t.wc = c - (m > 0 ? jobs.wc_end[m - 1] : 0);
    return t;
}

// Wave task (m, wc, rs): columns [wc*512, wc*512+512) of matrix m for the rows j in slice rs.
__global__ __launch_bounds__(256) void fetch_fp16_kernel(const FetchJobs jobs, const FinalizeArgs fa,
                                                        const int32_t* __restrict__ idx,
                                                        const uint16_t* __restrict__ xsel, int k, int K, int Ntot,
                                                        float* __restrict__ cpart, int wavecols, int slices) {
    const int lane = threadIdx.x & 63;
    const WaveTask t = wave_task(jobs, wavecols, slices);
    if (!t.valid) return;
    const int N = jobs.N[t.m];
    const uint4* __restrict__ R = jobs.R[t.m];
    const int oct = t.wc * 64 + lane;  // 8 columns = one 16-byte piece of a row
    const bool active = oct * 8 < N;
    const int rows_per = (k + slices - 1) / slices;
    const int j0 = t.rs * rows_per, j1 = min(j0 + rows_per, k);
    const size_t row16 = (size_t)(N / 8);

    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = j0; j < j1; j += kUnroll) {
        uint4 v[kUnroll];
        float xs[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            v[u] = make_uint4(0, 0, 0, 0);
            xs[u] = 0.f;
            if (j + u < j1) {
                const int row = idx[j + u];
                if (active && (unsigned)row < (unsigned)K) {
                    v[u] = R[(size_t)row * row16 + oct];
                    xs[u] = h2f(xsel[j + u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[2 * c] = fmaf(h2f(w[c] & 0xFFFFu), xs[u], acc[2 * c]);
                acc[2 * c + 1] = fmaf(h2f(w[c] >> 16), xs[u], acc[2 * c + 1]);
            }
        }
    }
    if (active) {
        float* out = cpart + (size_t)t.rs * Ntot + jobs.col0[t.m] + (size_t)oct * 8;
        if (fa.counters != nullptr) {
#pragma unroll
            for (int i = 0; i < 8; ++i) store_partial(out + i, acc[i], true);
        } else {
            reinterpret_cast<float4*>(out)[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            reinterpret_cast<float4*>(out)[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        }
    }
    if (fa.counters != nullptr) tiles_arrive_and_finalize(fa, t.m, t.wc * 8, min(8, N / 64 - t.wc * 8), lane);
}

// 4-bit residuals (Section 4.2): a 16-byte piece holds 32 columns; a wave
// covers 2048 columns.  o_dec[n] = S[n] * sum_j q[s_j][n] x[s_j].
__global__ __launch_bounds__(256) void fetch_int4_kernel(const FetchJobs jobs, const FinalizeArgs fa,
                                                        const int32_t* __restrict__ idx,
                                                        const uint16_t* __restrict__ xsel, int k, int K, int Ntot,
                                                        float* __restrict__ cpart, int wavecols, int slices) {
    const int lane = threadIdx.x & 63;
    const WaveTask t = wave_task(jobs, wavecols, slices);
    if (!t.valid) return;
    const int N = jobs.N[t.m];
    const uint4* __restrict__ R = jobs.R[t.m];
    const uint16_t* __restrict__ Rs = jobs.Rs[t.m];
    const int piece = t.wc * 64 + lane;  // 32 columns
    const bool active = piece * 32 < N;
    const int rows_per = (k + slices - 1) / slices;
    const int j0 = t.rs * rows_per, j1 = min(j0 + rows_per, k);
    const size_t row16 = (size_t)(N / 32);

    float acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.f;
    for (int j = j0; j < j1; j += kUnroll) {
        uint4 v[kUnroll];
        float xs[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            v[u] = make_uint4(0, 0, 0, 0);
            xs[u] = 0.f;
            if (j + u < j1) {
                const int row = idx[j + u];
                if (active && (unsigned)row < (unsigned)K) {
                    v[u] = R[(size_t)row * row16 + piece];
                    xs[u] = h2f(xsel[j + u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int q = (int)(w[c] << (28 - 4 * i)) >> 28;  // 4-bit two's complement
                    acc[8 * c + i] = fmaf((float)q, xs[u], acc[8 * c + i]);
                }
            }
        }
    }
    if (active) {
        const uint4* s4 = reinterpret_cast<const uint4*>(Rs + (size_t)piece * 32);
        float* out = cpart + (size_t)t.rs * Ntot + jobs.col0[t.m] + (size_t)piece * 32;
        const bool coherent = fa.counters != nullptr;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint4 sv = s4[b];
            const uint32_t sw[4] = {sv.x, sv.y, sv.z, sv.w};
            float r[8];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                r[2 * c] = acc[8 * b + 2 * c] * h2f(sw[c] & 0xFFFFu);
                r[2 * c + 1] = acc[8 * b + 2 * c + 1] * h2f(sw[c] >> 16);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) store_partial(out + 8 * b + i, r[i], coherent);
        }
    }
    if (fa.counters != nullptr) tiles_arrive_and_finalize(fa, t.m, t.wc * 32, min(32, N / 64 - t.wc * 32), lane);
}

inline int cols_per_wave(int rfmt) { return rfmt == 0 ? 512 : 2048; }

inline int total_wavecols(int rfmt, const MultiShape& sh) {
    int wc = 0;
    for (int m = 0; m < sh.n; ++m) wc += (sh.N[m] + cols_per_wave(rfmt) - 1) / cols_per_wave(rfmt);
    return wc;
}

}  // namespace

int fetch_slices(int rfmt, const MultiShape& sh, int k, int row_split) {
    const int wavecols = total_wavecols(rfmt, sh);
    int slices;
    if (row_split > 0) {
        slices = row_split;
    } else {
        // about 128 wavefronts x kUnroll rows x 1 KiB = 512 KiB of requests in flight
        slices = (128 + wavecols - 1) / wavecols;
    }
    if (slices > k) slices = k;
    if (slices > kMaxFetchSlices) slices = kMaxFetchSlices;
    if (slices < 1) slices = 1;
    return slices;
}

hipError_t launch_fetch(int rfmt, const MultiShape& sh, const FetchOperands& op, const int32_t* idx,
                        const void* xsel, int k, float* cpart, int slices, const FinalizeArgs& fa,
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
    const dim3 grid((unsigned)((tasks + 3) / 4)), block(256);
    const uint16_t* xs = static_cast<const uint16_t*>(xsel);
    const int Ntot = sh.col0[sh.n];
    if (rfmt == 0) {
        return launch_kernel(tm, fetch_fp16_kernel, grid, block, 0, stream, jobs, fa, idx, xs, k, sh.K, Ntot, cpart,
                             wc, slices);
    }
    return launch_kernel(tm, fetch_int4_kernel, grid, block, 0, stream, jobs, fa, idx, xs, k, sh.K, Ntot, cpart, wc,
                         slices);
}

}  // namespace decdec
