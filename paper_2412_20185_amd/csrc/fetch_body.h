// Device code of the residual kernel (included by fetch.hip and fused.hip).
//
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
//
// Selection inside the kernel (SELECT_NCH > 0): every workgroup first runs the
// exact top-k of select_block.h on x for itself and keeps sc_indices and
// x[sc_indices] in LDS, so step 1 costs no launch of its own and no trip
// through global memory (the paper's fused kernel does step 1 inside the
// kernel too, Section 4.3, but needs a grid-wide barrier because its
// selection is spread over the thread blocks; an exact select that is cheap
// enough to repeat per workgroup needs none).  Workgroup 0 also writes the
// selection to global memory for the caller.
#pragma once
#include <hip/hip_runtime.h>

#include "finalize.h"
#include "kernels.h"
#include "select_block.h"

namespace decdec {

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
__device__ __forceinline__ WaveTask wave_task(const FetchJobs& jobs, int wavecols, int slices, int bid) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int task = bid * kWavesPerBlock + wave;
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

// sc_indices / x[sc_indices] as the fetch loops see them: global memory, or LDS
// after an in-kernel selection.
struct Selection {
    const int32_t* idx;
    const uint16_t* xsel;
};

template <int SELECT_NCH>
__device__ __forceinline__ Selection obtain_selection(const uint16_t* __restrict__ x, int K, int k,
                                                      int32_t* idx_g, uint16_t* xsel_g, int bid) {
    if constexpr (SELECT_NCH > 0) {
        extern __shared__ uint4 s_sel_raw[];  // int32 idx[k], then fp16 xsel[k]
        __shared__ SelectShared sh;
        int32_t* idx_l = reinterpret_cast<int32_t*>(s_sel_raw);
        uint16_t* xs_l = reinterpret_cast<uint16_t*>(idx_l + k);
        block_select_topk<kBlockThreads, SELECT_NCH>(x, K, k, sh, idx_l, xs_l);
        __syncthreads();
        if (bid == 0) {
            for (int i = threadIdx.x; i < k; i += kBlockThreads) {
                idx_g[i] = idx_l[i];
                xsel_g[i] = xs_l[i];
            }
        }
        return Selection{idx_l, xs_l};
    } else {
        return Selection{idx_g, xsel_g};
    }
}

// Wave task (m, wc, rs): columns [wc*512, wc*512+512) of matrix m for the rows j in slice rs.
template <int SELECT_NCH>
__device__ __forceinline__ void fetch_fp16_block(const FetchJobs& jobs, const FinalizeArgs& fa,
                                                const uint16_t* __restrict__ x, int32_t* idx_g, uint16_t* xsel_g,
                                                int k, int K, int Ntot, float* __restrict__ cpart, int wavecols,
                                                int slices, int bid) {
    const int lane = threadIdx.x & 63;
    const Selection sel = obtain_selection<SELECT_NCH>(x, K, k, idx_g, xsel_g, bid);
    const int32_t* idx = sel.idx;
    const uint16_t* xsel = sel.xsel;
    const WaveTask t = wave_task(jobs, wavecols, slices, bid);
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
        int row[kUnroll];
        uint32_t xraw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {  // indices and activations first, so that no row load waits for them
            const int jj = min(j + u, j1 - 1);
            row[u] = idx[jj];
            xraw[u] = xsel[jj];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            v[u] = make_uint4(0, 0, 0, 0);
            if (j + u < j1 && active && (unsigned)row[u] < (unsigned)K) v[u] = R[(size_t)row[u] * row16 + oct];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            xs[u] = (j + u < j1 && (unsigned)row[u] < (unsigned)K) ? h2f(xraw[u]) : 0.f;
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

// Integer residuals (Section 4.2: 4-bit symmetric with one scale per output
// column; 2- and 8-bit are the variants of the paper's bit-width study, Table
// 2): a 16-byte piece holds CPL = 128/BITS columns; a wave covers 64*CPL
// columns.  o_dec[n] = S[n] * sum_j q[s_j][n] x[s_j].
template <int BITS, int SELECT_NCH>
__device__ __forceinline__ void fetch_int_block(const FetchJobs& jobs, const FinalizeArgs& fa,
                                               const uint16_t* __restrict__ x, int32_t* idx_g, uint16_t* xsel_g,
                                               int k, int K, int Ntot, float* __restrict__ cpart, int wavecols,
                                               int slices, int bid) {
    constexpr int CPL = 128 / BITS;  // columns per lane
    constexpr int CPW = 32 / BITS;   // codes per 32-bit word
    const int lane = threadIdx.x & 63;
    const Selection sel = obtain_selection<SELECT_NCH>(x, K, k, idx_g, xsel_g, bid);
    const int32_t* idx = sel.idx;
    const uint16_t* xsel = sel.xsel;
    const WaveTask t = wave_task(jobs, wavecols, slices, bid);
    if (!t.valid) return;
    const int N = jobs.N[t.m];
    const uint4* __restrict__ R = jobs.R[t.m];
    const uint16_t* __restrict__ Rs = jobs.Rs[t.m];
    const int piece = t.wc * 64 + lane;
    const bool active = piece * CPL < N;
    const int rows_per = (k + slices - 1) / slices;
    const int j0 = t.rs * rows_per, j1 = min(j0 + rows_per, k);
    const size_t row16 = (size_t)(N / CPL);

    // The column scales are requested before the rows, so that they arrive behind the first row loads
    // instead of costing a round trip of their own after the last one.
    uint4 sv[CPL / 8];
#pragma unroll
    for (int b = 0; b < CPL / 8; ++b)
        sv[b] = active ? reinterpret_cast<const uint4*>(Rs + (size_t)piece * CPL)[b] : make_uint4(0, 0, 0, 0);

    float acc[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) acc[i] = 0.f;
    for (int j = j0; j < j1; j += kUnroll) {
        uint4 v[kUnroll];
        float xs[kUnroll];
        int row[kUnroll];
        uint32_t xraw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {  // indices and activations first, so that no row load waits for them
            const int jj = min(j + u, j1 - 1);
            row[u] = idx[jj];
            xraw[u] = xsel[jj];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            v[u] = make_uint4(0, 0, 0, 0);
            if (j + u < j1 && active && (unsigned)row[u] < (unsigned)K) v[u] = R[(size_t)row[u] * row16 + piece];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            xs[u] = (j + u < j1 && (unsigned)row[u] < (unsigned)K) ? h2f(xraw[u]) : 0.f;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (j + u >= j1) break;  // wave-uniform: a short slice does not pay for the rows it does not have
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
#pragma unroll
                for (int i = 0; i < CPW; ++i) {
                    const int q = (int)(w[c] << (32 - BITS * (i + 1))) >> (32 - BITS);  // two's complement field
                    acc[CPW * c + i] = fmaf((float)q, xs[u], acc[CPW * c + i]);
                }
            }
        }
    }
    if (active) {
#pragma unroll
        for (int b = 0; b < CPL / 8; ++b) {
            const uint32_t sw[4] = {sv[b].x, sv[b].y, sv[b].z, sv[b].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[8 * b + 2 * c] *= h2f(sw[c] & 0xFFFFu);
                acc[8 * b + 2 * c + 1] *= h2f(sw[c] >> 16);
            }
        }
        float* out = cpart + (size_t)t.rs * Ntot + jobs.col0[t.m] + (size_t)piece * CPL;
        if (fa.counters != nullptr) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) store_partial(out + i, acc[i], true);
        } else {
#pragma unroll
            for (int i = 0; i < CPL / 4; ++i)
                reinterpret_cast<float4*>(out)[i] = make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
        }
    }
    if (fa.counters != nullptr)
        tiles_arrive_and_finalize(fa, t.m, t.wc * CPL, min(CPL, N / 64 - t.wc * CPL), lane);
}

// Columns one wavefront covers per row load, by residual format (decdec_rfmt).
__host__ __device__ constexpr int fetch_cols_per_wave(int rfmt) {
    return rfmt == 0 ? 512 : rfmt == 1 ? 2048 : rfmt == 2 ? 4096 : 1024;
}

}  // namespace decdec
