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
// (Section 4.3 "Kernel Fusion") the unit of ownership is a column segment: a
// workgroup owns the 1 KiB-per-row segment `wc` of the rows it handles, so its
// sum over those rows never leaves the compute unit.  The selected rows of a
// segment are spread over the wavefronts of the workgroup (and over `slices`
// workgroups when one workgroup does not put enough requests in flight: the
// knob that plays the role of n_tb in Section 4.4); the wavefronts' sums meet
// in LDS and the workgroup leaves ONE fp32 partial row per segment.
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
    int wc_end[kMaxMulti];  // cumulative count of column segments up to and including matrix m
    int n;
};

// Workgroup `bid` of the residual grid: row slice rs = bid / segments, column
// segment bid % segments of the concatenated matrices.
struct BlockTask {
    int m, wc, rs;
};

__device__ __forceinline__ BlockTask block_task(const FetchJobs& jobs, int segments, int bid) {
    BlockTask t;
    t.rs = bid / segments;
    const int c = bid - t.rs * segments;
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

// One workgroup = one column segment (64 lanes x 16 bytes of every row) x the
// rows of row slice rs; wavefront w < row_waves of it takes a contiguous share
// of those rows.  BITS = 16: fp16 rows.  BITS = 2, 4, 8: integer residuals
// (Section 4.2: 4-bit symmetric with one scale per output column; 2- and 8-bit
// are the variants of the paper's bit-width study, Table 2): a 16-byte piece
// holds CPL = 128/BITS columns,  o_dec[n] = S[n] * sum_j q[s_j][n] x[s_j].
//
// After the row loop the wavefronts' sums are added through LDS, eight columns
// of every lane per round, in the fixed order w = 0, 1, ...: thread t of the
// workgroup ends up with the segment's sum for CPL/8 columns.  It writes them
// to row rs of cpart; with in-kernel accumulation the workgroup then counts
// itself in on the 64-column tiles of its segment and adds up those it
// completes (finalize.h).
template <int BITS, int SELECT_NCH>
__device__ __forceinline__ void fetch_block(const FetchJobs& jobs, const FinalizeArgs& fa,
                                            const uint16_t* __restrict__ x, int32_t* idx_g, uint16_t* xsel_g, int k,
                                            int K, int Ntot, float* __restrict__ cpart, int segments, int slices,
                                            int row_waves, int bid) {
    constexpr int CPL = 128 / BITS;                // columns per lane (per 16-byte piece)
    constexpr int ROUNDS = CPL / 8;                // LDS rounds of 8 columns per lane
    constexpr int CPW = BITS == 16 ? 2 : 32 / BITS;  // columns per 32-bit word
    __shared__ float red[kWavesPerBlock][kBlockThreads];
    __shared__ unsigned tile_done[64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const Selection sel = obtain_selection<SELECT_NCH>(x, K, k, idx_g, xsel_g, bid);
    const int32_t* idx = sel.idx;
    const uint16_t* xsel = sel.xsel;
    const BlockTask t = block_task(jobs, segments, bid);
    const int N = jobs.N[t.m];
    const uint4* __restrict__ R = jobs.R[t.m];
    const int piece = t.wc * 64 + lane;  // 16-byte piece of a row this lane loads
    const bool active = piece * CPL < N;
    const size_t row16 = (size_t)(N / CPL);
    // rows of this wavefront: slice (rs, wave) out of slices * row_waves equal shares of the k selected rows
    const int rows_per = (k + slices * row_waves - 1) / (slices * row_waves);
    const int j0 = min((t.rs * row_waves + wave) * rows_per, k);
    const int j1 = wave < row_waves ? min(j0 + rows_per, k) : j0;

    // Columns this thread owns after the LDS rounds: round q gives it column ocol + 8 q of the matrix.
    const int ocol = (t.wc * 64 + (tid >> 3)) * CPL + (tid & 7);
    const bool owns = ocol < N;  // N is a multiple of 64, hence of 8 q steps inside a piece
    // The column scales are requested before the rows, so that they arrive behind the first row loads
    // instead of costing a round trip of their own after the last one.
    uint16_t sraw[ROUNDS];
    if constexpr (BITS != 16) {
        const uint16_t* __restrict__ Rs = jobs.Rs[t.m];
#pragma unroll
        for (int q = 0; q < ROUNDS; ++q) sraw[q] = owns ? Rs[ocol + 8 * q] : (uint16_t)0;
    }

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
                if constexpr (BITS == 16) {
                    acc[2 * c] = fmaf(h2f(w[c] & 0xFFFFu), xs[u], acc[2 * c]);
                    acc[2 * c + 1] = fmaf(h2f(w[c] >> 16), xs[u], acc[2 * c + 1]);
                } else {
#pragma unroll
                    for (int i = 0; i < CPW; ++i) {
                        const int q = (int)(w[c] << (32 - BITS * (i + 1))) >> (32 - BITS);  // two's complement field
                        acc[CPW * c + i] = fmaf((float)q, xs[u], acc[CPW * c + i]);
                    }
                }
            }
        }
    }

    // Sum over the wavefronts of the workgroup, 8 columns per lane and round.
    float val[ROUNDS];
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
        if (q > 0) __syncthreads();  // the reads of the round before are done
        if (wave < row_waves) {
            float4* dst = reinterpret_cast<float4*>(&red[wave][lane * 8]);
            dst[0] = make_float4(acc[8 * q], acc[8 * q + 1], acc[8 * q + 2], acc[8 * q + 3]);
            dst[1] = make_float4(acc[8 * q + 4], acc[8 * q + 5], acc[8 * q + 6], acc[8 * q + 7]);
        }
        __syncthreads();
        float s = red[0][tid];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w)
            if (w < row_waves) s += red[w][tid];  // wave-uniform
        if constexpr (BITS != 16) s *= h2f(sraw[q]);
        val[q] = s;
    }

    const bool coherent = fa.counters != nullptr;
    if (owns) {
        float* out = cpart + (size_t)t.rs * Ntot + jobs.col0[t.m] + ocol;
#pragma unroll
        for (int q = 0; q < ROUNDS; ++q) store_partial(out + 8 * q, val[q], coherent);
    }
    if (!coherent) return;

    // In-kernel accumulation: once every store of the workgroup has been performed, count the workgroup in
    // on the tiles of its segment; the wavefronts then share the tiles it has completed.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int tile0 = t.wc * CPL;                      // first 64-column tile of the segment inside matrix m
    const int ntiles = min(CPL, N / 64 - tile0);       // CPL <= 64 tiles per segment
    if (tid < ntiles) tile_done[tid] = tile_arrive(fa, t.m, tile0 + tid) ? 1u : 0u;
    __syncthreads();
    for (int j = wave; j < ntiles; j += kWavesPerBlock)
        if (tile_done[j]) finalize_tile(fa, t.m, tile0 + j, lane);
}

// Columns one workgroup covers (one 16-byte piece per lane and row), by residual format (decdec_rfmt).
__host__ __device__ constexpr int fetch_cols_per_wave(int rfmt) {
    return rfmt == 0 ? 512 : rfmt == 1 ? 2048 : rfmt == 2 ? 4096 : 1024;
}

// Host: kernel-side description of the matrices of one call.
inline FetchJobs make_fetch_jobs(int rfmt, const MultiShape& sh, const FetchOperands& op) {
    FetchJobs jobs{};
    jobs.n = sh.n;
    const int cpw = fetch_cols_per_wave(rfmt);
    int wc = 0;
    for (int m = 0; m < sh.n; ++m) {
        jobs.R[m] = static_cast<const uint4*>(op.R[m]);
        jobs.Rs[m] = static_cast<const uint16_t*>(op.R_scales[m]);
        jobs.N[m] = sh.N[m];
        jobs.col0[m] = sh.col0[m];
        wc += (sh.N[m] + cpw - 1) / cpw;
        jobs.wc_end[m] = wc;
    }
    return jobs;
}

}  // namespace decdec
