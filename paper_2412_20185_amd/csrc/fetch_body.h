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
// in LDS and the workgroup contributes ONE fp32 part sum per column of the segment.
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

constexpr int kFetchSegmentCols = 512;  // output columns of one column segment = threads of a workgroup

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

// What one lane loads of one row: 8 columns (16 of 2-bit codes), BITS bits each; never less than 4 bytes.
template <int BITS>
struct RowPiece;
template <>
struct RowPiece<16> {
    typedef uint4 type;
};
template <>
struct RowPiece<8> {
    typedef uint2 type;
};
template <>
struct RowPiece<4> {
    typedef uint32_t type;
};
template <>
struct RowPiece<2> {
    typedef uint32_t type;
};

// acc[i] += value of column i of the piece * xs.
template <int BITS, int CPL>
__device__ __forceinline__ void accumulate_piece(const typename RowPiece<BITS>::type& v, float xs, float (&acc)[CPL]) {
    if constexpr (BITS == 16) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            acc[2 * c] = fmaf(h2f(w[c] & 0xFFFFu), xs, acc[2 * c]);
            acc[2 * c + 1] = fmaf(h2f(w[c] >> 16), xs, acc[2 * c + 1]);
        }
    } else if constexpr (BITS == 8) {
        const uint32_t w[2] = {v.x, v.y};
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = fmaf((float)((int)(w[i >> 2] << (24 - 8 * (i & 3))) >> 24), xs, acc[i]);
    } else {
        const uint32_t w = v;  // CPL two's-complement fields of BITS bits
#pragma unroll
        for (int i = 0; i < CPL; ++i)
            acc[i] = fmaf((float)((int)(w << (32 - BITS * (i + 1))) >> (32 - BITS)), xs, acc[i]);
    }
}

// One workgroup = one column segment of 512 columns x the rows of row slice rs.  A lane reads 8 columns of a
// row (16, 8 or 4 bytes for fp16, 8-bit and 4-bit rows: a wavefront 1 KiB down to 256 bytes of contiguous
// row) or 16 columns of a 2-bit row (4 bytes; the two halves of a wavefront then take different rows).
// Wavefront w < row_waves takes a contiguous share of the workgroup's rows and keeps 4 KiB of row loads in
// flight in every format.  BITS = 16: fp16 rows.  BITS = 2, 4, 8: integer residuals (Section 4.2: 4-bit
// symmetric with one scale per output column; 2- and 8-bit are the variants of the paper's bit-width study,
// Table 2),  o_dec[n] = S[n] * sum_j q[s_j][n] x[s_j].
//
// After the row loop the sums of the wavefronts (and half-wavefronts) are added through LDS in a fixed
// order: thread t of the workgroup ends up with the segment's sum for column t and adds it into the
// column's accumulator (finalize.h), or, when a separate kernel does the adding, writes it to row rs of cpart.
template <int BITS, int SELECT_NCH>
__device__ __forceinline__ void fetch_block(const FetchJobs& jobs, const FinalizeArgs& fa,
                                            const uint16_t* __restrict__ x, int32_t* idx_g, uint16_t* xsel_g, int k,
                                            int K, int Ntot, float* __restrict__ cpart, int segments, int slices,
                                            int row_waves, int bid) {
    typedef typename RowPiece<BITS>::type piece_t;
    constexpr int CPL = BITS == 2 ? 16 : 8;             // columns per lane
    constexpr int LPR = kFetchSegmentCols / CPL;        // lanes that cover the segment's part of one row
    constexpr int SUB = 64 / LPR;                       // rows a wavefront loads with one instruction
    constexpr int UNROLL = (4096 / 64) / (int)sizeof(piece_t);  // loads in flight per lane: 4 KiB per wavefront
    static_assert(kBlockThreads == kFetchSegmentCols, "one thread per column of the segment");
    __shared__ float red[kWavesPerBlock * SUB][kFetchSegmentCols];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const Selection sel = obtain_selection<SELECT_NCH>(x, K, k, idx_g, xsel_g, bid);
    const int32_t* idx = sel.idx;
    const uint16_t* xsel = sel.xsel;
    const BlockTask t = block_task(jobs, segments, bid);
    const int N = jobs.N[t.m];
    const piece_t* __restrict__ R = reinterpret_cast<const piece_t*>(jobs.R[t.m]);
    const int sub = lane / LPR;                       // which of the SUB rows of a load instruction
    const int piece = t.wc * LPR + (lane % LPR);      // this lane's CPL columns of a row
    const bool active = piece * CPL < N;
    const size_t row_pieces = (size_t)(N / CPL);
    // rows of this wavefront: slice (rs, wave) out of slices * row_waves equal shares of the k selected rows
    const int rows_per = (k + slices * row_waves - 1) / (slices * row_waves);
    const int j0 = min((t.rs * row_waves + wave) * rows_per, k);
    const int j1 = wave < row_waves ? min(j0 + rows_per, k) : j0;

    const int ocol = t.wc * kFetchSegmentCols + tid;  // the column this thread owns after the LDS round
    const bool owns = ocol < N;
    // The column scale is requested before the rows, so that it arrives behind the first row loads instead
    // of costing a round trip of its own after the last one.
    uint16_t sraw = 0;
    if constexpr (BITS != 16) {
        if (owns) sraw = jobs.Rs[t.m][ocol];
    }

    float acc[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) acc[i] = 0.f;
    for (int j = j0; j < j1; j += UNROLL * SUB) {
        piece_t v[UNROLL];
        float xs[UNROLL];
        int row[UNROLL];
        uint32_t xraw[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {  // indices and activations first, so that no row load waits for them
            const int jj = min(j + u * SUB + sub, j1 - 1);
            row[u] = idx[jj];
            xraw[u] = xsel[jj];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            v[u] = piece_t{};
            if (j + u * SUB + sub < j1 && active && (unsigned)row[u] < (unsigned)K)
                v[u] = R[(size_t)row[u] * row_pieces + piece];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            xs[u] = (j + u * SUB + sub < j1 && (unsigned)row[u] < (unsigned)K) ? h2f(xraw[u]) : 0.f;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (j + u * SUB < j1) accumulate_piece<BITS, CPL>(v[u], xs[u], acc);  // wave-uniform: rows it does not have cost nothing
    }

    // Sum over the wavefronts (and their halves) of the workgroup.
    if (wave < row_waves) {
        float4* dst = reinterpret_cast<float4*>(&red[wave * SUB + sub][(lane % LPR) * CPL]);
#pragma unroll
        for (int i = 0; i < CPL / 4; ++i) dst[i] = make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
    }
    __syncthreads();
    float val = red[0][tid];
#pragma unroll
    for (int w = 1; w < kWavesPerBlock * SUB; ++w)
        if (w < row_waves * SUB) val += red[w][tid];  // wave-uniform
    if constexpr (BITS != 16) val *= h2f(sraw);

    if (owns) {
        if (fa.acc != nullptr) {
            arrive(fa, t.m, ocol, val);
        } else {
            cpart[(size_t)t.rs * Ntot + jobs.col0[t.m] + ocol] = val;
        }
    }
}

// Host: kernel-side description of the matrices of one call.
inline FetchJobs make_fetch_jobs(const MultiShape& sh, const FetchOperands& op) {
    FetchJobs jobs{};
    jobs.n = sh.n;
    const int cpw = kFetchSegmentCols;
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
