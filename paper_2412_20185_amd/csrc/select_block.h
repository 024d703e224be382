// Workgroup-level exact top-k of |x| (DecDEC Section 4.1 step 1 with the exact
// Top-K of Section 5.2; a tie at the cut goes to the lower index).  Used by the
// stand-alone selection kernel and by kernels that select for themselves.
//
// Radix select, nothing is sorted, x is read once and stays in registers:
//   * thread t owns the 8-key chunks t, t + THREADS, t + 2*THREADS, ... of x
//     (one 128-bit load each, at most NCH of them);
//   * the order of |x| is the order of the 15-bit key (fp16 bits, sign
//     cleared); an LDS histogram over the high 8 key bits, scanned by one
//     wavefront, finds the bin holding the k-th largest key; a second
//     histogram over the low 7 bits of the keys in that bin finds the key T
//     itself and how many keys equal to T are still needed;
//   * every thread counts, per chunk, its keys > T and == T; wave prefix sums
//     (DPP) plus per-wave totals in LDS give each chunk the number of such
//     keys at lower indices, hence each selected element its output position:
//     keys > T all go out, keys == T only the first `need` in index order.
//     Output is in ascending index order.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace decdec {

constexpr int kSelectMaxChunks = 8;  // 8-key chunks per thread at most

struct SelectShared {
    unsigned hist1[256];
    unsigned hist2[128];
    unsigned wtot[kSelectMaxChunks][16];  // per chunk round and wave: (keys > T) | (keys == T) << 16
    unsigned bin[2], rem[2];
};

template <int CTRL, int ROW_MASK, bool BOUND_CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned v) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, BOUND_CTRL);
}

// Inclusive prefix sum over the 64 lanes of a wavefront (DPP row shifts and row broadcasts).
__device__ __forceinline__ unsigned wave_incl_scan(unsigned v) {
    v += dpp_u32<0x111, 0xF, true>(v);   // row_shr:1, zero shifted in
    v += dpp_u32<0x112, 0xF, true>(v);   // row_shr:2
    v += dpp_u32<0x114, 0xF, true>(v);   // row_shr:4
    v += dpp_u32<0x118, 0xF, true>(v);   // row_shr:8 -> inclusive scan inside each row of 16
    v += dpp_u32<0x142, 0xA, false>(v);  // row_bcast15: rows 1 and 3 add the total of the row before
    v += dpp_u32<0x143, 0xC, false>(v);  // row_bcast31: rows 2 and 3 add the total of rows 0-1
    return v;
}

// Run by one wavefront.  hist holds NB = 64*PER bins in ascending key order and
// at least kk >= 1 keys in total.  Finds the bin b with fewer than kk keys in
// the bins above it and at least kk in the bins >= b; stores b and
// kk - (#keys above b).
template <int PER>
__device__ __forceinline__ void wave_find_bin(const unsigned* hist, unsigned kk, unsigned* out_bin,
                                              unsigned* out_rem, int lane) {
    constexpr int NB = 64 * PER;
    unsigned c[PER], tot = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        c[j] = hist[NB - 1 - (lane * PER + j)];  // descending key order
        tot += c[j];
    }
    unsigned above = wave_incl_scan(tot) - tot;  // keys in bins above this lane's bins
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (above < kk && kk <= above + c[j]) {
            *out_bin = (unsigned)(NB - 1 - (lane * PER + j));
            *out_rem = kk - above;
        }
        above += c[j];
    }
}

__device__ __forceinline__ unsigned key_of(const uint4& c, int e) {
    const uint32_t w = e < 2 ? c.x : e < 4 ? c.y : e < 6 ? c.z : c.w;
    return ((e & 1) ? (w >> 16) : w) & 0x7FFFu;
}
__device__ __forceinline__ uint16_t raw_of(const uint4& c, int e) {
    const uint32_t w = e < 2 ? c.x : e < 4 ? c.y : e < 6 ? c.z : c.w;
    return (uint16_t)((e & 1) ? (w >> 16) : (w & 0xFFFFu));
}

// All THREADS threads of the workgroup call this.  Requires K a multiple of 8,
// K <= 8*THREADS*NCH, x 16-byte aligned, 1 <= k <= K.  idx_out / xsel_out may
// point to global memory or LDS; xsel_out may be null.  Ends with the outputs
// written but not yet synchronised (the caller adds the barrier it needs).
template <int THREADS, int NCH>
__device__ __forceinline__ void block_select_topk(const uint16_t* __restrict__ x, int K, int k, SelectShared& sh,
                                                  int32_t* idx_out, uint16_t* xsel_out) {
    static_assert(THREADS % 64 == 0 && THREADS / 64 <= 16 && NCH <= kSelectMaxChunks, "select shape");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nchunks = K / 8;
    const uint4* x128 = reinterpret_cast<const uint4*>(x);

    uint4 ch[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int c = tid + j * THREADS;
        ch[j] = c < nchunks ? x128[c] : make_uint4(0, 0, 0, 0);
    }
    for (int i = tid; i < 256; i += THREADS) sh.hist1[i] = 0;
    for (int i = tid; i < 128; i += THREADS) sh.hist2[i] = 0;
    if (tid < 2) {
        sh.bin[tid] = 0;
        sh.rem[tid] = 1;
    }
    __syncthreads();

    // pass 1: high 8 bits of the key
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        if (tid + j * THREADS < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) atomicAdd(&sh.hist1[key_of(ch[j], e) >> 7], 1u);
        }
    }
    __syncthreads();
    if (wave == 0) wave_find_bin<4>(sh.hist1, (unsigned)k, &sh.bin[0], &sh.rem[0], lane);
    __syncthreads();
    const unsigned b1 = sh.bin[0];

    // pass 2: low 7 bits of the keys inside bin b1
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        if (tid + j * THREADS < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned key = key_of(ch[j], e);
                if ((key >> 7) == b1) atomicAdd(&sh.hist2[key & 127u], 1u);
            }
        }
    }
    __syncthreads();
    if (wave == 0) wave_find_bin<2>(sh.hist2, sh.rem[0], &sh.bin[1], &sh.rem[1], lane);
    __syncthreads();
    const unsigned T = (b1 << 7) | sh.bin[1];
    const unsigned need = sh.rem[1];  // keys equal to T still to take (>= 1)

    // compaction in index order: chunk c = tid + j*THREADS precedes c' > c
    unsigned cnt[NCH], incl[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        unsigned gt = 0, eq = 0;
        if (tid + j * THREADS < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned key = key_of(ch[j], e);
                gt += key > T;
                eq += key == T;
            }
        }
        cnt[j] = gt | (eq << 16);           // both counts <= 8 per chunk, <= 512 per wave: no carry between halves
        incl[j] = wave_incl_scan(cnt[j]);
        if (lane == 63) sh.wtot[j][wave] = incl[j];
    }
    __syncthreads();
    unsigned run_gt = 0, run_eq = 0;  // keys > T / == T in all chunks before round j
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        if (j * THREADS >= nchunks) break;
        unsigned before = incl[j] - cnt[j];
        unsigned round_tot = 0;
        for (int w = 0; w < THREADS / 64; ++w) {
            const unsigned t = sh.wtot[j][w];
            before += w < wave ? t : 0u;
            round_tot += t;
        }
        unsigned pos_gt = run_gt + (before & 0xFFFFu), seen_eq = run_eq + (before >> 16);
        run_gt += round_tot & 0xFFFFu;
        run_eq += round_tot >> 16;
        const int c = tid + j * THREADS;
        if (c < nchunks && cnt[j] != 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned key = key_of(ch[j], e);
                int pos = -1;
                if (key > T) {
                    pos = (int)(pos_gt + min(seen_eq, need));
                    ++pos_gt;
                } else if (key == T) {
                    if (seen_eq < need) pos = (int)(pos_gt + seen_eq);
                    ++seen_eq;
                }
                if (pos >= 0 && pos < k) {  // pos < k always holds; the bound keeps a logic error from writing outside
                    idx_out[pos] = c * 8 + e;
                    if (xsel_out) xsel_out[pos] = raw_of(ch[j], e);
                }
            }
        }
    }
}

}  // namespace decdec
