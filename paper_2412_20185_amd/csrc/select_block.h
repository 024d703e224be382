// Workgroup-level exact top-k of |x| (DecDEC Section 4.1 step 1 with the exact
// Top-K of Section 5.2; a tie at the cut goes to the lower index).  Used by the
// stand-alone selection kernel and by kernels that select for themselves.
//
// Radix select, nothing is sorted:
//   * x (K fp16 values) is copied into LDS once;
//   * the order of |x| is the order of the 15-bit key (fp16 bits, sign
//     cleared); an LDS histogram over the high 8 key bits, scanned by one
//     wavefront, finds the bin holding the k-th largest key; a second
//     histogram over the low 7 bits of the keys in that bin finds the key T
//     itself and how many keys equal to T are still needed;
//   * every thread owns a contiguous index range, counts its keys > T and
//     == T, and one workgroup prefix sum over both counts gives each selected
//     element its output position: keys > T all go out, keys == T only the
//     first `need` in index order.  Output is in ascending index order.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace decdec {

struct SelectShared {
    unsigned hist1[256];
    unsigned hist2[128];
    unsigned wtot_gt[16];
    unsigned wtot_eq[16];
    unsigned bin[2], rem[2];
};

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ unsigned wave_incl_scan(unsigned v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned o = __shfl_up(v, d);
        if (lane >= d) v += o;
    }
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
    unsigned above = wave_incl_scan(tot, lane) - tot;  // keys in bins above this lane's bins
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (above < kk && kk <= above + c[j]) {
            *out_bin = (unsigned)(NB - 1 - (lane * PER + j));
            *out_rem = kk - above;
        }
        above += c[j];
    }
}

// All THREADS threads of the workgroup call this.  keys: LDS, K fp16 values
// (K a multiple of 8, 16-byte aligned).  Requires 1 <= k <= K.
template <int THREADS>
__device__ __forceinline__ void block_select_topk(const uint16_t* __restrict__ x, int K, int k, uint4* keys,
                                                  SelectShared& sh, int32_t* __restrict__ idx_out,
                                                  uint16_t* __restrict__ xsel_out) {
    constexpr int WAVES = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint16_t* sx = reinterpret_cast<const uint16_t*>(keys);
    const uint32_t* sx32 = reinterpret_cast<const uint32_t*>(keys);

    const uint4* x128 = reinterpret_cast<const uint4*>(x);
    for (int i = tid; i < K / 8; i += THREADS) keys[i] = x128[i];
    for (int i = tid; i < 256; i += THREADS) sh.hist1[i] = 0;
    for (int i = tid; i < 128; i += THREADS) sh.hist2[i] = 0;
    if (tid < 2) {
        sh.bin[tid] = 0;
        sh.rem[tid] = 1;
    }
    __syncthreads();

    // pass 1: high 8 bits of the key
    for (int i = tid; i < K / 2; i += THREADS) {
        const uint32_t w = sx32[i];
        atomicAdd(&sh.hist1[(w & 0x7FFFu) >> 7], 1u);
        atomicAdd(&sh.hist1[(w >> 23) & 0xFFu], 1u);
    }
    __syncthreads();
    if (wave == 0) wave_find_bin<4>(sh.hist1, (unsigned)k, &sh.bin[0], &sh.rem[0], lane);
    __syncthreads();
    const unsigned b1 = sh.bin[0];

    // pass 2: low 7 bits of the keys inside bin b1
    for (int i = tid; i < K / 2; i += THREADS) {
        const uint32_t w = sx32[i];
        const uint32_t k0 = w & 0x7FFFu, k1 = (w >> 16) & 0x7FFFu;
        if ((k0 >> 7) == b1) atomicAdd(&sh.hist2[k0 & 127u], 1u);
        if ((k1 >> 7) == b1) atomicAdd(&sh.hist2[k1 & 127u], 1u);
    }
    __syncthreads();
    if (wave == 0) wave_find_bin<2>(sh.hist2, sh.rem[0], &sh.bin[1], &sh.rem[1], lane);
    __syncthreads();
    const unsigned T = (b1 << 7) | sh.bin[1];
    const unsigned need = sh.rem[1];  // keys equal to T still to take (>= 1)

    // compaction in index order
    const int C = (K + THREADS - 1) / THREADS;
    const int i0 = min(tid * C, K), i1 = min(i0 + C, K);
    unsigned n_gt = 0, n_eq = 0;
    for (int i = i0; i < i1; ++i) {
        const unsigned key = sx[i] & 0x7FFFu;
        n_gt += key > T;
        n_eq += key == T;
    }
    const unsigned inc_gt = wave_incl_scan(n_gt, lane), inc_eq = wave_incl_scan(n_eq, lane);
    if (lane == 63) {
        sh.wtot_gt[wave] = inc_gt;
        sh.wtot_eq[wave] = inc_eq;
    }
    __syncthreads();
    unsigned pos_gt = inc_gt - n_gt, seen_eq = inc_eq - n_eq;
    for (int w = 0; w < wave; ++w) {
        pos_gt += sh.wtot_gt[w];
        seen_eq += sh.wtot_eq[w];
    }
    for (int i = i0; i < i1; ++i) {
        const uint16_t raw = sx[i];
        const unsigned key = raw & 0x7FFFu;
        int pos = -1;
        if (key > T) {
            pos = (int)(pos_gt + min(seen_eq, need));
            ++pos_gt;
        } else if (key == T) {
            if (seen_eq < need) pos = (int)(pos_gt + seen_eq);
            ++seen_eq;
        }
        if (pos >= 0 && pos < k) {  // pos < k always holds; the bound keeps a logic error from writing outside
            idx_out[pos] = i;
            if (xsel_out) xsel_out[pos] = raw;
        }
    }
    static_assert(WAVES <= 16, "wtot arrays hold 16 wave totals");
}

}  // namespace decdec
