// Workgroup-level exact top-k of |x| (DecDEC Section 4.1 step 1 with the exact
// Top-K of Section 5.2; a tie at the cut goes to the lower index).  Used by the
// stand-alone selection kernel and by kernels that select for themselves.
//
// Radix select, nothing is sorted, x is read once and stays in registers:
//   * wavefront w owns the 64*NCH consecutive 8-key chunks starting at
//     w*64*NCH; lane l holds chunk w*64*NCH + j*64 + l for j = 0..NCH-1 (one
//     coalesced 128-bit load per j), so inside a wavefront the channel order
//     is (j, lane, position in the chunk) and wavefronts follow one another;
//   * the order of |x| is the order of the 15-bit key (fp16 bits, sign
//     cleared); an LDS histogram over the high 8 key bits finds the bin
//     holding the k-th largest key (kHistCopies copies picked by lane would
//     spread atomics that collide on few bins; measured, one copy is fastest); a
//     second histogram over the low 7 bits of the keys in that bin finds the
//     key T itself and how many keys equal to T are still needed.  Every
//     wavefront scans the histograms for itself (DPP prefix sum + readlane),
//     which saves the barriers a single scanning wavefront would need;
//   * per round j every thread counts its keys > T and == T; a wave prefix
//     sum per round, the round totals (readlane) and per-wave totals in LDS
//     give each thread the number of such keys at lower indices, hence each
//     selected element its output position: keys > T all go out, keys == T
//     only the first `need` in index order.  Only marked keys are visited when
//     writing.  Output is in ascending index order.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace decdec {

constexpr int kSelectMaxChunks = 8;  // 8-key chunks per thread at most
constexpr int kHistCopies = 1;

struct SelectShared {
    unsigned hist1[kHistCopies][256];
    unsigned hist2[128];
    unsigned wtot[16];  // per wave: (keys > T) | (keys == T) << 16
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

// Run by all 64 lanes of a wavefront.  hist holds COPIES histograms of
// NB = 64*PER bins in ascending key order whose sum has at least kk >= 1 keys.
// Finds the bin b with fewer than kk keys in the bins above it and at least kk
// in the bins >= b; returns b and kk - (#keys above b) in every lane.
template <int PER, int COPIES>
__device__ __forceinline__ void wave_find_bin(const unsigned* hist, unsigned kk, unsigned& bin, unsigned& rem,
                                              int lane) {
    constexpr int NB = 64 * PER;
    unsigned c[PER], tot = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int b = NB - 1 - (lane * PER + j);  // descending key order
        c[j] = 0;
#pragma unroll
        for (int r = 0; r < COPIES; ++r) c[j] += hist[r * NB + b];
        tot += c[j];
    }
    unsigned above = wave_incl_scan(tot) - tot;  // keys in bins above this lane's bins
    unsigned b_l = 0, r_l = 1;
    bool found = false;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (above < kk && kk <= above + c[j]) {
            b_l = (unsigned)(NB - 1 - (lane * PER + j));
            r_l = kk - above;
            found = true;
        }
        above += c[j];
    }
    const unsigned long long mask = __ballot(found);  // exactly one lane unless the histogram is short of kk keys
    const int src = mask ? __builtin_ctzll(mask) : 0;
    bin = (unsigned)__builtin_amdgcn_readlane((int)b_l, src);
    rem = (unsigned)__builtin_amdgcn_readlane((int)r_l, src);
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
    const int c0 = wave * 64 * NCH + lane;  // this thread's chunk of round j is c0 + 64*j
    const uint4* x128 = reinterpret_cast<const uint4*>(x);

    uint4 ch[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) ch[j] = c0 + 64 * j < nchunks ? x128[c0 + 64 * j] : make_uint4(0, 0, 0, 0);
    for (int i = tid; i < kHistCopies * 256; i += THREADS) (&sh.hist1[0][0])[i] = 0;
    for (int i = tid; i < 128; i += THREADS) sh.hist2[i] = 0;
    __syncthreads();

    // pass 1: high 8 bits of the key
    unsigned* h1 = sh.hist1[lane & (kHistCopies - 1)];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        if (c0 + 64 * j < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) atomicAdd(&h1[key_of(ch[j], e) >> 7], 1u);
        }
    }
    __syncthreads();
    unsigned b1, rem1;
    wave_find_bin<4, kHistCopies>(&sh.hist1[0][0], (unsigned)k, b1, rem1, lane);

    // pass 2: low 7 bits of the keys inside bin b1
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        if (c0 + 64 * j < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned key = key_of(ch[j], e);
                if ((key >> 7) == b1) atomicAdd(&sh.hist2[key & 127u], 1u);
            }
        }
    }
    __syncthreads();
    unsigned b2, need;  // need: keys equal to T still to take (>= 1)
    wave_find_bin<2, 1>(sh.hist2, rem1, b2, need, lane);
    const unsigned T = (b1 << 7) | b2;

    // compaction in index order.  Per round: bit e of gtm[j] / eqm[j] = key e of the chunk is > T / == T;
    // counts are packed as (> T) | (== T) << 16 (at most 4096 each per wavefront: no carry between the halves).
    unsigned gtm[NCH], eqm[NCH], excl[NCH];  // excl: this wave's marked keys at lower indices (earlier rounds, lower lanes)
    unsigned wave_cnt = 0;                    // uniform: marked keys of the rounds so far
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        unsigned g = 0, q = 0;
        if (c0 + 64 * j < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned key = key_of(ch[j], e);
                g |= (unsigned)(key > T) << e;
                q |= (unsigned)(key == T) << e;
            }
        }
        gtm[j] = g;
        eqm[j] = q;
        const unsigned cnt = (unsigned)__builtin_popcount(g) | ((unsigned)__builtin_popcount(q) << 16);
        const unsigned incl = wave_incl_scan(cnt);
        excl[j] = wave_cnt + incl - cnt;
        wave_cnt += (unsigned)__builtin_amdgcn_readlane((int)incl, 63);
    }
    if (lane == 0) sh.wtot[wave] = wave_cnt;
    __syncthreads();
    unsigned base_gt = 0, base_eq = 0;  // marked keys of the wavefronts before this one
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) {
        const unsigned t = sh.wtot[w];
        base_gt += w < wave ? (t & 0xFFFFu) : 0u;
        base_eq += w < wave ? (t >> 16) : 0u;
    }
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        unsigned m = gtm[j] | eqm[j];
        if (m == 0) continue;  // most threads: a chunk holds 8 keys, of which k/K are selected
        unsigned pos_gt = base_gt + (excl[j] & 0xFFFFu), seen_eq = base_eq + (excl[j] >> 16);
        while (m) {
            const int e = __builtin_ctz(m);
            m &= m - 1;
            const bool is_gt = (gtm[j] >> e) & 1u;
            const unsigned pos = pos_gt + min(seen_eq, need);
            // pos < k always holds for a taken key; the bound keeps a logic error from writing outside
            if ((is_gt || seen_eq < need) && pos < (unsigned)k) {
                idx_out[pos] = (c0 + 64 * j) * 8 + e;
                if (xsel_out) xsel_out[pos] = raw_of(ch[j], e);
            }
            pos_gt += is_gt;
            seen_eq += !is_gt;
        }
    }
}

}  // namespace decdec
