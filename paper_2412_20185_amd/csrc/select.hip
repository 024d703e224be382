// Step 1 of dynamic error compensation (DecDEC Section 4.1): sc_indices, the k
// input channels with the largest |x|, and x[sc_indices].
//
// The paper's kernel uses an approximate, chunked bucket Top-K (Section 4.3);
// this is the exact Top-K it uses as its quality reference (Section 5.2),
// with a tie at the cut going to the lower index, done as a radix select so
// that nothing is sorted:
//   * one workgroup of 1024 threads copies x (at most 128 KiB) into LDS once;
//   * the order of |x| is the order of the 15-bit key (fp16 bits with the sign
//     cleared); an LDS histogram over the high 8 key bits finds the bin that
//     holds the k-th largest key, a second one over the low 7 bits of the keys
//     in that bin finds the key T itself and how many keys equal to T are
//     still needed;
//   * every thread then owns a contiguous index range, counts its keys > T
//     and == T, two workgroup prefix sums give each selected element its
//     output position: keys > T all go out, keys == T only the first `need`
//     in index order.  The output is in ascending index order.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace decdec {
namespace {

constexpr int kWaves = kSelectThreads / 64;

// Inclusive prefix sum of v over the 1024 threads of the workgroup.
__device__ __forceinline__ unsigned block_incl_scan(unsigned v, unsigned* wtot, int lane, int wave) {
    unsigned incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    unsigned base = 0;
    for (int w = 0; w < wave; ++w) base += wtot[w];
    __syncthreads();
    return incl + base;
}

// hist has NB bins in ascending key order and holds at least kk keys in
// total (kk >= 1).  Finds the bin b such that fewer than kk keys lie in bins
// above b and at least kk in bins >= b; stores b and kk - (#keys above b).
template <int NB>
__device__ __forceinline__ void find_bin(const unsigned* hist, unsigned kk, unsigned* wtot, unsigned* out_bin,
                                         unsigned* out_rem, int tid, int lane, int wave) {
    const unsigned c = tid < NB ? hist[NB - 1 - tid] : 0u;
    const unsigned incl = block_incl_scan(c, wtot, lane, wave);
    const unsigned above = incl - c;
    if (tid < NB && above < kk && kk <= incl) {
        *out_bin = (unsigned)(NB - 1 - tid);
        *out_rem = kk - above;
    }
    __syncthreads();
}

__global__ __launch_bounds__(kSelectThreads) void select_topk_kernel(const uint16_t* __restrict__ x, int K, int k,
                                                                    int32_t* __restrict__ idx_out,
                                                                    uint16_t* __restrict__ xsel_out) {
    extern __shared__ uint4 s_raw[];  // K fp16 values
    __shared__ unsigned hist[256];
    __shared__ unsigned wtot[kWaves];
    __shared__ unsigned s_bin[2], s_rem[2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint16_t* sx = reinterpret_cast<const uint16_t*>(s_raw);
    const uint32_t* sx32 = reinterpret_cast<const uint32_t*>(s_raw);

    const uint4* x128 = reinterpret_cast<const uint4*>(x);
    for (int i = tid; i < K / 8; i += kSelectThreads) s_raw[i] = x128[i];
    if (tid < 256) hist[tid] = 0;
    if (tid < 2) {
        s_bin[tid] = 0;
        s_rem[tid] = 1;
    }
    __syncthreads();

    // pass 1: high 8 bits of the key
    for (int i = tid; i < K / 2; i += kSelectThreads) {
        const uint32_t w = sx32[i];
        atomicAdd(&hist[(w & 0x7FFFu) >> 7], 1u);
        atomicAdd(&hist[(w >> 23) & 0xFFu], 1u);
    }
    __syncthreads();
    find_bin<256>(hist, (unsigned)k, wtot, &s_bin[0], &s_rem[0], tid, lane, wave);
    const unsigned b1 = s_bin[0], k1 = s_rem[0];

    // pass 2: low 7 bits of the keys inside bin b1
    if (tid < 128) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < K / 2; i += kSelectThreads) {
        const uint32_t w = sx32[i];
        const uint32_t k0 = w & 0x7FFFu, k1v = (w >> 16) & 0x7FFFu;
        if ((k0 >> 7) == b1) atomicAdd(&hist[k0 & 127u], 1u);
        if ((k1v >> 7) == b1) atomicAdd(&hist[k1v & 127u], 1u);
    }
    __syncthreads();
    find_bin<128>(hist, k1, wtot, &s_bin[1], &s_rem[1], tid, lane, wave);
    const unsigned T = (b1 << 7) | s_bin[1];
    const unsigned need = s_rem[1];  // keys equal to T still to take (>= 1)

    // compaction in index order
    const int C = (K + kSelectThreads - 1) / kSelectThreads;
    const int i0 = min(tid * C, K), i1 = min(i0 + C, K);
    unsigned n_gt = 0, n_eq = 0;
    for (int i = i0; i < i1; ++i) {
        const unsigned key = sx[i] & 0x7FFFu;
        n_gt += key > T;
        n_eq += key == T;
    }
    unsigned pos_gt = block_incl_scan(n_gt, wtot, lane, wave) - n_gt;
    unsigned seen_eq = block_incl_scan(n_eq, wtot, lane, wave) - n_eq;
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
}

}  // namespace

hipError_t launch_select_topk(const void* x, int K, int k, int32_t* idx_out, void* xsel_out, hipStream_t stream) {
    const size_t lds = (size_t)K * 2;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(select_topk_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kSelectMaxK * 2);
    if (attr != hipSuccess) return attr;
    select_topk_kernel<<<dim3(1), dim3(kSelectThreads), lds, stream>>>(
        static_cast<const uint16_t*>(x), K, k, idx_out, static_cast<uint16_t*>(xsel_out));
    return hipGetLastError();
}

}  // namespace decdec
