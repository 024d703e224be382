// The paper's fast approximate Top-K (DecDEC Section 4.3): x is cut into chunks
// of 1024 channels, every chunk contributes k_chunk channels, and inside a
// chunk magnitudes are scattered into 32 buckets whose boundaries follow from
// two calibrated values b_0 and b_15 (the only two the kernel receives, as in
// the paper):
//     b_i = b_0 - i (b_0 - b_15) / 15   (i <= 15),   b_i = b_15 (31 - i) / 16   (i >= 15);
// channels are gathered from bucket 0 (largest magnitudes) upwards, and the
// bucket that overflows gives its lowest channel indices (the paper fills it at
// random; a deterministic rule keeps the result checkable).
//
// The paper maps the 32 buckets onto the 32 lanes of a warp and one thread
// block onto several chunks.  Here one 64-lane wavefront owns one chunk: each
// lane keeps 16 magnitudes in registers, a 32-bin LDS histogram plus one wave
// prefix sum finds the overflowing bucket, and a second wave prefix sum places
// the selected channels in ascending index order.  Chunks are independent, so
// the grid is K/1024 single-wave workgroups and nothing is synchronised across
// them.  The bucket of a value is computed with the same fp32 operations as the
// reference so that the selection is reproducible bit for bit.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "select_block.h"

namespace decdec {
namespace {

__device__ __forceinline__ int bucket_of(uint32_t raw16, float b0, float b15, float w_hi, float w_lo) {
    const uint16_t mag = (uint16_t)(raw16 & 0x7FFFu);
    if (mag > 0x7C00u) return 0;  // NaN ranks above everything
    const float a = (float)__builtin_bit_cast(_Float16, mag);
    if (a >= b0) return 0;
    if (a >= b15) {
        if (!(w_hi > 0.f)) return 1;
        const float t = ceilf((b0 - a) / w_hi);
        return (int)fminf(fmaxf(t, 1.f), 15.f);
    }
    if (!(w_lo > 0.f)) return 31;
    const float t = floorf(a / w_lo);
    return 31 - (int)fminf(fmaxf(t, 0.f), 15.f);
}

__global__ __launch_bounds__(64) void select_bucket_kernel(const uint16_t* __restrict__ x, int k_chunk, float b0,
                                                          float b15, int32_t* __restrict__ idx_out,
                                                          uint16_t* __restrict__ xsel_out) {
    __shared__ unsigned hist[32];
    __shared__ unsigned s_cut[2];
    const int lane = threadIdx.x, chunk = blockIdx.x;
    const uint4* x128 = reinterpret_cast<const uint4*>(x) + (size_t)chunk * 128;
    const float w_hi = (b0 - b15) / 15.f, w_lo = b15 / 16.f;

    uint4 ch[2] = {x128[lane], x128[lane + 64]};
    if (lane < 32) hist[lane] = 0;
    if (lane < 2) s_cut[lane] = 0;
    __syncthreads();
    unsigned char bk[2][8];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int b = bucket_of(raw_of(ch[j], e), b0, b15, w_hi, w_lo);
            bk[j][e] = (unsigned char)b;
            atomicAdd(&hist[b], 1u);
        }
    }
    __syncthreads();
    // the bucket in which the running count reaches k_chunk, and how many of its channels are still needed
    const unsigned c = lane < 32 ? hist[lane] : 0u;
    const unsigned incl = wave_incl_scan(c);
    if (lane < 32 && incl - c < (unsigned)k_chunk && (unsigned)k_chunk <= incl) {
        s_cut[0] = (unsigned)lane;
        s_cut[1] = (unsigned)k_chunk - (incl - c);
    }
    __syncthreads();
    const unsigned cut = s_cut[0], need = s_cut[1];

    unsigned run_lt = 0, run_eq = 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        unsigned lt = 0, eq = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            lt += bk[j][e] < cut;
            eq += bk[j][e] == cut;
        }
        const unsigned cnt = lt | (eq << 16);
        const unsigned inc = wave_incl_scan(cnt);
        const unsigned tot = (unsigned)__builtin_amdgcn_readlane((int)inc, 63);
        unsigned pos_lt = run_lt + ((inc - cnt) & 0xFFFFu), seen_eq = run_eq + ((inc - cnt) >> 16);
        run_lt += tot & 0xFFFFu;
        run_eq += tot >> 16;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int pos = -1;
            if (bk[j][e] < cut) {
                pos = (int)(pos_lt + min(seen_eq, need));
                ++pos_lt;
            } else if (bk[j][e] == cut) {
                if (seen_eq < need) pos = (int)(pos_lt + seen_eq);
                ++seen_eq;
            }
            if (pos >= 0 && pos < k_chunk) {  // pos < k_chunk always holds; the bound guards the store
                const size_t o = (size_t)chunk * k_chunk + pos;
                idx_out[o] = chunk * 1024 + (lane + 64 * j) * 8 + e;
                if (xsel_out) xsel_out[o] = raw_of(ch[j], e);
            }
        }
    }
}

}  // namespace

hipError_t launch_select_bucket(const void* x, int K, int k_chunk, float b0, float b15, int32_t* idx_out,
                                void* xsel_out, hipStream_t stream, const KernelTimer* tm) {
    return launch_kernel(tm, select_bucket_kernel, dim3((unsigned)(K / 1024)), dim3(64), 0, stream,
                         static_cast<const uint16_t*>(x), k_chunk, b0, b15, idx_out, static_cast<uint16_t*>(xsel_out));
}

}  // namespace decdec
