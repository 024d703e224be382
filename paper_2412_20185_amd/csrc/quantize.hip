// Offline preparation on the device: uniform min/max group-128 quantiser that
// writes the packed codes (layout.h), the fp16 scales and zero points, and the
// fp16 residual R = W - W_hat that DecDEC keeps in CPU memory (Section 3.1).
// The paper takes its base quantisers from third-party work (Section 5.2) and
// prints no formula; the formula is stated in decdec.h.  Every decision is one
// IEEE fp32 operation (correctly rounded divide, no fusion that changes a
// result), so the codes are reproducible bit for bit on a CPU.
//
// One wavefront handles one tile (128 input channels x 64 columns), one lane
// per column: rows of W are read 256 B per wave-load, the column's 128 values
// stay in registers, and the lane packs its own words of the tile.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "layout.h"

namespace decdec {
namespace {

template <int KIND, int BITS>
__global__ __launch_bounds__(256) void quantize_uniform_kernel(const float* __restrict__ W, uint32_t* __restrict__ Wq,
                                                              _Float16* __restrict__ scales,
                                                              _Float16* __restrict__ zeros, _Float16* __restrict__ R,
                                                              int N, int G, int tiles) {
    const int lane = threadIdx.x & 63;
    const int tile_id = blockIdx.x * 4 + (threadIdx.x >> 6);  // = nt * G + g
    if (tile_id >= tiles) return;
    const int nt = tile_id / G, g = tile_id - nt * G;
    const int n = nt * kTileCols + lane;
    const float* src = W + (size_t)g * kGroup * N + n;

    float w[kGroup];
#pragma unroll
    for (int i = 0; i < kGroup; ++i) w[i] = src[(size_t)i * N];
    float lo = w[0], hi = w[0];
#pragma unroll
    for (int i = 1; i < kGroup; ++i) {
        lo = fminf(lo, w[i]);
        hi = fmaxf(hi, w[i]);
    }
    constexpr float qmax = (float)((1 << BITS) - 1);
    _Float16 s16 = (_Float16)((hi - lo) / qmax);
    if (s16 == (_Float16)0.f) s16 = (_Float16)1.f;
    const float s = (float)s16;
    const float z = fminf(fmaxf(rintf(-lo / s), 0.f), qmax) + 0.f;  // + 0: a zero point is never -0

    uint32_t words[words_per_lane(KIND)];
#pragma unroll
    for (int i = 0; i < words_per_lane(KIND); ++i) words[i] = 0u;
#pragma unroll
    for (int i = 0; i < kGroup; ++i) {
        const float qf = fminf(fmaxf(rintf(w[i] / s) + z, 0.f), qmax);
        const uint32_t q = (uint32_t)qf;
        constexpr int kind = KIND;
        const CodeSlot slot = code_slot(kind, i);
#pragma unroll
        for (int r = 0; r < slot.nruns; ++r) {
            const BitRun br = slot.run[r];
            words[br.word] |= ((q >> br.code_bit) & ((1u << br.nbits) - 1u)) << br.bit;
        }
        if (R != nullptr) {
            R[((size_t)g * kGroup + i) * N + n] = (_Float16)(w[i] - s * (qf - z));
        }
    }
    uint32_t* tile = Wq + (size_t)tile_id * (tile_bytes(KIND) / 4);
#pragma unroll
    for (int p = 0; p < words_per_lane(KIND) / 4; ++p) {
        uint4 v = make_uint4(words[4 * p], words[4 * p + 1], words[4 * p + 2], words[4 * p + 3]);
        reinterpret_cast<uint4*>(tile)[p * kTileCols + lane] = v;
    }
    scales[(size_t)g * N + n] = s16;
    zeros[(size_t)g * N + n] = (_Float16)z;
}

}  // namespace

hipError_t launch_quantize_uniform(int bits, const float* W, void* Wq, void* scales, void* zeros, void* R, int K,
                                   int N, hipStream_t stream) {
    const int G = K / kGroup, tiles = (N / kTileCols) * G;
    const dim3 grid((unsigned)((tiles + 3) / 4)), block(256);
    if (bits == 4) {
        quantize_uniform_kernel<PACK_U4, 4><<<grid, block, 0, stream>>>(
            W, static_cast<uint32_t*>(Wq), static_cast<_Float16*>(scales), static_cast<_Float16*>(zeros),
            static_cast<_Float16*>(R), N, G, tiles);
    } else if (bits == 3) {
        quantize_uniform_kernel<PACK_U3, 3><<<grid, block, 0, stream>>>(
            W, static_cast<uint32_t*>(Wq), static_cast<_Float16*>(scales), static_cast<_Float16*>(zeros),
            static_cast<_Float16*>(R), N, G, tiles);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace decdec
