// Offline preparation of the residuals on the device (DecDEC Section 4.2).
//
//   residual_f32_kernel     R = W - W_hat for weights already quantised and
//                           packed (any base quantiser: the paper applies
//                           DecDEC on top of third-party quantisers, Section
//                           5.2), one fp32 subtraction per element.
//   residual_scale_kernel   per output column the scale S of the b-bit
//                           symmetric quantiser  Q(r) = clip(rint(r / S),
//                           -qmax, qmax),  qmax = 2^(b-1) - 1, found by grid
//                           search for the least squared error over
//                           S = fp16(alpha * max|r| / qmax), alpha = 0.30,
//                           0.31, ..., 1.00 (a tie keeps the larger alpha).
//   residual_encode_kernel  the codes, packed row by row for the fetch kernel.
//
// The search is written so that a CPU can reproduce it bit for bit: every
// step is one IEEE fp64 operation (no contraction into fused multiply-adds),
// the error of a column is summed over its rows in ascending order, and the
// conversion of a scale to fp16 is one round-to-nearest-even done with integer
// arithmetic.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "layout.h"

namespace decdec {
namespace {

#pragma clang fp contract(off)

template <int KIND>
__global__ __launch_bounds__(256) void residual_f32_kernel(const float* __restrict__ W,
                                                          const uint32_t* __restrict__ Wq,
                                                          const _Float16* __restrict__ scales,
                                                          const _Float16* __restrict__ zeros_or_lut,
                                                          float* __restrict__ R, int N, int G, int tiles) {
    const int lane = threadIdx.x & 63;
    const int tile_id = blockIdx.x * 4 + (threadIdx.x >> 6);  // = nt * G + g
    if (tile_id >= tiles) return;
    const int nt = tile_id / G, g = tile_id - nt * G;
    const int n = nt * kTileCols + lane;

    uint32_t words[words_per_lane(KIND)];
    const uint4* tile = reinterpret_cast<const uint4*>(Wq + (size_t)tile_id * (tile_bytes(KIND) / 4));
#pragma unroll
    for (int p = 0; p < words_per_lane(KIND) / 4; ++p) {
        const uint4 v = tile[p * kTileCols + lane];
        words[4 * p] = v.x;
        words[4 * p + 1] = v.y;
        words[4 * p + 2] = v.z;
        words[4 * p + 3] = v.w;
    }
    float s = 0.f, z = 0.f, lut[8];
    if constexpr (KIND == PACK_LUT3) {
#pragma unroll
        for (int c = 0; c < 8; ++c) lut[c] = (float)zeros_or_lut[(size_t)n * 8 + c];
    } else {
        s = (float)scales[(size_t)g * N + n];
        z = (float)zeros_or_lut[(size_t)g * N + n];
    }
#pragma unroll
    for (int i = 0; i < kGroup; ++i) {
        constexpr int kind = KIND;
        const CodeSlot slot = code_slot(kind, i);
        uint32_t q = 0;
#pragma unroll
        for (int r = 0; r < slot.nruns; ++r) {
            const BitRun br = slot.run[r];
            q |= ((words[br.word] >> br.bit) & ((1u << br.nbits) - 1u)) << br.code_bit;
        }
        float w_hat;
        if constexpr (KIND == PACK_LUT3) {
            w_hat = lut[0];
#pragma unroll
            for (int c = 1; c < 8; ++c) w_hat = q == (uint32_t)c ? lut[c] : w_hat;
        } else {
            w_hat = s * ((float)q - z);  // exact: an 11-bit scale times an integer below 16
        }
        const size_t at = ((size_t)g * kGroup + i) * N + n;
        R[at] = W[at] - w_hat;
    }
}

// fp16 bits of v >= 0 (finite), rounded to nearest even: what a correctly
// rounded conversion of the fp64 value gives.
__device__ __forceinline__ uint16_t half_bits_rne(double v) {
    if (!(v > 0.0)) return 0;
    if (v >= 65520.0) return 0x7C00;                       // rounds to infinity
    if (v < 6.103515625e-05) return (uint16_t)rint(v * 16777216.0);  // below 2^-14: multiples of 2^-24
    const int e = (int)((__double_as_longlong(v) >> 52) & 0x7FF) - 1023;  // 2^e <= v < 2^(e+1), -14 <= e <= 15
    const double scaled = v * __longlong_as_double((long long)(1023 + 10 - e) << 52);  // in [1024, 2048), exact
    const int r = (int)rint(scaled);                        // 1024 .. 2048
    return (uint16_t)(((e + 15) << 10) + (r - 1024));       // r = 2048 carries into the exponent
}

__device__ __forceinline__ double half_bits_to_double(uint16_t h) {
    return (double)(float)__builtin_bit_cast(_Float16, h);
}

constexpr int kAlphas = 71;      // 0.30 ... 1.00
constexpr int kAlphaChunk = 12;  // accumulators kept in registers per pass over the column

// One thread per output column.
__global__ __launch_bounds__(64) void residual_scale_kernel(const float* __restrict__ R, int K, int N, double qmax,
                                                           _Float16* __restrict__ scales_out) {
    const int n = blockIdx.x * 64 + threadIdx.x;
    if (n >= N) return;
    double m = 0.0;
    for (int k = 0; k < K; ++k) m = fmax(m, fabs((double)R[(size_t)k * N + n]));
    double best_err = __longlong_as_double(0x7FF0000000000000LL);  // +inf
    uint16_t best = 0x3C00;                                        // 1.0
    for (int a0 = 0; a0 < kAlphas; a0 += kAlphaChunk) {
        double S[kAlphaChunk], err[kAlphaChunk];
        uint16_t Sh[kAlphaChunk];
#pragma unroll
        for (int a = 0; a < kAlphaChunk; ++a) {
            const double alpha = (double)(30 + min(a0 + a, kAlphas - 1)) / 100.0;
            uint16_t h = half_bits_rne(alpha * m / qmax);
            if (h == 0) h = 0x3C00;  // an all-zero (or vanishing) column gets S = 1
            Sh[a] = h;
            S[a] = half_bits_to_double(h);
            err[a] = 0.0;
        }
        for (int k = 0; k < K; ++k) {
            const double r = (double)R[(size_t)k * N + n];
#pragma unroll
            for (int a = 0; a < kAlphaChunk; ++a) {
                const double q = fmin(fmax(rint(r / S[a]), -qmax), qmax);
                const double d = r - S[a] * q;
                err[a] = err[a] + d * d;
            }
        }
#pragma unroll
        for (int a = 0; a < kAlphaChunk; ++a) {
            if (a0 + a < kAlphas && err[a] <= best_err) {
                best_err = err[a];
                best = Sh[a];
            }
        }
    }
    scales_out[n] = __builtin_bit_cast(_Float16, best);
}

// One thread per 32-bit word of the packed rows: 32 / BITS columns of one row.
template <int BITS>
__global__ __launch_bounds__(256) void residual_encode_kernel(const float* __restrict__ R,
                                                             const _Float16* __restrict__ scales,
                                                             uint32_t* __restrict__ out, int K, int N) {
    constexpr int CPW = 32 / BITS;
    const double qmax = (double)((1 << (BITS - 1)) - 1);
    const int words_per_row = N / CPW;
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= (size_t)K * words_per_row) return;
    const int k = (int)(id / words_per_row), w = (int)(id - (size_t)k * words_per_row);
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int n = w * CPW + i;
        const double S = (double)(float)scales[n];
        const int q = (int)fmin(fmax(rint((double)R[(size_t)k * N + n] / S), -qmax), qmax);
        word |= ((uint32_t)q & ((1u << BITS) - 1u)) << (BITS * i);
    }
    out[id] = word;
}

}  // namespace

hipError_t launch_residual_f32(int kind, const float* W, const void* Wq, const void* scales, const void* zeros_or_lut,
                               float* R, int K, int N, hipStream_t stream) {
    const int G = K / kGroup, tiles = (N / kTileCols) * G;
    const dim3 grid((unsigned)((tiles + 3) / 4)), block(256);
    const uint32_t* q = static_cast<const uint32_t*>(Wq);
    const _Float16* s = static_cast<const _Float16*>(scales);
    const _Float16* z = static_cast<const _Float16*>(zeros_or_lut);
    switch (kind) {
        case PACK_U4: residual_f32_kernel<PACK_U4><<<grid, block, 0, stream>>>(W, q, s, z, R, N, G, tiles); break;
        case PACK_U3: residual_f32_kernel<PACK_U3><<<grid, block, 0, stream>>>(W, q, s, z, R, N, G, tiles); break;
        case PACK_LUT3: residual_f32_kernel<PACK_LUT3><<<grid, block, 0, stream>>>(W, q, s, z, R, N, G, tiles); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_quantize_residual(int bits, const float* R, void* codes_out, void* scales_out, int K, int N,
                                    hipStream_t stream) {
    if (bits != 2 && bits != 4 && bits != 8) return hipErrorInvalidValue;
    const double qmax = (double)((1 << (bits - 1)) - 1);
    _Float16* S = static_cast<_Float16*>(scales_out);
    residual_scale_kernel<<<dim3((unsigned)((N + 63) / 64)), dim3(64), 0, stream>>>(R, K, N, qmax, S);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t words = (size_t)K * (size_t)(N / (32 / bits));
    const dim3 grid((unsigned)((words + 255) / 256)), block(256);
    uint32_t* out = static_cast<uint32_t*>(codes_out);
    if (bits == 2) residual_encode_kernel<2><<<grid, block, 0, stream>>>(R, S, out, K, N);
    if (bits == 4) residual_encode_kernel<4><<<grid, block, 0, stream>>>(R, S, out, K, N);
    if (bits == 8) residual_encode_kernel<8><<<grid, block, 0, stream>>>(R, S, out, K, N);
    return hipGetLastError();
}

}  // namespace decdec
