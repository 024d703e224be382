// Step 4 of dynamic error compensation (DecDEC Section 4.1), o = o_b + o_dec,
// folded into the kernels that produce the two terms.
//
// The paper adds o_dec into o_b with atomics from its fused kernel (Section
// 4.3 "Kernel Fusion").  So does this: every producer of a column (the base
// GEMV once per K-slice, the residual kernel once per slice of the selected
// channels) adds its fp32 part sum into one 64-bit word per output column with
// a single returning atomic.  Floating-point atomics would make the result
// depend on who came first; the word therefore holds the sum in fixed point
// (integer addition is associative, so every arrival order gives the same
// bits) and, in its low six bits, the number of producers that have arrived:
//
//     word = (sum of rint(v * 2^30)) * 64  +  arrivals
//
// The producer whose atomic returns arrivals == producers - 1 holds the whole
// sum (returned value + own term), rounds it once to fp16, writes y and stores
// zero to the word for the next call.  One memory round trip per producer, no
// partial rows, no fences (each column is a location of its own), nobody
// waits, and no extra launch.
//
// Range and resolution: a part sum is clamped to +-2^21 before conversion
// (far outside fp16's +-65504, so a clamped term can only make y infinite, or
// meet a clamped term of the other sign: inputs are assumed finite and y
// representable); up to 32 producers then stay below 2^57 in the 58-bit signed
// sum field.  The step 2^-30 is finer than the last place of an fp32 part sum
// of magnitude 2^-7 or more, and 2^-6 of fp16's smallest subnormal: the fixed
// point sum is at least as accurate as an fp32 sum in any order.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace decdec {

struct FinalizeArgs {
    _Float16* y[kMaxMulti];
    int col0[kMaxMulti];           // first concatenated column of matrix m
    unsigned long long* acc;       // one word per concatenated column, zero between calls; null: the
                                   // producers leave fp32 partial rows and a separate kernel adds them
    float* gpart;                  // [gslices][Ntot]   (acc == null only)
    float* cpart;                  // [cslices][Ntot]   (acc == null only)
    int gslices, cslices, Ntot;
    int direct;                    // 1: the base GEMV is the only producer and has one slice: it writes y itself
};

constexpr float kFixedScale = 1073741824.f;       // 2^30
constexpr float kFixedInvScale = 1.f / 1073741824.f;
constexpr float kFixedLimit = 2097152.f;          // 2^21
constexpr int kArrivalBits = 6;                   // producers per column <= 32 < 2^6
static_assert(kMaxGemvSlices + kMaxFetchSlices <= 32, "32 clamped terms of 2^51 stay below 2^57");
static_assert(kMaxGemvSlices + kMaxFetchSlices < (1 << kArrivalBits), "the arrival count must fit its field");

// fp32 part sum -> fixed point (round to nearest even; NaN takes the lower clamp, so it leaves -inf in y).
__device__ __forceinline__ long long to_fixed(float v) {
    v = fminf(fmaxf(v, -kFixedLimit), kFixedLimit);
    return (long long)rintf(v * kFixedScale);
}

// Fixed-point sum -> the fp16 result (one rounding to fp32, exact scaling, one rounding to fp16).
__device__ __forceinline__ _Float16 from_fixed(long long s) { return (_Float16)((float)s * kFixedInvScale); }

// One thread per column: add part sum v of column n of matrix m.  Called once by every one of the
// gslices + cslices producers of that column; the last one writes y[n].
__device__ __forceinline__ void arrive(const FinalizeArgs& fa, int m, int n, float v) {
    unsigned long long* word = fa.acc + fa.col0[m] + n;
    const unsigned long long term = ((unsigned long long)to_fixed(v) << kArrivalBits) + 1ull;
    const unsigned long long old = __hip_atomic_fetch_add(word, term, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((int)(old & ((1ull << kArrivalBits) - 1)) + 1 == fa.gslices + fa.cslices) {
        fa.y[m][n] = from_fixed((long long)(old + term) >> kArrivalBits);
        __hip_atomic_store(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next call
    }
}

}  // namespace decdec
