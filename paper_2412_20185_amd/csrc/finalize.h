// Step 4 of dynamic error compensation (DecDEC Section 4.1), o = o_b + o_dec,
// folded into the kernels that produce the two terms.
//
// The base GEMV leaves `gslices` fp32 partial rows and the residual kernel
// `cslices` (one per workgroup and column segment in both); every 64-column
// tile of the output has a counter.  A producer
// that has written its part of a tile increments the tile's counter; whichever
// producer brings the counter to gslices + cslices adds all partial rows of
// that tile in a fixed order, rounds once to fp16, writes y and resets the
// counter.  Nobody waits for anybody, the sum does not depend on who came
// last, and no extra launch is needed.  (The paper adds o_dec into o_b with
// atomics from its fused kernel, Section 4.3; this keeps the "no extra kernel"
// property without making the result depend on the order of floating-point
// atomics.)
//
// Visibility across the eight L2 caches of the chip without flushing them: a
// device-scope fence writes back and invalidates a whole L2, which costs more
// than the kernels themselves when a thousand workgroups do it.  Instead the
// partial rows are written with device-scope atomic stores (they write through
// the L2), the wave waits until those stores have completed (s_waitcnt
// vmcnt(0)) before it increments the counter with a device-scope atomic, and
// the finalizing wave reads the partial rows with device-scope atomic loads
// (they do not hit in a stale L2 line).  That is release/acquire on exactly
// these locations.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace decdec {

struct FinalizeArgs {
    _Float16* y[kMaxMulti];
    int col0[kMaxMulti];    // first concatenated column of matrix m
    int tile0[kMaxMulti];   // first tile (64 columns) of matrix m among all tiles
    const float* gpart;     // [gslices][Ntot]
    const float* cpart;     // [cslices][Ntot]
    unsigned* counters;     // one per tile, zero between calls; null: a separate kernel accumulates
    int gslices, cslices, Ntot;
    int direct;             // 1: the base GEMV is the only producer and has one slice: it writes y itself
};

// Store of a partial result that other workgroups (possibly behind another L2) will read.
__device__ __forceinline__ void store_partial(float* p, float v, bool coherent) {
    if (coherent) {
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *p = v;
    }
}

__device__ __forceinline__ float load_partial(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All 64 lanes: add the partial rows of tile nt of matrix m, write y, reset the counter.
// The summation order of accumulate_kernel: eight interleaved part sums per producer (rows p, p + 8, ...
// in ascending order), v_p = o_b,p + o_dec,p, combined as a fixed tree.  Rows are loaded eight at a
// time, all eight requests in flight together; a missing row contributes +0, which leaves a sum that
// started at +0 unchanged bit for bit.
__device__ __forceinline__ void finalize_tile(const FinalizeArgs& fa, int m, int nt, int lane) {
    const int cc = fa.col0[m] + nt * 64 + lane;
    float ob[8], odec[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) ob[p] = odec[p] = 0.f;
    for (int s0 = 0; s0 < fa.gslices; s0 += 8) {
        float t[8];
#pragma unroll
        for (int p = 0; p < 8; ++p)
            t[p] = s0 + p < fa.gslices ? load_partial(fa.gpart + (size_t)(s0 + p) * fa.Ntot + cc) : 0.f;
#pragma unroll
        for (int p = 0; p < 8; ++p) ob[p] += t[p];
    }
    for (int r0 = 0; r0 < fa.cslices; r0 += 8) {
        float t[8];
#pragma unroll
        for (int p = 0; p < 8; ++p)
            t[p] = r0 + p < fa.cslices ? load_partial(fa.cpart + (size_t)(r0 + p) * fa.Ntot + cc) : 0.f;
#pragma unroll
        for (int p = 0; p < 8; ++p) odec[p] += t[p];
    }
    float v[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) v[p] = ob[p] + odec[p];
    fa.y[m][nt * 64 + lane] = (_Float16)(((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
    if (lane == 0) fa.counters[fa.tile0[m] + nt] = 0;  // ready for the next call (stream-ordered after this one)
}

// One thread: count a producer in on tile nt of matrix m, after the partial rows it contributes to that
// tile have been performed (store_partial coherent, then s_waitcnt vmcnt(0), then - if other wavefronts of
// the workgroup stored too - a workgroup barrier).  True for the producer that completes the tile.
__device__ __forceinline__ bool tile_arrive(const FinalizeArgs& fa, int m, int nt) {
    const unsigned old =
        __hip_atomic_fetch_add(&fa.counters[fa.tile0[m] + nt], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return old + 1 == (unsigned)(fa.gslices + fa.cslices);
}

// Called by all 64 lanes of a wavefront after it has written (store_partial,
// coherent) its partial row for tile nt of matrix m: counts the wave in and
// adds the tile up if that completed it.
__device__ __forceinline__ void wave_arrive_and_finalize(const FinalizeArgs& fa, int m, int nt, int lane) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's partial row has been performed
    const bool last = lane == 0 ? tile_arrive(fa, m, nt) : false;
    if (__ballot(last)) finalize_tile(fa, m, nt, lane);
}

}  // namespace decdec
