// Device code of the base GEMV (included by gemv.hip and fused.hip).
//
// Base GEMV  o_b = W_hat x  for 3/4-bit weights at batch 1 (DecDEC Section 4.1:
// the base GEMV the compensation runs beside; Section 2.2: weights are
// de-quantised on the fly and multiplied with fp16 activations).
//
// gfx950 design.  The work is a stream over the packed weights (HBM bound), so
// there is no MFMA here; what has to be kept small is the number of vector
// instructions per weight:
//   * one wavefront = 64 output columns, one lane per column, walking along K
//     one 128-channel quantisation group (= one tile, see layout.h) at a time;
//     each wave-wide 128-bit load is one contiguous 1 KiB piece of the stream;
//   * a lane never converts a code: a masked code field inside the fp16
//     mantissa is the subnormal  code * 2^(p-24), which v_dot2_f32_f16
//     multiplies with an (x[2j], x[2j+1]) pair and accumulates in fp32; fields
//     are used at two bit positions p (4 and 7), each with its own
//     accumulators, combined once per group;
//   * all lanes of a wave need the same activations, so x is read through the
//     scalar cache into SGPRs and used as the scalar operand of the dot;
//   * the zero point is factored out of the inner loop:
//     sum_k s (q_k - z) x_k = s (sum_k q_k x_k - z sum_k x_k), with the
//     group's sum of x formed once per wave by a DPP reduction;
//   * K is split over the waves of a workgroup and, where one workgroup per
//     64-column tile would leave compute units idle, over workgroups; a
//     workgroup reduces its waves through LDS and either writes y itself (one
//     K-slice, no residual term) or adds its sums into the per-column
//     accumulators with one atomic per column (finalize.h).
#pragma once
#include <hip/hip_runtime.h>

#include "finalize.h"
#include "kernels.h"
#include "layout.h"

namespace decdec {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), acc, false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}

// Sum over the 64 lanes of a wavefront, returned as a wave-uniform value.
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_move<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xF>(v);  // row_half_mirror
    v += dpp_move<0x140, 0xF>(v);  // row_mirror: every lane holds its row's sum
    v += dpp_move<0x142, 0xA>(v);  // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xC>(v);  // row_bcast31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// A field at bits p..p+b-1 of an fp16 pattern with nothing else set is the
// subnormal code * 2^(p-24).  The dot unit keeps full fp32 accuracy for such
// operands only when the field's top bit is mantissa bit 6 or above, so every
// field is moved to p = 4 or p = 7 first; accumulators are rescaled by 2^-p
// and by 2^24 once per group.
constexpr float kTwoPow24 = 16777216.f;

// sum_k q_k x_k over one group for one lane, 4-bit layout.  xs: the group's 64
// activation pairs (wave-uniform address).
__device__ __forceinline__ float group_dot_u4(const uint4 (&q)[4], const uint32_t* __restrict__ xs) {
    float a = 0.f, b = 0.f, c = 0.f, d = 0.f;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t wd[4] = {q[p].x, q[p].y, q[p].z, q[p].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int w = 4 * p + i;
            const uint32_t t = wd[i];
            a = dot2((t << 4) & 0x00F000F0u, xs[4 * w + 0], a);
            b = dot2(t & 0x00F000F0u, xs[4 * w + 1], b);
            c = dot2((t >> 4) & 0x00F000F0u, xs[4 * w + 2], c);
            d = dot2((t >> 8) & 0x00F000F0u, xs[4 * w + 3], d);
        }
    }
    return ((a + b) + (c + d)) * (kTwoPow24 / 16.f);
}

// Same for the 3-bit layout: fields at bits 0-2, 4-6, 7-9, 10-12, 13-15 of
// each half and a spare bit 3 that carries one bit of pairs 60..63.
__device__ __forceinline__ float group_dot_u3(const uint4 (&q)[3], const uint32_t* __restrict__ xs) {
    float a4 = 0.f, b4 = 0.f, c4 = 0.f, a7 = 0.f, b7 = 0.f;
    float e[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const uint32_t wd[4] = {q[p].x, q[p].y, q[p].z, q[p].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int w = 4 * p + i;
            const uint32_t t = wd[i], lo = t << 4, hi = t >> 6;
            a4 = dot2(lo & 0x00700070u, xs[5 * w + 0], a4);   // bits 0-2
            b4 = dot2(t & 0x00700070u, xs[5 * w + 1], b4);    // bits 4-6
            a7 = dot2(t & 0x03800380u, xs[5 * w + 2], a7);    // bits 7-9
            c4 = dot2(hi & 0x00700070u, xs[5 * w + 3], c4);   // bits 10-12
            b7 = dot2(hi & 0x03800380u, xs[5 * w + 4], b7);   // bits 13-15
            e[w % 3] = dot2(lo & 0x00800080u, xs[60 + w / 3], e[w % 3]);  // spare bit 3
        }
    }
    const float at7 = (a7 + b7) + ((e[0] + 2.f * e[1]) + 4.f * e[2]);
    return (((a4 + b4) + c4) * 0.0625f + at7 * 0.0078125f) * kTwoPow24;
}

// Per-lane codebook as byte tables for v_perm_b32 lookups.
struct LutTables {
    uint32_t lo03, lo47, hi03, hi47;
};

__device__ __forceinline__ LutTables make_lut_tables(uint4 l) {
    // l.x = (e0,e1)  l.y = (e2,e3)  l.z = (e4,e5)  l.w = (e6,e7) as fp16 pairs
    LutTables t;
    t.lo03 = __builtin_amdgcn_perm(l.y, l.x, 0x06040200u);
    t.hi03 = __builtin_amdgcn_perm(l.y, l.x, 0x07050301u);
    t.lo47 = __builtin_amdgcn_perm(l.w, l.z, 0x06040200u);
    t.hi47 = __builtin_amdgcn_perm(l.w, l.z, 0x07050301u);
    return t;
}

// sum_k lut[c_k] x_k over one group for one lane, LUT layout.
__device__ __forceinline__ float group_dot_lut3(const uint4 (&q)[3], const LutTables& T,
                                                const uint32_t* __restrict__ xs) {
    const uint32_t wd[12] = {q[0].x, q[0].y, q[0].z, q[0].w, q[1].x, q[1].y,
                             q[1].z, q[1].w, q[2].x, q[2].y, q[2].z, q[2].w};
    float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint32_t w0 = wd[3 * b], w1 = wd[3 * b + 1], w2 = wd[3 * b + 2];
        uint32_t sel[8];
        sel[0] = w0 & 0x07070707u;
        sel[1] = (w0 >> 3) & 0x07070707u;
        sel[2] = w1 & 0x07070707u;
        sel[3] = (w1 >> 3) & 0x07070707u;
        sel[4] = w2 & 0x07070707u;
        sel[5] = (w2 >> 3) & 0x07070707u;
        sel[6] = ((w0 >> 6) & 0x03030303u) | ((w2 >> 4) & 0x04040404u);
        sel[7] = ((w1 >> 6) & 0x03030303u) | ((w2 >> 5) & 0x04040404u);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const uint32_t lo = __builtin_amdgcn_perm(T.lo47, T.lo03, sel[s]);
            const uint32_t hi = __builtin_amdgcn_perm(T.hi47, T.hi03, sel[s]);
            const uint32_t p01 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
            const uint32_t p23 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
            acc0 = dot2(p01, xs[16 * b + 2 * s], acc0);
            acc1 = dot2(p23, xs[16 * b + 2 * s + 1], acc1);
        }
    }
    return acc0 + acc1;
}


typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// 128-bit load of data that is read exactly once (the weight stream).
__device__ __forceinline__ uint4 load_streaming(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// What one lane holds of one tile while it is in flight.
template <int KIND>
struct TileRegs {
    uint4 q[words_per_lane(KIND) / 4];
    uint16_t s, z;   // fp16 scale and zero point of (group, column)   (uniform formats)
    uint32_t xp;     // this lane's activation pair, for the group's sum of x
};

template <int KIND>
__device__ __forceinline__ void load_tile(TileRegs<KIND>& r, const uint4* __restrict__ tile,
                                          const uint16_t* __restrict__ scales,
                                          const uint16_t* __restrict__ zeros, const uint32_t* __restrict__ x32,
                                          int g, int N, int n, int lane) {
    constexpr int P = words_per_lane(KIND) / 4;
#pragma unroll
    for (int p = 0; p < P; ++p) r.q[p] = load_streaming(tile + p * kTileCols);
    if constexpr (KIND != PACK_LUT3) {
        r.s = scales[(size_t)g * N + n];
        r.z = zeros[(size_t)g * N + n];
        r.xp = x32[g * 64 + lane];
    }
}

template <int KIND>
__device__ __forceinline__ float tile_dot(const TileRegs<KIND>& r, const LutTables& T,
                                          const uint32_t* __restrict__ xs) {
    if constexpr (KIND == PACK_LUT3) {
        return group_dot_lut3(r.q, T, xs);
    } else {
        const float gs = wave_sum(dot2(r.xp, 0x3C003C00u, 0.f));  // sum of the group's 128 activations
        float d;
        if constexpr (KIND == PACK_U4) {
            d = group_dot_u4(r.q, xs);
        } else {
            d = group_dot_u3(r.q, xs);
        }
        const float s = (float)__builtin_bit_cast(_Float16, r.s);
        const float z = (float)__builtin_bit_cast(_Float16, r.z);
        return s * (d - z * gs);
    }
}

struct GemvJobs {
    const uint4* Wq[kMaxMulti];
    const uint16_t* scales[kMaxMulti];
    const uint16_t* zeros_or_lut[kMaxMulti];
    int N[kMaxMulti];
    int col0[kMaxMulti];
    int tile_end[kMaxMulti];  // cumulative count of 64-column tiles up to and including matrix m
    int n;
};

// Work of workgroup `bid` out of (total tiles) * slices workgroups of WPB wavefronts; workgroup (nt, ks)
// covers column tile nt (of whichever matrix it falls in) and groups
// [ks*WPB*gpw, (ks+1)*WPB*gpw), wave w of it the gpw groups starting at
// (ks*WPB + w)*gpw.  part is fp32 [slices][Ntot].  A wave keeps the loads of
// NBUF tiles in flight: the tile NBUF groups ahead is requested as soon as the
// registers of the current one are free.  With fa.direct (one slice, nothing
// else to add) the workgroup rounds its sums to fp16 and writes y itself.
template <int KIND, int WPB, int NBUF>
__device__ __forceinline__ void gemv_block(const GemvJobs& jobs, const FinalizeArgs& fa,
                                           const uint32_t* __restrict__ x32, float* __restrict__ part, int Ntot,
                                           int G, int slices, int gpw, int bid) {
    constexpr int P = words_per_lane(KIND) / 4;  // 16-byte pieces per lane per tile
    constexpr int kTileStride = P * kTileCols;   // uint4 per tile
    __shared__ float red[WPB][kTileCols];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gt = bid / slices;  // tile index over all matrices
    const int ks = bid - gt * slices;
    int m = 0;
#pragma unroll
    for (int i = 0; i < kMaxMulti - 1; ++i) m += (i + 1 < jobs.n && gt >= jobs.tile_end[i]) ? 1 : 0;
    const int nt = gt - (m > 0 ? jobs.tile_end[m - 1] : 0);
    const int N = jobs.N[m];
    const int n = nt * kTileCols + lane;
    const uint16_t* __restrict__ scales = jobs.scales[m];
    const uint16_t* __restrict__ zeros_or_lut = jobs.zeros_or_lut[m];

    int g = (ks * WPB + wave) * gpw;
    const int g_end = min(g + gpw, G);

    LutTables T{};
    if constexpr (KIND == PACK_LUT3) {
        T = make_lut_tables(reinterpret_cast<const uint4*>(zeros_or_lut)[n]);
    }

    float total = 0.f;
    const uint4* tile = jobs.Wq[m] + ((size_t)nt * G + g) * kTileStride + lane;
    if constexpr (NBUF == 2) {
        TileRegs<KIND> ra, rb;
        if (g < g_end) load_tile<KIND>(ra, tile, scales, zeros_or_lut, x32, g, N, n, lane);
        while (g < g_end) {
            if (g + 1 < g_end) load_tile<KIND>(rb, tile + kTileStride, scales, zeros_or_lut, x32, g + 1, N, n, lane);
            total += tile_dot<KIND>(ra, T, x32 + g * 64);
            if (++g >= g_end) break;
            tile += 2 * kTileStride;
            if (g + 1 < g_end) load_tile<KIND>(ra, tile, scales, zeros_or_lut, x32, g + 1, N, n, lane);
            total += tile_dot<KIND>(rb, T, x32 + g * 64);
            ++g;
        }
    } else {
        TileRegs<KIND> r[NBUF];
#pragma unroll
        for (int i = 0; i < NBUF; ++i)
            if (g + i < g_end)
                load_tile<KIND>(r[i], tile + i * kTileStride, scales, zeros_or_lut, x32, g + i, N, n, lane);
        while (g < g_end) {
#pragma unroll
            for (int i = 0; i < NBUF; ++i) {
                if (g + i >= g_end) break;  // wave-uniform
                total += tile_dot<KIND>(r[i], T, x32 + (g + i) * 64);
                if (g + i + NBUF < g_end)
                    load_tile<KIND>(r[i], tile + (i + NBUF) * kTileStride, scales, zeros_or_lut, x32, g + i + NBUF, N,
                                    n, lane);
            }
            g += NBUF;
            tile += NBUF * kTileStride;
        }
    }

    red[wave][lane] = total;
    __syncthreads();
    if (wave == 0) {
        // a fixed tree over the waves, so that the loads from LDS are independent of one another
        float v[WPB];
#pragma unroll
        for (int w = 0; w < WPB; ++w) v[w] = red[w][lane];
#pragma unroll
        for (int span = 1; span < WPB; span *= 2)
#pragma unroll
            for (int w = 0; w + span < WPB; w += 2 * span) v[w] += v[w + span];
        if (fa.direct) {
            fa.y[m][n] = (_Float16)v[0];
        } else if (fa.acc != nullptr) {
            arrive(fa, m, n, v[0]);
        } else {
            part[(size_t)ks * Ntot + jobs.col0[m] + n] = v[0];
        }
    }
}

}  // namespace decdec
