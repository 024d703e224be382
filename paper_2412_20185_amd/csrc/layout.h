// Private packed layout of the quantised weight matrix (host packer, device
// quantiser and GEMV kernels all include this file; nothing outside the
// library depends on it).
//
// The K x N code matrix is cut into tiles of 128 input channels (one
// quantisation group) x 64 output columns.  Tiles are stored column-tile
// major: tile (nt, g) starts at ((nt * K/128) + g) * tile_bytes, so one
// wavefront walking along K for its 64 columns reads one contiguous stream.
// Inside a tile lane l (= column nt*64 + l) owns `bits` 16-byte pieces; piece
// p of lane l sits at byte p*1024 + l*16, so every wave-wide 128-bit load is
// one fully coalesced 1 KiB access.  A lane's pieces, read as 32-bit words
// w = 4p + c, hold that column's 128 codes of the group.
//
// Codes are placed so that a code can be turned into an fp16 operand of
// v_dot2_f32_f16 with at most one shift and one AND: a 3- or 4-bit field that
// lies inside mantissa bits 0..9 of a 16-bit half, with every other bit
// cleared, *is* the fp16 subnormal  code * 2^(p - 24)  (p = lowest bit of the
// field).  The dot unit does not normalise subnormal inputs, it only keeps
// full fp32 accuracy when the field's top bit is mantissa bit 6 or higher, so
// every field is used at p = 4 (bits 4-6 / 4-7) or p = 7 (bits 7-9), in place
// or after one shift of the whole word.  The two halves of a word pair up
// with two consecutive activations (x[2j], x[2j+1]) = one 32-bit word of x.
// "pair" j in 0..63 below means k_local = 2j (low half) and 2j + 1 (high
// half).
//
// 4-bit (16 words/lane):  word w, nibble i in 0..3 of each half -> pair 4w + i.
// 3-bit (12 words/lane):  per half: fields f = 0..4 at bits 0-2, 4-6, 7-9,
//     10-12, 13-15 and one spare bit 3.  Field f of word w -> pair 5w + f
//     (pairs 0..59).  Pairs 60..63: pair 60 + b takes bit e of its code from
//     the spare bit of word 3b + e (e = 0,1,2).
// LUT 3-bit (12 words/lane): codes are kept byte-aligned so that they serve
//     directly as v_perm_b32 byte selectors.  Block b = 0..3 is words 3b..3b+2.
//     Byte y of word 3b+i holds code A in bits 0-2 and code B in bits 3-5.
//     Selector s = 2i (A codes) / 2i+1 (B codes), i = 0..2; selector 6 / 7 are
//     built from the left-over bits 6-7: selector 6 byte y = bits 6-7 of
//     word 3b byte y (code bits 0-1) and bit 6 of word 3b+2 byte y (code
//     bit 2); selector 7 likewise from word 3b+1 and bit 7 of word 3b+2.
//     Selector s byte y is code number 4s + y of the block; codes (0,1) of a
//     selector form pair 16b + 2s, codes (2,3) pair 16b + 2s + 1.
#pragma once
#include <cstddef>
#include <cstdint>

#if defined(__HIPCC__)
#define DD_HD __host__ __device__
#else
#define DD_HD
#endif

namespace decdec {

constexpr int kGroup = 128;    // input channels per quantisation group / tile
constexpr int kTileCols = 64;  // output columns per tile = lanes per wavefront

enum PackKind : int { PACK_U4 = 0, PACK_U3 = 1, PACK_LUT3 = 2 };

DD_HD constexpr int words_per_lane(int kind) { return kind == PACK_U4 ? 16 : 12; }
DD_HD constexpr int tile_bytes(int kind) { return words_per_lane(kind) * 4 * kTileCols; }

// Where the bits of the code for k_local (0..127) live in a lane's words.
// A code occupies up to three (word, bit) runs.
struct BitRun {
    int word, bit, nbits, code_bit;  // nbits code bits starting at code_bit stored at word:bit
};
struct CodeSlot {
    int nruns;
    BitRun run[3];
};

DD_HD constexpr CodeSlot code_slot(int kind, int k_local) {
    const int j = k_local >> 1, h = k_local & 1;
    CodeSlot s{};
    if (kind == PACK_U4) {
        s.nruns = 1;
        s.run[0] = BitRun{j >> 2, 16 * h + 4 * (j & 3), 4, 0};
    } else if (kind == PACK_U3) {
        if (j < 60) {
            const int w = j / 5, f = j % 5;
            s.nruns = 1;
            s.run[0] = BitRun{w, 16 * h + (f == 0 ? 0 : 1 + 3 * f), 3, 0};
        } else {
            const int b = j - 60;
            s.nruns = 3;
            for (int e = 0; e < 3; ++e) s.run[e] = BitRun{3 * b + e, 16 * h + 3, 1, e};
        }
    } else {  // PACK_LUT3
        const int b = j >> 4;        // block of 32 codes
        const int jj = j & 15;       // pair inside block
        const int sel = jj >> 1;     // selector 0..7
        const int y = 2 * (jj & 1) + h;  // byte inside selector
        if (sel < 6) {
            s.nruns = 1;
            s.run[0] = BitRun{3 * b + (sel >> 1), 8 * y + 3 * (sel & 1), 3, 0};
        } else {
            const int u = sel - 6;   // 0: low bits in word 3b, 1: in word 3b+1
            s.nruns = 2;
            s.run[0] = BitRun{3 * b + u, 8 * y + 6, 2, 0};
            s.run[1] = BitRun{3 * b + 2, 8 * y + 6 + u, 1, 2};
        }
    }
    return s;
}

// Byte offset of 32-bit word w of lane l inside a tile.
DD_HD constexpr size_t word_offset_in_tile(int w, int lane) {
    return (size_t)(w >> 2) * 1024 + (size_t)lane * 16 + (size_t)(w & 3) * 4;
}

}  // namespace decdec
