// Geometry and number coding of the block-scaled matrix-core layout (MX_LAYOUT_MATRIX).
//
// gfx950 has MFMA instructions that take, per lane, 32 consecutive K elements of one row in an
// 8/6/4-bit float code plus one power-of-two scale per lane (an E8M0 byte), i.e. a hardware form
// of "one shared exponent per 32-element block" (the MX idea of Section 2 of the paper).  MXInt
// mantissas are integers, so they are carried in the 6-bit E2M3 code, which holds every multiple
// of 1/2 up to 7.5 exactly: a mantissa piece v with |v| <= 15 is stored as v/2.  A mantissa of up
// to 4 stored bits is one piece; a wider one (|q| <= 128) is split as q = 16*h + l with
// l in [-8, 7] and h in [-8, 8], two pieces whose scales differ by 2^4.  Products of pieces and
// their sums inside one 32-element block are small integers over 4 and exact in the instruction's
// arithmetic; the block's scaled value is added into the fp32 accumulator.
//
// Layout of one operand (rows x K, blocks of 32 or 64 along K), pieces P = 1 or 2:
//   fragment (row tile rt of 32 rows, K step ks of 64 elements, piece p): lane 32*h + i holds
//     row 32*rt + i, elements 64*ks + 32*h + e (e = 0..31) as 6-bit codes at bits [6e, 6e+6) of six
//     dwords.
//   unit = two fragments F0, F1 stored as four planes, 3072 bytes:
//     [F0 dwords 0..3: 64 lanes x 16 B][F1 dwords 0..3: 64 x 16 B][F0 dwords 4,5: 64 x 8 B][F1 dwords 4,5: 64 x 8 B]
//     so that a lane fetches a fragment with one 16-byte and one 8-byte read into six consecutive
//     registers, and a linear copy of the unit into LDS is conflict-free for both reads.
//     P = 2: unit (rt, ks) = (high piece, low piece).   P = 1: unit (rt/2, ks) = (tile 2u, tile 2u+1).
//   units are stored [unit][ks] (ks padded to a multiple of 4), then the scales
//     [row tile][ks/4][lane][4 bytes]: byte j = exponent byte (rebased to bias 127) of the block that
//     holds the lane's elements at K step 4*(ks/4) + j.  The high piece uses that byte + 4.
#pragma once

#include "mx_common.h"

namespace mx {

constexpr int kUnitBytes = 3072;

struct MatGeom {
    int32_t pieces;
    int64_t row_tiles;    // even when pieces == 1
    int64_t units;
    int64_t ksteps;       // multiple of 4
    int64_t frag_bytes;
    int64_t scale_bytes;
    int64_t matrix;       // multiple of 256
};

__host__ __device__ inline int mat_pieces(int w) { return w <= 4 ? 1 : 2; }

__host__ __device__ inline MatGeom mat_geom(int64_t rows, int64_t cols, int w) {
    MatGeom g;
    g.pieces = mat_pieces(w);
    g.row_tiles = (rows + 31) / 32;
    if (g.pieces == 1) g.row_tiles = (g.row_tiles + 1) / 2 * 2;
    g.units = g.pieces == 2 ? g.row_tiles : g.row_tiles / 2;
    g.ksteps = ((cols + 63) / 64 + 3) / 4 * 4;
    g.frag_bytes = g.units * g.ksteps * kUnitBytes;
    g.scale_bytes = g.row_tiles * (g.ksteps / 4) * 256;
    g.matrix = (g.frag_bytes + g.scale_bytes + 255) / 256 * 256;
    return g;
}

// Byte offsets inside a unit of the two parts of fragment f (0 or 1) for `lane`.
__host__ __device__ inline int frag_lo(int f, int lane) { return f * 1024 + lane * 16; }
__host__ __device__ inline int frag_hi(int f, int lane) { return 2048 + f * 512 + lane * 8; }
// Byte offset of unit (u, ks).
__host__ __device__ inline int64_t mat_unit(const MatGeom& g, int64_t u, int64_t ks) {
    return (u * g.ksteps + ks) * kUnitBytes;
}

}  // namespace mx
