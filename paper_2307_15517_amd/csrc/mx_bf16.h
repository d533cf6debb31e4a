// MX_LAYOUT_MATRIX for blocks of 16 elements.
//
// The block-scaled matrix instruction of gfx950 scales runs of 32 elements, so it cannot carry
// one exponent per 16.  For block 16 the shared exponent is folded into the elements instead:
// element k of a block is stored as the bfloat16 number q_k * 2^(E - bias - (w - 2)), which is
// exact (|q_k| <= 128 needs 8 significant bits, bfloat16 has 8) and keeps the full exponent range
// of the format.  The product is then a plain v_mfma_f32_32x32x16_bf16 per block pair: every
// mantissa product is exact in fp32 and the sums are taken in the instruction's fp32
// accumulation (Section 3.2 of the paper: mantissa products summed per block, the two shared
// exponents applied once per block -- here once per element, at packing time).
//
// Restriction: a nonzero element must be a normal bfloat16 number, i.e. for 8-bit exponents the
// exponent byte of a block with nonzero mantissas must lie in [w - 1, 253] (blocks quantized from
// fp32 data of magnitude >= 2^-120 always do).
//
// Layout of one operand (rows x K):
//   fragment (row tile rt of 32 rows, 16 elements): lane 32*h + i holds row 32*rt + i, elements
//     8*h .. 8*h + 7 as eight bfloat16 = 16 bytes; 64 lanes x 16 B = 1 KiB.
//   unit (rt, ks) = the two fragments of K step ks (32 elements), 2 KiB; units are stored
//     [row tile][ks] with ks padded to a multiple of 2.
//   Behind the units: the exponent bytes [row][K/16] of the logical rows (read by mx_unpack only).
#pragma once

#include "mx_common.h"

namespace mx {

constexpr int kBfUnitBytes = 2048;

struct BfGeom {
    int64_t row_tiles;
    int64_t ksteps;       // K steps of 32 elements, multiple of 2
    int64_t nblk;         // blocks per row
    int64_t frag_bytes;
    int64_t matrix;       // multiple of 256
};

__host__ __device__ inline BfGeom bf_geom(int64_t rows, int64_t cols) {
    BfGeom g;
    g.row_tiles = (rows + 31) / 32;
    g.ksteps = ((cols + 31) / 32 + 1) / 2 * 2;
    g.nblk = cols / 16;
    g.frag_bytes = g.row_tiles * g.ksteps * kBfUnitBytes;
    g.matrix = (g.frag_bytes + rows * g.nblk + 255) / 256 * 256;
    return g;
}

// Byte offset of fragment f (0 or 1) of unit (rt, ks) for `lane`.
__host__ __device__ inline int64_t bf_frag(const BfGeom& g, int64_t rt, int64_t ks, int f, int lane) {
    return (rt * g.ksteps + ks) * kBfUnitBytes + f * 1024 + lane * 16;
}

// bfloat16 bits of q * 2^s (exact when the result is a normal number or zero).
__device__ __forceinline__ uint32_t bf16_of(float q, int s) {
    return __float_as_uint(__builtin_ldexpf(q, s)) >> 16;
}

}  // namespace mx
