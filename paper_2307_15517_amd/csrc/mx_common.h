// Shared host/device helpers of the MXInt library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mx.h"

namespace mx {

constexpr int kWave = 64;

// ---- format checks (host) ------------------------------------------------------------------
inline bool format_ok_quant(const mx_format& f) {
    return (f.block == 8 || f.block == 16 || f.block == 32 || f.block == 64) && f.exp_bits >= 2 && f.exp_bits <= 8 &&
           f.mant_bits >= 2 && f.mant_bits <= 8 && (f.rounding == MX_RNE || f.rounding == MX_RTZ);
}
inline bool format_ok_gemm(const mx_format& f) {
    return format_ok_quant(f) && (f.block == 16 || f.block == 32 || f.block == 64);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- fragment layout geometry (host and device) ---------------------------------------------
// Rows in groups of 32, columns in chunks of 4 blocks.  One (group, chunk) record holds
//   64 lane pieces of P = block*w/4 bytes: lane = 32*h + i carries, for each of the 4 blocks j of
//     the chunk, elements [h*block/2, (h+1)*block/2) of row i as a (block/2)*w-bit stream;
//   then 128 exponent bytes: [row i][block j].
struct FragGeom {
    int64_t groups;      // ceil(rows / 32)
    int64_t chunks;      // ceil(cols / (4*block))
    int32_t piece;       // bytes per lane per record
    int32_t record;      // bytes per (group, chunk) record
    int64_t matrix;      // bytes per matrix, a multiple of 256
};
__host__ __device__ inline FragGeom frag_geom(int64_t rows, int64_t cols, int block, int w) {
    FragGeom g;
    g.groups = (rows + 31) / 32;
    g.chunks = (cols + 4 * block - 1) / (4 * block);
    g.piece = block * w / 4;
    g.record = 64 * g.piece + 128;
    int64_t bytes = g.groups * g.chunks * (int64_t)g.record;
    g.matrix = (bytes + 255) / 256 * 256;
    return g;
}

#define MX_HIP_LAUNCH_CHECK()                                  \
    do {                                                       \
        hipError_t e__ = hipGetLastError();                    \
        if (e__ != hipSuccess) return MX_ERR_DEVICE;           \
    } while (0)

// ---- device bit helpers ------------------------------------------------------------------------
// Sign-extended w-bit field at bit offset `bit` of a little-endian stream held in dwords.
template <int W>
__device__ __forceinline__ int stream_get(const uint32_t* s, int bit) {
    const int d = bit >> 5, sh = bit & 31;
    uint32_t lo = s[d];
    uint32_t v;
    if (sh + W <= 32) {
        v = lo >> sh;
    } else {
        v = (lo >> sh) | (s[d + 1] << (32 - sh));
    }
    return ((int)(v << (32 - W))) >> (32 - W);
}

}  // namespace mx
