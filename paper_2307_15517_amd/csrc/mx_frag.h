// Device helpers shared by the kernels that read MX_LAYOUT_FRAGMENT operands: lane pieces, their
// unpacking to int8, and the exact per-block integer product on the matrix cores (Section 3.2 of the
// paper: mantissa products are summed as integers inside a block, the shared exponents come after).
#pragma once

#include "mx_common.h"

namespace mx {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

// dwords of one lane piece: four half blocks of B/2 elements, W bits each
template <int W, int B> struct Piece { static constexpr int kDw = B * W / 16; };

template <int NDW>
__device__ __forceinline__ void load_dwords(const uint8_t* p, uint32_t* out) {
    if constexpr (NDW % 4 == 0) {
#pragma unroll
        for (int d = 0; d < NDW / 4; ++d) {
            uint4 v = reinterpret_cast<const uint4*>(p)[d];
            out[4 * d] = v.x; out[4 * d + 1] = v.y; out[4 * d + 2] = v.z; out[4 * d + 3] = v.w;
        }
    } else if constexpr (NDW % 2 == 0) {
#pragma unroll
        for (int d = 0; d < NDW / 2; ++d) {
            uint2 v = reinterpret_cast<const uint2*>(p)[d];
            out[2 * d] = v.x; out[2 * d + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int d = 0; d < NDW; ++d) out[d] = reinterpret_cast<const uint32_t*>(p)[d];
    }
}

// Half-block j of a lane piece -> B/2 sign-extended int8 in B/8 dwords.  For W = 4 the bytes come
// out multiplied by 16 (kScaleLog2 = 4), which the exponent offset takes back: the nibbles of every
// group of 8 elements are stored e0 e4 e1 e5 e2 e6 e3 e7, so two masks give the bytes in element order.
template <int W, int B> struct Unpack {
    static constexpr int kScaleLog2 = (W == 4) ? 4 : 0;
    __device__ __forceinline__ static void run(const uint32_t* piece, int j, uint32_t* out) {
        constexpr int kOut = B / 8;
        if constexpr (W == 8) {
#pragma unroll
            for (int d = 0; d < kOut; ++d) out[d] = piece[j * kOut + d];
        } else if constexpr (W == 4) {
#pragma unroll
            for (int d = 0; d < kOut / 2; ++d) {
                const uint32_t x = piece[j * (kOut / 2) + d];
                out[2 * d] = (x << 4) & 0xF0F0F0F0u;
                out[2 * d + 1] = x & 0xF0F0F0F0u;
            }
        } else {
#pragma unroll
            for (int d = 0; d < kOut; ++d) {
                uint32_t o = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int bit = (j * (B / 2) + d * 4 + t) * W;
                    o |= ((uint32_t)stream_get<W>(piece, bit) & 0xFFu) << (8 * t);
                }
                out[d] = o;
            }
        }
    }
};

// Exact int32 dot products of one block: D (32x32) = A half-blocks x B half-blocks.
template <int B>
__device__ __forceinline__ v16i_t block_mfma(const uint32_t* a, const uint32_t* b) {
    v16i_t z = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (B == 16) {
        const long la = (long)(((uint64_t)a[1] << 32) | a[0]);
        const long lb = (long)(((uint64_t)b[1] << 32) | b[0]);
        return __builtin_amdgcn_mfma_i32_32x32x16_i8(la, lb, z, 0, 0, 0);
    } else {
#pragma unroll
        for (int s = 0; s < B / 32; ++s) {
            v4i_t va = {(int)a[4 * s], (int)a[4 * s + 1], (int)a[4 * s + 2], (int)a[4 * s + 3]};
            v4i_t vb = {(int)b[4 * s], (int)b[4 * s + 1], (int)b[4 * s + 2], (int)b[4 * s + 3]};
            z = __builtin_amdgcn_mfma_i32_32x32x32_i8(va, vb, z, 0, 0, 0);
        }
        return z;
    }
}

}  // namespace mx
