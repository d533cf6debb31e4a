// Shared host/device helpers of the MXInt library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "mx.h"

namespace mx {

constexpr int kWave = 64;

// ---- format checks (host) ------------------------------------------------------------------
inline bool format_ok_quant(const mx_format& f) {
    return (f.block == 8 || f.block == 16 || f.block == 32 || f.block == 64) && f.exp_bits >= 2 && f.exp_bits <= 8 &&
           f.mant_bits >= 2 && f.mant_bits <= 8 && (f.rounding == MX_RNE || f.rounding == MX_RTZ) &&
           (f.block_rows == 1 || f.block_rows == 2);
}
inline bool format_ok_gemm(const mx_format& f) {
    return format_ok_quant(f) && (f.block == 16 || f.block == 32 || f.block == 64);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Raises a kernel's dynamic-LDS limit above the 64 KB default.  The attribute belongs to the (kernel, device) pair,
// so it is set once per device; `done` is the caller's per-kernel bit set of devices (a static of the launch
// function).  Safe from several host threads: at worst two of them set the same value.
inline bool allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return false;
    const uint64_t bit = 1ull << dev;
    if (done.load(std::memory_order_acquire) & bit) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    done.fetch_or(bit, std::memory_order_release);
    return true;
}

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

// 16 bytes of an fp32 input tensor that its kernel reads exactly once: a streaming load, so that the tensor does not
// displace what later calls read again (packed weights stay in the last-level cache from one call to the next).
// Used where it was measured to pay (the quantize+pack of the prefill path); the plain quantizers run about a tenth
// slower with it on large inputs and keep ordinary loads.
typedef float f4v_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_once4(const float* p) {
    const f4v_t t = __builtin_nontemporal_load(reinterpret_cast<const f4v_t*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

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

// Buffer loads: a lane whose byte offset lies at or beyond `bytes` gets zeros and touches no memory,
// so a load past the end needs no branch around it -- the number of loads a wave has in flight is
// then the same on every path, and the waits the compiler places stay exact (a load inside a
// conditional makes every later wait a wait for all outstanding loads).
using BufRsrc = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ BufRsrc make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
template <int NDW>
__device__ __forceinline__ void buf_load_dwords(BufRsrc r, uint32_t off, uint32_t* out) {
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u2 __attribute__((ext_vector_type(2)));
    if constexpr (NDW % 4 == 0) {
#pragma unroll
        for (int d = 0; d < NDW / 4; ++d) {
            const u4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off + 16 * d, 0, 0);
            out[4 * d] = v.x; out[4 * d + 1] = v.y; out[4 * d + 2] = v.z; out[4 * d + 3] = v.w;
        }
    } else if constexpr (NDW % 2 == 0) {
#pragma unroll
        for (int d = 0; d < NDW / 2; ++d) {
            const u2 v = __builtin_amdgcn_raw_buffer_load_b64(r, off + 8 * d, 0, 0);
            out[2 * d] = v.x; out[2 * d + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int d = 0; d < NDW; ++d) out[d] = __builtin_amdgcn_raw_buffer_load_b32(r, off + 4 * d, 0, 0);
    }
}

}  // namespace mx
