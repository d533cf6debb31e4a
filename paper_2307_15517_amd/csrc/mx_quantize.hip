// MXInt block quantizer and its inverse for gfx950.
//
// Format: Section 4.1 of the paper (a block shares one e-bit exponent; every element keeps a
// sign and an m-bit mantissa; w = m + 1 stored bits).  The arithmetic per block is
//   E = floor(log2 max|x|) clamped to the e-bit range, q = round(x * 2^(w-2-E)) clamped to +-qmax.
// Everything is done on the fp32 bit pattern (exponent field, v_ldexp_f32, v_rndne_f32), so the
// result does not depend on any transcendental and is bit-exact by construction.
//
// The kernels are bound by HBM traffic: 4 bytes read and w/8 + 1/block bytes written per element.
#include "mx_common.h"

namespace mx {
namespace {

// Maximum of v over aligned groups of LPB consecutive lanes (LPB in 1, 2, 4, 8), on the DPP path.
template <int LPB>
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v) {
    if constexpr (LPB >= 2) {
        uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);  // lane ^ 1
        v = v > o ? v : o;
    }
    if constexpr (LPB >= 4) {
        uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);  // lane ^ 2
        v = v > o ? v : o;
    }
    if constexpr (LPB >= 8) {
        uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);  // 7 - lane within 8
        v = v > o ? v : o;
    }
    return v;
}

// Shared exponent of a block from the bit pattern of its largest magnitude.
// Returns E (unbiased, clamped); a zero or subnormal maximum gives the lower clamp.
__device__ __forceinline__ int block_exponent(uint32_t amax_bits, int bias, int emax) {
    const int ef = (int)(amax_bits >> 23);
    int E = ef == 0 ? -127 : ef - 127;   // subnormal maxima have floor(log2) <= -127 <= any lower clamp
    E = E < -bias ? -bias : E;
    E = E > emax ? emax : E;
    return E;
}

template <int W, int RND>
__device__ __forceinline__ int quantize_one(float x, int shift) {
    constexpr float qmax = (float)((1 << (W - 1)) - 1);
    float v = __builtin_ldexpf(x, shift);
    float r = RND == MX_RNE ? __builtin_rintf(v) : __builtin_truncf(v);
    r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
    return (int)r;
}

// Eight mantissas -> 8*W bits, element i at bits [i*W, (i+1)*W).
template <int W>
__device__ __forceinline__ uint64_t pack8(const int* q) {
    uint64_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s |= (uint64_t)((uint32_t)q[i] & ((1u << W) - 1u)) << (i * W);
    return s;
}

template <int W>
__device__ __forceinline__ void store_stream(uint8_t* dst, uint64_t s) {
    // dst = base + octet*W: alignment is gcd(W, 8)-ish; pick the widest store that is always aligned
    if constexpr (W == 8) {
        *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)s, (uint32_t)(s >> 32));
    } else if constexpr (W == 4) {
        *reinterpret_cast<uint32_t*>(dst) = (uint32_t)s;
    } else if constexpr (W == 2 || W == 6) {
#pragma unroll
        for (int i = 0; i < W / 2; ++i) reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)(s >> (16 * i));
    } else {
#pragma unroll
        for (int i = 0; i < W; ++i) dst[i] = (uint8_t)(s >> (8 * i));
    }
}

template <int W>
__device__ __forceinline__ uint64_t load_stream(const uint8_t* src) {
    if constexpr (W == 8) {
        uint2 v = *reinterpret_cast<const uint2*>(src);
        return (uint64_t)v.x | ((uint64_t)v.y << 32);
    } else if constexpr (W == 4) {
        return *reinterpret_cast<const uint32_t*>(src);
    } else if constexpr (W == 2 || W == 6) {
        uint64_t s = 0;
#pragma unroll
        for (int i = 0; i < W / 2; ++i) s |= (uint64_t)reinterpret_cast<const uint16_t*>(src)[i] << (16 * i);
        return s;
    } else {
        uint64_t s = 0;
#pragma unroll
        for (int i = 0; i < W; ++i) s |= (uint64_t)src[i] << (8 * i);
        return s;
    }
}

struct QuantArgs {
    const float* x;
    uint8_t* mant;
    uint8_t* exps;
    int64_t octets;        // batch*rows*cols/8
    int64_t row_octets;    // cols/8
    int64_t rows;          // rows per batch entry
    int64_t row_stride;
    int64_t batch_stride;
    int32_t bias;
    int32_t emax;
    int32_t dense;         // x is dense and 16-byte aligned: octet o starts at x + 8*o
};

// Blocks along the contiguous axis.  One lane owns 8 consecutive elements (two 16-byte loads),
// LPB = B/8 adjacent lanes own one block.
template <int W, int B, int RND>
__global__ __launch_bounds__(256) void quantize_axis1_kernel(QuantArgs a) {
    constexpr int LPB = B / 8;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    // every lane of a wave runs the same number of iterations (the DPP reductions need whole groups)
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t wave_first = first - (threadIdx.x & 63);
    for (int64_t wo = wave_first, o = first; wo < a.octets; wo += stride, o += stride) {
        const bool live = o < a.octets;
        float v[8];
        if (live) {
            const float* src;
            if (a.dense) {
                src = a.x + o * 8;
            } else {
                const int64_t row = o / a.row_octets, c8 = o - row * a.row_octets;
                const int64_t b = row / a.rows, r = row - b * a.rows;
                src = a.x + b * a.batch_stride + r * a.row_stride + c8 * 8;
            }
            if (a.dense) {
                const float4 lo = reinterpret_cast<const float4*>(src)[0];
                const float4 hi = reinterpret_cast<const float4*>(src)[1];
                v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
                v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = src[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = 0.f;
        }
        uint32_t am = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t ab = __float_as_uint(v[i]) & 0x7fffffffu;
            am = ab > am ? ab : am;
        }
        am = group_max_u32<LPB>(am);
        const int E = block_exponent(am, a.bias, a.emax);
        const int shift = (W - 2) - E;
        int q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = quantize_one<W, RND>(v[i], shift);
        if (live) {
            store_stream<W>(a.mant + o * W, pack8<W>(q));
            if ((threadIdx.x & (LPB - 1)) == 0) a.exps[o / LPB] = (uint8_t)(E + a.bias);
        }
    }
}

// Two-row blocks (the paper's block shape (B, 2), Section 4.1): rows 2p and 2p+1 share the exponents
// of their blocks.  One lane owns the same 8 consecutive columns of both rows, LPB = B/8 adjacent
// lanes own one block; a workgroup takes 256 consecutive octets of one row pair.
struct QuantRows2Args {
    const float* x;
    uint8_t* mant;
    uint8_t* exps;
    int64_t items;         // batch * (rows/2) * (cols/8)
    int64_t row_octets;    // cols/8
    int64_t pairs;         // rows/2 per batch entry
    int64_t row_stride;
    int64_t batch_stride;
    int32_t bias;
    int32_t emax;
    int32_t vec;           // 16-byte loads are aligned
    int32_t flat;          // the batch entries follow each other at rows * row_stride
    int64_t chunks;        // workgroups per row pair: ceil(row_octets / 256)
};

// VEC: 16-byte loads.  A template parameter, not a run-time branch: with both forms in one function
// the compiler folds them into the element-wise one.
template <int W, int B, int RND, bool VEC>
__global__ __launch_bounds__(256) void quantize_rows2_kernel(QuantRows2Args a) {
    constexpr int LPB = B / 8;
    // one workgroup per (row pair, run of 256 octets): no per-item index arithmetic
    const int64_t pr = blockIdx.x / a.chunks;                       // pair index over the batch (scalar)
    const int64_t c8 = (blockIdx.x - pr * a.chunks) * 256 + threadIdx.x;
    const bool live = c8 < a.row_octets;                            // whole blocks: row_octets is a multiple of LPB
    const float* pair0;                                             // first row of the pair
    if (a.flat) {
        pair0 = a.x + 2 * pr * a.row_stride;
    } else {
        const int64_t b = pr / a.pairs, p = pr - b * a.pairs;
        pair0 = a.x + b * a.batch_stride + 2 * p * a.row_stride;
    }
    float v[2][8];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        if (live) {
            const float* src = pair0 + r * a.row_stride + c8 * 8;
            if constexpr (VEC) {
                const float4 lo = reinterpret_cast<const float4*>(src)[0];
                const float4 hi = reinterpret_cast<const float4*>(src)[1];
                v[r][0] = lo.x; v[r][1] = lo.y; v[r][2] = lo.z; v[r][3] = lo.w;
                v[r][4] = hi.x; v[r][5] = hi.y; v[r][6] = hi.z; v[r][7] = hi.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[r][i] = src[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[r][i] = 0.f;
        }
    }
    uint32_t am = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t ab = __float_as_uint(v[r][i]) & 0x7fffffffu;
            am = ab > am ? ab : am;
        }
    am = group_max_u32<LPB>(am);
    const int E = block_exponent(am, a.bias, a.emax);
    const int shift = (W - 2) - E;
    if (live) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            int q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = quantize_one<W, RND>(v[r][i], shift);
            store_stream<W>(a.mant + ((pr * 2 + r) * a.row_octets + c8) * W, pack8<W>(q));
        }
        if ((threadIdx.x & (LPB - 1)) == 0) a.exps[(pr * a.row_octets + c8) / LPB] = (uint8_t)(E + a.bias);
    }
}

struct QuantAxis0Args {
    const float* x;
    uint8_t* mant;
    uint8_t* exps;
    int64_t batch, rows, cols, row_stride, batch_stride;
    int32_t bias, emax;
    int32_t brows;             // 2: columns 2p and 2p+1 (rows 2p, 2p+1 of the transposed matrix) share exponents
};

// Blocks down the rows of each column; the output is the canonical form of the transposed
// matrix.  A workgroup takes 256 rows x 32 columns: the tile is read as row segments of 128 bytes
// and written into LDS transposed, so that a thread then finds 8 consecutive rows of one column as
// two 16-byte reads; consecutive lanes take consecutive octets of a column, i.e. the B/8 lanes of a
// block are neighbours (DPP maximum) and a half wave stores 32*W contiguous bytes of one output row.
constexpr int kAxis0Rows = 256, kAxis0Cols = 32, kAxis0Pitch = kAxis0Rows + 4;

template <int W, int B, int RND>
__global__ __launch_bounds__(256) void quantize_axis0_kernel(QuantAxis0Args a) {
    constexpr int LPB = B / 8;
    __shared__ __attribute__((aligned(16))) float tile[kAxis0Cols * kAxis0Pitch];
    const int64_t r0 = (int64_t)blockIdx.x * kAxis0Rows, c0 = (int64_t)blockIdx.y * kAxis0Cols;
    const int64_t b = blockIdx.z;
    const float* xb = a.x + b * a.batch_stride;
    const bool vec = (((uintptr_t)a.x & 15) == 0) && (a.row_stride & 3) == 0 && (a.batch_stride & 3) == 0;
    const int tc = (threadIdx.x & 7) * 4, tr = threadIdx.x >> 3;       // 8 threads cover a row segment, 32 rows per pass
    float4 v[kAxis0Rows / 32];
#pragma unroll
    for (int p = 0; p < kAxis0Rows / 32; ++p) {
        const int64_t row = r0 + p * 32 + tr, col = c0 + tc;
        v[p] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < a.rows) {
            const float* src = xb + row * a.row_stride + col;
            if (vec && col + 3 < a.cols) {
                v[p] = *reinterpret_cast<const float4*>(src);
            } else {
                if (col < a.cols) v[p].x = src[0];
                if (col + 1 < a.cols) v[p].y = src[1];
                if (col + 2 < a.cols) v[p].z = src[2];
                if (col + 3 < a.cols) v[p].w = src[3];
            }
        }
    }
#pragma unroll
    for (int p = 0; p < kAxis0Rows / 32; ++p) {
        float* dst = tile + tc * kAxis0Pitch + p * 32 + tr;
        dst[0] = v[p].x;
        dst[kAxis0Pitch] = v[p].y;
        dst[2 * kAxis0Pitch] = v[p].z;
        dst[3 * kAxis0Pitch] = v[p].w;
    }
    __syncthreads();

    const int64_t nb = a.rows / B, row_octets = a.rows / 8;
#pragma unroll
    for (int k = 0; k < kAxis0Cols * (kAxis0Rows / 8) / 256; ++k) {
        const int idx = threadIdx.x + 256 * k;
        const int cl = idx >> 5, o = idx & 31;                          // column of the tile, octet of its 256 rows
        const float4 lo = *reinterpret_cast<const float4*>(tile + cl * kAxis0Pitch + 8 * o);
        const float4 hi = *reinterpret_cast<const float4*>(tile + cl * kAxis0Pitch + 8 * o + 4);
        const float x8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        uint32_t am = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t ab = __float_as_uint(x8[i]) & 0x7fffffffu;
            am = ab > am ? ab : am;
        }
        am = group_max_u32<LPB>(am);
        if (a.brows == 2) {             // the two halves of a wave hold the same octets of columns 2p and 2p+1
            const uint32_t other = (uint32_t)__shfl_xor((int)am, 32, 64);
            am = other > am ? other : am;
        }
        const int E = block_exponent(am, a.bias, a.emax);
        const int shift = (W - 2) - E;
        int q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = quantize_one<W, RND>(x8[i], shift);
        const int64_t col = c0 + cl, row = r0 + 8 * o;                  // rows is a multiple of B: whole blocks or none
        if (col < a.cols && row < a.rows) {
            store_stream<W>(a.mant + ((b * a.cols + col) * row_octets + row / 8) * W, pack8<W>(q));
            const int rs = a.brows - 1;                                   // 0 or 1: rows per exponent as a shift
            if ((o & (LPB - 1)) == 0 && (col & rs) == 0)
                a.exps[(b * (a.cols >> rs) + (col >> rs)) * nb + row / B] = (uint8_t)(E + a.bias);
        }
    }
}

struct DequantArgs {
    const uint8_t* mant;
    const uint8_t* exps;
    float* y;
    int64_t octets;
    int64_t row_octets;    // cols/8
    int32_t bias;
    int32_t block_rows;    // 1 or 2 rows per exponent
};

template <int W, int B>
__global__ __launch_bounds__(256) void dequantize_kernel(DequantArgs a) {
    constexpr int LPB = B / 8;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < a.octets; o += stride) {
        const uint64_t s = load_stream<W>(a.mant + o * W);
        int64_t eidx = o / LPB;
        if (a.block_rows == 2) {                    // rows 2p and 2p+1 read the exponents of pair p
            const int64_t row = o / a.row_octets, c8 = o - row * a.row_octets;
            eidx = ((row >> 1) * a.row_octets + c8) / LPB;
        }
        const int sh = (int)a.exps[eidx] - a.bias - (W - 2);
        float r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int q = (int)((uint32_t)(s >> (i * W)) << (32 - W)) >> (32 - W);
            r[i] = __builtin_ldexpf((float)q, sh);
        }
        float4* dst = reinterpret_cast<float4*>(a.y + o * 8);
        dst[0] = make_float4(r[0], r[1], r[2], r[3]);
        dst[1] = make_float4(r[4], r[5], r[6], r[7]);
    }
}

inline int grid_for(int64_t items, int threads, int max_blocks) {
    int64_t g = ceil_div(items, threads);
    if (g < 1) g = 1;
    if (g > max_blocks) g = max_blocks;
    return (int)g;
}

template <int W, int B>
mx_status launch_axis1(const QuantArgs& a, int rnd, hipStream_t st) {
    // enough resident waves to cover HBM latency; each lane then walks the tensor with a grid stride
    const int grid = grid_for(a.octets, 256, 256 * 16);
    if (rnd == MX_RNE)
        hipLaunchKernelGGL((quantize_axis1_kernel<W, B, MX_RNE>), dim3(grid), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((quantize_axis1_kernel<W, B, MX_RTZ>), dim3(grid), dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int W, int B>
mx_status launch_rows2(const QuantRows2Args& a, int rnd, hipStream_t st) {
    const int64_t wgs = a.items / a.row_octets * a.chunks;
    if (wgs > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)wgs);
    if (rnd == MX_RNE) {
        if (a.vec) hipLaunchKernelGGL((quantize_rows2_kernel<W, B, MX_RNE, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((quantize_rows2_kernel<W, B, MX_RNE, false>), grid, dim3(256), 0, st, a);
    } else {
        if (a.vec) hipLaunchKernelGGL((quantize_rows2_kernel<W, B, MX_RTZ, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((quantize_rows2_kernel<W, B, MX_RTZ, false>), grid, dim3(256), 0, st, a);
    }
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int W, int B>
mx_status launch_axis0(const QuantAxis0Args& a, int rnd, hipStream_t st) {
    if (ceil_div(a.cols, kAxis0Cols) > 65535) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)ceil_div(a.rows, kAxis0Rows), (unsigned)ceil_div(a.cols, kAxis0Cols), (unsigned)a.batch);
    if (rnd == MX_RNE)
        hipLaunchKernelGGL((quantize_axis0_kernel<W, B, MX_RNE>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((quantize_axis0_kernel<W, B, MX_RTZ>), grid, dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int W, int B>
mx_status launch_dequant(const DequantArgs& a, hipStream_t st) {
    const int grid = grid_for(a.octets, 256, 256 * 16);
    hipLaunchKernelGGL((dequantize_kernel<W, B>), dim3(grid), dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

// Expand (w, block) runtime values into template instances.
#define MX_SWITCH_W(W_, ...)                                                         \
    switch (W_) {                                                                    \
        case 2: { constexpr int kW = 2; __VA_ARGS__; } break;                        \
        case 3: { constexpr int kW = 3; __VA_ARGS__; } break;                        \
        case 4: { constexpr int kW = 4; __VA_ARGS__; } break;                        \
        case 5: { constexpr int kW = 5; __VA_ARGS__; } break;                        \
        case 6: { constexpr int kW = 6; __VA_ARGS__; } break;                        \
        case 7: { constexpr int kW = 7; __VA_ARGS__; } break;                        \
        case 8: { constexpr int kW = 8; __VA_ARGS__; } break;                        \
        default: return MX_ERR_BAD_ARG;                                              \
    }
#define MX_SWITCH_B(B_, ...)                                                         \
    switch (B_) {                                                                    \
        case 8: { constexpr int kB = 8; __VA_ARGS__; } break;                        \
        case 16: { constexpr int kB = 16; __VA_ARGS__; } break;                      \
        case 32: { constexpr int kB = 32; __VA_ARGS__; } break;                      \
        case 64: { constexpr int kB = 64; __VA_ARGS__; } break;                      \
        default: return MX_ERR_UNSUPPORTED;                                          \
    }

}  // namespace
}  // namespace mx

namespace mx {
namespace {

// One workgroup per 1024-element piece of a row: a lane looks at four elements and the workgroup raises the flag
// when any of them has all exponent bits set (NaN or infinity).
__global__ __launch_bounds__(256) void nonfinite_kernel(const float* x, int64_t rows, int64_t cols, int64_t row_stride,
                                                        int64_t batch_stride, int64_t pieces, int32_t* flag) {
    const int64_t item = blockIdx.x;
    const int64_t line = item / pieces, piece = item - line * pieces;
    const int64_t b = line / rows, r = line - b * rows;
    const float* row = x + b * batch_stride + r * row_stride;
    bool bad = false;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t c = piece * 1024 + u * 256 + threadIdx.x;
        if (c < cols) bad = bad || ((__float_as_uint(row[c]) & 0x7F800000u) == 0x7F800000u);
    }
    if (bad) *flag = 1;                       // every writer writes the same value
}

__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

}  // namespace
}  // namespace mx

using namespace mx;

extern "C" size_t mx_mant_bytes(int64_t batch, int64_t rows, int64_t cols, mx_format f) {
    if (!format_ok_quant(f) || batch < 0 || rows < 0 || cols < 0) return 0;
    return (size_t)(batch * rows * cols) * f.mant_bits / 8;
}

extern "C" size_t mx_exps_bytes(int64_t batch, int64_t rows, int64_t cols, mx_format f) {
    if (!format_ok_quant(f) || batch < 0 || rows < 0 || cols < 0 || rows % f.block_rows != 0) return 0;
    return (size_t)(batch * rows * cols) / (f.block * f.block_rows);
}

extern "C" mx_status mx_quantize(const float* x, int64_t batch, int64_t rows, int64_t cols,
                                 int64_t row_stride, int64_t batch_stride, int32_t axis, mx_format f,
                                 uint8_t* mant, uint8_t* exps, void* stream) {
    if (!format_ok_quant(f)) return MX_ERR_BAD_ARG;
    if (batch < 0 || rows < 0 || cols < 0 || row_stride < cols) return MX_ERR_BAD_ARG;
    if (axis != 0 && axis != 1) return MX_ERR_BAD_ARG;
    if ((axis == 1 ? cols : rows) % f.block != 0) return MX_ERR_BAD_ARG;
    if (f.block_rows == 2 && (axis == 1 ? rows : cols) % 2 != 0) return MX_ERR_BAD_ARG;
    if (batch > 1 && batch_stride < (rows - 1) * row_stride + cols) return MX_ERR_BAD_ARG;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!x || !mant || !exps) return MX_ERR_BAD_ARG;
    if (((uintptr_t)x & 3) || ((uintptr_t)mant & 15)) return MX_ERR_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int bias = (1 << (f.exp_bits - 1)) - 1;
    const int emax = ((1 << f.exp_bits) - 1) - bias;
    if (axis == 1 && f.block_rows == 2) {
        QuantRows2Args a;
        a.x = x; a.mant = mant; a.exps = exps;
        a.items = batch * (rows / 2) * (cols / 8);
        a.row_octets = cols / 8;
        a.pairs = rows / 2; a.row_stride = row_stride; a.batch_stride = batch_stride;
        a.bias = bias; a.emax = emax;
        a.vec = (((uintptr_t)x & 15) == 0 && (row_stride & 3) == 0 && (batch_stride & 3) == 0) ? 1 : 0;
        a.chunks = ceil_div(a.row_octets, 256);
        a.flat = (batch == 1 || batch_stride == rows * row_stride) ? 1 : 0;
        MX_SWITCH_W(f.mant_bits, MX_SWITCH_B(f.block, return (launch_rows2<kW, kB>(a, f.rounding, st))));
    } else if (axis == 1) {
        QuantArgs a;
        a.x = x; a.mant = mant; a.exps = exps;
        a.octets = batch * rows * (cols / 8);
        a.row_octets = cols / 8;
        a.rows = rows; a.row_stride = row_stride; a.batch_stride = batch_stride;
        a.bias = bias; a.emax = emax;
        const bool dense_rows = row_stride == cols && (batch == 1 || batch_stride == rows * cols);
        a.dense = dense_rows && (((uintptr_t)x & 15) == 0);
        MX_SWITCH_W(f.mant_bits, MX_SWITCH_B(f.block, return (launch_axis1<kW, kB>(a, f.rounding, st))));
    } else {
        if (cols > 0x7fffffffLL || rows / f.block > 65535 || batch > 65535) return MX_ERR_UNSUPPORTED;
        QuantAxis0Args a;
        a.x = x; a.mant = mant; a.exps = exps;
        a.batch = batch; a.rows = rows; a.cols = cols;
        a.row_stride = row_stride; a.batch_stride = batch_stride;
        a.bias = bias; a.emax = emax; a.brows = f.block_rows;
        MX_SWITCH_W(f.mant_bits, MX_SWITCH_B(f.block, return (launch_axis0<kW, kB>(a, f.rounding, st))));
    }
    return MX_ERR_UNSUPPORTED;
}

extern "C" mx_status mx_check_finite(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                     int64_t batch_stride, int32_t* flag, void* stream) {
    if (batch < 0 || rows < 0 || cols < 0 || row_stride < cols) return MX_ERR_BAD_ARG;
    if (batch > 1 && batch_stride < (rows - 1) * row_stride + cols) return MX_ERR_BAD_ARG;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!x || !flag || ((uintptr_t)x & 3) || ((uintptr_t)flag & 3)) return MX_ERR_BAD_ARG;
    const int64_t pieces = ceil_div(cols, 1024), items = batch * rows * pieces;
    if (items > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    clear_flag_kernel<<<1, 1, 0, st>>>(flag);
    nonfinite_kernel<<<(uint32_t)items, 256, 0, st>>>(x, rows, cols, row_stride, batch_stride, pieces, flag);
    if (hipGetLastError() != hipSuccess) return MX_ERR_DEVICE;
    int32_t found = 0;
    if (hipMemcpyAsync(&found, flag, sizeof(found), hipMemcpyDeviceToHost, st) != hipSuccess) return MX_ERR_DEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return MX_ERR_DEVICE;
    return found ? MX_ERR_BAD_ARG : MX_OK;
}

extern "C" mx_status mx_dequantize(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows,
                                   int64_t cols, mx_format f, float* y, void* stream) {
    if (!format_ok_quant(f)) return MX_ERR_BAD_ARG;
    if (batch < 0 || rows < 0 || cols < 0 || cols % f.block != 0 || rows % f.block_rows != 0) return MX_ERR_BAD_ARG;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!mant || !exps || !y) return MX_ERR_BAD_ARG;
    if (((uintptr_t)y & 15) || ((uintptr_t)mant & 15)) return MX_ERR_BAD_ARG;
    DequantArgs a;
    a.mant = mant; a.exps = exps; a.y = y;
    a.octets = batch * rows * (cols / 8);
    a.row_octets = cols / 8;
    a.block_rows = f.block_rows;
    a.bias = (1 << (f.exp_bits - 1)) - 1;
    hipStream_t st = (hipStream_t)stream;
    MX_SWITCH_W(f.mant_bits, MX_SWITCH_B(f.block, return (launch_dequant<kW, kB>(a, st))));
    return MX_ERR_UNSUPPORTED;
}
