// Canonical MXInt form <-> fragment layout (see FragGeom in mx_common.h).
//
// The fragment layout keeps the density of the format (Eq. 1 of the paper: w bits per element
// plus e/block bits of exponent) and orders the bytes the way the lanes of a 32x32 integer MFMA
// consume them: lane 32*h + i holds half h of each block of row i.  For w = 4 the eight nibbles of
// every dword are stored in the order e0 e4 e1 e5 e2 e6 e3 e7, so that (d << 4) & 0xF0F0F0F0 and
// d & 0xF0F0F0F0 are the two int8x4 words (times 16) in element order.
#include "mx_common.h"
#include "mx_bf16.h"
#include "mx_matrix.h"

namespace mx {

// defined in mx_pack_matrix.hip / mx_linear.hip
bool matrix_format_ok(const mx_format& f);
mx_status pack_matrix(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                      mx_format f, uint8_t* packed, bool pack, hipStream_t st);
mx_status quantize_pack_matrix(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                               int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st);
mx_status quantize_pack_fragment(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                 int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st);

namespace {

__device__ __forceinline__ uint32_t nibble_interleave(uint32_t d) {
    // in: nibble t at position t;  out: nibble t at position p(t), p = 0 2 4 6 1 3 5 7
    uint32_t r = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int p = t < 4 ? 2 * t : 2 * (t - 4) + 1;
        r |= ((d >> (4 * t)) & 0xFu) << (4 * p);
    }
    return r;
}
__device__ __forceinline__ uint32_t nibble_deinterleave(uint32_t d) {
    uint32_t r = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int p = t < 4 ? 2 * t : 2 * (t - 4) + 1;
        r |= ((d >> (4 * p)) & 0xFu) << (4 * t);
    }
    return r;
}

struct PackArgs {
    const uint8_t* mant;   // canonical (pack: source; unpack: destination)
    const uint8_t* exps;
    uint8_t* packed;
    int64_t rows, cols;    // logical
    int64_t groups, chunks;
    int64_t matrix_bytes;  // packed bytes per batch entry
    int32_t block, w, piece, record;
    int32_t brows;         // rows per exponent of the canonical form (1 or 2)
};

// One thread per (record, lane); grid.y = batch.
template <bool PACK>
__global__ __launch_bounds__(256) void pack_kernel(PackArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rec = t >> 6;
    const int lane = (int)(t & 63);
    if (rec >= a.groups * a.chunks) return;
    const int64_t b = blockIdx.y;
    const int64_t g = rec / a.chunks, c = rec - g * a.chunks;
    const int i = lane & 31, h = lane >> 5;
    const int64_t row = g * 32 + i;
    const int half_bytes = a.piece / 4;                    // (block/2)*w/8
    const int64_t row_bytes = a.cols * a.w / 8;
    const int64_t nblk = a.cols / a.block;
    uint8_t* mant = const_cast<uint8_t*>(a.mant) + b * a.rows * row_bytes;
    uint8_t* exps = const_cast<uint8_t*>(a.exps) + b * (a.rows / a.brows) * nblk;
    uint8_t* rec_base = a.packed + b * a.matrix_bytes + rec * a.record;
    uint8_t* piece = rec_base + (int64_t)lane * a.piece;
    for (int j = 0; j < 4; ++j) {
        const int64_t blk = c * 4 + j;
        const bool inside = row < a.rows && blk < nblk;
        uint8_t* canon = mant + row * row_bytes + (blk * a.block + h * (a.block / 2)) * a.w / 8;
        uint8_t* dst = piece + j * half_bytes;
        if (a.w == 4) {
            // half_bytes = block/4 is a multiple of 4; canonical offset is a multiple of 4 as well
            for (int d = 0; d < half_bytes; d += 4) {
                if (PACK) {
                    uint32_t v = inside ? *reinterpret_cast<const uint32_t*>(canon + d) : 0u;
                    *reinterpret_cast<uint32_t*>(dst + d) = nibble_interleave(v);
                } else if (inside) {
                    uint32_t v = *reinterpret_cast<const uint32_t*>(dst + d);
                    *reinterpret_cast<uint32_t*>(canon + d) = nibble_deinterleave(v);
                }
            }
        } else {
            for (int d = 0; d < half_bytes; ++d) {
                if (PACK) dst[d] = inside ? canon[d] : (uint8_t)0;
                else if (inside) canon[d] = dst[d];
            }
        }
        if (h == 0) {
            uint8_t* pe = rec_base + 64 * a.piece + i * 4 + j;
            // two-row blocks: both rows carry the pair's byte in the layout; the even row writes it back
            if (PACK) *pe = inside ? exps[(row / a.brows) * nblk + blk] : (uint8_t)0;
            else if (inside && row % a.brows == 0) exps[(row / a.brows) * nblk + blk] = *pe;
        }
    }
}

mx_status check_pack_args(int64_t batch, int64_t rows, int64_t cols, const mx_format& f, int32_t layout) {
    if (layout != MX_LAYOUT_FRAGMENT && layout != MX_LAYOUT_MATRIX) return MX_ERR_BAD_ARG;
    if (!format_ok_quant(f)) return MX_ERR_BAD_ARG;
    if (layout == MX_LAYOUT_FRAGMENT ? !format_ok_gemm(f) : !matrix_format_ok(f)) return MX_ERR_UNSUPPORTED;
    if (batch < 0 || rows < 0 || cols < 0 || cols % f.block != 0 || rows % f.block_rows != 0) return MX_ERR_BAD_ARG;
    return MX_OK;
}

template <bool PACK>
mx_status run_pack(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                   mx_format f, int32_t layout, uint8_t* packed, void* stream) {
    mx_status s = check_pack_args(batch, rows, cols, f, layout);
    if (s != MX_OK) return s;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!mant || !exps || !packed) return MX_ERR_BAD_ARG;
    if (((uintptr_t)packed & 255) || ((uintptr_t)mant & 15)) return MX_ERR_BAD_ARG;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    if (layout == MX_LAYOUT_MATRIX) return pack_matrix(mant, exps, batch, rows, cols, f, packed, PACK, (hipStream_t)stream);
    FragGeom g = frag_geom(rows, cols, f.block, f.mant_bits);
    PackArgs a;
    a.mant = mant; a.exps = exps; a.packed = packed;
    a.rows = rows; a.cols = cols; a.groups = g.groups; a.chunks = g.chunks;
    a.matrix_bytes = g.matrix; a.block = f.block; a.w = f.mant_bits; a.piece = g.piece; a.record = g.record;
    a.brows = f.block_rows;
    const int64_t threads = g.groups * g.chunks * 64;
    dim3 grid((unsigned)ceil_div(threads, 256), (unsigned)batch);
    hipLaunchKernelGGL((pack_kernel<PACK>), grid, dim3(256), 0, (hipStream_t)stream, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

}  // namespace
}  // namespace mx

using namespace mx;

extern "C" size_t mx_packed_bytes(int64_t batch, int64_t rows, int64_t cols, mx_format f, int32_t layout) {
    if (check_pack_args(batch, rows, cols, f, layout) != MX_OK) return 0;
    if (layout == MX_LAYOUT_MATRIX && f.block == 16) return (size_t)(batch * bf_geom(rows, cols).matrix);
    if (layout == MX_LAYOUT_MATRIX) return (size_t)(batch * mat_geom(rows, cols, f.mant_bits).matrix);
    return (size_t)(batch * frag_geom(rows, cols, f.block, f.mant_bits).matrix);
}

extern "C" mx_status mx_pack(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows,
                             int64_t cols, mx_format f, int32_t layout, void* packed, void* stream) {
    return run_pack<true>(mant, exps, batch, rows, cols, f, layout, (uint8_t*)packed, stream);
}

extern "C" mx_status mx_unpack(const void* packed, int64_t batch, int64_t rows, int64_t cols, mx_format f,
                               int32_t layout, uint8_t* mant, uint8_t* exps, void* stream) {
    return run_pack<false>(mant, exps, batch, rows, cols, f, layout,
                           const_cast<uint8_t*>((const uint8_t*)packed), stream);
}

extern "C" mx_status mx_quantize_pack(const float* x, int64_t batch, int64_t rows, int64_t cols,
                                      int64_t row_stride, int64_t batch_stride, mx_format f, int32_t layout,
                                      void* packed, void* stream) {
    mx_status s = check_pack_args(batch, rows, cols, f, layout);
    if (s != MX_OK) return s;
    if (row_stride < cols) return MX_ERR_BAD_ARG;
    if (batch > 1 && batch_stride < (rows - 1) * row_stride + cols) return MX_ERR_BAD_ARG;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!x || !packed || ((uintptr_t)x & 3) || ((uintptr_t)packed & 255)) return MX_ERR_BAD_ARG;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    if (layout == MX_LAYOUT_MATRIX)
        return quantize_pack_matrix(x, batch, rows, cols, row_stride, batch_stride, f, (uint8_t*)packed,
                                    (hipStream_t)stream);
    return quantize_pack_fragment(x, batch, rows, cols, row_stride, batch_stride, f, (uint8_t*)packed,
                                  (hipStream_t)stream);
}

namespace mx {
mx_status quantize_pack_bf16_axis0(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                   int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st);
}

extern "C" mx_status mx_quantize_pack_axis0(const float* x, int64_t batch, int64_t rows, int64_t cols,
                                            int64_t row_stride, int64_t batch_stride, mx_format f, int32_t layout,
                                            void* packed, void* stream) {
    // the operand that comes out is x^T: cols x rows, blocks along its columns (the rows of x)
    mx_status s = check_pack_args(batch, cols, rows, f, layout);
    if (s != MX_OK) return s;
    if (row_stride < cols) return MX_ERR_BAD_ARG;
    if (batch > 1 && batch_stride < (rows - 1) * row_stride + cols) return MX_ERR_BAD_ARG;
    if (layout != MX_LAYOUT_MATRIX || f.block != 16) return MX_ERR_UNSUPPORTED;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!x || !packed || ((uintptr_t)x & 3) || ((uintptr_t)packed & 255)) return MX_ERR_BAD_ARG;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    return quantize_pack_bf16_axis0(x, batch, rows, cols, row_stride, batch_stride, f, (uint8_t*)packed,
                                    (hipStream_t)stream);
}
