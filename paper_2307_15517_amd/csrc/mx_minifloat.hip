// Quantizer and dequantizer of the paper's two other block formats (Section 2): Block Minifloat
// (elements are small floats sharing the exponent bias of their block) and, with no mantissa bits,
// Block Logarithm.  The bit-level definition is in include/mx.h.
//
// HBM-bound: 4 bytes read and 1 byte (+ 1/block) written per element.  An item is four
// consecutive elements (a 16-byte load, a 4-byte store); the threads of a wave take consecutive
// items of the row, a thread four items 256 apart (all four loads are issued first), so a block is block/4 neighbouring lanes and its maximum takes log2(block/4) DPP
// steps.  All rounding decisions are taken in integer arithmetic on the 24-bit significand.
#include "mx_common.h"

namespace mx {
namespace {

struct MiniArgs {
    const float* x;
    uint8_t* codes;
    uint8_t* shared;
    float* y;
    int64_t rows, cols, row_stride, batch_stride;
    int64_t items_per_row;     // cols / 4
    int32_t e, m, rnd;
};

// |x| (fp32 bits without the sign) as sig * 2^(ex - 23) with sig in [2^23, 2^24), also for fp32 subnormals;
// zero gives sig = 0.
__device__ __forceinline__ void significand(uint32_t ab, uint32_t& sig, int& ex) {
    const uint32_t ef = ab >> 23, fr = ab & 0x7fffffu;
    if (ef != 0) {
        sig = fr | 0x800000u;
        ex = (int)ef - 127;
    } else {
        const int lz = fr == 0 ? 0 : __builtin_clz(fr) - 8;
        sig = fr << lz;
        ex = -126 - lz;
    }
}

constexpr int kMiniItems = 4;      // items (of four elements) per thread, 256 threads apart: all loads first

template <int B>
__global__ __launch_bounds__(256) void quantize_minifloat_kernel(MiniArgs a) {
    const int64_t b = blockIdx.z;
    const int m = a.m, e = a.e;
    const int cmax = (1 << e) - 1;
    // a workgroup takes 1024 consecutive items of one row; cols % block == 0 and 256 % (block/4) == 0, so the
    // lanes of a block are all inside the row or all outside
    for (int64_t r = blockIdx.y; r < a.rows; r += gridDim.y) {
        const float* xrow = a.x + b * a.batch_stride + r * a.row_stride;
        uint8_t* crow = a.codes + (b * a.rows + r) * a.cols;
        uint8_t* srow = a.shared + (b * a.rows + r) * (a.cols / B);
        float4 v[kMiniItems];
#pragma unroll
        for (int u = 0; u < kMiniItems; ++u) {
            const int64_t it = (int64_t)blockIdx.x * (256 * kMiniItems) + u * 256 + threadIdx.x;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (it < a.items_per_row) v[u] = *reinterpret_cast<const float4*>(xrow + it * 4);
        }
#pragma unroll
        for (int u = 0; u < kMiniItems; ++u) {
            const int64_t it = (int64_t)blockIdx.x * (256 * kMiniItems) + u * 256 + threadIdx.x;
            const int64_t c = it * 4;
            const float xv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            uint32_t am = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t ab = __float_as_uint(xv[i]) & 0x7fffffffu;
                am = ab > am ? ab : am;
            }
            uint32_t o;
            if (B >= 8)  { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);  am = o > am ? o : am; }   // lane ^ 1
            if (B >= 16) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0x4E, 0xF, 0xF, true);  am = o > am ? o : am; }   // lane ^ 2
            if (B >= 32) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0x141, 0xF, 0xF, true); am = o > am ? o : am; }   // 7 - lane within 8
            if (B >= 64) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0x140, 0xF, 0xF, true); am = o > am ? o : am; }   // 15 - lane within 16
            if (it >= a.items_per_row) continue;

            uint32_t out = 0;
            uint8_t sbyte = 0;
            if (am != 0) {
                // T = floor(log2 amax), plus one when the maximum rounds up into the next binade: its m+1
                // leading fraction bits are all ones and what follows is at least half of the last place,
                // i.e. the 24-bit significand is >= 2^24 - 2^(22-m)
                uint32_t sm;
                int fl;
                significand(am, sm, fl);
                int T = fl;
                if (a.rnd == MX_RNE && sm >= (1u << 24) - (1u << (22 - m))) T += 1;
                T = T < -126 ? -126 : T;
                T = T > 127 ? 127 : T;
                const int L = T - cmax + 1;
                // Rounding happens in the fp32 bit pattern.  At or above the format's smallest normal value
                // 2^L the result keeps m fraction bits: add half of the dropped field (less one, plus the
                // parity bit that sends a tie to the even code) and drop the field -- a carry runs into the
                // exponent by itself -- and the code integer c << m | f is the kept bits minus a constant.
                // Below 2^L the step is fixed at 2^(L-m): adding 2^(L-m+23) makes the fp32 adder round to
                // that step (ties to even), and the code integer is the low bits of the sum.
                const int sb = 23 - m;                                          // dropped fraction bits
                const uint32_t half_m1 = (1u << (sb - 1)) - 1u;
                const uint32_t code_max = (1u << (e + m)) - 1u;
                const uint32_t rebase = (uint32_t)(126 + L) << m;               // may wrap: used modulo 2^32
                const bool low_ok = L >= -126;                                  // 2^L is an fp32 normal
                const uint32_t minnorm = low_ok ? (uint32_t)(L + 127) << 23 : 0x00800000u;
                const bool magic_overflows = L - m + 23 > 127;
                const float magic = __uint_as_float((uint32_t)((low_ok && !magic_overflows ? L : -126) - m + 23 + 127) << 23);
                const uint32_t par0 = m == 0 ? (uint32_t)(L & 1) : 0u;         // m = 0: the code's parity is the exponent's
                // Ordinary data has no element below the format's smallest normal value (2^-cmax of the block
                // maximum; zeros count as below): when no lane of the wave holds one, only the first rule runs.
                uint32_t lowest = __float_as_uint(xv[0]) & 0x7fffffffu;
#pragma unroll
                for (int i = 1; i < 4; ++i) {
                    const uint32_t ab = __float_as_uint(xv[i]) & 0x7fffffffu;
                    lowest = ab < lowest ? ab : lowest;
                }
                if (__builtin_amdgcn_ballot_w64(lowest < minnorm) == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t bits = __float_as_uint(xv[i]);
                        const uint32_t ab = bits & 0x7fffffffu;
                        uint32_t r = ab;
                        if (a.rnd == MX_RNE) r += half_m1 + (((ab >> sb) & 1u) ^ par0);
                        uint32_t code = (r >> sb) - rebase;
                        code = code > code_max ? code_max : code;
                        out |= (((bits >> 31) << (e + m)) | code) << (8 * i);
                    }
                } else
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t bits = __float_as_uint(xv[i]);
                    const uint32_t ab = bits & 0x7fffffffu;
                    const uint32_t sign = bits >> 31;
                    uint32_t code;
                    if (ab != 0 && ab < minnorm && (!low_ok || magic_overflows)) {
                        // rare: an fp32 subnormal that the format still resolves (very wide exponent fields), or an
                        // underflow step too large for the addition trick (blocks near the top of the fp32 range): integers
                        uint32_t sig;
                        int ex;
                        significand(ab, sig, ex);
                        int k = ex < L ? L : ex;
                        int sh = 23 - m + (k - ex);
                        sh = sh > 31 ? 31 : sh;
                        uint32_t n = sig >> sh;
                        const uint32_t rem = sig & ((1u << sh) - 1u), half = 1u << (sh - 1);
                        if (a.rnd == MX_RNE) {
                            const uint32_t c_lo = n >= (1u << m) ? (uint32_t)(k - L + 1) : 0u;
                            const uint32_t odd = m == 0 ? (c_lo & 1u) : (n & 1u);
                            n += (rem > half || (rem == half && odd)) ? 1u : 0u;
                        }
                        if (n == (2u << m)) { k += 1; n = 1u << m; }
                        const uint32_t cf = n >= (1u << m) ? (uint32_t)(k - L + 1) : 0u;
                        code = (cf << m) | (n & ((1u << m) - 1u));
                    } else {
                        // normal range of the format
                        uint32_t r = ab;
                        if (a.rnd == MX_RNE) r += half_m1 + (((ab >> sb) & 1u) ^ par0);
                        uint32_t code_n = (r >> sb) - rebase;               // the shift drops the rounded-away field
                        // underflow range of the format
                        uint32_t code_s;
                        if (a.rnd == MX_RNE) code_s = __float_as_uint(__uint_as_float(ab) + magic) & 0x7fffffu;
                        else code_s = (uint32_t)__builtin_ldexpf(__uint_as_float(ab), m - L);   // conversion truncates
                        code = ab < minnorm ? (low_ok ? code_s : 0u) : code_n;     // zero: minnorm > 0 and code_s = 0
                    }
                    code = code > code_max ? code_max : code;                   // saturate (clamped T only)
                    out |= ((sign << (e + m)) | code) << (8 * i);
                }
                sbyte = (uint8_t)(T + 127);
            }
            *reinterpret_cast<uint32_t*>(crow + c) = out;
            if ((c & (B - 1)) == 0) srow[c / B] = sbyte;
        }
    }
}

__global__ __launch_bounds__(256) void dequantize_minifloat_kernel(MiniArgs a, int block) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.rows * a.items_per_row) return;
    const int64_t b = blockIdx.y;
    const int64_t r = t / a.items_per_row, c = (t - r * a.items_per_row) * 4;
    const uint32_t codes = *reinterpret_cast<const uint32_t*>(a.codes + (b * a.rows + r) * a.cols + c);
    const int sb = a.shared[(b * a.rows + r) * (a.cols / block) + c / block];
    const int m = a.m, e = a.e, cmax = (1 << e) - 1;
    float out[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t code = (codes >> (8 * i)) & 0xFFu;
        const uint32_t sign = (code >> (e + m)) & 1u, cf = (code >> m) & (uint32_t)cmax, ff = code & ((1u << m) - 1u);
        float v = 0.f;
        if (sb != 0) {
            const int T = sb - 127;
            // (2^m + f) * 2^(c - cmax + T - m) for c >= 1, f * 2^(1 - cmax + T - m) for c == 0
            const float mant = (float)(cf >= 1 ? (1u << m) + ff : ff);
            v = __builtin_ldexpf(mant, (cf >= 1 ? (int)cf : 1) - cmax + T - m);
        }
        out[i] = sign ? -v : v;
    }
    *reinterpret_cast<float4*>(a.y + ((b * a.rows + r) * a.cols + c)) = make_float4(out[0], out[1], out[2], out[3]);
}

bool minifloat_ok(const mx_minifloat_format& f) {
    return (f.block == 8 || f.block == 16 || f.block == 32 || f.block == 64) && f.exp_bits >= 1 && f.mant_bits >= 0 &&
           1 + f.exp_bits + f.mant_bits <= 8 && (f.rounding == MX_RNE || f.rounding == MX_RTZ);
}

}  // namespace
}  // namespace mx

using namespace mx;

extern "C" mx_status mx_quantize_minifloat(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                           int64_t batch_stride, mx_minifloat_format f, uint8_t* codes, uint8_t* shared,
                                           void* stream) {
    if (!minifloat_ok(f)) return MX_ERR_BAD_ARG;
    if (batch < 0 || rows < 0 || cols < 0 || cols % f.block != 0 || row_stride < cols) return MX_ERR_BAD_ARG;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!x || !codes || !shared || ((uintptr_t)codes & 3)) return MX_ERR_BAD_ARG;
    if (((uintptr_t)x & 15) || (row_stride & 3) || (batch_stride & 3)) return MX_ERR_UNSUPPORTED;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    MiniArgs a;
    a.x = x; a.codes = codes; a.shared = shared; a.y = nullptr;
    // blocks never cross a row (cols % block == 0), so contiguous rows, and contiguous matrices, are one long row:
    // no workgroup is left with the short tail of a row
    if (row_stride == cols) {
        cols *= rows; rows = 1; row_stride = cols;
        if (batch_stride == cols) { cols *= batch; batch = 1; batch_stride = cols; }
    }
    a.rows = rows; a.cols = cols; a.row_stride = row_stride; a.batch_stride = batch_stride;
    a.items_per_row = cols / 4;
    a.e = f.exp_bits; a.m = f.mant_bits; a.rnd = f.rounding;
    const int64_t blocks = ceil_div(a.items_per_row, 256 * kMiniItems);
    if (blocks > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)blocks, (unsigned)(rows < 65535 ? rows : 65535), (unsigned)batch);
    hipStream_t st = (hipStream_t)stream;
    switch (f.block) {
        case 8: hipLaunchKernelGGL(quantize_minifloat_kernel<8>, grid, dim3(256), 0, st, a); break;
        case 16: hipLaunchKernelGGL(quantize_minifloat_kernel<16>, grid, dim3(256), 0, st, a); break;
        case 32: hipLaunchKernelGGL(quantize_minifloat_kernel<32>, grid, dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL(quantize_minifloat_kernel<64>, grid, dim3(256), 0, st, a); break;
    }
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

extern "C" mx_status mx_dequantize_minifloat(const uint8_t* codes, const uint8_t* shared, int64_t batch, int64_t rows,
                                             int64_t cols, mx_minifloat_format f, float* y, void* stream) {
    if (!minifloat_ok(f)) return MX_ERR_BAD_ARG;
    if (batch < 0 || rows < 0 || cols < 0 || cols % f.block != 0) return MX_ERR_BAD_ARG;
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!y || !codes || !shared || ((uintptr_t)codes & 3) || ((uintptr_t)y & 15)) return MX_ERR_BAD_ARG;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    MiniArgs a;
    a.x = nullptr; a.codes = const_cast<uint8_t*>(codes); a.shared = const_cast<uint8_t*>(shared); a.y = y;
    a.rows = rows; a.cols = cols; a.row_stride = cols; a.batch_stride = rows * cols;
    a.items_per_row = cols / 4;
    a.e = f.exp_bits; a.m = f.mant_bits; a.rnd = f.rounding;
    const int64_t blocks = ceil_div(rows * a.items_per_row, 256);
    if (blocks > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)blocks, (unsigned)batch);
    hipLaunchKernelGGL(dequantize_minifloat_kernel, grid, dim3(256), 0, (hipStream_t)stream, a, (int)f.block);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}
