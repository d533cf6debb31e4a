// Decode-time linear layer: fp32 activations (M <= 8 rows) are quantized to MXInt and written
// straight into the fragment layout, then the decode kernel of mx_gemm streams the packed weights.
// The quantizer arithmetic is the one of mx_quantize (Section 4.1 format; Section 3.2 emulation
// semantics: quantize the input, then the operator).
#include "mx_gemm.h"

namespace mx {
namespace {

struct LinQuantArgs {
    const float* x;
    uint8_t* packed;
    int64_t M;           // rows holding data
    int64_t rows_out;    // rows written: M (decode: the rest of the row group is never read) or M padded to 32
    int64_t K, row_stride, batch_stride, chunks, matrix_bytes;
    int32_t piece, record, bias, emax;
};

// One thread per (row m < rows_out, block slot b < 4*chunks); grid.y = batch.  Slots past K and
// rows past M hold zero mantissas and exponent byte 0.
template <int W, int B, int RND>
__global__ __launch_bounds__(256) void quantize_to_fragments_kernel(LinQuantArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t slots = a.chunks * 4;
    if (t >= a.rows_out * slots) return;
    const int64_t m = t / slots, b = t - m * slots;
    const int64_t c = b >> 2;
    const int j = (int)(b & 3);
    const bool inside = b * B < a.K && m < a.M;
    const float* xrow = a.x + blockIdx.y * a.batch_stride + m * a.row_stride;
    float v[B];
    uint32_t am = 0;
#pragma unroll
    for (int k = 0; k < B; ++k) {
        v[k] = inside ? xrow[b * B + k] : 0.f;
        uint32_t ab = __float_as_uint(v[k]) & 0x7fffffffu;
        am = ab > am ? ab : am;
    }
    const int ef = (int)(am >> 23);
    int E = ef == 0 ? -127 : ef - 127;
    E = E < -a.bias ? -a.bias : E;
    E = E > a.emax ? a.emax : E;
    const int shift = (W - 2) - E;
    constexpr float qmax = (float)((1 << (W - 1)) - 1);
    uint8_t* rec = a.packed + blockIdx.y * a.matrix_bytes + ((m >> 5) * a.chunks + c) * a.record;
    const int i = (int)(m & 31);
    constexpr int kHalfBytes = B * W / 16;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // (B/2)*W bits of half h, as bytes
        uint8_t out[kHalfBytes];
#pragma unroll
        for (int d = 0; d < kHalfBytes; ++d) out[d] = 0;
#pragma unroll
        for (int k = 0; k < B / 2; ++k) {
            float s = __builtin_ldexpf(v[h * (B / 2) + k], shift);
            float r = RND == MX_RNE ? __builtin_rintf(s) : __builtin_truncf(s);
            r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
            const uint32_t code = (uint32_t)(int)r & ((1u << W) - 1u);
            int pos = k;                                   // element position inside the half block
            if (W == 4) {                                  // nibble order e0 e4 e1 e5 e2 e6 e3 e7 per 8
                const int t8 = k & 7;
                pos = (k & ~7) + (t8 < 4 ? 2 * t8 : 2 * (t8 - 4) + 1);
            }
            const int bit = pos * W;
            out[bit >> 3] |= (uint8_t)(code << (bit & 7));
            if ((bit & 7) + W > 8) out[(bit >> 3) + 1] |= (uint8_t)(code >> (8 - (bit & 7)));
        }
        uint8_t* dst = rec + (int64_t)(32 * h + i) * a.piece + j * kHalfBytes;
#pragma unroll
        for (int d = 0; d < kHalfBytes; ++d) dst[d] = out[d];
    }
    rec[64 * a.piece + i * 4 + j] = inside ? (uint8_t)(E + a.bias) : (uint8_t)0;
}

template <int W, int B>
mx_status launch_lq(const LinQuantArgs& a, int64_t batch, int rnd, hipStream_t st) {
    const int64_t threads = a.rows_out * a.chunks * 4;
    dim3 grid((unsigned)ceil_div(threads, 256), (unsigned)batch);
    if (rnd == MX_RNE)
        hipLaunchKernelGGL((quantize_to_fragments_kernel<W, B, MX_RNE>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((quantize_to_fragments_kernel<W, B, MX_RTZ>), grid, dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

#define MX_SW(W_, NAME, ...)                                        \
    switch (W_) {                                                   \
        case 2: { constexpr int NAME = 2; __VA_ARGS__; } break;     \
        case 3: { constexpr int NAME = 3; __VA_ARGS__; } break;     \
        case 4: { constexpr int NAME = 4; __VA_ARGS__; } break;     \
        case 5: { constexpr int NAME = 5; __VA_ARGS__; } break;     \
        case 6: { constexpr int NAME = 6; __VA_ARGS__; } break;     \
        case 7: { constexpr int NAME = 7; __VA_ARGS__; } break;     \
        case 8: { constexpr int NAME = 8; __VA_ARGS__; } break;     \
        default: return MX_ERR_BAD_ARG;                             \
    }

mx_status run_lq(const float* x, int64_t batch, int64_t M, int64_t rows_out, int64_t K, int64_t row_stride,
                 int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st) {
    const FragGeom ga = frag_geom(M, K, f.block, f.mant_bits);
    LinQuantArgs a;
    a.x = x; a.packed = packed;
    a.M = M; a.rows_out = rows_out; a.K = K; a.row_stride = row_stride; a.batch_stride = batch_stride;
    a.chunks = ga.chunks; a.matrix_bytes = ga.matrix;
    a.piece = ga.piece; a.record = ga.record;
    a.bias = (1 << (f.exp_bits - 1)) - 1;
    a.emax = ((1 << f.exp_bits) - 1) - a.bias;
    if (ceil_div(rows_out * ga.chunks * 4, 256) > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    switch (f.block) {
        case 16: MX_SW(f.mant_bits, kW, return (launch_lq<kW, 16>(a, batch, f.rounding, st))); break;
        case 32: MX_SW(f.mant_bits, kW, return (launch_lq<kW, 32>(a, batch, f.rounding, st))); break;
        case 64: MX_SW(f.mant_bits, kW, return (launch_lq<kW, 64>(a, batch, f.rounding, st))); break;
    }
    return MX_ERR_UNSUPPORTED;
}

}  // namespace

// fp32 -> fragment layout for any number of rows (the padding rows of the last group are zeroed).
mx_status quantize_pack_fragment(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                 int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st) {
    return run_lq(x, batch, rows, ceil_div(rows, 32) * 32, cols, row_stride, batch_stride, f, packed, st);
}

}  // namespace mx

using namespace mx;

extern "C" mx_status mx_linear(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx,
                               void* A_scratch, const void* B_packed, int64_t N, mx_format fb,
                               int32_t layout, float* Y, int64_t ldy, void* stream) {
    if (!format_ok_quant(fx) || !format_ok_quant(fb)) return MX_ERR_BAD_ARG;
    if (fx.block != fb.block || fx.exp_bits != fb.exp_bits) return MX_ERR_BAD_ARG;
    if (!format_ok_gemm(fx)) return MX_ERR_UNSUPPORTED;
    if (layout != MX_LAYOUT_FRAGMENT) return layout == MX_LAYOUT_MATRIX ? MX_ERR_UNSUPPORTED : MX_ERR_BAD_ARG;
    if (M < 0 || N < 0 || K < 0 || K % fx.block != 0 || row_stride < K || ldy < N) return MX_ERR_BAD_ARG;
    if (M > 8) return MX_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return MX_OK;
    if (K > 0 && (!x || !A_scratch || !B_packed)) return MX_ERR_BAD_ARG;
    if (((uintptr_t)x & 3) || ((uintptr_t)A_scratch & 255)) return MX_ERR_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (K > 0 && M <= 2) {
        // one launch: the dot-product decode kernel quantizes the activations on its way into LDS
        // (same arithmetic, same accumulation order as the two-launch form); A_scratch is not touched
        const GemmArgs g = fragment_args(M, N, K, A_scratch, fx, B_packed, fb, Y, ldy, M * ldy);
        const mx_status s = gemv_dot(g, fx.mant_bits, fb.mant_bits, fx.block, 1, st, x, row_stride, &fx);
        if (s != MX_ERR_UNSUPPORTED) return s;
    }
    if (K > 0) {
        // rows M..31 of the row group stay as they are: the decode kernel does not read them
        mx_status s = run_lq(x, 1, M, M, K, row_stride, 0, fx, (uint8_t*)A_scratch, st);
        if (s != MX_OK) return s;
    }
    return mx_gemm(1, M, N, K, A_scratch, fx, B_packed, fb, layout, Y, ldy, M * ldy, stream);
}
