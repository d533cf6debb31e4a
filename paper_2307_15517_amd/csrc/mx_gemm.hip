// Host entry point of the MXInt x MXInt product: argument checks and dispatch on the block size.
#include "mx_gemm.h"

namespace mx {
bool matrix_format_ok(const mx_format& f);
mx_status gemm_scaled(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, mx_format fa, const void* B,
                      mx_format fb, float* Y, int64_t ldy, int64_t batch_stride_y, hipStream_t st);
mx_status gemm_bf16(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, const void* B, float* Y,
                    int64_t ldy, int64_t batch_stride_y, hipStream_t st);
mx_status gemm_bf16_q(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, const void* B,
                      const uint8_t* bias_mant, const uint8_t* bias_exps, mx_format fbias, mx_format fo, void* out,
                      hipStream_t st);
mx_status gemm_scaled_q(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, mx_format fa,
                        const void* B, mx_format fb, const uint8_t* bias_mant, const uint8_t* bias_exps,
                        mx_format fbias, mx_format fo, void* out, hipStream_t st);
}  // namespace mx

namespace mx {
GemmArgs fragment_args(int64_t M, int64_t N, int64_t K, const void* A, mx_format fa, const void* B, mx_format fb,
                       float* Y, int64_t ldy, int64_t batch_stride_y) {
    const FragGeom ga = frag_geom(M, K, fa.block, fa.mant_bits);
    const FragGeom gb = frag_geom(N, K, fb.block, fb.mant_bits);
    GemmArgs g;
    g.A = (const uint8_t*)A; g.B = (const uint8_t*)B; g.Y = Y;
    g.M = M; g.N = N; g.K = K;
    g.groupsA = ga.groups; g.groupsB = gb.groups; g.chunks = ga.chunks;
    g.matrixA = ga.matrix; g.matrixB = gb.matrix;
    g.ldy = ldy; g.batch_stride_y = batch_stride_y;
    g.recordA = ga.record; g.recordB = gb.record;
    const int bias = (1 << (fa.exp_bits - 1)) - 1;
    g.eadj = -2 * bias - (fa.mant_bits - 2) - (fb.mant_bits - 2);
    return g;
}
}  // namespace mx

using namespace mx;

extern "C" mx_status mx_gemm(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A_packed,
                             mx_format fa, const void* B_packed, mx_format fb, int32_t layout, float* Y,
                             int64_t ldy, int64_t batch_stride_y, void* stream) {
    if (!format_ok_quant(fa) || !format_ok_quant(fb)) return MX_ERR_BAD_ARG;
    if (fa.block != fb.block || fa.exp_bits != fb.exp_bits) return MX_ERR_BAD_ARG;
    if (layout != MX_LAYOUT_FRAGMENT && layout != MX_LAYOUT_MATRIX) return MX_ERR_BAD_ARG;
    if (layout == MX_LAYOUT_FRAGMENT ? !format_ok_gemm(fa) : !matrix_format_ok(fa)) return MX_ERR_UNSUPPORTED;
    if (batch < 0 || M < 0 || N < 0 || K < 0 || K % fa.block != 0 || ldy < N) return MX_ERR_BAD_ARG;
    if (batch > 1 && batch_stride_y < (M - 1) * ldy + N) return MX_ERR_BAD_ARG;
    if (batch == 0 || M == 0 || N == 0) return MX_OK;
    if (!Y || ((uintptr_t)Y & 3)) return MX_ERR_BAD_ARG;
    if (K > 0 && (!A_packed || !B_packed)) return MX_ERR_BAD_ARG;
    if (((uintptr_t)A_packed & 255) || ((uintptr_t)B_packed & 255)) return MX_ERR_BAD_ARG;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    if (layout == MX_LAYOUT_MATRIX && fa.block == 16)      // bfloat16 form of the layout
        return gemm_bf16(batch, M, N, K, A_packed, B_packed, Y, ldy, batch_stride_y, (hipStream_t)stream);
    if (layout == MX_LAYOUT_MATRIX)
        return gemm_scaled(batch, M, N, K, A_packed, fa, B_packed, fb, Y, ldy, batch_stride_y, (hipStream_t)stream);
    const FragGeom ga = frag_geom(M, K, fa.block, fa.mant_bits);
    if (ceil_div(ga.groups, 4) > 65535) return MX_ERR_UNSUPPORTED;
    const GemmArgs g = fragment_args(M, N, K, A_packed, fa, B_packed, fb, Y, ldy, batch_stride_y);
    hipStream_t st = (hipStream_t)stream;
    if (M <= 2) {      // one or two rows: dot-product kernel; three to eight: MFMA streaming kernel
        const mx_status s = gemv_dot(g, fa.mant_bits, fb.mant_bits, fa.block, batch, st);
        if (s != MX_ERR_UNSUPPORTED) return s;
    }
    switch (fa.block) {
        case 16: return gemm_block16(g, fa.mant_bits, fb.mant_bits, batch, st);
        case 32: return gemm_block32(g, fa.mant_bits, fb.mant_bits, batch, st);
        case 64: return gemm_block64(g, fa.mant_bits, fb.mant_bits, batch, st);
    }
    return MX_ERR_UNSUPPORTED;
}

extern "C" mx_status mx_gemm_q(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A_packed, mx_format fa,
                               const void* B_packed, mx_format fb, int32_t layout, const uint8_t* bias_mant,
                               const uint8_t* bias_exps, mx_format fbias, mx_format fo, void* out_packed,
                               void* stream) {
    if (!format_ok_quant(fa) || !format_ok_quant(fb) || !format_ok_quant(fo)) return MX_ERR_BAD_ARG;
    if (fa.block != fb.block || fa.exp_bits != fb.exp_bits) return MX_ERR_BAD_ARG;
    const bool with_bias = bias_mant != nullptr || bias_exps != nullptr;
    if (with_bias && (!bias_mant || !bias_exps || !format_ok_quant(fbias) || fbias.block != fo.block ||
                      fbias.block_rows != 1)) return MX_ERR_BAD_ARG;
    if (layout != MX_LAYOUT_FRAGMENT && layout != MX_LAYOUT_MATRIX) return MX_ERR_BAD_ARG;
    if (batch < 0 || M < 0 || N < 0 || K < 0 || K % fa.block != 0 || N % fo.block != 0 || M % fo.block_rows != 0)
        return MX_ERR_BAD_ARG;
    // built for the matrix layout, inputs and output in the same form of it (blocks of 16, or of 32/64)
    if (layout != MX_LAYOUT_MATRIX || !matrix_format_ok(fa) || !matrix_format_ok(fo)) return MX_ERR_UNSUPPORTED;
    if ((fa.block == 16) != (fo.block == 16)) return MX_ERR_UNSUPPORTED;
    if (batch == 0 || M == 0 || N == 0) return MX_OK;
    if (!out_packed || ((uintptr_t)out_packed & 255)) return MX_ERR_BAD_ARG;
    if (K > 0 && (!A_packed || !B_packed)) return MX_ERR_BAD_ARG;
    if (((uintptr_t)A_packed & 255) || ((uintptr_t)B_packed & 255)) return MX_ERR_BAD_ARG;
    if (batch > 65535) return MX_ERR_UNSUPPORTED;
    if (fa.block == 16)
        return gemm_bf16_q(batch, M, N, K, A_packed, B_packed, bias_mant, bias_exps, fbias, fo, out_packed,
                           (hipStream_t)stream);
    return gemm_scaled_q(batch, M, N, K, A_packed, fa, B_packed, fb, bias_mant, bias_exps, fbias, fo, out_packed,
                         (hipStream_t)stream);
}
