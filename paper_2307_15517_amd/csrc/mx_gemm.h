// Arguments shared by the product kernels and their host dispatch.
#pragma once
#include "mx_common.h"

namespace mx {

struct GemmArgs {
    const uint8_t* A;
    const uint8_t* B;
    float* Y;
    int64_t M, N;
    int64_t groupsA, groupsB, chunks;
    int64_t matrixA, matrixB;     // packed bytes per batch entry
    int64_t ldy, batch_stride_y;
    int32_t recordA, recordB;
    int32_t eadj;                 // -2*bias - (wa-2) - (wb-2)
    int64_t K;
};

// One instance per block size, each compiled in its own translation unit.
mx_status gemm_block16(const GemmArgs& g, int wa, int wb, int64_t batch, hipStream_t st);
mx_status gemm_block32(const GemmArgs& g, int wa, int wb, int64_t batch, hipStream_t st);
mx_status gemm_block64(const GemmArgs& g, int wa, int wb, int64_t batch, hipStream_t st);

// Decode path for M <= 4, used for M <= 2 (mx_gemv_dot.hip); MX_ERR_UNSUPPORTED when it does not apply.
mx_status gemv_dot(const GemmArgs& g, int wa, int wb, int block, int64_t batch, hipStream_t st,
                   const float* x = nullptr, int64_t x_stride = 0, const mx_format* fx = nullptr);
// Fills the kernel arguments of the fragment-layout product (shared by mx_gemm and mx_linear).
GemmArgs fragment_args(int64_t M, int64_t N, int64_t K, const void* A, mx_format fa, const void* B, mx_format fb,
                       float* Y, int64_t ldy, int64_t batch_stride_y);

}  // namespace mx
