// Host interface of the one-launch decode linear (mx_decode.hip) and the layout of mx_linear's workspace.
#pragma once
#include "mx_common.h"

namespace mx {

// Workspace of mx_linear: [arrival counters][partial sums of the K slices][packed activations of the
// two-launch form].  The counters must be zero when a call starts; every call leaves them zero.
constexpr int64_t kDecodeMaxGroups = 4096;                       // column groups of 32: N <= 131072
constexpr int64_t kDecodeCounterBytes = kDecodeMaxGroups * 4;
constexpr int64_t kDecodeMaxSplit = 64;

struct DecodePlan {
    bool ok;                 // the one-launch kernel takes the shape
    int32_t ksplit, slice;   // K slices, records (chunks of four blocks) per slice
    int64_t partial_floats;  // fp32 partial sums kept in the workspace (0 with one slice)
};
DecodePlan decode_plan(int64_t M, int64_t K, int64_t N, int block, int wb);

// Byte offset of the packed activations inside the workspace, and the workspace's size.
inline int64_t decode_packed_offset(const DecodePlan& p) {
    return kDecodeCounterBytes + (p.partial_floats * 4 + 255) / 256 * 256;
}

// x: fp32 [M x K], 16-byte aligned rows.  MX_ERR_UNSUPPORTED when decode_plan says no.
mx_status linear_decode(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx, void* workspace,
                        const void* B_packed, int64_t N, mx_format fb, float* Y, int64_t ldy, hipStream_t st);

}  // namespace mx
