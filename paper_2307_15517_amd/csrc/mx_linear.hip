// Decode-time linear layer: fp32 activations (M <= 8 rows) are quantized to MXInt and written
// straight into the fragment layout, then the decode kernel of mx_gemm streams the packed weights.
// The quantizer arithmetic is the one of mx_quantize (Section 4.1 format; Section 3.2 emulation
// semantics: quantize the input, then the operator).
#include "mx_decode.h"
#include "mx_gemm.h"

namespace mx {
namespace {

struct LinQuantArgs {
    const float* x;
    uint8_t* packed;
    int64_t M;           // rows holding data
    int64_t rows_out;    // rows covered by the launch; whole row groups of 32 are written
    int64_t K, row_stride, batch_stride, chunks, matrix_bytes;
    int32_t piece, record, bias, emax;
    int32_t vec;         // x and its strides allow 16-byte loads
    int32_t brows;       // 2: rows 2p and 2p+1 (adjacent lanes) share their exponents
};

// One wave per record of the fragment layout (32 rows x 4 blocks); four waves, i.e. four consecutive
// chunks, per workgroup; grid.y = batch.  A record is built in passes of 64 columns: the wave reads
// 32 rows x 256 bytes as whole row segments (four rows per load instruction) and turns them through
// its own LDS tile, after which lane 32*h + i holds half h of every block of row i that the pass
// covers; the block maximum is completed with the partner lane.  The finished pieces and exponent
// bytes go back through the same LDS tile, so that the record leaves as one contiguous run of
// 16-byte stores.  Slots past K and rows in [M, 32*groups) hold zero mantissas and exponent byte 0.
constexpr int kLqRowPitch = 256 + 16;     // bytes; the 16-byte skew spreads the lanes' rows over the banks
constexpr int kLqTile = 32 * kLqRowPitch; // also holds the largest record (64 * 128 + 128 bytes)

// VEC: 16-byte loads (x and its strides allow them).  A template parameter, not a run-time branch: with
// both forms in one function the compiler folds them into the element-wise one.
template <int W, int B, int RND, bool VEC>
__global__ __launch_bounds__(256) void quantize_to_fragments_kernel(LinQuantArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * kLqTile];
    constexpr int kPieceDw = B * W / 16;          // dwords of one lane piece: four half blocks
    constexpr int kPasses = 4 * B / 64;           // 64 columns per pass
    constexpr int kBlocksPerPass = 64 / B > 0 ? 64 / B : 1;
    constexpr int kHalf = B / 2;
    constexpr int kPerPass = B >= 64 ? 32 : kBlocksPerPass * kHalf;   // elements of a lane per pass (always 32)
    static_assert(kPerPass == 32, "a lane quantizes 32 elements per pass");
    constexpr float qmax = (float)((1 << (W - 1)) - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    uint8_t* lds = lds_all + wv * kLqTile;
    const int i = lane & 31, h = lane >> 5;
    const int64_t cq = (a.chunks + 3) / 4;
    const int64_t grp = blockIdx.x / cq, c = (blockIdx.x - grp * cq) * 4 + wv;
    if (c >= a.chunks) return;                    // whole wave; no workgroup barrier below
    const float* xb = a.x + blockIdx.y * a.batch_stride;

    uint32_t piece[kPieceDw];
#pragma unroll
    for (int d = 0; d < kPieceDw; ++d) piece[d] = 0;
    uint32_t exps = 0;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        float4 in[8];
        const int64_t col = c * (4 * B) + p * 64 + (lane & 15) * 4;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int64_t row = grp * 32 + 4 * r + (lane >> 4);
            in[r] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < a.M && col < a.K) {
                const float* src = xb + row * a.row_stride + col;
                if constexpr (VEC) in[r] = *reinterpret_cast<const float4*>(src);
                else in[r] = make_float4(src[0], src[1], src[2], src[3]);
            }
        }
        if (p > 0) __builtin_amdgcn_wave_barrier();          // the previous pass has read its tile
#pragma unroll
        for (int r = 0; r < 8; ++r)
            *reinterpret_cast<float4*>(lds + (4 * r + (lane >> 4)) * kLqRowPitch + (lane & 15) * 16) = in[r];
        __builtin_amdgcn_wave_barrier();

        // the lane's 32 elements of this pass: B/2 consecutive floats of each of its 64/B blocks
        float v[32];
#pragma unroll
        for (int jj = 0; jj < kBlocksPerPass; ++jj) {
            constexpr int kRun = B >= 64 ? 32 : kHalf;       // consecutive floats per block
            const uint8_t* src = lds + i * kLqRowPitch + (jj * (B >= 64 ? 64 : B) + h * kRun) * 4;
#pragma unroll
            for (int q4 = 0; q4 < kRun / 4; ++q4) {
                const float4 t = *reinterpret_cast<const float4*>(src + q4 * 16);
                v[jj * kRun + 4 * q4] = t.x; v[jj * kRun + 4 * q4 + 1] = t.y;
                v[jj * kRun + 4 * q4 + 2] = t.z; v[jj * kRun + 4 * q4 + 3] = t.w;
            }
        }
        const bool row_in = grp * 32 + i < a.M;
#pragma unroll
        for (int jj = 0; jj < kBlocksPerPass; ++jj) {
            constexpr int kRun = B >= 64 ? 32 : kHalf;
            const int j = p * kBlocksPerPass + jj;           // block slot inside the chunk (compile time)
            uint32_t am = 0;
#pragma unroll
            for (int k = 0; k < kRun; ++k) {
                const uint32_t ab = __float_as_uint(v[jj * kRun + k]) & 0x7fffffffu;
                am = ab > am ? ab : am;
            }
            const uint32_t o = (uint32_t)__shfl_xor((int)am, 32, 64);
            am = o > am ? o : am;
            if (a.brows == 2) {         // two-row blocks: the neighbouring lane holds the other row
                const uint32_t o2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);
                am = o2 > am ? o2 : am;
            }
            const int ef = (int)(am >> 23);
            int E = ef == 0 ? -127 : ef - 127;
            E = E < -a.bias ? -a.bias : E;
            E = E > a.emax ? a.emax : E;
            const int shift = (W - 2) - E;
            const bool inside = row_in && (c * 4 + j) * B < a.K;
            exps |= (inside ? (uint32_t)(E + a.bias) : 0u) << (8 * j);
#pragma unroll
            for (int k = 0; k < kRun; ++k) {
                const float s = __builtin_ldexpf(v[jj * kRun + k], shift);
                float r = RND == MX_RNE ? __builtin_rintf(s) : __builtin_truncf(s);
                r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
                const uint32_t code = (uint32_t)(int)r & ((1u << W) - 1u);
                int pos = k;                                   // element position inside the half block
                if (W == 4) {                                  // nibble order e0 e4 e1 e5 e2 e6 e3 e7 per 8
                    const int t8 = k & 7;
                    pos = (k & ~7) + (t8 < 4 ? 2 * t8 : 2 * (t8 - 4) + 1);
                }
                const int bit = (j * kHalf + pos) * W;         // compile time after unrolling
                piece[bit >> 5] |= code << (bit & 31);
                if ((bit & 31) + W > 32) piece[(bit >> 5) + 1] |= code >> (32 - (bit & 31));
            }
        }
    }
    // record image in LDS: 64 pieces, then the 32 exponent dwords
    __builtin_amdgcn_wave_barrier();
    uint32_t* img = reinterpret_cast<uint32_t*>(lds);
#pragma unroll
    for (int d = 0; d < kPieceDw; ++d) img[lane * kPieceDw + d] = piece[d];
    if (h == 0) img[64 * kPieceDw + i] = exps;
    __builtin_amdgcn_wave_barrier();
    constexpr int kRec16 = (64 * kPieceDw * 4 + 128) / 16;
    uint4* dst = reinterpret_cast<uint4*>(a.packed + blockIdx.y * a.matrix_bytes + (grp * a.chunks + c) * a.record);
#pragma unroll
    for (int it = 0; it < (kRec16 + 63) / 64; ++it) {
        const int idx = it * 64 + lane;
        if (idx < kRec16) dst[idx] = reinterpret_cast<const uint4*>(lds)[idx];
    }
}

template <int W, int B>
mx_status launch_lq(const LinQuantArgs& a, int64_t batch, int rnd, hipStream_t st) {
    dim3 grid((unsigned)(ceil_div(a.rows_out, 32) * ceil_div(a.chunks, 4)), (unsigned)batch);
    if (rnd == MX_RNE) {
        if (a.vec) hipLaunchKernelGGL((quantize_to_fragments_kernel<W, B, MX_RNE, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((quantize_to_fragments_kernel<W, B, MX_RNE, false>), grid, dim3(256), 0, st, a);
    } else {
        if (a.vec) hipLaunchKernelGGL((quantize_to_fragments_kernel<W, B, MX_RTZ, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((quantize_to_fragments_kernel<W, B, MX_RTZ, false>), grid, dim3(256), 0, st, a);
    }
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
    a.vec = (((uintptr_t)x & 15) == 0 && (row_stride & 3) == 0 && (batch_stride & 3) == 0) ? 1 : 0;
    a.brows = f.block_rows;
    if (ceil_div(rows_out, 32) * ceil_div(ga.chunks, 4) > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
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

// Bytes of the workspace mx_linear needs for this call: arrival counters, partial sums of the K slices, and the
// packed activations of the two-launch form.  0 on a bad argument.
extern "C" size_t mx_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, mx_format fx, mx_format fb,
                                            int32_t layout) {
    if (!format_ok_gemm(fx) || !format_ok_gemm(fb) || fx.block != fb.block || layout != MX_LAYOUT_FRAGMENT) return 0;
    if (M < 0 || M > 8 || N < 0 || K < 0 || K % fx.block != 0) return 0;
    const DecodePlan p = decode_plan(M, K, N, fb.block, fb.mant_bits);
    return (size_t)(decode_packed_offset(p) + frag_geom(M, K, fx.block, fx.mant_bits).matrix);
}

namespace {

// Argument checks of mx_linear that need no workspace.  MX_OK means "go on"; *done is set when there is nothing to do.
mx_status linear_check(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx, const void* B_packed,
                       int64_t N, mx_format fb, int32_t layout, float* Y, int64_t ldy, bool* done) {
    *done = false;
    if (!format_ok_quant(fx) || !format_ok_quant(fb)) return MX_ERR_BAD_ARG;
    if (fx.block != fb.block || fx.exp_bits != fb.exp_bits) return MX_ERR_BAD_ARG;
    if (!format_ok_gemm(fx)) return MX_ERR_UNSUPPORTED;
    if (fx.block_rows == 2 && M % 2 != 0) return MX_ERR_BAD_ARG;      // rows 2p and 2p+1 share their exponents
    if (layout != MX_LAYOUT_FRAGMENT) return layout == MX_LAYOUT_MATRIX ? MX_ERR_UNSUPPORTED : MX_ERR_BAD_ARG;
    if (M < 0 || N < 0 || K < 0 || K % fx.block != 0 || row_stride < K || ldy < N) return MX_ERR_BAD_ARG;
    if (M > 8) return MX_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) { *done = true; return MX_OK; }
    if (!Y || ((uintptr_t)Y & 3)) return MX_ERR_BAD_ARG;
    if (K > 0 && (!x || !B_packed)) return MX_ERR_BAD_ARG;
    if (((uintptr_t)x & 3) || ((uintptr_t)B_packed & 255)) return MX_ERR_BAD_ARG;
    return MX_OK;
}

// The work of mx_linear on checked arguments and a workspace whose counters are zero.
mx_status linear_run(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx, void* workspace,
                     const void* B_packed, int64_t N, mx_format fb, int32_t layout, float* Y, int64_t ldy,
                     void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const DecodePlan p = decode_plan(M, K, N, fb.block, fb.mant_bits);
    const bool fused_ok = K > 0 && fx.block_rows == 1 && ((uintptr_t)x & 15) == 0 && (row_stride & 3) == 0;
    if (fused_ok && M <= 2) {
        // one launch, one workgroup per column group: the dot-product decode kernel quantizes the activations on
        // its way into LDS; nothing passes between workgroups, the workspace is not touched
        const GemmArgs g = fragment_args(M, N, K, nullptr, fx, B_packed, fb, Y, ldy, M * ldy);
        const mx_status s = gemv_dot(g, fx.mant_bits, fb.mant_bits, fx.block, 1, st, x, row_stride, &fx);
        if (s != MX_ERR_UNSUPPORTED) return s;
    }
    if (fused_ok && M > 2 && p.ok) {
        // one launch: column groups x K slices, the activations of a slice quantized inside the kernel
        const mx_status s = linear_decode(x, M, K, row_stride, fx, workspace, B_packed, N, fb, Y, ldy, st);
        if (s != MX_ERR_UNSUPPORTED) return s;
    }
    // two launches: quantize into the fragment layout, then the decode product of mx_gemm
    void* packed = (uint8_t*)workspace + decode_packed_offset(p);
    if (K > 0) {
        mx_status s = run_lq(x, 1, M, M, K, row_stride, 0, fx, (uint8_t*)packed, st);
        if (s != MX_OK) return s;
    }
    return mx_gemm(1, M, N, K, packed, fx, B_packed, fb, layout, Y, ldy, M * ldy, stream);
}

// Device memory the library owns, for callers that cannot hand over a workspace: one array per GPU, there from the
// moment the library is loaded until the process ends.  Host code never uses this name as an address -- it is the
// host-side stand-in of a device symbol; the address on the current device comes from hipGetSymbolAddress (below).
constexpr int64_t kStaticWorkspaceBytes = 8 << 20;
static __device__ __align__(256) uint8_t static_workspace[kStaticWorkspaceBytes];

__global__ void clear_counters_kernel(uint32_t* counters) {
    for (int64_t i = threadIdx.x; i < kDecodeCounterBytes / 4; i += blockDim.x) counters[i] = 0u;
}

// Address of static_workspace on the current device, looked up once per device.
void* static_workspace_ptr() {
    static std::atomic<void*> ptrs[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return nullptr;
    void* p = ptrs[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(static_workspace)) != hipSuccess || !p) return nullptr;
    ptrs[dev].store(p, std::memory_order_release);
    return p;
}

}  // namespace

extern "C" mx_status mx_linear(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx,
                               void* workspace, const void* B_packed, int64_t N, mx_format fb,
                               int32_t layout, float* Y, int64_t ldy, void* stream) {
    bool done;
    const mx_status s = linear_check(x, M, K, row_stride, fx, B_packed, N, fb, layout, Y, ldy, &done);
    if (s != MX_OK || done) return s;
    if (K > 0 && !workspace) return MX_ERR_BAD_ARG;
    if ((uintptr_t)workspace & 255) return MX_ERR_BAD_ARG;
    return linear_run(x, M, K, row_stride, fx, workspace, B_packed, N, fb, layout, Y, ldy, stream);
}

extern "C" size_t mx_linear_static_workspace_max(void) { return (size_t)kStaticWorkspaceBytes; }

extern "C" mx_status mx_linear_static_workspace(const float* x, int64_t M, int64_t K, int64_t row_stride,
                                                mx_format fx, const void* B_packed, int64_t N, mx_format fb,
                                                int32_t layout, float* Y, int64_t ldy, void* stream) {
    bool done;
    const mx_status s = linear_check(x, M, K, row_stride, fx, B_packed, N, fb, layout, Y, ldy, &done);
    if (s != MX_OK || done) return s;
    const size_t need = mx_linear_workspace_bytes(M, K, N, fx, fb, layout);
    if (need == 0) return MX_ERR_BAD_ARG;
    if (need > (size_t)kStaticWorkspaceBytes) return MX_ERR_UNSUPPORTED;      // the shape needs more than the library holds
    void* ws = static_workspace_ptr();
    if (!ws) return MX_ERR_DEVICE;
    // the array keeps what the last call on this GPU left: the counters start every call at zero (a fill kernel,
    // not a memset node, so that the call can be captured into a graph)
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, (uint32_t*)ws);
    MX_HIP_LAUNCH_CHECK();
    return linear_run(x, M, K, row_stride, fx, ws, B_packed, N, fb, layout, Y, ldy, stream);
}
