// mx_cast: MXInt (block, es, ws) -> MXInt (block, ed, wd) on the canonical form, in integer
// arithmetic, without going through floating point (Section 4 of the paper, the paragraph on
// mixed-precision quantization: casting mantissas is bit extension or truncation, the exponent
// takes a shift).  The result is what quantizing the block's exact values to the destination
// format gives: with mx = max |q_i| and p = floor(log2 mx) the new shared exponent is
// E' = E - (ws-2) + p, clamped to the destination's range, and every mantissa becomes
// q_i * 2^sh, sh = (E - (ws-2)) - (E' - (wd-2)): a left shift (exact) or a right shift with the
// destination's rounding, then saturation at +-qmax.  A block of zeros stores exponent byte 0.
//
// The canonical arrays are contiguous over batch, rows and columns, so the tensor is treated as
// one run of blocks.  One thread converts 32 consecutive elements (ws dwords in, wd dwords out;
// four, two or one block, or half of a block of 64 whose maximum is completed with the
// neighbouring lane).  HBM-bound: (ws + wd)/8 + 2/block bytes per element.
#include "mx_common.h"

namespace mx {
namespace {

struct CastArgs {
    const uint8_t* mant;
    const uint8_t* exps;
    uint8_t* mant_out;
    uint8_t* exps_out;
    int64_t elems;             // batch * rows * cols
    int32_t bias_s, bias_d, emin_d, emax_d;
    int32_t vec;               // both mantissa arrays are 16-byte aligned
    int64_t runs_per_row;      // two-row blocks: cols / 32
};

template <int WS, int WD, int B, int RND>
__global__ __launch_bounds__(256) void cast_kernel(CastArgs a) {
    constexpr int NB = B >= 32 ? 1 : 32 / B;          // blocks (or the half block) of a thread
    constexpr int BE = B >= 32 ? 32 : B;              // elements of each
    constexpr int qmax = (1 << (WD - 1)) - 1;
    const int64_t run = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t e0 = run * 32;
    // elements of this run that exist: 32, or a whole number of blocks at the end of the tensor
    // (every lane goes through the arithmetic: a block of 64 needs its neighbour)
    const int n = e0 >= a.elems ? 0 : (a.elems - e0 >= 32 ? 32 : (int)(a.elems - e0));

    uint32_t in[WS + 1];
#pragma unroll
    for (int d = 0; d <= WS; ++d) in[d] = 0;
    const uint8_t* src = a.mant + run * (4 * WS);
    if (n == 32) {
        if (WS % 4 == 0 && a.vec) {                   // 16 or 32 bytes per lane, 16-byte aligned
#pragma unroll
            for (int d = 0; d < WS / 4; ++d) {
                const uint4 v = reinterpret_cast<const uint4*>(src)[d];
                in[4 * d] = v.x; in[4 * d + 1] = v.y; in[4 * d + 2] = v.z; in[4 * d + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int d = 0; d < WS; ++d) in[d] = reinterpret_cast<const uint32_t*>(src)[d];
        }
    } else {
        for (int byte = 0; byte < n * WS / 8; ++byte) in[byte >> 2] |= (uint32_t)src[byte] << (8 * (byte & 3));
    }
    int q[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) q[i] = stream_get<WS>(in, i * WS);

    uint32_t out[WD];
#pragma unroll
    for (int d = 0; d < WD; ++d) out[d] = 0;
    const int64_t blk0 = e0 / B;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        int mx = 0;
#pragma unroll
        for (int i = 0; i < BE; ++i) {
            const int v = q[j * BE + i];
            const int m = v < 0 ? -v : v;
            mx = m > mx ? m : mx;
        }
        if (B == 64) {                                // lanes 2t, 2t+1 hold the halves of one block
            const int o = __builtin_amdgcn_update_dpp(0, mx, 0xB1, 0xF, 0xF, true);
            mx = o > mx ? o : mx;
        }
        const bool have = j * BE < n;
        int ebyte = 0;
        if (have && mx != 0) {
            const int E = (int)a.exps[blk0 + j] - a.bias_s;
            int E2 = E - (WS - 2) + (31 - __builtin_clz((unsigned)mx));
            E2 = E2 < a.emin_d ? a.emin_d : E2;
            E2 = E2 > a.emax_d ? a.emax_d : E2;
            int sh = (E - (WS - 2)) - (E2 - (WD - 2));
            ebyte = E2 + a.bias_d;
            // |q| <= 128: any shift beyond 16 either way gives the same result as 16
            sh = sh > 16 ? 16 : (sh < -16 ? -16 : sh);
#pragma unroll
            for (int i = 0; i < BE; ++i) {
                const int v = q[j * BE + i];
                int r;
                if (sh >= 0) {
                    r = v << sh;                       // |v| << 16 stays inside int32
                } else {
                    // arithmetic right shift = floor; to nearest with ties to even: add half - 1 + (the bit
                    // that becomes the last one), then floor; toward zero: add 2^k - 1 to negatives, then floor
                    const int k = -sh;
                    if (RND == MX_RNE) r = (v + ((1 << (k - 1)) - 1) + ((v >> k) & 1)) >> k;
                    else r = (v + ((v >> 31) & ((1 << k) - 1))) >> k;
                }
                r = r > qmax ? qmax : (r < -qmax ? -qmax : r);
                const int bit = (j * BE + i) * WD;    // compile time after unrolling
                const uint32_t code = (uint32_t)r & ((1u << WD) - 1u);
                out[bit >> 5] |= code << (bit & 31);
                if ((bit & 31) + WD > 32) out[(bit >> 5) + 1] |= code >> (32 - (bit & 31));
            }
        }
        // one exponent byte per block: every block of the thread, or the even lane for a block of 64
        if (have && (B < 64 || (e0 & 63) == 0)) a.exps_out[blk0 + j] = (uint8_t)ebyte;
    }
    uint8_t* dst = a.mant_out + run * (4 * WD);
    if (n == 32) {
        if (WD % 4 == 0 && a.vec) {
#pragma unroll
            for (int d = 0; d < WD / 4; ++d)
                reinterpret_cast<uint4*>(dst)[d] = make_uint4(out[4 * d], out[4 * d + 1], out[4 * d + 2], out[4 * d + 3]);
        } else {
#pragma unroll
            for (int d = 0; d < WD; ++d) reinterpret_cast<uint32_t*>(dst)[d] = out[d];
        }
    } else {
        for (int byte = 0; byte < n * WD / 8; ++byte) dst[byte] = (uint8_t)(out[byte >> 2] >> (8 * (byte & 3)));
    }
}

// Two-row blocks (block shape (B, 2)): one thread converts the same 32 columns of rows 2p and 2p+1, which
// share their exponents; the block maximum runs over both rows.  cols is a multiple of 32 here, so every
// run is whole and dword-aligned.
template <int WS, int WD, int B, int RND>
__global__ __launch_bounds__(256) void cast_rows2_kernel(CastArgs a) {
    constexpr int NB = B >= 32 ? 1 : 32 / B;
    constexpr int BE = B >= 32 ? 32 : B;
    constexpr int qmax = (1 << (WD - 1)) - 1;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t pairs = a.elems / (64 * a.runs_per_row);
    const bool live = t < pairs * a.runs_per_row;
    const int64_t pr = live ? t / a.runs_per_row : 0, rr = live ? t - pr * a.runs_per_row : 0;
    int q[2][32];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        uint32_t in[WS + 1];
#pragma unroll
        for (int d = 0; d <= WS; ++d) in[d] = 0;
        if (live) {
            const uint32_t* src = reinterpret_cast<const uint32_t*>(a.mant + ((2 * pr + r) * a.runs_per_row + rr) * (4 * WS));
#pragma unroll
            for (int d = 0; d < WS; ++d) in[d] = src[d];
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) q[r][i] = stream_get<WS>(in, i * WS);
    }
    uint32_t out[2][WD];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int d = 0; d < WD; ++d) out[r][d] = 0;
    const int64_t blk0 = (pr * a.runs_per_row + rr) * 32 / B;        // exponent index: [pair][block]
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        int mx = 0;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < BE; ++i) {
                const int v = q[r][j * BE + i];
                const int m = v < 0 ? -v : v;
                mx = m > mx ? m : mx;
            }
        if (B == 64) {
            const int o = __builtin_amdgcn_update_dpp(0, mx, 0xB1, 0xF, 0xF, true);
            mx = o > mx ? o : mx;
        }
        int ebyte = 0;
        if (live && mx != 0) {
            const int E = (int)a.exps[blk0 + j] - a.bias_s;
            int E2 = E - (WS - 2) + (31 - __builtin_clz((unsigned)mx));
            E2 = E2 < a.emin_d ? a.emin_d : E2;
            E2 = E2 > a.emax_d ? a.emax_d : E2;
            int sh = (E - (WS - 2)) - (E2 - (WD - 2));
            ebyte = E2 + a.bias_d;
            sh = sh > 16 ? 16 : (sh < -16 ? -16 : sh);
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int i = 0; i < BE; ++i) {
                    const int v = q[r][j * BE + i];
                    int res;
                    if (sh >= 0) {
                        res = v << sh;
                    } else {
                        const int k = -sh;
                        if (RND == MX_RNE) res = (v + ((1 << (k - 1)) - 1) + ((v >> k) & 1)) >> k;
                        else res = (v + ((v >> 31) & ((1 << k) - 1))) >> k;
                    }
                    res = res > qmax ? qmax : (res < -qmax ? -qmax : res);
                    const int bit = (j * BE + i) * WD;
                    const uint32_t code = (uint32_t)res & ((1u << WD) - 1u);
                    out[r][bit >> 5] |= code << (bit & 31);
                    if ((bit & 31) + WD > 32) out[r][(bit >> 5) + 1] |= code >> (32 - (bit & 31));
                }
        }
        if (live && (B < 64 || (rr & 1) == 0)) a.exps_out[blk0 + j] = (uint8_t)ebyte;
    }
    if (live) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(a.mant_out + ((2 * pr + r) * a.runs_per_row + rr) * (4 * WD));
#pragma unroll
            for (int d = 0; d < WD; ++d) dst[d] = out[r][d];
        }
    }
}

template <int WS, int WD, int B>
mx_status launch_cast(const CastArgs& a, int rnd, hipStream_t st) {
    if (a.runs_per_row > 0) {
        const int64_t items = a.elems / 64;
        if (ceil_div(items, 256) > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
        dim3 grid((unsigned)ceil_div(items, 256));
        if (rnd == MX_RNE) hipLaunchKernelGGL((cast_rows2_kernel<WS, WD, B, MX_RNE>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((cast_rows2_kernel<WS, WD, B, MX_RTZ>), grid, dim3(256), 0, st, a);
        MX_HIP_LAUNCH_CHECK();
        return MX_OK;
    }
    const int64_t runs = ceil_div(a.elems, 32);
    if (ceil_div(runs, 256) > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)ceil_div(runs, 256));
    if (rnd == MX_RNE) hipLaunchKernelGGL((cast_kernel<WS, WD, B, MX_RNE>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((cast_kernel<WS, WD, B, MX_RTZ>), grid, dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int WS, int WD>
mx_status dispatch_block(const CastArgs& a, int block, int rnd, hipStream_t st) {
    switch (block) {
        case 8: return launch_cast<WS, WD, 8>(a, rnd, st);
        case 16: return launch_cast<WS, WD, 16>(a, rnd, st);
        case 32: return launch_cast<WS, WD, 32>(a, rnd, st);
        case 64: return launch_cast<WS, WD, 64>(a, rnd, st);
    }
    return MX_ERR_BAD_ARG;
}

template <int WS>
mx_status dispatch_wd(const CastArgs& a, int wd, int block, int rnd, hipStream_t st) {
    switch (wd) {
        case 2: return dispatch_block<WS, 2>(a, block, rnd, st);
        case 3: return dispatch_block<WS, 3>(a, block, rnd, st);
        case 4: return dispatch_block<WS, 4>(a, block, rnd, st);
        case 5: return dispatch_block<WS, 5>(a, block, rnd, st);
        case 6: return dispatch_block<WS, 6>(a, block, rnd, st);
        case 7: return dispatch_block<WS, 7>(a, block, rnd, st);
        case 8: return dispatch_block<WS, 8>(a, block, rnd, st);
    }
    return MX_ERR_BAD_ARG;
}

}  // namespace
}  // namespace mx

using namespace mx;

extern "C" mx_status mx_cast(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                             mx_format fs, mx_format fd, uint8_t* mant_out, uint8_t* exps_out, void* stream) {
    if (!format_ok_quant(fs) || !format_ok_quant(fd) || fs.block != fd.block) return MX_ERR_BAD_ARG;
    if (batch < 0 || rows < 0 || cols < 0 || cols % fs.block != 0) return MX_ERR_BAD_ARG;
    if (fs.block_rows != fd.block_rows) return MX_ERR_BAD_ARG;
    if (fs.block_rows == 2 && rows % 2 != 0) return MX_ERR_BAD_ARG;
    if (fs.block_rows == 2 && cols % 32 != 0) return MX_ERR_UNSUPPORTED;     // two-row blocks: whole 32-element runs per row
    if (batch == 0 || rows == 0 || cols == 0) return MX_OK;
    if (!mant || !exps || !mant_out || !exps_out) return MX_ERR_BAD_ARG;
    if (((uintptr_t)mant & 3) || ((uintptr_t)mant_out & 3)) return MX_ERR_BAD_ARG;
    if (mant == mant_out || exps == exps_out) return MX_ERR_BAD_ARG;
    CastArgs a;
    a.mant = mant; a.exps = exps; a.mant_out = mant_out; a.exps_out = exps_out;
    a.elems = batch * rows * cols;
    a.vec = ((((uintptr_t)mant) | ((uintptr_t)mant_out)) & 15) == 0 ? 1 : 0;
    a.runs_per_row = fs.block_rows == 2 ? cols / 32 : 0;
    a.bias_s = (1 << (fs.exp_bits - 1)) - 1;
    a.bias_d = (1 << (fd.exp_bits - 1)) - 1;
    a.emin_d = -a.bias_d;
    a.emax_d = ((1 << fd.exp_bits) - 1) - a.bias_d;
    hipStream_t st = (hipStream_t)stream;
    switch (fs.mant_bits) {
        case 2: return dispatch_wd<2>(a, fd.mant_bits, fs.block, fd.rounding, st);
        case 3: return dispatch_wd<3>(a, fd.mant_bits, fs.block, fd.rounding, st);
        case 4: return dispatch_wd<4>(a, fd.mant_bits, fs.block, fd.rounding, st);
        case 5: return dispatch_wd<5>(a, fd.mant_bits, fs.block, fd.rounding, st);
        case 6: return dispatch_wd<6>(a, fd.mant_bits, fs.block, fd.rounding, st);
        case 7: return dispatch_wd<7>(a, fd.mant_bits, fs.block, fd.rounding, st);
        case 8: return dispatch_wd<8>(a, fd.mant_bits, fs.block, fd.rounding, st);
    }
    return MX_ERR_BAD_ARG;
}
