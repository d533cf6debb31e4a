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

typedef short s2v __attribute__((ext_vector_type(2)));
typedef unsigned short u2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ s2v splat(int v) { s2v r; r.x = (short)v; r.y = (short)v; return r; }

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
    // Two elements per register as 16-bit halves (|q| <= 128, and every intermediate of the shift below fits
    // 16 bits), so the arithmetic runs as packed 16-bit instructions: of the four elements 4g..4g+3, pair
    // 2g holds (4g, 4g+2) and pair 2g+1 holds (4g+1, 4g+3) -- for 8-bit sources these are the even and the
    // odd bytes of one dword, sign-extended in place.
    s2v pr[16];
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        if (WS == 8) {
            const s2v x = __builtin_bit_cast(s2v, in[g]);
            pr[2 * g] = __builtin_bit_cast(s2v, __builtin_bit_cast(u2v, in[g]) << (unsigned short)8) >> splat(8);
            pr[2 * g + 1] = x >> splat(8);
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                s2v v;
                v.x = (short)stream_get<WS>(in, (4 * g + p) * WS);
                v.y = (short)stream_get<WS>(in, (4 * g + p + 2) * WS);
                pr[2 * g + p] = v;
            }
        }
    }

    uint32_t out[WD];
#pragma unroll
    for (int d = 0; d < WD; ++d) out[d] = 0;
    const int64_t blk0 = e0 / B;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        constexpr int NP = BE / 2;                    // pairs of the block
        s2v hi = pr[j * NP], lo = pr[j * NP];
#pragma unroll
        for (int t = 1; t < NP; ++t) {
            hi = __builtin_elementwise_max(hi, pr[j * NP + t]);
            lo = __builtin_elementwise_min(lo, pr[j * NP + t]);
        }
        int mx = max(max((int)hi.x, (int)hi.y), max(-(int)lo.x, -(int)lo.y));
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
            const int sh = (E - (WS - 2)) - (E2 - (WD - 2));
            ebyte = E2 + a.bias_d;
            // |q| <= 128 and qmax <= 127: a left shift beyond 7 saturates every nonzero element like 7 does, a
            // right shift beyond 9 gives zero like 9 does, and within these limits nothing leaves 16 bits
            const int up = sh > 0 ? (sh > 7 ? 7 : sh) : 0;
            const int k = sh < 0 ? (sh < -9 ? 9 : -sh) : 0;
            // arithmetic right shift = floor; to nearest with ties to even: add half - 1 + (the bit that becomes
            // the last one), then floor; toward zero: add 2^k - 1 to negatives, then floor.  k = 0 adds nothing.
            const s2v ups = splat(up), ks = splat(k);
            const s2v add = splat(RND == MX_RNE ? (k > 0 ? (1 << (k - 1)) - 1 : 0) : (1 << k) - 1);
            const s2v one = splat(k > 0 ? 1 : 0);
#pragma unroll
            for (int t = 0; t < NP; ++t) {
                const s2v v = pr[j * NP + t] << ups;
                s2v r;
                if (RND == MX_RNE) r = (v + add + ((v >> ks) & one)) >> ks;
                else r = (v + ((v >> splat(15)) & add)) >> ks;
                r = __builtin_elementwise_min(__builtin_elementwise_max(r, splat(-qmax)), splat(qmax));
                pr[j * NP + t] = r;
            }
        } else {
#pragma unroll
            for (int t = 0; t < NP; ++t) pr[j * NP + t] = splat(0);
        }
        // one exponent byte per block: every block of the thread, or the even lane for a block of 64
        if (have && (B < 64 || (e0 & 63) == 0)) a.exps_out[blk0 + j] = (uint8_t)ebyte;
    }
    // back into the bit stream
    if (WD == 8) {
#pragma unroll
        for (int g = 0; g < 8; ++g)                   // bytes: pair 2g gives 0 and 2, pair 2g+1 gives 1 and 3
            out[g] = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, pr[2 * g + 1]),
                                           __builtin_bit_cast(uint32_t, pr[2 * g]), 0x06020400u);
    } else if (WD == 4) {
#pragma unroll
        for (int G = 0; G < 4; ++G) {                 // eight elements per dword
            uint32_t x[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t ev = __builtin_bit_cast(uint32_t, pr[4 * G + 2 * h]) & 0x000F000Fu;
                const uint32_t od = __builtin_bit_cast(uint32_t, pr[4 * G + 2 * h + 1]) & 0x000F000Fu;
                x[h] = (od << 4) | ev;                // byte 0: elements 0, 1; byte 2: elements 2, 3 of the group
            }
            out[G] = __builtin_amdgcn_perm(x[1], x[0], 0x06040200u);
        }
    } else {
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const uint32_t c = __builtin_bit_cast(uint32_t, pr[t]) & (((1u << WD) - 1u) * 0x00010001u);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int bit = (4 * (t >> 1) + (t & 1) + 2 * h) * WD;   // compile time after unrolling
                const uint32_t code = h == 0 ? (c & 0xFFFFu) : (c >> 16);
                out[bit >> 5] |= code << (bit & 31);
                if ((bit & 31) + WD > 32) out[(bit >> 5) + 1] |= code >> (32 - (bit & 31));
            }
        }
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

// Two-row blocks whose rows are not whole runs of 32 elements (cols a multiple of the block only): one
// thread per block, widths and block size as run-time values.  A block of one row is a whole number of
// bytes (8 | block), so eight elements at a time travel as ws (wd) bytes through a 64-bit word and no two
// threads write the same byte.  Not a fast path: the shapes of the workloads never come here.
struct CastAnyArgs {
    CastArgs c;
    int64_t pairs, cols;
    int32_t ws, wd, block, rnd;
};

__global__ __launch_bounds__(256) void cast_rows2_any_kernel(CastAnyArgs a) {
    const int64_t nb = a.cols / a.block;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= a.pairs * nb) return;
    const int64_t pr = t / nb, j = t - pr * nb;
    const int ws = a.ws, wd = a.wd, octets = a.block / 8;
    const int qmax = (1 << (wd - 1)) - 1;
    auto octet = [&](const uint8_t* base, int64_t first_elem, int w) {      // 8 elements = w bytes
        uint64_t bits = 0;
        const uint8_t* p = base + first_elem * w / 8;
        for (int k = 0; k < w; ++k) bits |= (uint64_t)p[k] << (8 * k);
        return bits;
    };
    int mx = 0;
    for (int r = 0; r < 2; ++r)
        for (int o = 0; o < octets; ++o) {
            const uint64_t bits = octet(a.c.mant, ((2 * pr + r) * a.cols + j * a.block) + 8 * o, ws);
            for (int i = 0; i < 8; ++i) {
                const int v = (int)((int64_t)(bits << (64 - ws * (i + 1))) >> (64 - ws));
                const int m = v < 0 ? -v : v;
                mx = m > mx ? m : mx;
            }
        }
    int ebyte = 0, sh = 0;
    if (mx != 0) {
        const int E = (int)a.c.exps[pr * nb + j] - a.c.bias_s;
        int E2 = E - (ws - 2) + (31 - __builtin_clz((unsigned)mx));
        E2 = E2 < a.c.emin_d ? a.c.emin_d : E2;
        E2 = E2 > a.c.emax_d ? a.c.emax_d : E2;
        sh = (E - (ws - 2)) - (E2 - (wd - 2));
        sh = sh > 16 ? 16 : (sh < -16 ? -16 : sh);
        ebyte = E2 + a.c.bias_d;
    }
    for (int r = 0; r < 2; ++r)
        for (int o = 0; o < octets; ++o) {
            const int64_t first = ((2 * pr + r) * a.cols + j * a.block) + 8 * o;
            const uint64_t bits = octet(a.c.mant, first, ws);
            uint64_t out = 0;
            for (int i = 0; i < 8; ++i) {
                const int v = (int)((int64_t)(bits << (64 - ws * (i + 1))) >> (64 - ws));
                int res = 0;
                if (mx != 0) {
                    if (sh >= 0) {
                        res = v << sh;
                    } else {
                        const int k = -sh;
                        if (a.rnd == MX_RNE) res = (v + ((1 << (k - 1)) - 1) + ((v >> k) & 1)) >> k;
                        else res = (v + ((v >> 31) & ((1 << k) - 1))) >> k;
                    }
                    res = res > qmax ? qmax : (res < -qmax ? -qmax : res);
                }
                out |= (uint64_t)((uint32_t)res & ((1u << wd) - 1u)) << (wd * i);
            }
            uint8_t* p = a.c.mant_out + first * wd / 8;
            for (int k = 0; k < wd; ++k) p[k] = (uint8_t)(out >> (8 * k));
        }
    a.c.exps_out[pr * nb + j] = (uint8_t)ebyte;
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
    if (fs.block_rows == 2 && cols % 32 != 0) {                              // rows are not whole 32-element runs
        CastAnyArgs g;
        g.c = a; g.pairs = batch * rows / 2; g.cols = cols;
        g.ws = fs.mant_bits; g.wd = fd.mant_bits; g.block = fs.block; g.rnd = fd.rounding;
        const int64_t wgs = ceil_div(g.pairs * (cols / fs.block), 256);
        if (wgs > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(cast_rows2_any_kernel, dim3((unsigned)wgs), dim3(256), 0, st, g);
        MX_HIP_LAUNCH_CHECK();
        return MX_OK;
    }
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
