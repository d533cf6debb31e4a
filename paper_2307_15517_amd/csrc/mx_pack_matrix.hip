// Writers and reader of the block-scaled matrix-core layout (see mx_matrix.h):
//   pack_matrix      canonical MXInt form -> layout (software E2M3 coding; offline for weights)
//   unpack_matrix    layout -> canonical form (exact inverse, used to check the layout)
//   quantize_pack    fp32 activations -> layout in one pass (the quantizer arithmetic of
//                    mx_quantize, Section 4.1 format, fused with the store; hardware fp6 packing)
#include "mx_matrix.h"

namespace mx {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v6i __attribute__((ext_vector_type(6)));

// E2M3 code of v/2 for an integer piece |v| <= 15.
__device__ __forceinline__ uint32_t e2m3_half_code(int v) {
    const uint32_t m = (uint32_t)(v < 0 ? -v : v);
    const uint32_t c = m < 4 ? 4 * m : (m < 8 ? 2 * m + 8 : m + 16);
    return c | (v < 0 ? 0x20u : 0u);
}
// Inverse of the above on the codes it produces.
__device__ __forceinline__ int e2m3_half_value(uint32_t code) {
    const uint32_t c = code & 31u;
    const int m = c >= 24 ? (int)c - 16 : (c >= 16 ? ((int)c - 8) / 2 : (int)c / 4);
    return (code & 0x20u) ? -m : m;
}

// q = 16*h + l with l in [-8, 7]
__device__ __forceinline__ void split_piece(int q, int& h, int& l) {
    l = ((q + 8) & 15) - 8;
    h = (q - l) >> 4;
}

struct MatPackArgs {
    uint8_t* mant;      // canonical
    uint8_t* exps;
    uint8_t* packed;
    int64_t rows, cols;
    MatGeom g;
    int32_t block, w, bias;
    int32_t brows;      // rows per exponent of the canonical form (1 or 2)
};

// Mantissa of element k of a canonical row (w-bit two's complement at bit k*w).
__device__ __forceinline__ int canon_get(const uint8_t* row, int64_t k, int w) {
    const int64_t bit = k * w;
    const int sh = (int)(bit & 7);
    uint32_t v = row[bit >> 3];
    if (sh + w > 8) v |= (uint32_t)row[(bit >> 3) + 1] << 8;
    v >>= sh;
    return ((int)(v << (32 - w))) >> (32 - w);
}

// One thread per (row tile, K step, lane); grid.y = batch.
__global__ __launch_bounds__(256) void pack_matrix_kernel(MatPackArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = (int)(t & 63);
    const int64_t fk = t >> 6;
    if (fk >= a.g.row_tiles * a.g.ksteps) return;
    const int64_t rt = fk / a.g.ksteps, ks = fk - rt * a.g.ksteps;
    const int64_t b = blockIdx.y;
    const int i = lane & 31, h = lane >> 5;
    const int64_t row = rt * 32 + i;
    const int64_t k0 = ks * 64 + h * 32;
    const int64_t row_bytes = a.cols * a.w / 8, nblk = a.cols / a.block;
    const uint8_t* mrow = a.mant + (b * a.rows + row) * row_bytes;
    const bool inside = row < a.rows && k0 < a.cols;
    uint32_t f[2][6];
#pragma unroll
    for (int d = 0; d < 6; ++d) f[0][d] = f[1][d] = 0;
    if (inside) {
        for (int e = 0; e < 32; ++e) {
            const int q = canon_get(mrow, k0 + e, a.w);
            int hi = 0, lo = q;
            if (a.g.pieces == 2) split_piece(q, hi, lo);
            const uint32_t c1 = e2m3_half_code(lo);          // last piece: the low (or only) one
            const uint32_t c0 = e2m3_half_code(hi);
            const int bit = e * 6, d = bit >> 5, sh = bit & 31;
            f[1][d] |= c1 << sh;
            f[0][d] |= c0 << sh;
            if (sh > 26) {
                f[1][d + 1] |= c1 >> (32 - sh);
                f[0][d + 1] |= c0 >> (32 - sh);
            }
        }
    }
    uint8_t* base = a.packed + b * a.g.matrix;
    // fragment 0 / 1 of the unit: (high, low) piece, or (even, odd) row tile
    const int64_t u = a.g.pieces == 2 ? rt : rt >> 1;
    uint8_t* unit = base + mat_unit(a.g, u, ks);
    for (int fi = (a.g.pieces == 2 ? 0 : 1); fi < 2; ++fi) {
        const int slot = a.g.pieces == 2 ? fi : (int)(rt & 1);
        uint32_t* lo = reinterpret_cast<uint32_t*>(unit + frag_lo(slot, lane));
        uint32_t* hi = reinterpret_cast<uint32_t*>(unit + frag_hi(slot, lane));
#pragma unroll
        for (int d = 0; d < 4; ++d) lo[d] = f[fi][d];
        hi[0] = f[fi][4]; hi[1] = f[fi][5];
    }
    // scale byte of this lane's block
    uint8_t sb = 0;
    if (inside) sb = (uint8_t)((int)a.exps[((b * a.rows + row) / a.brows) * nblk + k0 / a.block] + (127 - a.bias));
    base[a.g.frag_bytes + ((rt * (a.g.ksteps / 4) + (ks >> 2)) * 64 + lane) * 4 + (ks & 3)] = sb;
}

// One thread per (row, run of 32 elements); grid.y = batch.
__global__ __launch_bounds__(256) void unpack_matrix_kernel(MatPackArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t runs = a.cols / 32;
    if (t >= a.rows * runs) return;
    const int64_t row = t / runs, run = t - row * runs;
    const int64_t b = blockIdx.y;
    const int64_t rt = row >> 5, ks = run >> 1;
    const int lane = (int)((run & 1) * 32 + (row & 31));
    const uint8_t* base = a.packed + b * a.g.matrix;
    uint32_t f[2][6];
#pragma unroll
    for (int d = 0; d < 6; ++d) f[0][d] = f[1][d] = 0;
    const int64_t u = a.g.pieces == 2 ? rt : rt >> 1;
    const uint8_t* unit = base + mat_unit(a.g, u, ks);
    for (int fi = (a.g.pieces == 2 ? 0 : 1); fi < 2; ++fi) {
        const int slot = a.g.pieces == 2 ? fi : (int)(rt & 1);
        const uint32_t* lo = reinterpret_cast<const uint32_t*>(unit + frag_lo(slot, lane));
        const uint32_t* hi = reinterpret_cast<const uint32_t*>(unit + frag_hi(slot, lane));
#pragma unroll
        for (int d = 0; d < 4; ++d) f[fi][d] = lo[d];
        f[fi][4] = hi[0]; f[fi][5] = hi[1];
    }
    const int64_t row_bytes = a.cols * a.w / 8, nblk = a.cols / a.block;
    uint8_t* out = a.mant + (b * a.rows + row) * row_bytes + run * 4 * a.w;
    uint64_t acc = 0;
    int nbits = 0;
    for (int e = 0; e < 32; ++e) {
        const int bit = e * 6, d = bit >> 5, sh = bit & 31;
        uint32_t c1 = f[1][d] >> sh, c0 = f[0][d] >> sh;
        if (sh > 26) { c1 |= f[1][d + 1] << (32 - sh); c0 |= f[0][d + 1] << (32 - sh); }
        int q = e2m3_half_value(c1 & 63u);
        if (a.g.pieces == 2) q += 16 * e2m3_half_value(c0 & 63u);
        acc |= (uint64_t)((uint32_t)q & ((1u << a.w) - 1u)) << nbits;
        nbits += a.w;
        while (nbits >= 8) { *out++ = (uint8_t)acc; acc >>= 8; nbits -= 8; }
    }
    if ((run * 32) % a.block == 0 && row % a.brows == 0) {
        const uint8_t sb = base[a.g.frag_bytes + ((rt * (a.g.ksteps / 4) + (ks >> 2)) * 64 + lane) * 4 + (ks & 3)];
        a.exps[((b * a.rows + row) / a.brows) * nblk + run * 32 / a.block] = (uint8_t)((int)sb - (127 - a.bias));
    }
}

// ------------------------------------------------------------------------------------------------
// fp32 -> layout in one pass.  One workgroup of four waves per (row tile, group of four K steps);
// wave j owns K step j of the group: 32 rows x 64 floats, read as 256-byte row segments (four
// rows per load instruction), turned through LDS so that each lane ends up with the 32
// consecutive elements of its row that it has to emit.  Small work items keep several waves per
// SIMD resident, so the arithmetic of the waves whose data has arrived overlaps the loads that are
// still in flight.
// ------------------------------------------------------------------------------------------------
struct QPackArgs {
    const float* x;
    uint8_t* packed;
    int64_t rows, cols, row_stride, batch_stride;
    MatGeom g;
    int32_t bias, emax;
    int32_t brows;      // 2: rows 2p and 2p+1 (adjacent lanes) share their exponents
};

constexpr int kQpRowPitch = 256 + 16;     // bytes; the 16-byte skew spreads the lanes' rows over the banks

template <int W, int B, int RND>
__global__ __launch_bounds__(256) void quantize_pack_matrix_kernel(QPackArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 32 * kQpRowPitch];
    __shared__ uint32_t scale_bytes[4][64];
    constexpr int P = (W <= 4) ? 1 : 2;
    constexpr float qmax = (float)((1 << (W - 1)) - 1);
    const int j = threadIdx.x >> 6, lane = threadIdx.x & 63;        // j: K step of the group
    uint8_t* lds = lds_all + j * 32 * kQpRowPitch;
    const int i = lane & 31, h = lane >> 5;
    const int64_t ks4n = a.g.ksteps / 4;
    const int64_t rt = blockIdx.x / ks4n, ks4 = blockIdx.x - rt * ks4n;
    const int64_t b = blockIdx.y;
    const float* xb = a.x + b * a.batch_stride;
    const int64_t ks = ks4 * 4 + j;

    // 32 rows x 256 bytes, zero outside the matrix: instruction r covers rows 4r .. 4r+3
    float4 in[8];
    const int64_t c = ks * 64 + (lane & 15) * 4;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int64_t row = rt * 32 + 4 * r + (lane >> 4);
        in[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < a.rows && c < a.cols) in[r] = load_once4(xb + row * a.row_stride + c);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r)
        *reinterpret_cast<float4*>(lds + (4 * r + (lane >> 4)) * kQpRowPitch + (lane & 15) * 16) = in[r];
    __builtin_amdgcn_wave_barrier();

    uint8_t* base = a.packed + b * a.g.matrix;
    float v[32];
    const uint8_t* src = lds + i * kQpRowPitch + h * 128;
#pragma unroll
    for (int q4 = 0; q4 < 8; ++q4) {
        const float4 t = *reinterpret_cast<const float4*>(src + q4 * 16);
        v[4 * q4] = t.x; v[4 * q4 + 1] = t.y; v[4 * q4 + 2] = t.z; v[4 * q4 + 3] = t.w;
    }
    uint32_t am = 0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const uint32_t ab = __float_as_uint(v[e]) & 0x7fffffffu;
        am = ab > am ? ab : am;
    }
    if (B == 64) {                      // the two halves of a lane pair form one block
        const uint32_t o = (uint32_t)__shfl_xor((int)am, 32, 64);
        am = o > am ? o : am;
    }
    if (a.brows == 2) {                 // two-row blocks: the neighbouring lane holds the other row
        const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);
        am = o > am ? o : am;
    }
    const int ef = (int)(am >> 23);
    int E = ef == 0 ? -127 : ef - 127;
    E = E < -a.bias ? -a.bias : E;
    E = E > a.emax ? a.emax : E;
    const int shift = (W - 2) - E;
    v16f lo0, lo1, hi0, hi1;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        float s = __builtin_ldexpf(v[e], shift);
        float r = RND == MX_RNE ? __builtin_rintf(s) : __builtin_truncf(s);
        r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
        float hi = 0.f, lo = r;
        if (P == 2) {
            hi = __builtin_floorf(r * 0.0625f + 0.5f);      // h = floor((q + 8) / 16)
            lo = r - 16.f * hi;
        }
        lo += 0.0f;                                          // -0.0 (a small negative rounded to zero) -> +0.0
        // the packing instruction interleaves its two sources: element 2t from the first, 2t+1 from the second
        if (e & 1) { lo1[e >> 1] = lo; hi1[e >> 1] = hi; }
        else       { lo0[e >> 1] = lo; hi0[e >> 1] = hi; }
    }
    const v6i fl = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(lo0, lo1, 2.0f);   // codes of piece / 2
    uint8_t* unit = base + mat_unit(a.g, P == 2 ? rt : rt >> 1, ks);
    const int lslot = P == 2 ? 1 : (int)(rt & 1);
    *reinterpret_cast<uint4*>(unit + frag_lo(lslot, lane)) =
        make_uint4((uint32_t)fl[0], (uint32_t)fl[1], (uint32_t)fl[2], (uint32_t)fl[3]);
    *reinterpret_cast<uint2*>(unit + frag_hi(lslot, lane)) = make_uint2((uint32_t)fl[4], (uint32_t)fl[5]);
    if (P == 2) {
        const v6i fh = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(hi0, hi1, 2.0f);
        *reinterpret_cast<uint4*>(unit + frag_lo(0, lane)) =
            make_uint4((uint32_t)fh[0], (uint32_t)fh[1], (uint32_t)fh[2], (uint32_t)fh[3]);
        *reinterpret_cast<uint2*>(unit + frag_hi(0, lane)) = make_uint2((uint32_t)fh[4], (uint32_t)fh[5]);
    }
    // the four waves' scale bytes of a lane make one dword
    const bool inside = (rt * 32 + i) < a.rows && (ks * 64 + h * 32) < a.cols;
    scale_bytes[j][lane] = inside ? (uint32_t)(E + 127) : 0u;          // E + bias + (127 - bias)
    __syncthreads();
    if (j == 0) {
        const uint32_t d = scale_bytes[0][lane] | (scale_bytes[1][lane] << 8) | (scale_bytes[2][lane] << 16) |
                           (scale_bytes[3][lane] << 24);
        *reinterpret_cast<uint32_t*>(base + a.g.frag_bytes + ((rt * ks4n + ks4) * 64 + lane) * 4) = d;
    }
}

template <int W, int B>
mx_status launch_qpack(const QPackArgs& a, int64_t batch, int rnd, hipStream_t st) {
    dim3 grid((unsigned)(a.g.row_tiles * (a.g.ksteps / 4)), (unsigned)batch);
    if (rnd == MX_RNE)
        hipLaunchKernelGGL((quantize_pack_matrix_kernel<W, B, MX_RNE>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((quantize_pack_matrix_kernel<W, B, MX_RTZ>), grid, dim3(256), 0, st, a);
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

}  // namespace

// defined in mx_pack_bf16.hip: blocks of 16 use the bfloat16 form of the layout
mx_status pack_bf16(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                    mx_format f, uint8_t* packed, bool pack, hipStream_t st);
mx_status quantize_pack_bf16(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                             int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st);

bool matrix_format_ok(const mx_format& f) {
    return format_ok_quant(f) && (f.block == 16 || f.block == 32 || f.block == 64);
}

mx_status pack_matrix(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                      mx_format f, uint8_t* packed, bool pack, hipStream_t st) {
    if (f.block == 16) return pack_bf16(mant, exps, batch, rows, cols, f, packed, pack, st);
    MatPackArgs a;
    a.mant = const_cast<uint8_t*>(mant); a.exps = const_cast<uint8_t*>(exps); a.packed = packed;
    a.rows = rows; a.cols = cols; a.g = mat_geom(rows, cols, f.mant_bits);
    a.block = f.block; a.w = f.mant_bits; a.bias = (1 << (f.exp_bits - 1)) - 1;
    a.brows = f.block_rows;
    if (pack) {
        const int64_t threads = a.g.row_tiles * a.g.ksteps * 64;
        dim3 grid((unsigned)ceil_div(threads, 256), (unsigned)batch);
        hipLaunchKernelGGL(pack_matrix_kernel, grid, dim3(256), 0, st, a);
    } else {
        const int64_t threads = rows * (cols / 32);
        dim3 grid((unsigned)ceil_div(threads, 256), (unsigned)batch);
        hipLaunchKernelGGL(unpack_matrix_kernel, grid, dim3(256), 0, st, a);
    }
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

mx_status quantize_pack_matrix(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                               int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st) {
    if (f.block == 16) return quantize_pack_bf16(x, batch, rows, cols, row_stride, batch_stride, f, packed, st);
    if (((uintptr_t)x & 15) || (row_stride & 3) || (batch_stride & 3)) return MX_ERR_UNSUPPORTED;
    QPackArgs a;
    a.x = x; a.packed = packed; a.rows = rows; a.cols = cols;
    a.row_stride = row_stride; a.batch_stride = batch_stride;
    a.g = mat_geom(rows, cols, f.mant_bits);
    a.bias = (1 << (f.exp_bits - 1)) - 1;
    a.emax = ((1 << f.exp_bits) - 1) - a.bias;
    a.brows = f.block_rows;
    if (a.g.row_tiles * (a.g.ksteps / 4) > 0x7fffffffLL || batch > 65535) return MX_ERR_UNSUPPORTED;
    if (f.block == 32) { MX_SW(f.mant_bits, kW, return (launch_qpack<kW, 32>(a, batch, f.rounding, st))); }
    else               { MX_SW(f.mant_bits, kW, return (launch_qpack<kW, 64>(a, batch, f.rounding, st))); }
    return MX_ERR_UNSUPPORTED;
}

}  // namespace mx
