// Writers and reader of the block-16 matrix-core layout (see mx_bf16.h):
//   pack_bf16           canonical MXInt form -> layout (offline for weights)
//   unpack (same call)  layout -> canonical form (exact inverse, used to check the layout)
//   quantize_pack_bf16  fp32 activations -> layout in one pass (the quantizer arithmetic of
//                       mx_quantize, Section 4.1 format, fused with the store)
#include "mx_bf16.h"

namespace mx {
namespace {

struct BfPackArgs {
    uint8_t* mant;      // canonical
    uint8_t* exps;
    uint8_t* packed;
    int64_t rows, cols;
    BfGeom g;
    int32_t w, bias;
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

// One thread per (row tile, block slot, lane); grid.y = batch.  Slots past K and rows past the
// matrix hold zeros.
__global__ __launch_bounds__(256) void pack_bf16_kernel(BfPackArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = (int)(t & 63);
    const int64_t fk = t >> 6, slots = a.g.ksteps * 2;
    if (fk >= a.g.row_tiles * slots) return;
    const int64_t rt = fk / slots, kf = fk - rt * slots;
    const int64_t b = blockIdx.y;
    const int i = lane & 31, h = lane >> 5;
    const int64_t row = rt * 32 + i;
    uint8_t* base = a.packed + b * a.g.matrix;
    uint32_t out[4] = {0, 0, 0, 0};
    if (row < a.rows && kf < a.g.nblk) {
        const uint8_t* mrow = a.mant + (b * a.rows + row) * (a.cols * a.w / 8);
        const uint8_t ebyte = a.exps[((b * a.rows + row) / a.brows) * a.g.nblk + kf];
        const int s = (int)ebyte - a.bias - (a.w - 2);
        for (int e = 0; e < 8; ++e) {
            const int q = canon_get(mrow, kf * 16 + 8 * h + e, a.w);
            out[e >> 1] |= bf16_of((float)q, s) << (16 * (e & 1));
        }
        if (h == 0) base[a.g.frag_bytes + row * a.g.nblk + kf] = ebyte;
    }
    *reinterpret_cast<uint4*>(base + bf_frag(a.g, rt, kf >> 1, (int)(kf & 1), lane)) =
        make_uint4(out[0], out[1], out[2], out[3]);
}

// One thread per (row, block); grid.y = batch.
__global__ __launch_bounds__(256) void unpack_bf16_kernel(BfPackArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= a.rows * a.g.nblk) return;
    const int64_t row = t / a.g.nblk, kf = t - row * a.g.nblk;
    const int64_t b = blockIdx.y;
    const uint8_t* base = a.packed + b * a.g.matrix;
    const uint8_t ebyte = base[a.g.frag_bytes + row * a.g.nblk + kf];
    const int s = (int)ebyte - a.bias - (a.w - 2);
    uint8_t* out = a.mant + (b * a.rows + row) * (a.cols * a.w / 8) + kf * 2 * a.w;
    uint64_t acc = 0;
    int nbits = 0;
    for (int h = 0; h < 2; ++h) {
        const uint4 v = *reinterpret_cast<const uint4*>(base + bf_frag(a.g, row >> 5, kf >> 1, (int)(kf & 1),
                                                                       32 * h + (int)(row & 31)));
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
        for (int e = 0; e < 8; ++e) {
            const uint32_t bits = (d[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
            const int q = (int)__builtin_ldexpf(__uint_as_float(bits << 16), -s);
            acc |= (uint64_t)((uint32_t)q & ((1u << a.w) - 1u)) << nbits;
            nbits += a.w;
            while (nbits >= 8) { *out++ = (uint8_t)acc; acc >>= 8; nbits -= 8; }
        }
    }
    if (row % a.brows == 0) a.exps[((b * a.rows + row) / a.brows) * a.g.nblk + kf] = ebyte;
}

// ------------------------------------------------------------------------------------------------
// fp32 -> layout in one pass.  One workgroup of four waves per (row tile, 256 columns); wave j owns
// 64 columns (four blocks, two K steps): 32 rows x 256 bytes read as whole row segments (four rows
// per load instruction), turned through the wave's LDS tile so that lane 32*h + i holds half h of
// each of the four blocks of row i; the block maximum is completed with the partner lane.
// ------------------------------------------------------------------------------------------------
struct BfQPackArgs {
    const float* x;
    uint8_t* packed;
    int64_t rows, cols, row_stride, batch_stride;
    BfGeom g;
    int32_t bias, emax;
    int32_t brows;      // 2: rows 2p and 2p+1 (adjacent lanes) share their exponents
};

constexpr int kBfRowPitch = 256 + 16;     // bytes; the 16-byte skew spreads the lanes' rows over the banks

template <int W, int RND>
__global__ __launch_bounds__(256) void quantize_pack_bf16_kernel(BfQPackArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 32 * kBfRowPitch];
    constexpr float qmax = (float)((1 << (W - 1)) - 1);
    const int j = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    uint8_t* lds = lds_all + j * 32 * kBfRowPitch;
    const int i = lane & 31, h = lane >> 5;
    const int64_t spans = a.g.ksteps / 2, spq = (spans + 3) / 4;      // spans of 64 columns
    const int64_t rt = blockIdx.x / spq, sp = (blockIdx.x - rt * spq) * 4 + j;
    if (sp >= spans) return;                                         // whole wave; no workgroup barrier below
    const int64_t b = blockIdx.y;
    const float* xb = a.x + b * a.batch_stride;

    float4 in[8];
    const int64_t c = sp * 64 + (lane & 15) * 4;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int64_t row = rt * 32 + 4 * r + (lane >> 4);
        in[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < a.rows && c < a.cols) in[r] = *reinterpret_cast<const float4*>(xb + row * a.row_stride + c);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r)
        *reinterpret_cast<float4*>(lds + (4 * r + (lane >> 4)) * kBfRowPitch + (lane & 15) * 16) = in[r];
    __builtin_amdgcn_wave_barrier();

    uint8_t* base = a.packed + b * a.g.matrix;
    const int64_t row = rt * 32 + i;
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        const uint8_t* src = lds + i * kBfRowPitch + (f * 16 + h * 8) * 4;
        const float4 t0 = *reinterpret_cast<const float4*>(src), t1 = *reinterpret_cast<const float4*>(src + 16);
        const float v[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
        uint32_t am = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t ab = __float_as_uint(v[e]) & 0x7fffffffu;
            am = ab > am ? ab : am;
        }
        const uint32_t o = (uint32_t)__shfl_xor((int)am, 32, 64);
        am = o > am ? o : am;
        if (a.brows == 2) {             // two-row blocks: the neighbouring lane holds the other row
            const uint32_t o2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);
            am = o2 > am ? o2 : am;
        }
        const int ef = (int)(am >> 23);
        int E = ef == 0 ? -127 : ef - 127;
        E = E < -a.bias ? -a.bias : E;
        E = E > a.emax ? a.emax : E;
        uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float sc = __builtin_ldexpf(v[e], (W - 2) - E);
            float r = RND == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
            r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
            r += 0.0f;                                   // -0.0 (a small negative rounded to zero) -> +0.0
            out[e >> 1] |= bf16_of(r, E - (W - 2)) << (16 * (e & 1));
        }
        *reinterpret_cast<uint4*>(base + bf_frag(a.g, rt, sp * 2 + (f >> 1), f & 1, lane)) =
            make_uint4(out[0], out[1], out[2], out[3]);
        const int64_t blk = sp * 4 + f;
        if (h == 0 && row < a.rows && blk < a.g.nblk) base[a.g.frag_bytes + row * a.g.nblk + blk] = (uint8_t)(E + a.bias);
    }
}

template <int W>
mx_status launch_bf_qpack(const BfQPackArgs& a, int64_t batch, int rnd, hipStream_t st) {
    dim3 grid((unsigned)(a.g.row_tiles * ((a.g.ksteps / 2 + 3) / 4)), (unsigned)batch);
    if (rnd == MX_RNE)
        hipLaunchKernelGGL((quantize_pack_bf16_kernel<W, MX_RNE>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((quantize_pack_bf16_kernel<W, MX_RTZ>), grid, dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}


// ------------------------------------------------------------------------------------------------
// fp32 -> layout with the blocks running DOWN the columns of x (the strided axis), i.e. the packed
// operand of x^T [cols x rows]: what mx_quantize with axis 0 followed by mx_pack gives.  This is the
// V operand of attention: V [keys x d] is reduced over the keys in P V, so its blocks run along the
// keys and the operand is V^T [d x keys].
// One workgroup of four waves per 64 rows (four blocks) x 128 columns of x: the tile is read as whole
// row segments of 512 bytes (two rows per wave instruction) into LDS; wave j then owns output row tile
// j of the workgroup (32 columns of x), lane 32*h + i reads half h of each block of column i down the
// LDS tile (32 consecutive floats per half wave: conflict-free with the pitch below), completes the
// block maximum with the partner lane, quantizes and stores 16 bytes per fragment.
// ------------------------------------------------------------------------------------------------
struct BfQPackTArgs {
    const float* x;
    uint8_t* packed;
    int64_t rows, cols, row_stride, batch_stride;     // of x
    BfGeom g;                                          // of the operand: cols x rows
    int32_t bias, emax;
    int32_t vec;                                       // 16-byte loads are aligned
    int32_t brows;                                     // 2: columns 2p and 2p+1 of x (rows of the operand) share exponents
};

constexpr int kBfTPitch = 128 + 4;     // floats per LDS tile row: the two lane halves (8 rows apart) land 32 banks apart

template <int W, int RND>
__global__ __launch_bounds__(256) void quantize_pack_bf16_axis0_kernel(BfQPackTArgs a) {
    __shared__ __attribute__((aligned(16))) float tile[64 * kBfTPitch];
    constexpr float qmax = (float)((1 << (W - 1)) - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int64_t r0 = (int64_t)blockIdx.x * 64;       // first row of x (first key) of the tile
    const int64_t c0 = (int64_t)blockIdx.y * 128;      // first column of x
    const int64_t b = blockIdx.z;
    const float* xb = a.x + b * a.batch_stride;

    // 64 rows x 128 columns: a thread loads four columns of a row; 32 threads cover a row, a workgroup 8 rows
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int rr = p * 8 + (threadIdx.x >> 5);
        const int64_t row = r0 + rr, col = c0 + (threadIdx.x & 31) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < a.rows) {
            const float* src = xb + row * a.row_stride + col;
            if (a.vec && col + 3 < a.cols) {
                v = *reinterpret_cast<const float4*>(src);
            } else {
                if (col < a.cols) v.x = src[0];
                if (col + 1 < a.cols) v.y = src[1];
                if (col + 2 < a.cols) v.z = src[2];
                if (col + 3 < a.cols) v.w = src[3];
            }
        }
        *reinterpret_cast<float4*>(tile + rr * kBfTPitch + (threadIdx.x & 31) * 4) = v;
    }
    __syncthreads();

    const int64_t rt = blockIdx.y * 4 + wave;          // output row tile: columns c0 + 32*wave .. of x
    if (rt >= a.g.row_tiles) return;
    uint8_t* base = a.packed + b * a.g.matrix;
    const int64_t orow = rt * 32 + i;                  // output row = column of x
#pragma unroll
    for (int f = 0; f < 4; ++f) {                      // block f of the tile: rows 16*f .. 16*f+15 of x
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = tile[(16 * f + 8 * h + e) * kBfTPitch + 32 * wave + i];
        uint32_t am = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t ab = __float_as_uint(v[e]) & 0x7fffffffu;
            am = ab > am ? ab : am;
        }
        const uint32_t o = (uint32_t)__shfl_xor((int)am, 32, 64);
        am = o > am ? o : am;
        if (a.brows == 2) {             // two-row blocks: the neighbouring lane holds the neighbouring column of x
            const uint32_t o2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);
            am = o2 > am ? o2 : am;
        }
        const int ef = (int)(am >> 23);
        int E = ef == 0 ? -127 : ef - 127;
        E = E < -a.bias ? -a.bias : E;
        E = E > a.emax ? a.emax : E;
        uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float sc = __builtin_ldexpf(v[e], (W - 2) - E);
            float r = RND == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
            r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
            r += 0.0f;                                   // -0.0 (a small negative rounded to zero) -> +0.0
            out[e >> 1] |= bf16_of(r, E - (W - 2)) << (16 * (e & 1));
        }
        const int64_t kf = blockIdx.x * 4 + f;           // block along the operand's K (the rows of x)
        if (kf < a.g.ksteps * 2)
            *reinterpret_cast<uint4*>(base + bf_frag(a.g, rt, kf >> 1, (int)(kf & 1), lane)) =
                make_uint4(out[0], out[1], out[2], out[3]);
        if (h == 0 && orow < a.cols && kf < a.g.nblk) base[a.g.frag_bytes + orow * a.g.nblk + kf] = (uint8_t)(E + a.bias);
    }
}

template <int W>
mx_status launch_bf_qpack_t(const BfQPackTArgs& a, int64_t batch, int rnd, hipStream_t st) {
    // the K steps of the operand are padded to a multiple of 2 (64 rows of x): the grid covers the padding too
    dim3 grid((unsigned)(a.g.ksteps / 2), (unsigned)ceil_div(a.g.row_tiles, 4), (unsigned)batch);
    if (rnd == MX_RNE)
        hipLaunchKernelGGL((quantize_pack_bf16_axis0_kernel<W, MX_RNE>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((quantize_pack_bf16_axis0_kernel<W, MX_RTZ>), grid, dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

}  // namespace

mx_status pack_bf16(const uint8_t* mant, const uint8_t* exps, int64_t batch, int64_t rows, int64_t cols,
                    mx_format f, uint8_t* packed, bool pack, hipStream_t st) {
    BfPackArgs a;
    a.mant = const_cast<uint8_t*>(mant); a.exps = const_cast<uint8_t*>(exps); a.packed = packed;
    a.rows = rows; a.cols = cols; a.g = bf_geom(rows, cols);
    a.w = f.mant_bits; a.bias = (1 << (f.exp_bits - 1)) - 1;
    a.brows = f.block_rows;
    const int64_t threads = pack ? a.g.row_tiles * a.g.ksteps * 2 * 64 : rows * a.g.nblk;
    if (ceil_div(threads, 256) > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)ceil_div(threads, 256), (unsigned)batch);
    if (pack) hipLaunchKernelGGL(pack_bf16_kernel, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(unpack_bf16_kernel, grid, dim3(256), 0, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

mx_status quantize_pack_bf16(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                             int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st) {
    if (((uintptr_t)x & 15) || (row_stride & 3) || (batch_stride & 3)) return MX_ERR_UNSUPPORTED;
    BfQPackArgs a;
    a.x = x; a.packed = packed; a.rows = rows; a.cols = cols;
    a.row_stride = row_stride; a.batch_stride = batch_stride;
    a.g = bf_geom(rows, cols);
    a.bias = (1 << (f.exp_bits - 1)) - 1;
    a.emax = ((1 << f.exp_bits) - 1) - a.bias;
    a.brows = f.block_rows;
    if (a.g.row_tiles * ((a.g.ksteps / 2 + 3) / 4) > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    switch (f.mant_bits) {
        case 2: return launch_bf_qpack<2>(a, batch, f.rounding, st);
        case 3: return launch_bf_qpack<3>(a, batch, f.rounding, st);
        case 4: return launch_bf_qpack<4>(a, batch, f.rounding, st);
        case 5: return launch_bf_qpack<5>(a, batch, f.rounding, st);
        case 6: return launch_bf_qpack<6>(a, batch, f.rounding, st);
        case 7: return launch_bf_qpack<7>(a, batch, f.rounding, st);
        case 8: return launch_bf_qpack<8>(a, batch, f.rounding, st);
    }
    return MX_ERR_BAD_ARG;
}

// x [rows x cols] with blocks down the columns -> packed operand of x^T [cols x rows].
mx_status quantize_pack_bf16_axis0(const float* x, int64_t batch, int64_t rows, int64_t cols, int64_t row_stride,
                                   int64_t batch_stride, mx_format f, uint8_t* packed, hipStream_t st) {
    BfQPackTArgs a;
    a.x = x; a.packed = packed; a.rows = rows; a.cols = cols;
    a.row_stride = row_stride; a.batch_stride = batch_stride;
    a.g = bf_geom(cols, rows);
    a.bias = (1 << (f.exp_bits - 1)) - 1;
    a.emax = ((1 << f.exp_bits) - 1) - a.bias;
    a.vec = (((uintptr_t)x & 15) == 0 && (row_stride & 3) == 0 && (batch_stride & 3) == 0) ? 1 : 0;
    a.brows = f.block_rows;
    if (a.g.ksteps / 2 > 0x7fffffffLL || ceil_div(a.g.row_tiles, 4) > 65535) return MX_ERR_UNSUPPORTED;
    switch (f.mant_bits) {
        case 2: return launch_bf_qpack_t<2>(a, batch, f.rounding, st);
        case 3: return launch_bf_qpack_t<3>(a, batch, f.rounding, st);
        case 4: return launch_bf_qpack_t<4>(a, batch, f.rounding, st);
        case 5: return launch_bf_qpack_t<5>(a, batch, f.rounding, st);
        case 6: return launch_bf_qpack_t<6>(a, batch, f.rounding, st);
        case 7: return launch_bf_qpack_t<7>(a, batch, f.rounding, st);
        case 8: return launch_bf_qpack_t<8>(a, batch, f.rounding, st);
    }
    return MX_ERR_BAD_ARG;
}

}  // namespace mx

