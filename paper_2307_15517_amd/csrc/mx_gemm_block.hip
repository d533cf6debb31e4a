// MXInt x MXInt product on the integer matrix cores of gfx950, operands in the fragment layout.
//
// Arithmetic (Section 3.2 of the paper, the MXInt dot-product operator): per K-block the mantissa
// products are summed exactly in int32 by one MFMA whose K extent equals the block (32x32x16 for
// block 16, 32x32x32 for block 32, two chained 32x32x32 for block 64); the block's value is that
// integer times 2^(Ea + Eb - (wa-2) - (wb-2)), applied with v_ldexp_f32 and added into an fp32
// accumulator.  The left operand feeds the MFMA "A" side, so in the 32x32 result a lane owns one
// output column n and its 16 registers are 16 rows m: the right operand's block exponent is one
// value per lane, the left operand's is one value per register.
#include "mx_gemm.h"
#include "mx_frag.h"

#ifndef MX_GEMM_BLOCK
#error "compile with -DMX_GEMM_BLOCK=16, 32 or 64"
#endif

namespace mx {
namespace {

typedef v4i_t v4i;
typedef v16i_t v16i;

// ------------------------------------------------------------------------------------------------
// General kernel: a workgroup of four waves owns a 128 x 128 tile of Y; each wave a 64 x 64
// quarter (2 x 2 row groups).  Fragments come straight from global memory in lane order.
// ------------------------------------------------------------------------------------------------
template <int WA, int WB, int B>
__global__ __launch_bounds__(256) void gemm_fragment_kernel(GemmArgs g) {
    constexpr int kDwA = Piece<WA, B>::kDw, kDwB = Piece<WB, B>::kDw;
    constexpr int kHalfDw = B / 8;       // int8 dwords per lane per block
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int64_t ga0 = (int64_t)blockIdx.y * 4 + (wave >> 1) * 2;
    const int64_t gb0 = (int64_t)blockIdx.x * 4 + (wave & 1) * 2;
    const int64_t bz = blockIdx.z;
    const uint8_t* Abase = g.A + bz * g.matrixA;
    const uint8_t* Bbase = g.B + bz * g.matrixB;
    const int eadj = g.eadj - Unpack<WA, B>::kScaleLog2 - Unpack<WB, B>::kScaleLog2;

    float acc[2][2][16];
#pragma unroll
    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ta][tb][r] = 0.f;

    for (int64_t c = 0; c < g.chunks; ++c) {
        uint32_t pa[2][kDwA], pb[2][kDwB];
        uint32_t ea[2][16];     // [group][4*gq + r]: the four block exponents of row 8*gq + 4*h + r
        uint32_t eb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (ga0 + t < g.groupsA) {
                const uint8_t* rec = Abase + ((ga0 + t) * g.chunks + c) * g.recordA;
                load_dwords<kDwA>(rec + lane * (kDwA * 4), pa[t]);
                const uint8_t* ex = rec + 64 * (kDwA * 4);
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) load_dwords<4>(ex + (8 * gq + 4 * h) * 4, &ea[t][4 * gq]);
            } else {
#pragma unroll
                for (int d = 0; d < kDwA; ++d) pa[t][d] = 0;
#pragma unroll
                for (int d = 0; d < 16; ++d) ea[t][d] = 0;
            }
            if (gb0 + t < g.groupsB) {
                const uint8_t* rec = Bbase + ((gb0 + t) * g.chunks + c) * g.recordB;
                load_dwords<kDwB>(rec + lane * (kDwB * 4), pb[t]);
                eb[t] = reinterpret_cast<const uint32_t*>(rec + 64 * (kDwB * 4))[i];
            } else {
#pragma unroll
                for (int d = 0; d < kDwB; ++d) pb[t][d] = 0;
                eb[t] = 0;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t fa[2][kHalfDw], fb[2][kHalfDw];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                Unpack<WA, B>::run(pa[t], j, fa[t]);
                Unpack<WB, B>::run(pb[t], j, fb[t]);
            }
#pragma unroll
            for (int ta = 0; ta < 2; ++ta) {
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const v16i d = block_mfma<B>(fa[ta], fb[tb]);
                    const int ebj = (int)((eb[tb] >> (8 * j)) & 0xFFu) + eadj;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int e = (int)((ea[ta][r] >> (8 * j)) & 0xFFu) + ebj;
                        acc[ta][tb][r] += __builtin_ldexpf((float)d[r], e);
                    }
                }
            }
        }
    }

    float* Y = g.Y + bz * g.batch_stride_y;
#pragma unroll
    for (int ta = 0; ta < 2; ++ta) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int64_t n = (gb0 + tb) * 32 + i;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = (ga0 + ta) * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                // written once and not read again by this kernel: a streaming store keeps the operands in the L2
                if (m < g.M && n < g.N) __builtin_nontemporal_store(acc[ta][tb][r], &Y[m * g.ldy + n]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Decode kernel (M <= 8): bound by one pass over the packed right operand.  A workgroup of NW
// waves owns 32 output columns; its waves take the K chunks round-robin, each keeping four fp32
// partial sums per lane (rows 4*h .. 4*h+3), which are added through LDS at the end.
// ------------------------------------------------------------------------------------------------
template <int WA, int WB, int B, int NW>
__global__ __launch_bounds__(NW * 64) void gemv_fragment_kernel(GemmArgs g) {
    constexpr int kDwA = Piece<WA, B>::kDw, kDwB = Piece<WB, B>::kDw;
    constexpr int kHalfDw = B / 8;
    __shared__ float red[NW][4][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int64_t gb = blockIdx.x;
    const int64_t bz = blockIdx.y;
    const uint8_t* Abase = g.A + bz * g.matrixA;                       // group 0 holds all M <= 8 rows
    const uint8_t* Bbase = g.B + bz * g.matrixB + gb * g.chunks * g.recordB;
    const int eadj = g.eadj - Unpack<WA, B>::kScaleLog2 - Unpack<WB, B>::kScaleLog2;
    const bool arow = i < g.M;

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int64_t c = wave; c < g.chunks; c += NW) {
        uint32_t pa[kDwA], pb[kDwB], ea[4], eb;
        const uint8_t* recB = Bbase + c * g.recordB;
        load_dwords<kDwB>(recB + lane * (kDwB * 4), pb);
        eb = reinterpret_cast<const uint32_t*>(recB + 64 * (kDwB * 4))[i];
        const uint8_t* recA = Abase + c * g.recordA;
        if (arow) {
            load_dwords<kDwA>(recA + lane * (kDwA * 4), pa);
        } else {
#pragma unroll
            for (int d = 0; d < kDwA; ++d) pa[d] = 0;
        }
        load_dwords<4>(recA + 64 * (kDwA * 4) + (4 * h) * 4, ea);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t fa[kHalfDw], fb[kHalfDw];
            Unpack<WA, B>::run(pa, j, fa);
            Unpack<WB, B>::run(pb, j, fb);
            const v16i d = block_mfma<B>(fa, fb);
            const int ebj = (int)((eb >> (8 * j)) & 0xFFu) + eadj;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = (int)((ea[r] >> (8 * j)) & 0xFFu) + ebj;
                acc[r] += __builtin_ldexpf((float)d[r], e);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][r][lane] = acc[r];
    __syncthreads();
    // 256 (r, lane) sums, one per thread of the first four waves
    for (int t = threadIdx.x; t < 256; t += NW * 64) {
        const int r = t >> 6, l = t & 63;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[w][r][l];
        const int64_t m = 4 * (l >> 5) + r;
        const int64_t n = gb * 32 + (l & 31);
        if (m < g.M && n < g.N) g.Y[bz * g.batch_stride_y + m * g.ldy + n] = s;
    }
}

constexpr int kGemvWaves = 8;

// ------------------------------------------------------------------------------------------------
// Streaming decode kernel (M <= 8, K small enough for the activations to sit in LDS): the same
// arithmetic as above, arranged for HBM bandwidth.  The workgroup copies the (tiny) left
// operand's fragments into LDS once; every wave keeps D chunks of its share of the packed right
// operand in flight in registers (a ring that is refilled as soon as a slot has been consumed),
// so the weight stream never waits for the arithmetic.
//   MR: rows per lane half that are computed (1 for M == 1, else 4).
// ------------------------------------------------------------------------------------------------
template <int WA, int WB, int B, int NW, int D, int MR>
__global__ __launch_bounds__(NW * 64) void gemv_stream_kernel(GemmArgs g) {
    constexpr int kDwA = Piece<WA, B>::kDw, kDwB = Piece<WB, B>::kDw;
    constexpr int kHalfDw = B / 8;
    constexpr int XD = 16 * kDwA + 8;            // dwords kept per chunk: 16 lane pieces (rows 0..7, both halves) + 8 rows of exponents
    extern __shared__ __attribute__((aligned(16))) uint32_t xs[];
    float* red = reinterpret_cast<float*>(xs + g.chunks * XD);          // [NW][MR][64]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int64_t gb = blockIdx.x;
    const int64_t bz = blockIdx.y;
    const uint8_t* Abase = g.A + bz * g.matrixA;
    const uint8_t* Bbase = g.B + bz * g.matrixB + gb * g.chunks * g.recordB;
    const int eadj = g.eadj - Unpack<WA, B>::kScaleLog2 - Unpack<WB, B>::kScaleLog2;
    const int chunks = (int)g.chunks;

    // ring of D chunks of weights per wave; chunk number t of this wave is chunk wave + t*NW, and a
    // chunk number past the end of the column group reads zeros (no branch around a load: the waits
    // the compiler places then count exactly the loads that are in flight)
    const BufRsrc rB = make_rsrc(Bbase, (uint32_t)(chunks * g.recordB));
    uint32_t pb[D][kDwB], eb[D];
    auto fetch = [&](int slot, int t) {
        const uint32_t off = (uint32_t)(wave + t * NW) * (uint32_t)g.recordB;
        buf_load_dwords<kDwB>(rB, off + lane * (kDwB * 4), pb[slot]);
        buf_load_dwords<1>(rB, off + 64 * (kDwB * 4) + i * 4, &eb[slot]);
    };

    // left operand -> LDS (rows 0..7 of row group 0), in units of UD dwords, several loads in flight.
    // Loads return in the order of issue: the first batch of the left operand is requested before the
    // ring of weights, so that it does not wait behind them.
    {
        constexpr int UD = (kDwA % 4 == 0) ? 4 : 1;          // dwords per unit
        constexpr int UPC = XD / UD;                         // units per chunk (XD = 16*kDwA + 8)
        constexpr int UNROLL = 4;
        const int total = chunks * UPC;
        auto batch_load = [&](int base, uint32_t (*v)[UD]) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int idx = base + u * NW * 64;
                if (idx < total) {
                    const int c = idx / UPC, d = (idx - c * UPC) * UD;
                    const uint8_t* rec = Abase + (int64_t)c * g.recordA;
                    const uint8_t* src;
                    int row;                                  // first row the unit belongs to
                    if (d < 16 * kDwA) {
                        const int l16 = d / kDwA, dd = d - l16 * kDwA;
                        row = l16 & 7;
                        src = rec + ((l16 >> 3) * 32 + row) * (kDwA * 4) + dd * 4;
                    } else {
                        row = d - 16 * kDwA;
                        src = rec + 64 * (kDwA * 4) + row * 4;
                    }
                    // rows >= M feed accumulator rows that are never stored: their slots keep whatever LDS holds
                    if (row < g.M) load_dwords<UD>(src, v[u]);
                }
            }
        };
        auto batch_store = [&](int base, uint32_t (*v)[UD]) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int idx = base + u * NW * 64;
                if (idx < total) {
#pragma unroll
                    for (int d = 0; d < UD; ++d) xs[idx * UD + d] = v[u][d];
                }
            }
        };
        uint32_t v[UNROLL][UD];
        batch_load(threadIdx.x, v);
#pragma unroll
        for (int u = 0; u < D; ++u) fetch(u, u);
        batch_store(threadIdx.x, v);
        for (int base = threadIdx.x + NW * 64 * UNROLL; base < total; base += NW * 64 * UNROLL) {
            batch_load(base, v);
            batch_store(base, v);
        }
    }
    __syncthreads();

    float acc[MR];
#pragma unroll
    for (int r = 0; r < MR; ++r) acc[r] = 0.f;
    const int per_wave = (chunks - wave + NW - 1) / NW;          // chunks of this wave, wave-uniform (chunks >= NW is not required)
    for (int t0 = 0; t0 < per_wave; t0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int t = t0 + u;
            const bool live = t < per_wave;                       // scalar condition: no load depends on it
            const int c = wave + t * NW;
            uint32_t fbv[4][kHalfDw];
            uint32_t ebv = 0;
            if (live) {
#pragma unroll
                for (int j = 0; j < 4; ++j) Unpack<WB, B>::run(pb[u], j, fbv[j]);
                ebv = eb[u];
            }
            fetch(u, t + D);                                      // the slot is free: refill it
            if (live) {
                const uint32_t* xc = xs + c * XD;
                uint32_t pa[kDwA], ea[4];
                if (i < 8) {
#pragma unroll
                    for (int d = 0; d < kDwA; ++d) pa[d] = xc[(h * 8 + i) * kDwA + d];
                } else {
#pragma unroll
                    for (int d = 0; d < kDwA; ++d) pa[d] = 0;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) ea[r] = xc[16 * kDwA + 4 * h + r];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t fa[kHalfDw];
                    Unpack<WA, B>::run(pa, j, fa);
                    const v16i d = block_mfma<B>(fa, fbv[j]);
                    const int ebj = (int)((ebv >> (8 * j)) & 0xFFu) + eadj;
#pragma unroll
                    for (int r = 0; r < MR; ++r) {
                        const int e = (int)((ea[r] >> (8 * j)) & 0xFFu) + ebj;
                        acc[r] += __builtin_ldexpf((float)d[r], e);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < MR; ++r) red[(wave * MR + r) * 64 + lane] = acc[r];
    __syncthreads();
    for (int t = threadIdx.x; t < MR * 64; t += NW * 64) {
        const int r = t >> 6, l = t & 63;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[(w * MR + r) * 64 + l];
        const int64_t m = 4 * (l >> 5) + r;
        const int64_t n = gb * 32 + (l & 31);
        if (m < g.M && n < g.N) g.Y[bz * g.batch_stride_y + m * g.ldy + n] = s;
    }
}

constexpr int kStreamDepth = 5;

template <int WA, int WB, int B, int MR, int NW>
mx_status launch_stream(const GemmArgs& g, int64_t batch, size_t smem, hipStream_t st) {
    auto kern = gemv_stream_kernel<WA, WB, B, NW, kStreamDepth, MR>;
    static std::atomic<uint64_t> done{0};
    if (!allow_dynamic_lds((const void*)kern, 160 * 1024, done)) return MX_ERR_DEVICE;
    dim3 grid((unsigned)g.groupsB, (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), smem, st, g);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int WA, int WB, int B>
mx_status launch(const GemmArgs& g, int64_t batch, hipStream_t st) {
    if (g.M <= 8) {
        // streaming kernel when the left operand fits in LDS next to the reduction buffer; 16 waves per
        // workgroup when there are too few column groups to fill the chip with 8
        constexpr int XD = 16 * Piece<WA, B>::kDw + 8;
        const int nw = g.groupsB * batch < 256 ? 16 : 8;
        const size_t smem = (size_t)g.chunks * XD * 4 + (size_t)nw * 4 * 64 * 4;
        if (g.chunks > 0 && (g.chunks + 1024) * g.recordB < (1LL << 31) && smem <= 160 * 1024) {
            if (nw == 16) {
                if (g.M == 1) return launch_stream<WA, WB, B, 1, 16>(g, batch, smem, st);
                return launch_stream<WA, WB, B, 4, 16>(g, batch, smem, st);
            }
            if (g.M == 1) return launch_stream<WA, WB, B, 1, 8>(g, batch, smem, st);
            return launch_stream<WA, WB, B, 4, 8>(g, batch, smem, st);
        }
        dim3 grid((unsigned)g.groupsB, (unsigned)batch);
        hipLaunchKernelGGL((gemv_fragment_kernel<WA, WB, B, kGemvWaves>), grid, dim3(kGemvWaves * 64), 0, st, g);
    } else {
        dim3 grid((unsigned)ceil_div(g.groupsB, 4), (unsigned)ceil_div(g.groupsA, 4), (unsigned)batch);
        hipLaunchKernelGGL((gemm_fragment_kernel<WA, WB, B>), grid, dim3(256), 0, st, g);
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

template <int B>
mx_status dispatch_widths(const GemmArgs& g, int wa, int wb, int64_t batch, hipStream_t st) {
    MX_SW(wa, kWA, MX_SW(wb, kWB, return (launch<kWA, kWB, B>(g, batch, st))));
    return MX_ERR_BAD_ARG;
}

}  // namespace

#define MX_CAT2(a, b) a##b
#define MX_CAT(a, b) MX_CAT2(a, b)
mx_status MX_CAT(gemm_block, MX_GEMM_BLOCK)(const GemmArgs& g, int wa, int wb, int64_t batch, hipStream_t st) {
    return dispatch_widths<MX_GEMM_BLOCK>(g, wa, wb, batch, st);
}

}  // namespace mx
