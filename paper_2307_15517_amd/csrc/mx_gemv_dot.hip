// Decode kernel for very few activation rows (M <= 4), right operand in the fragment layout.
//
// Arithmetic as in the MFMA kernels (Section 3.2 of the paper: exact integer block dots, the two
// shared exponents applied once per block), but the dots are taken with v_dot4_i32_i8: with one
// to four rows the 32x32 MFMA would spend three quarters of its work, and all of its epilogue,
// on rows that do not exist, and the kernel is bound by instruction issue, not by the matrix
// cores.  Lane 32*h + i owns output column 32*gb + i and half h of every block (that is what the
// fragment layout gives it); the two half dots of a block are added as integers across the wave
// halves, so that the block's dot is exact before its scale is applied; half h then accumulates
// every second block in fp32 and the halves meet in one cross-lane add at the end.  The
// activations are unpacked to int8 once per workgroup into LDS and read back as broadcasts.
#include "mx_gemm.h"
#include "mx_frag.h"

namespace mx {
namespace {

template <int W, int B> using UnpackB = Unpack<W, B>;

// Mantissa t of half-block j of a left-operand lane piece (runtime width), sign-extended.
__device__ __forceinline__ int piece_get(const uint8_t* piece, int j, int t, int w, int B) {
    int pos = j * (B / 2) + t;
    if (w == 4) {                        // nibbles of every group of 8 are stored e0 e4 e1 e5 e2 e6 e3 e7
        const int t8 = t & 7;
        pos = j * (B / 2) + (t & ~7) + (t8 < 4 ? 2 * t8 : 2 * (t8 - 4) + 1);
    }
    const int bit = pos * w, sh = bit & 7;
    uint32_t v = piece[bit >> 3];
    if (sh + w > 8) v |= (uint32_t)piece[(bit >> 3) + 1] << 8;
    v >>= sh;
    return ((int)(v << (32 - w))) >> (32 - w);
}

struct DotArgs {
    GemmArgs g;
    int32_t wa;          // stored width of the left operand
    // fused form (mx_linear): the left operand is still fp32 and is quantized on the way into LDS
    const float* x;      // null: take the packed left operand g.A
    int64_t x_stride;
    int32_t bias, emax, rounding;
};

// MP: rows computed (1, 2 or 4; M <= MP, missing rows are fed zeros).  NW waves per workgroup, each
// keeping a ring of D chunks of weights in flight.
template <int WB, int B, int MP, int NW, int D>
__global__ __launch_bounds__(NW * 64) void gemv_dot_kernel(DotArgs a) {
    const GemmArgs& g = a.g;
    constexpr int kDwB = Piece<WB, B>::kDw;
    constexpr int kHalfDw = B / 8;               // int8 dwords of a half block
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    const int chunks = (int)g.chunks;
    // LDS: x8[MP][chunks*4 blocks][2 halves][kHalfDw dwords], xe[MP][chunks] exponent dwords, red[NW][MP][64]
    uint32_t* x8 = lds;
    uint32_t* xe = x8 + MP * chunks * 4 * 2 * kHalfDw;
    float* red = reinterpret_cast<float*>(xe + MP * chunks);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int64_t gb = blockIdx.x;
    const int64_t bz = blockIdx.y;
    const uint8_t* Abase = g.A + bz * g.matrixA;
    const uint8_t* Bbase = g.B + bz * g.matrixB + gb * g.chunks * g.recordB;
    const int eadj = g.eadj - UnpackB<WB, B>::kScaleLog2;
    const int pieceA = B * a.wa / 4;             // bytes of a left-operand lane piece

    // ring of D chunks of this column group's records; a chunk number past the end reads zeros
    const BufRsrc rB = make_rsrc(Bbase, (uint32_t)(chunks * g.recordB));
    uint32_t pb[D][kDwB], eb[D];
    auto fetch = [&](int slot, int t) {
        const uint32_t off = (uint32_t)(wave + t * NW) * (uint32_t)g.recordB;
        buf_load_dwords<kDwB>(rB, off + lane * (kDwB * 4), pb[slot]);
        buf_load_dwords<1>(rB, off + 64 * (kDwB * 4) + i * 4, &eb[slot]);
    };
    // Loads return in the order of issue, so whatever the workgroup needs first is requested first:
    // the activations, then the ring of weights; the arithmetic on the activations then runs while
    // the weights are in flight.
    if (a.x != nullptr) {
        // fp32 activations -> MXInt (the arithmetic of mx_quantize) -> int8 in LDS.  One item is four
        // consecutive elements of a row, items of consecutive lanes are consecutive (a wave reads 1 KB
        // per instruction), so a block is B/4 consecutive lanes and its maximum takes log2(B/4) DPP
        // steps.  Every workgroup reads the same activations; each starts at a different sweep so that
        // they do not all ask the same cache channel at the same time.
        constexpr int T = NW * 64;
        constexpr int XU = 8;                                   // items per thread requested before the weights
        const int kpad = chunks * 4 * B;                        // row length in LDS (slots past K hold zeros)
        const int sweeps = (kpad / 4 + T - 1) / T;
        const int n_it = MP * sweeps;
        const int rot = (int)(gb % sweeps);
        const float qmax = (float)((1 << (a.wa - 1)) - 1);
        uint8_t* xeb = reinterpret_cast<uint8_t*>(xe);
        auto item_pos = [&](int it, int& m, int& e) {
            m = it / sweeps;
            int kk = it - m * sweeps + rot;
            kk = kk >= sweeps ? kk - sweeps : kk;
            e = 4 * ((int)threadIdx.x + T * kk);
        };
        auto item_load = [&](int it) -> float4 {
            int m, e;
            item_pos(it, m, e);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m < g.M && e < g.K) {                           // K is a multiple of 4: all four or none
                const float* src = a.x + (int64_t)m * a.x_stride + e;
                v = *reinterpret_cast<const float4*>(src);       // the fused form is only entered with 16-byte aligned rows
            }
            return v;
        };
        auto item_store = [&](int it, const float4& v) {
            int m, e;
            item_pos(it, m, e);
            const uint32_t b0 = __float_as_uint(v.x) & 0x7fffffffu, b1 = __float_as_uint(v.y) & 0x7fffffffu;
            const uint32_t b2 = __float_as_uint(v.z) & 0x7fffffffu, b3 = __float_as_uint(v.w) & 0x7fffffffu;
            uint32_t am = b0 > b1 ? b0 : b1, a2 = b2 > b3 ? b2 : b3;
            am = am > a2 ? am : a2;
            uint32_t o;
            o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);  am = o > am ? o : am;   // lane ^ 1
            o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0x4E, 0xF, 0xF, true);  am = o > am ? o : am;   // lane ^ 2
            if (B >= 32) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0x141, 0xF, 0xF, true); am = o > am ? o : am; }   // 7 - lane within 8
            if (B >= 64) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0x140, 0xF, 0xF, true); am = o > am ? o : am; }   // 15 - lane within 16
            const int ef = (int)(am >> 23);
            int E = ef == 0 ? -127 : ef - 127;
            E = E < -a.bias ? -a.bias : E;
            E = E > a.emax ? a.emax : E;
            const int shift = (a.wa - 2) - E;
            auto code = [&](float x) -> uint32_t {
                const float sc = __builtin_ldexpf(x, shift);
                float r = a.rounding == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
                r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
                return (uint32_t)(int)r & 0xFFu;
            };
            if (e < kpad) {
                x8[(m * kpad + e) >> 2] = code(v.x) | (code(v.y) << 8) | (code(v.z) << 16) | (code(v.w) << 24);
                if ((e & (B - 1)) == 0) xeb[m * chunks * 4 + e / B] = (m < g.M && e < g.K) ? (uint8_t)(E + a.bias) : (uint8_t)0;
            }
        };
        float4 xv[XU];
#pragma unroll
        for (int it = 0; it < XU; ++it)
            if (it < n_it) xv[it] = item_load(it);
#pragma unroll
        for (int u = 0; u < D; ++u) fetch(u, u);
#pragma unroll
        for (int it = 0; it < XU; ++it)
            if (it < n_it) item_store(it, xv[it]);
        for (int it = XU; it < n_it; ++it) item_store(it, item_load(it));
    } else {
    // packed activations -> int8 in LDS: one item per (row, chunk, half)
    for (int idx = threadIdx.x; idx < MP * chunks * 2; idx += NW * 64) {
        const int hh = idx & 1, c = (idx >> 1) % chunks, m = (idx >> 1) / chunks;
        const uint8_t* rec = Abase + (int64_t)c * g.recordA;
        const uint8_t* piece = rec + (32 * hh + m) * pieceA;
        uint32_t* dst = x8 + ((m * chunks + c) * 4 * 2 + hh) * kHalfDw;      // + j*2*kHalfDw per block
        if (m < g.M) {
            if (a.wa == 8) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int d = 0; d < kHalfDw; ++d)
                        dst[j * 2 * kHalfDw + d] = reinterpret_cast<const uint32_t*>(piece)[j * kHalfDw + d];
            } else {
                for (int j = 0; j < 4; ++j)
                    for (int d = 0; d < kHalfDw; ++d) {
                        uint32_t o = 0;
                        for (int t = 0; t < 4; ++t)
                            o |= ((uint32_t)piece_get(piece, j, d * 4 + t, a.wa, B) & 0xFFu) << (8 * t);
                        dst[j * 2 * kHalfDw + d] = o;
                    }
            }
            if (hh == 0) xe[m * chunks + c] = reinterpret_cast<const uint32_t*>(rec + 64 * pieceA)[m];
        } else {
            for (int j = 0; j < 4; ++j)
                for (int d = 0; d < kHalfDw; ++d) dst[j * 2 * kHalfDw + d] = 0;
            if (hh == 0) xe[m * chunks + c] = 0;
        }
    }
#pragma unroll
    for (int u = 0; u < D; ++u) fetch(u, u);
    }
    __syncthreads();

    float acc[MP];
#pragma unroll
    for (int m = 0; m < MP; ++m) acc[m] = 0.f;
    const int per_wave = (chunks - wave + NW - 1) / NW;          // wave-uniform
    for (int t0 = 0; t0 < per_wave; t0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int t = t0 + u;
            const bool live = t < per_wave;                       // scalar condition: no load depends on it
            const int c = wave + t * NW;
            uint32_t fb[4][kHalfDw];
            uint32_t ebv = 0;
            if (live) {
#pragma unroll
                for (int j = 0; j < 4; ++j) UnpackB<WB, B>::run(pb[u], j, fb[j]);
                ebv = eb[u];
            }
            fetch(u, t + D);                                      // the slot is free: refill it
            if (live) {
                uint32_t exm[MP];
#pragma unroll
                for (int m = 0; m < MP; ++m) exm[m] = xe[m * chunks + c];
                // A block's dot must be exact before it is scaled: its two half dots (this lane's and the
                // other wave half's) are added as integers -- in fp32, halves that cancel would leave their
                // rounding behind, next to much smaller blocks.  One swap of the wave halves between the
                // registers of blocks 2*jp and 2*jp + 1 puts both half dots of block 2*jp + h into half h,
                // which scales and accumulates that block.
#pragma unroll
                for (int jp = 0; jp < 2; ++jp) {
                    const int sh = 16 * jp + 8 * h;               // exponent byte of block 2*jp + h
                    const int ebj = (int)((ebv >> sh) & 0xFFu) + eadj;
#pragma unroll
                    for (int m = 0; m < MP; ++m) {
                        int dh[2];
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) {
                            const int j = 2 * jp + jj;
                            const uint32_t* xv = x8 + (((m * chunks + c) * 4 + j) * 2 + h) * kHalfDw;
                            dh[jj] = 0;
#pragma unroll
                            for (int q = 0; q < kHalfDw; ++q) dh[jj] = __builtin_amdgcn_sdot4((int)fb[j][q], (int)xv[q], dh[jj], false);
                        }
                        // first result: lanes 0..31 keep theirs of block 2*jp, lanes 32..63 get the lower half's of
                        // block 2*jp + 1; second result: lanes 0..31 get the upper half's of block 2*jp, lanes
                        // 32..63 keep theirs of block 2*jp + 1
                        const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)dh[0], (unsigned)dh[1], false, false);
                        const int d = (int)(sw[0] + sw[1]);
                        const int e = (int)((exm[m] >> sh) & 0xFFu) + ebj;
                        acc[m] += __builtin_ldexpf((float)d, e);
                    }
                }
            }
        }
    }
    // the two halves of a column, then the waves
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        acc[m] += __shfl_xor(acc[m], 32, 64);
        if (h == 0) red[(wave * MP + m) * 32 + i] = acc[m];
    }
    __syncthreads();
    for (int t = threadIdx.x; t < MP * 32; t += NW * 64) {
        const int m = t >> 5, col = t & 31;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += red[(w * MP + m) * 32 + col];
        const int64_t n = gb * 32 + col;
        if (m < g.M && n < g.N) g.Y[bz * g.batch_stride_y + (int64_t)m * g.ldy + n] = s;
    }
}

constexpr int kDotDepth = 5;

// NW: 8 waves per workgroup when there are enough column groups to fill the chip, 16 when there are
// few (each workgroup then has to keep twice as many bytes in flight).
template <int WB, int B, int MP, int NW>
mx_status launch_dot_nw(const DotArgs& a, int64_t batch, hipStream_t st) {
    const size_t smem = ((size_t)MP * a.g.chunks * 4 * 2 * (B / 8) + (size_t)MP * a.g.chunks) * 4 +
                        (size_t)NW * MP * 32 * 4;
    if (smem > 160 * 1024) return MX_ERR_UNSUPPORTED;
    auto kern = gemv_dot_kernel<WB, B, MP, NW, kDotDepth>;
    static std::atomic<uint64_t> done{0};
    if (!allow_dynamic_lds((const void*)kern, 160 * 1024, done)) return MX_ERR_DEVICE;
    dim3 grid((unsigned)a.g.groupsB, (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), smem, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int WB, int B, int MP>
mx_status launch_dot(const DotArgs& a, int64_t batch, hipStream_t st) {
    if (a.g.groupsB * batch < 256) return launch_dot_nw<WB, B, MP, 16>(a, batch, st);
    return launch_dot_nw<WB, B, MP, 8>(a, batch, st);
}

template <int B, int MP>
mx_status dispatch_wb(const DotArgs& a, int wb, int64_t batch, hipStream_t st) {
    switch (wb) {
        case 2: return launch_dot<2, B, MP>(a, batch, st);
        case 3: return launch_dot<3, B, MP>(a, batch, st);
        case 4: return launch_dot<4, B, MP>(a, batch, st);
        case 5: return launch_dot<5, B, MP>(a, batch, st);
        case 6: return launch_dot<6, B, MP>(a, batch, st);
        case 7: return launch_dot<7, B, MP>(a, batch, st);
        case 8: return launch_dot<8, B, MP>(a, batch, st);
    }
    return MX_ERR_BAD_ARG;
}

template <int B>
mx_status dispatch_m(const DotArgs& a, int wb, int64_t batch, hipStream_t st) {
    if (a.g.M == 1) return dispatch_wb<B, 1>(a, wb, batch, st);
    if (a.g.M == 2) return dispatch_wb<B, 2>(a, wb, batch, st);
    return dispatch_wb<B, 4>(a, wb, batch, st);
}

}  // namespace

// M <= 4.  MX_ERR_UNSUPPORTED when the activations do not fit in LDS (the caller falls back).
// x != null: fused form, the left operand is quantized from fp32 (format fx) inside the kernel.
mx_status gemv_dot(const GemmArgs& g, int wa, int wb, int block, int64_t batch, hipStream_t st, const float* x,
                   int64_t x_stride, const mx_format* fx) {
    DotArgs a;
    a.g = g;
    a.wa = wa;
    a.x = x;
    a.x_stride = x_stride;
    if (x != nullptr && (((uintptr_t)x & 15) != 0 || (x_stride & 3) != 0)) return MX_ERR_UNSUPPORTED;
    a.bias = a.emax = a.rounding = 0;
    if (x != nullptr) {
        a.bias = (1 << (fx->exp_bits - 1)) - 1;
        a.emax = ((1 << fx->exp_bits) - 1) - a.bias;
        a.rounding = fx->rounding;
    }
    if (g.chunks <= 0) return MX_ERR_UNSUPPORTED;
    if ((g.chunks + 1024) * g.recordB >= (1LL << 31)) return MX_ERR_UNSUPPORTED;   // 32-bit ring offsets
    switch (block) {
        case 16: return dispatch_m<16>(a, wb, batch, st);
        case 32: return dispatch_m<32>(a, wb, batch, st);
        case 64: return dispatch_m<64>(a, wb, batch, st);
    }
    return MX_ERR_UNSUPPORTED;
}

}  // namespace mx
