// Attention with both matrix products in MXInt, in one kernel (blocks of 16, operands in the
// bfloat16 form of MX_LAYOUT_MATRIX, see mx_bf16.h).
//
// What is computed, per head (Fig. 1 of the paper: both products of the attention layer take
// quantized operands; Section 3.2: an emulated operator computes on quantized inputs, here the
// probabilities are quantized before the second product like any other operand):
//     S = Q K^T,  P = softmax(scale * S) along the keys (fp32),  P^ = MXInt(P) in blocks of 16 keys,
//     O = P^ V.
// The quantizer scales a block by a power of two chosen from the block's maximum, so P^ needs the
// final row maximum and row sum: the kernel sweeps the keys twice.  Sweep 1 takes S tile by tile
// and keeps a running maximum and sum per query; sweep 2 takes S again (34 GOP at the full size,
// far cheaper than the 537 MB of fp32 scores it replaces), forms P, quantizes it in registers and
// feeds it to the second product.
//
// Register-only hand-over between the products: S is computed transposed, S^T = K Q^T, so that in
// the result a lane holds one query (column) and 16 keys; the rows of the K operand are permuted
// when they are read from LDS (bits 2 and 3 of the row number swapped) so that those 16 keys are
// two whole blocks, elements 8h..8h+7 of each in lane half h -- exactly the operand layout of
// v_mfma_f32_32x32x16_bf16 for O^T = V^T P^T.  The block maximum is completed with the lane of the
// other half (one exchange per block).
//
// Work split: a workgroup of four waves owns 256 queries of one head (a wave: two tiles of 32, its
// Q fragments stay in registers); the K (and in sweep 2 the V^T) units of one tile of 32 keys are
// copied global -> LDS with 16-byte direct-to-LDS loads, four stages, one barrier per key tile.
#include <type_traits>

#include "mx_bf16.h"

namespace mx {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

struct AttnArgs {
    const uint8_t* Q;
    const uint8_t* K;
    const uint8_t* V;              // V^T: [D x Sk]
    float* O;
    int64_t Sq, Sk, D;
    int64_t matrixQ, matrixK, matrixV;
    int64_t q_tiles;               // row tiles of Q
    int64_t nt;                    // key tiles of 32
    int64_t v_ksteps;              // K steps of the V^T geometry
    int64_t ldo, o_batch_stride;
    int64_t tiles_q, total;        // workgroup tiles per head, and in all
    float c;                       // scale * log2(e)
    int32_t wp, bias_p, emax_p;
    int32_t vec;                   // O rows may be stored as float4
};

// 16 bytes per lane from global memory straight into LDS: lane L's bytes land at lds_addr + 16*L.
// Completion is awaited explicitly with s_waitcnt vmcnt(n) before the barrier that publishes a stage.
__device__ __forceinline__ void copy16_to_lds(const uint8_t* uniform_src, uint32_t lane_offset, uint32_t lds_addr) {
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, %1\n\t"
        :
        : "v"(lane_offset), "s"(uniform_src), "s"(lds_addr)
        : "memory", "m0");
}

// s_waitcnt vmcnt(n), every other counter left alone (gfx9 encoding: vmcnt = bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

constexpr int kAttnStages = 4;
constexpr int kAttnRQ = 2;         // query tiles of 32 per wave

// KS: K steps of 32 along the head dimension (2 or 4); DT: tiles of 32 along the head dimension of V.
template <int KS, int DT, int RND>
__global__ __launch_bounds__(256) void attention_bf16_kernel(AttnArgs g) {
    constexpr int RQ = kAttnRQ, S = kAttnStages;
    constexpr int NK = 2 * KS;                          // matrix instructions (16 elements) along the head dimension
    constexpr int STAGE = (KS + DT) * kBfUnitBytes;     // K units, then V^T units
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    // Workgroup n runs on XCD n % 8, each with its own L2: every XCD gets one contiguous range of
    // (head, query tile) pairs, so that the workgroups resident on it share the K and V of few heads.
    const int64_t per_xcd = (g.total + 7) / 8;
    const int64_t lin = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (lin >= g.total) return;
    const int64_t bz = lin / g.tiles_q, bq = lin - bz * g.tiles_q;
    const uint8_t* Qbase = g.Q + bz * g.matrixQ;
    const uint8_t* Kbase = g.K + bz * g.matrixK;
    const uint8_t* Vbase = g.V + bz * g.matrixV;
    const uint32_t lane16 = lane * 16;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

    // the wave's Q fragments (right operand of S^T = K Q^T): lane 32h + i holds query i, elements 8h..8h+7
    const int64_t qt0 = (bq * 4 + wave) * RQ;
    v4i qf[RQ][NK];
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        int64_t rt = qt0 + q;
        rt = rt < g.q_tiles ? rt : g.q_tiles - 1;       // tiles past the matrix re-read its last tile (never stored)
#pragma unroll
        for (int kk = 0; kk < NK; ++kk)
            qf[q][kk] = *reinterpret_cast<const v4i*>(Qbase + (rt * KS + (kk >> 1)) * kBfUnitBytes + (kk & 1) * 1024 + lane16);
    }

    // K rows are read permuted (bits 2 and 3 of the row swapped): result register r of lane 32h + i is
    // then key 16*(r/8) + 8h + r%8 of the tile.
    const int sig = (i & 0x13) | ((i & 4) << 1) | ((i & 8) >> 1);
    const int koff = (32 * h + sig) * 16;

    float m_run[RQ], l_run[RQ];                         // sweep 1: running maximum and sum of this lane's keys
    float mrow[RQ];                                     // sweep 2: row maximum + log2(row sum), in the exp2 domain
#pragma unroll
    for (int q = 0; q < RQ; ++q) { m_run[q] = -__builtin_inff(); l_run[q] = 0.f; mrow[q] = 0.f; }
    v16f o[DT][RQ];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int q = 0; q < RQ; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][q][r] = 0.f;
    const float qmax = (float)((1 << (g.wp - 1)) - 1);

    auto sweep = [&](auto pvc) {
        constexpr bool PV = decltype(pvc)::value;
        constexpr int NP = 2 * (PV ? KS + DT : KS);     // 1 KiB pieces per key tile
        constexpr int NL = (NP + 3) / 4;                // per wave
        const uint8_t* src[NL];
        int64_t adv[NL];
        int dst[NL];
#pragma unroll
        for (int q = 0; q < NL; ++q) {
            int t = q * 4 + wave;
            if (t >= NP) t = NP - 1;                    // duplicate the last copy instead of branching
            const int n = t >> 1, part = t & 1;
            if (n < KS) {
                src[q] = Kbase + n * kBfUnitBytes + part * 1024;
                adv[q] = KS * kBfUnitBytes;
            } else {
                src[q] = Vbase + (n - KS) * g.v_ksteps * kBfUnitBytes + part * 1024;
                adv[q] = kBfUnitBytes;
            }
            dst[q] = n * kBfUnitBytes + part * 1024;
        }
        // Copies are always issued in full, with the key tile clamped to the last one, so that the
        // number of copies in flight is the same at every step and the vmcnt waits stay exact.
        auto issue = [&](int64_t kt, int stage) {
            kt = kt < g.nt ? kt : g.nt - 1;
#pragma unroll
            for (int q = 0; q < NL; ++q) copy16_to_lds(src[q] + kt * adv[q], lane16, lds0 + stage * STAGE + dst[q]);
        };
#pragma unroll
        for (int st = 0; st < S - 1; ++st) issue(st, st);
        int cur = 0;
        for (int64_t kt = 0; kt < g.nt; ++kt) {
            // copies in flight, oldest first: tiles kt .. kt+S-2.  Tile kt has landed once only the newest
            // S-2 tiles' copies are outstanding; the barrier publishes it and tells that every wave is done
            // with the stage of tile kt-1, which the copy of tile kt+S-1 overwrites.
            wait_vmcnt<(S - 2) * NL>();
            __syncthreads();
            issue(kt + S - 1, cur == 0 ? S - 1 : cur - 1);
            const uint8_t* st = smem + cur * STAGE;
            cur = cur + 1 == S ? 0 : cur + 1;

            v4i kf[NK];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
                kf[kk] = *reinterpret_cast<const v4i*>(st + (kk >> 1) * kBfUnitBytes + (kk & 1) * 1024 + koff);
            v16f s[RQ];
#pragma unroll
            for (int q = 0; q < RQ; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[q][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
#pragma unroll
                for (int q = 0; q < RQ; ++q)
                    s[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, kf[kk]),
                                                                   __builtin_bit_cast(v8bf, qf[q][kk]), s[q], 0, 0, 0);
            const bool ragged = (kt + 1) * 32 > g.Sk;   // keys past the end take no part (uniform branch)
            const int64_t key0 = kt * 32 + 8 * h;
            if constexpr (!PV) {
#pragma unroll
                for (int q = 0; q < RQ; ++q) {
                    float t[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) t[r] = s[q][r] * g.c;
                    if (ragged) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (key0 + 16 * (r >> 3) + (r & 7) >= g.Sk) t[r] = -__builtin_inff();
                    }
                    float tm = t[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) tm = __builtin_fmaxf(tm, t[r]);
                    const float m_new = __builtin_fmaxf(m_run[q], tm);
                    const float m_use = m_new == -__builtin_inff() ? 0.f : m_new;
                    float sum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(t[r] - m_use);
                    l_run[q] = l_run[q] * __builtin_amdgcn_exp2f(m_run[q] - m_use) + sum;
                    m_run[q] = m_new;
                }
            } else {
                v4i vf[DT][2];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        vf[dt][b] = *reinterpret_cast<const v4i*>(st + (KS + dt) * kBfUnitBytes + b * 1024 + lane16);
#pragma unroll
                for (int q = 0; q < RQ; ++q) {
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        // one block of 16 keys of query i: this lane's half, quantized with the arithmetic of mx_quantize
                        float p[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[q][8 * b + e], g.c, -mrow[q]));
                        if (ragged) {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (key0 + 16 * b + e >= g.Sk) p[e] = 0.f;
                        }
                        float am = p[0];
#pragma unroll
                        for (int e = 1; e < 8; ++e) am = __builtin_fmaxf(am, p[e]);
                        am = __builtin_fmaxf(am, __shfl_xor(am, 32, 64));
                        const int ef = (int)(__float_as_uint(am) >> 23);
                        int E = ef == 0 ? -127 : ef - 127;
                        E = E < -g.bias_p ? -g.bias_p : E;
                        E = E > g.emax_p ? g.emax_p : E;
                        const int sh = (g.wp - 2) - E;
                        uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float sc = __builtin_ldexpf(p[e], sh);
                            float r = RND == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
                            r = __builtin_fminf(r, qmax);                      // probabilities are not negative
                            out[e >> 1] |= bf16_of(r, -sh) << (16 * (e & 1));
                        }
                        v4i pf;
                        pf[0] = (int)out[0]; pf[1] = (int)out[1]; pf[2] = (int)out[2]; pf[3] = (int)out[3];
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
                            o[dt][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, vf[dt][b]),
                                                                               __builtin_bit_cast(v8bf, pf), o[dt][q], 0, 0, 0);
                    }
                }
            }
        }
        wait_vmcnt<0>();                                  // the clamped tail copies must not outlive the stage's next use
        __syncthreads();
    };

    sweep(std::false_type{});
    // row statistics: the two lane halves hold disjoint keys of the same query
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        const float mo = __shfl_xor(m_run[q], 32, 64), lo = __shfl_xor(l_run[q], 32, 64);
        const float mf = __builtin_fmaxf(m_run[q], mo);  // finite: there is at least one key
        const float a = __fmul_rn(l_run[q], __builtin_amdgcn_exp2f(m_run[q] - mf));
        const float b = __fmul_rn(lo, __builtin_amdgcn_exp2f(mo - mf));
        mrow[q] = mf + __builtin_amdgcn_logf(__fadd_rn(a, b));             // the same value in both halves
    }
    sweep(std::true_type{});

    // O^T registers: register r of lane 32h + i is element 8*(r/4) + 4h + r%4 of the tile's 32, query i
    float* O = g.O + bz * g.o_batch_stride;
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        const int64_t row = (qt0 + q) * 32 + i;
        if (row >= g.Sq) continue;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int64_t d = dt * 32 + 8 * gq + 4 * h;
                if (d >= g.D) continue;                   // D is a multiple of 16: four elements or none
                float* dst = O + row * g.ldo + d;
                if (g.vec) {
                    *reinterpret_cast<float4*>(dst) = make_float4(o[dt][q][4 * gq], o[dt][q][4 * gq + 1],
                                                                  o[dt][q][4 * gq + 2], o[dt][q][4 * gq + 3]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) dst[j] = o[dt][q][4 * gq + j];
                }
            }
    }
}

template <int KS, int DT>
mx_status launch_attention(const AttnArgs& g, int rnd, hipStream_t st) {
    constexpr int smem = kAttnStages * (KS + DT) * kBfUnitBytes;
    static_assert(smem <= 160 * 1024, "LDS budget of one compute unit");
    auto k0 = attention_bf16_kernel<KS, DT, MX_RNE>;
    auto k1 = attention_bf16_kernel<KS, DT, MX_RTZ>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)k0, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess ||
            hipFuncSetAttribute((const void*)k1, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return MX_ERR_DEVICE;
        configured = true;
    }
    if (g.total > 0x7fffff00LL) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)(ceil_div(g.total, 8) * 8));
    hipLaunchKernelGGL(rnd == MX_RNE ? k0 : k1, grid, dim3(256), smem, st, g);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

}  // namespace

bool matrix_format_ok(const mx_format& f);

}  // namespace mx

using namespace mx;

extern "C" mx_status mx_attention(int64_t batch, int64_t Sq, int64_t Sk, int64_t D, const void* Q_packed, mx_format fq,
                                  const void* K_packed, mx_format fk, const void* Vt_packed, mx_format fv, mx_format fp,
                                  float scale, int32_t layout, float* O, int64_t ldo, int64_t o_batch_stride,
                                  void* stream) {
    if (!format_ok_quant(fq) || !format_ok_quant(fk) || !format_ok_quant(fv) || !format_ok_quant(fp))
        return MX_ERR_BAD_ARG;
    if (fq.block != fk.block || fq.exp_bits != fk.exp_bits || fp.block != fv.block || fp.exp_bits != fv.exp_bits)
        return MX_ERR_BAD_ARG;
    if (layout != MX_LAYOUT_FRAGMENT && layout != MX_LAYOUT_MATRIX) return MX_ERR_BAD_ARG;
    if (batch < 0 || Sq < 0 || Sk < 1 || D < 1 || D % fq.block != 0 || Sk % fp.block != 0 || ldo < D) return MX_ERR_BAD_ARG;
    if (!(scale == scale) || __builtin_isinf(scale)) return MX_ERR_BAD_ARG;
    // built for the bfloat16 form of the matrix layout: blocks of 16 (one row each) in all four formats
    if (layout != MX_LAYOUT_MATRIX || !matrix_format_ok(fq) || !matrix_format_ok(fk) || !matrix_format_ok(fv) ||
        !matrix_format_ok(fp))
        return MX_ERR_UNSUPPORTED;
    if (fq.block != 16 || fp.block != 16 || fq.block_rows != 1 || fk.block_rows != 1 || fv.block_rows != 1 ||
        fp.block_rows != 1 || D > 128)
        return MX_ERR_UNSUPPORTED;
    if (batch == 0 || Sq == 0) return MX_OK;
    if (!Q_packed || !K_packed || !Vt_packed || !O) return MX_ERR_BAD_ARG;
    if (((uintptr_t)Q_packed & 255) || ((uintptr_t)K_packed & 255) || ((uintptr_t)Vt_packed & 255)) return MX_ERR_BAD_ARG;
    const BfGeom gq = bf_geom(Sq, D), gk = bf_geom(Sk, D), gv = bf_geom(D, Sk);
    AttnArgs g;
    g.Q = (const uint8_t*)Q_packed; g.K = (const uint8_t*)K_packed; g.V = (const uint8_t*)Vt_packed; g.O = O;
    g.Sq = Sq; g.Sk = Sk; g.D = D;
    g.matrixQ = gq.matrix; g.matrixK = gk.matrix; g.matrixV = gv.matrix;
    g.q_tiles = gq.row_tiles; g.nt = gk.row_tiles; g.v_ksteps = gv.ksteps;
    g.ldo = ldo; g.o_batch_stride = o_batch_stride;
    g.tiles_q = ceil_div(Sq, 128 * kAttnRQ);
    g.total = g.tiles_q * batch;
    g.c = scale * 1.4426950408889634f;
    g.wp = fp.mant_bits; g.bias_p = (1 << (fp.exp_bits - 1)) - 1;
    g.emax_p = ((1 << fp.exp_bits) - 1) - g.bias_p;
    g.vec = (((uintptr_t)O & 15) == 0 && ldo % 4 == 0 && o_batch_stride % 4 == 0) ? 1 : 0;
    const int dt = (int)ceil_div(D, 32);
    hipStream_t st = (hipStream_t)stream;
    if (gq.ksteps == 2) return dt == 1 ? launch_attention<2, 1>(g, fp.rounding, st) : launch_attention<2, 2>(g, fp.rounding, st);
    return dt == 3 ? launch_attention<4, 3>(g, fp.rounding, st) : launch_attention<4, 4>(g, fp.rounding, st);
}
