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
// Work split: a workgroup of four waves owns 128 queries of one head (a wave: one tile of 32, its
// Q fragments stay in registers), two workgroups per compute unit; the K (and in sweep 2 the V^T)
// units of one tile of 32 keys are copied global -> LDS with 16-byte direct-to-LDS loads, four
// stages, one barrier per key tile.
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
    float pair;                    // 0 when two neighbouring queries share the exponents of P, else -inf
    float wide;                    // 0 when P is quantized in blocks of 32 keys (a whole key tile), else -inf
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

// The value is computed before this point of the program: an empty volatile statement is ordered with the
// scheduling fences, and so, through it, is the (otherwise freely movable) arithmetic that produces v.
__device__ __forceinline__ void pin(float v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ void pin(int v) { asm volatile("" ::"v"(v)); }

constexpr int kAttnStages = 4;
// Query tiles of 32 per wave.  1: 205 registers, two workgroups per compute unit, accumulators in ordinary
// registers (123 us at 32 x 2048 x 2048 x 128); 2: 363 registers, one workgroup, half the LDS reads per matrix
// instruction but every score copied out of the accumulation registers (128 us).
constexpr int kAttnRQ = 1;

// KS: K steps of 32 along the head dimension (2 or 4); DT: tiles of 32 along the head dimension of V;
// RQ: query tiles of 32 per wave.  RQ = 2 needs more than 256 registers (one wave per SIMD); RQ = 1 leaves
// room for two workgroups per compute unit, whose waves fill each other's waits.
template <int KS, int DT, int RND, int RQ>
__global__ __launch_bounds__(256, RQ == 1 ? 2 : 1) void attention_bf16_kernel(AttnArgs g) {
    constexpr int S = kAttnStages;
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

    // the wave's Q fragments (right operand of S^T = K Q^T): lane 32h + i holds query i, elements 8h..8h+7.
    // A negative scale is carried by the operand (sign bits flipped: every product and sum changes
    // sign exactly), so that below the largest score is the largest argument of exp.
    const int64_t qt0 = (bq * 4 + wave) * RQ;
    const int flip = g.c < 0.f ? (int)0x80008000u : 0;
    const float c = __builtin_fabsf(g.c);
    v4i qf[RQ][NK];
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        int64_t rt = qt0 + q;
        rt = rt < g.q_tiles ? rt : g.q_tiles - 1;       // tiles past the matrix re-read its last tile (never stored)
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
            qf[q][kk] = *reinterpret_cast<const v4i*>(Qbase + (rt * KS + (kk >> 1)) * kBfUnitBytes + (kk & 1) * 1024 + lane16);
#pragma unroll
            for (int d = 0; d < 4; ++d) qf[q][kk][d] ^= flip;
        }
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
    const int wm2 = g.wp - 2;

    // scores of two consecutive key tiles live in two register sets: while the arithmetic on one tile's
    // scores runs on the vector units, the matrix cores take the next tile's.
    v16f s[2][RQ];

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
        // S^T of the key tile in `stage` into register set `set`: fragments first, then matrix instruction
        // m = 0 .. 2*NK-1 one at a time (the caller slots vector work between them)
        v4i kf[NK];
        auto read_k = [&](int stage) {
            const uint8_t* st = smem + stage * STAGE;
#pragma unroll
            for (int kk = 0; kk < NK; ++kk)
                kf[kk] = *reinterpret_cast<const v4i*>(st + (kk >> 1) * kBfUnitBytes + (kk & 1) * 1024 + koff);
        };
        auto score_mfma = [&](int m, auto setc) {
            constexpr int set = decltype(setc)::value;
            const int kk = m / RQ, q = m % RQ;              // consecutive instructions never share an accumulator
            v16f zero;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.f;
            s[set][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, kf[kk]), __builtin_bit_cast(v8bf, qf[q][kk]),
                                                                kk == 0 ? zero : s[set][q], 0, 0, 0);
        };
        // One key tile: tile kt's scores are in set kt % 2, tile kt+1's are started into the other set.
        // RAG: keys past Sk are masked (only the last tile can have them).
        // The instruction order is written out and pinned: one matrix instruction, then its share of the
        // vector work (given as numbered units), so that both pipes stay busy with one wave per SIMD.
        auto body = [&](int64_t kt, int cur, auto setc, auto ragc) {
            constexpr int set = decltype(setc)::value;
            constexpr bool RAG = decltype(ragc)::value;
            const auto nset = std::integral_constant<int, set ^ 1>{};
            const int nxt = cur + 1 == S ? 0 : cur + 1;
            const uint8_t* st = smem + cur * STAGE;
            v4i vf[PV ? DT : 1][2];
            if constexpr (PV) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        vf[dt][b] = *reinterpret_cast<const v4i*>(st + (KS + dt) * kBfUnitBytes + b * 1024 + lane16);
            }
            // copies in flight, oldest first: tiles kt+1 .. kt+S-1.  Tile kt+1 has landed once only the newest
            // S-2 tiles' copies are outstanding; the barrier publishes it and tells that every wave has taken
            // what it needs of tile kt's stage, which the copy of tile kt+S overwrites.
            wait_vmcnt<(S - 2) * NL>();
            __syncthreads();
            issue(kt + S, cur);
            read_k(nxt);
            const int valid = (int)(g.Sk - kt * 32) - 8 * h;   // this lane's key 16*b + e is real iff 16*b + e < valid
            auto masked = [&](int r) { return RAG && 16 * (r >> 3) + (r & 7) >= valid; };
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!PV) {
                // units of one query tile: 0 = tile maximum and the new running maximum, 1..4 = four
                // exponentials each, 5 = the running sum
                constexpr int NU = 6;
                float m_old[RQ], m_use[RQ], sum[RQ];
                auto unit = [&](int q, int u) {
                    if (u == 0) {
                        float sm = -__builtin_inff();
#pragma unroll
                        for (int r = 0; r < 16; ++r) sm = __builtin_fmaxf(sm, masked(r) ? -__builtin_inff() : s[set][q][r]);
                        m_old[q] = m_run[q];
                        m_run[q] = __builtin_fmaxf(m_run[q], sm * c);
                        m_use[q] = m_run[q] == -__builtin_inff() ? 0.f : m_run[q];
                        sum[q] = 0.f;
                        pin(m_use[q]);
                    } else if (u < 5) {
#pragma unroll
                        for (int r = 4 * (u - 1); r < 4 * u; ++r) {
                            float arg = __builtin_fmaf(s[set][q][r], c, -m_use[q]);
                            if (masked(r)) arg = -__builtin_inff();   // also when c is 0
                            sum[q] += __builtin_amdgcn_exp2f(arg);
                        }
                        pin(sum[q]);
                    } else {
                        l_run[q] = l_run[q] * __builtin_amdgcn_exp2f(m_old[q] - m_use[q]) + sum[q];
                        pin(l_run[q]);
                    }
                };
                constexpr int NM = RQ * NK;
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    score_mfma(m, nset);
#pragma unroll
                    for (int x = m * (RQ * NU) / NM; x < (m + 1) * (RQ * NU) / NM; ++x) unit(x / NU, x % NU);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // One query tile = two blocks of 16 keys, this lane's half of each.  With a = log2 of the
                // probability, the block exponent is the integer part of the largest a (the quantizer's
                // floor(log2 max)) and the mantissas are round(2^(a - E + w - 2)): the arithmetic of mx_quantize
                // on P.  exp2 grows with the score, so the maximum is taken over the scores themselves.
                // Units: 0 = half-block maxima, their exchange with the other lane half, the exponents;
                // 1..16 = one element each; 17, 18 = operand registers.  (Taking the elements four at a time,
                // operation by operation, measured slower: the exponentials then queue behind each other.)
                constexpr int NU = 19;
                float el[RQ][16], off[RQ][2];
                int sh[RQ][2];
                v4i pf[RQ][2];
                auto unit = [&](int q, int u) {
                    if (u == 0) {
                        float mb[2];
#pragma unroll
                        for (int b = 0; b < 2; ++b) {
                            float sm = -__builtin_inff();
#pragma unroll
                            for (int e = 0; e < 8; ++e) sm = __builtin_fmaxf(sm, masked(8 * b + e) ? -__builtin_inff() : s[set][q][8 * b + e]);
                            // both lane halves get the larger of the two halves' values
                            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(sm), __float_as_uint(sm), false, false);
                            sm = __builtin_fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                            float m = __builtin_fmaf(sm, c, -mrow[q]);
                            // two-row blocks: queries 2t and 2t+1 (neighbouring lanes) share the exponent, the larger
                            // of the two log-probabilities; one-row blocks add -inf to the neighbour's and keep their own
                            m = __builtin_fmaxf(m, g.pair + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                                                                0, __builtin_bit_cast(int, m), 0xB1, 0xF, 0xF, true)));
                            mb[b] = m;
                        }
#pragma unroll
                        for (int b = 0; b < 2; ++b) {
                            // blocks of 32: the tile's two runs of 16 keys are one block (the same trick: + 0 or + -inf)
                            float m = __builtin_fmaxf(mb[b], g.wide + mb[b ^ 1]);
                            m = __builtin_fmaxf(m, -200.f);                   // also for all keys masked, or c = 0 with them
                            int E = (int)__builtin_floorf(m);
                            E = E < -g.bias_p ? -g.bias_p : E;
                            E = E > g.emax_p ? g.emax_p : E;
                            sh[q][b] = wm2 - E;
                            off[q][b] = (float)sh[q][b] - mrow[q];
                            pin(off[q][b]);
                        }
                    } else if (u < 17) {
                        const int r = u - 1, b = r >> 3;
                        float arg = __builtin_fmaf(s[set][q][r], c, off[q][b]);
                        if (masked(r)) arg = -__builtin_inff();
                        const float sc = __builtin_amdgcn_exp2f(arg);
                        float v = RND == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
                        v = __builtin_fminf(v, qmax);                         // probabilities are not negative
                        el[q][r] = __builtin_ldexpf(v, -sh[q][b]);            // an exact bfloat16 number
                        pin(el[q][r]);
                    } else {
                        const int b = u - 17;
#pragma unroll
                        for (int d = 0; d < 4; ++d)                           // the upper halves of two fp32 values
                            pf[q][b][d] = (int)__builtin_amdgcn_perm(__float_as_uint(el[q][8 * b + 2 * d + 1]),
                                                                     __float_as_uint(el[q][8 * b + 2 * d]), 0x07060302u);
#pragma unroll
                        for (int d = 0; d < 4; ++d) pin(pf[q][b][d]);
                    }
                };
                auto out_mfma = [&](int q, int m) {
                    const int b = m / DT, dt = m % DT;
                    o[dt][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, vf[dt][b]),
                                                                       __builtin_bit_cast(v8bf, pf[q][b]), o[dt][q], 0, 0, 0);
                };
                // the next tile's scores under the vector work of the first query tile, every query tile's
                // second product under the vector work of the following one, the last one's bare
                constexpr int NM = RQ * NK;
                unit(0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    score_mfma(m, nset);
#pragma unroll
                    for (int x = 1 + m * (NU - 1) / NM; x < 1 + (m + 1) * (NU - 1) / NM; ++x) unit(0, x);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int q = 1; q < RQ; ++q)
#pragma unroll
                    for (int m = 0; m < 2 * DT; ++m) {
                        out_mfma(q - 1, m);
#pragma unroll
                        for (int x = m * NU / (2 * DT); x < (m + 1) * NU / (2 * DT); ++x) unit(q, x);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                for (int m = 0; m < 2 * DT; ++m) out_mfma(RQ - 1, m);
                __builtin_amdgcn_sched_barrier(0);
            }
        };

#pragma unroll
        for (int st = 0; st < S; ++st) issue(st, st);
        wait_vmcnt<(S - 1) * NL>();
        __syncthreads();
        read_k(0);
#pragma unroll
        for (int m = 0; m < RQ * NK; ++m) score_mfma(m, std::integral_constant<int, 0>{});
        // tiles in pairs (the register sets alternate); the last one or two tiles take the masking form
        int64_t kt = 0;
        int cur = 0;
        auto advance = [&]() { cur = cur + 1 == S ? 0 : cur + 1; ++kt; };
        while (kt + 2 < g.nt) {
            body(kt, cur, std::integral_constant<int, 0>{}, std::false_type{}); advance();
            body(kt, cur, std::integral_constant<int, 1>{}, std::false_type{}); advance();
        }
        body(kt, cur, std::integral_constant<int, 0>{}, std::true_type{}); advance();
        if (kt < g.nt) { body(kt, cur, std::integral_constant<int, 1>{}, std::true_type{}); advance(); }
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
    auto store = [&](auto vecc) {
        constexpr bool VEC = decltype(vecc)::value;
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            const int64_t row = (qt0 + q) * 32 + i;
            if (row < g.Sq) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int d = dt * 32 + 8 * gq + 4 * h;
                        if (d < (int)g.D) {                  // D is a multiple of 16: four elements or none
                            float* dst = O + row * g.ldo + d;
                            if constexpr (VEC) {
                                *reinterpret_cast<float4*>(dst) = make_float4(o[dt][q][4 * gq], o[dt][q][4 * gq + 1],
                                                                              o[dt][q][4 * gq + 2], o[dt][q][4 * gq + 3]);
                            } else {
#pragma unroll
                                for (int j = 0; j < 4; ++j) dst[j] = o[dt][q][4 * gq + j];
                            }
                        }
                    }
            }
        }
    };
    if (g.vec) store(std::true_type{}); else store(std::false_type{});
}

template <int KS, int DT, int RQ>
mx_status launch_attention(AttnArgs& g, int64_t batch, int rnd, hipStream_t st) {
    constexpr int smem = kAttnStages * (KS + DT) * kBfUnitBytes;
    static_assert(smem * (RQ == 1 ? 2 : 1) <= 160 * 1024, "LDS budget of one compute unit");
    auto k0 = attention_bf16_kernel<KS, DT, MX_RNE, RQ>;
    auto k1 = attention_bf16_kernel<KS, DT, MX_RTZ, RQ>;
    static std::atomic<uint64_t> done0{0}, done1{0};
    if (!allow_dynamic_lds((const void*)k0, smem, done0) || !allow_dynamic_lds((const void*)k1, smem, done1))
        return MX_ERR_DEVICE;
    g.tiles_q = ceil_div(g.Sq, 128 * RQ);
    g.total = g.tiles_q * batch;
    if (g.total > 0x7fffff00LL) return MX_ERR_UNSUPPORTED;
    dim3 grid((unsigned)(ceil_div(g.total, 8) * 8));
    hipLaunchKernelGGL(rnd == MX_RNE ? k0 : k1, grid, dim3(256), smem, st, g);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int KS, int DT>
mx_status launch_attention_rq(AttnArgs& g, int64_t batch, int rnd, hipStream_t st) {
    return launch_attention<KS, DT, kAttnRQ>(g, batch, rnd, st);
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
    if (fq.block != fk.block || fq.exp_bits != fk.exp_bits || fp.block % fv.block != 0 || fp.exp_bits != fv.exp_bits)
        return MX_ERR_BAD_ARG;
    if (layout != MX_LAYOUT_FRAGMENT && layout != MX_LAYOUT_MATRIX) return MX_ERR_BAD_ARG;
    if (batch < 0 || Sq < 0 || Sk < 1 || D < 1 || D % fq.block != 0 || Sk % fp.block != 0 || ldo < D) return MX_ERR_BAD_ARG;
    if (!(scale == scale) || __builtin_isinf(scale)) return MX_ERR_BAD_ARG;
    // two-row blocks: whole pairs of queries (Q, P), of keys (K), of columns of V (the rows of V^T)
    if (((fq.block_rows == 2 || fp.block_rows == 2) && Sq % 2 != 0) || (fk.block_rows == 2 && Sk % 2 != 0) ||
        (fv.block_rows == 2 && D % 2 != 0))
        return MX_ERR_BAD_ARG;
    // built for the bfloat16 form of the matrix layout, which is declared with blocks of 16.  The packed operands carry
    // their exponents inside the elements, so their block shape (one or two rows) makes no difference here; P's does:
    // its blocks are 16 keys, or 32 (one key tile of the kernel).
    if (layout != MX_LAYOUT_MATRIX || !matrix_format_ok(fq) || !matrix_format_ok(fk) || !matrix_format_ok(fv) ||
        !matrix_format_ok(fp))
        return MX_ERR_UNSUPPORTED;
    if (fq.block != 16 || fv.block != 16 || (fp.block != 16 && fp.block != 32) || D > 128) return MX_ERR_UNSUPPORTED;
    if (batch == 0 || Sq == 0) return MX_OK;
    if (!Q_packed || !K_packed || !Vt_packed || !O || ((uintptr_t)O & 3)) return MX_ERR_BAD_ARG;
    if (batch > 1 && o_batch_stride < (Sq - 1) * ldo + D) return MX_ERR_BAD_ARG;      // heads would overlap
    if (((uintptr_t)Q_packed & 255) || ((uintptr_t)K_packed & 255) || ((uintptr_t)Vt_packed & 255)) return MX_ERR_BAD_ARG;
    const BfGeom gq = bf_geom(Sq, D), gk = bf_geom(Sk, D), gv = bf_geom(D, Sk);
    AttnArgs g;
    g.Q = (const uint8_t*)Q_packed; g.K = (const uint8_t*)K_packed; g.V = (const uint8_t*)Vt_packed; g.O = O;
    g.Sq = Sq; g.Sk = Sk; g.D = D;
    g.matrixQ = gq.matrix; g.matrixK = gk.matrix; g.matrixV = gv.matrix;
    g.q_tiles = gq.row_tiles; g.nt = gk.row_tiles; g.v_ksteps = gv.ksteps;
    g.ldo = ldo; g.o_batch_stride = o_batch_stride;
    g.tiles_q = g.total = 0;
    g.c = scale * 1.4426950408889634f;
    g.wp = fp.mant_bits; g.bias_p = (1 << (fp.exp_bits - 1)) - 1;
    g.emax_p = ((1 << fp.exp_bits) - 1) - g.bias_p;
    g.vec = (((uintptr_t)O & 15) == 0 && ldo % 4 == 0 && o_batch_stride % 4 == 0) ? 1 : 0;
    g.pair = fp.block_rows == 2 ? 0.f : -__builtin_inff();
    g.wide = fp.block == 32 ? 0.f : -__builtin_inff();
    const int dt = (int)ceil_div(D, 32);
    hipStream_t st = (hipStream_t)stream;
    if (gq.ksteps == 2)
        return dt == 1 ? launch_attention_rq<2, 1>(g, batch, fp.rounding, st) : launch_attention_rq<2, 2>(g, batch, fp.rounding, st);
    return dt == 3 ? launch_attention_rq<4, 3>(g, batch, fp.rounding, st) : launch_attention_rq<4, 4>(g, batch, fp.rounding, st);
}
