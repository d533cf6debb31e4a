// MXInt x MXInt product on the block-scaled fp6 matrix cores of gfx950 (operands in
// MX_LAYOUT_MATRIX, see mx_matrix.h), for block sizes 32 and 64.
//
// Arithmetic (Section 3.2 of the paper: mantissa products summed per block, the two shared
// exponents applied once per block): every v_mfma_scale_f32_32x32x64_f8f6f4 takes two 32-element
// blocks per lane pair with their two exponent bytes and adds
//     (sum_k a_k*b_k) * 2^(Ea + Eb)
// into the fp32 accumulator; the mantissa pieces are exact in the 6-bit code, so the block sums
// are exact and only the accumulation over blocks rounds (to fp32), as on the integer path.
// A mantissa wider than 4 bits takes two pieces (q = 16h + l), i.e. two MFMAs per operand pair.
//
// Structure: a workgroup of four waves (2 x 2) owns a (64*TM) x (64*TN) tile of Y.  Per K step of
// 64 the operand units are copied global -> LDS with 16-byte direct-to-LDS loads (the layout in
// HBM is the LDS image, so the copy is linear and the fragment reads are conflict-free b128
// reads), double buffered with one barrier per step.
#include <type_traits>

#include "mx_gemm.h"
#include "mx_matrix.h"

namespace mx {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

struct ScaledArgs {
    const uint8_t* A;
    const uint8_t* B;
    float* Y;
    int64_t M, N;
    int64_t unitsA, unitsB;        // units per matrix (for clamping)
    int64_t tilesA, tilesB;        // row tiles per matrix
    int64_t ksteps;
    int64_t fragA, fragB;          // byte offset of the scale region
    int64_t matrixA, matrixB;
    int64_t ldy, batch_stride_y;
    int32_t eadj;
    int32_t tiles_n;               // workgroup tiles along N
};

// 16 bytes per lane from global memory straight into LDS: lane L's bytes land at lds_addr + 16*L.
// Written as inline assembly so that the compiler does not serialize every later LDS read behind
// the copy (it cannot tell the two stages apart); completion is awaited explicitly with
// s_waitcnt vmcnt(0) before the barrier that publishes a stage.
__device__ __forceinline__ void copy16_to_lds(const uint8_t* uniform_src, uint32_t lane_offset,
                                              uint32_t lds_addr) {
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, %1\n\t"
        :
        : "v"(lane_offset), "s"(uniform_src), "s"(lds_addr)
        : "memory", "m0");
}

template <int PA, int PB, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_scaled_kernel(ScaledArgs g) {
    constexpr int UA = (PA == 2) ? 2 * TM : TM;        // units of the A tile per K step
    constexpr int UB = (PB == 2) ? 2 * TN : TN;
    constexpr int NU = UA + UB;
    constexpr int STAGE = NU * kUnitBytes;
    constexpr int NLOAD = (3 * NU + 3) / 4;            // 1 KiB wave loads per wave per K step
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t bn = blockIdx.x % g.tiles_n, bm = blockIdx.x / g.tiles_n;
    const int64_t bz = blockIdx.y;
    const uint8_t* Abase = g.A + bz * g.matrixA;
    const uint8_t* Bbase = g.B + bz * g.matrixB;

    // this wave's share of the global -> LDS copy: load t moves plane (t % 3) of stage unit (t / 3)
    const uint8_t* src[NLOAD];
    int dst[NLOAD];
#pragma unroll
    for (int q = 0; q < NLOAD; ++q) {
        int t = q * 4 + wave;
        if (t >= 3 * NU) t = 3 * NU - 1;               // duplicate the last load instead of branching
        const int n = t / 3, plane = t - 3 * n;
        int64_t u;
        const uint8_t* base;
        if (n < UA) {
            u = bm * UA + n;
            u = u < g.unitsA ? u : g.unitsA - 1;
            base = Abase;
        } else {
            u = bn * UB + (n - UA);
            u = u < g.unitsB ? u : g.unitsB - 1;
            base = Bbase;
        }
        src[q] = base + u * g.ksteps * kUnitBytes + plane * 1024;
        dst[q] = n * kUnitBytes + plane * 1024;
    }
    const uint32_t lane16 = lane * 16;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

    // scale dwords: one per row tile per four K steps, read straight from global
    constexpr int RA = TM, RB = TN;      // row tiles per wave: the wave tile is (32*RA) x (32*RB)
    const uint32_t* sA[RA];
    const uint32_t* sB[RB];
    const int64_t rtA0 = (bm * 2 + wm) * RA, rtB0 = (bn * 2 + wn) * RB;
#pragma unroll
    for (int t = 0; t < RA; ++t) {
        int64_t rt = rtA0 + t;
        rt = rt < g.tilesA ? rt : g.tilesA - 1;
        sA[t] = reinterpret_cast<const uint32_t*>(Abase + g.fragA) + rt * (g.ksteps / 4) * 64 + lane;
    }
#pragma unroll
    for (int t = 0; t < RB; ++t) {
        int64_t rt = rtB0 + t;
        rt = rt < g.tilesB ? rt : g.tilesB - 1;
        sB[t] = reinterpret_cast<const uint32_t*>(Bbase + g.fragB) + rt * (g.ksteps / 4) * 64 + lane;
    }

    v16f acc[RA][RB];
#pragma unroll
    for (int ta = 0; ta < RA; ++ta)
#pragma unroll
        for (int tb = 0; tb < RB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ta][tb][r] = 0.f;

    auto issue = [&](int64_t ks, int stage) {
#pragma unroll
        for (int q = 0; q < NLOAD; ++q)
            copy16_to_lds(src[q] + ks * kUnitBytes, lane16, lds0 + stage * STAGE + dst[q]);
    };

    // fragment registers, two sets: the MFMAs of a K step run from one set while the LDS reads of
    // the next step fill the other.  [set][tile][piece] -> 8 dwords (6 used)
    struct Frag { int d[6]; };
    Frag fa[2][RA][PA], fb[2][RB][PB];
    auto load_unit = [&](const uint8_t* u, Frag& f0, Frag& f1) {     // u: unit base in LDS
        const uint4 l0 = *reinterpret_cast<const uint4*>(u + frag_lo(0, lane));
        const uint2 h0 = *reinterpret_cast<const uint2*>(u + frag_hi(0, lane));
        const uint4 l1 = *reinterpret_cast<const uint4*>(u + frag_lo(1, lane));
        const uint2 h1 = *reinterpret_cast<const uint2*>(u + frag_hi(1, lane));
        f0.d[0] = (int)l0.x; f0.d[1] = (int)l0.y; f0.d[2] = (int)l0.z; f0.d[3] = (int)l0.w;
        f0.d[4] = (int)h0.x; f0.d[5] = (int)h0.y;
        f1.d[0] = (int)l1.x; f1.d[1] = (int)l1.y; f1.d[2] = (int)l1.z; f1.d[3] = (int)l1.w;
        f1.d[4] = (int)h1.x; f1.d[5] = (int)h1.y;
    };
    auto operand = [](const Frag& f) {       // the fp6 forms read six of the eight operand dwords
        return v8i{f.d[0], f.d[1], f.d[2], f.d[3], f.d[4], f.d[5], 0, 0};
    };
    auto read_frags = [&](int stage, auto setc) {
        constexpr int set = decltype(setc)::value;
        const uint8_t* st = smem + stage * STAGE;
        if constexpr (PA == 2) {
#pragma unroll
            for (int t = 0; t < RA; ++t) load_unit(st + (wm * RA + t) * kUnitBytes, fa[set][t][0], fa[set][t][1]);
        } else {
#pragma unroll
            for (int t = 0; t < RA; t += 2)
                load_unit(st + ((wm * RA + t) / 2) * kUnitBytes, fa[set][t][0], fa[set][t + 1][0]);
        }
        if constexpr (PB == 2) {
#pragma unroll
            for (int t = 0; t < RB; ++t)
                load_unit(st + (UA + wn * RB + t) * kUnitBytes, fb[set][t][0], fb[set][t][1]);
        } else {
#pragma unroll
            for (int t = 0; t < RB; t += 2)
                load_unit(st + (UA + (wn * RB + t) / 2) * kUnitBytes, fb[set][t][0], fb[set][t + 1][0]);
        }
    };

    // Pipeline: at the top of step ks the copy of step ks+1 (issued one step earlier) is awaited
    // and published with one barrier; that barrier also means every wave has finished reading the
    // stage of step ks into registers, so the copy of step ks+2 may overwrite it.
    uint32_t nxA[RA], nxB[RB];           // scale dwords of the next group of four K steps
#pragma unroll
    for (int t = 0; t < RA; ++t) nxA[t] = g.ksteps > 0 ? sA[t][0] : 0u;
#pragma unroll
    for (int t = 0; t < RB; ++t) nxB[t] = g.ksteps > 0 ? sB[t][0] : 0u;
    if (g.ksteps > 0) {
        issue(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        issue(1, 1);                      // ksteps is a multiple of 4
        read_frags(0, std::integral_constant<int, 0>{});
    }
    for (int64_t ks4 = 0; ks4 < g.ksteps / 4; ++ks4) {
        const bool last_group = ks4 + 1 == g.ksteps / 4;
        uint32_t scA[RA], scAh[RA], scB[RB], scBh[RB];
#pragma unroll
        for (int t = 0; t < RA; ++t) {
            scA[t] = nxA[t];
            scAh[t] = scA[t] + 0x04040404u;
        }
#pragma unroll
        for (int t = 0; t < RB; ++t) {
            scB[t] = nxB[t];
            scBh[t] = scB[t] + 0x04040404u;
        }
        // one K step; j (the byte of the scale dwords it uses) must be a compile-time constant
        auto kstep = [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            constexpr int set = j & 1;
            const int64_t ks = ks4 * 4 + j;
            __builtin_amdgcn_sched_barrier(0);
            // ksteps is a multiple of four: steps ks+1 and ks+2 can only be missing in the last group
            const bool have1 = j < 3 || !last_group;
            const bool have2 = j < 2 || !last_group;
            if (have1) {
                __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): this wave's copy of step ks+1 landed
                __syncthreads();
                if (j == 2 && have2) {                    // next group's scales, one step before their use
#pragma unroll
                    for (int t = 0; t < RA; ++t) nxA[t] = sA[t][(ks4 + 1) * 64];
#pragma unroll
                    for (int t = 0; t < RB; ++t) nxB[t] = sB[t][(ks4 + 1) * 64];
                }
                if (have2) issue(ks + 2, set);
                read_frags(set ^ 1, std::integral_constant<int, set ^ 1>{});
            }
            __builtin_amdgcn_sched_barrier(0);            // keep the LDS reads ahead of this step's MFMAs
            // all high-piece MFMAs first: consecutive instructions never share an accumulator
#pragma unroll
            for (int pa = 0; pa < PA; ++pa) {
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
#pragma unroll
                    for (int ta = 0; ta < RA; ++ta) {
#pragma unroll
                        for (int tb = 0; tb < RB; ++tb) {
                            // piece 0 of a two-piece operand is the high one: scale byte + 4
                            const int sa = (int)((PA == 2 && pa == 0) ? scAh[ta] : scA[ta]);
                            const int sb = (int)((PB == 2 && pb == 0) ? scBh[tb] : scB[tb]);
                            acc[ta][tb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                operand(fa[set][ta][pa]), operand(fb[set][tb][pb]), acc[ta][tb], 2, 2, j, sa,
                                j, sb);
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        kstep(std::integral_constant<int, 0>{});
        kstep(std::integral_constant<int, 1>{});
        kstep(std::integral_constant<int, 2>{});
        kstep(std::integral_constant<int, 3>{});
    }

    float* Y = g.Y + bz * g.batch_stride_y;
    const int i = lane & 31, h = lane >> 5;
#pragma unroll
    for (int ta = 0; ta < RA; ++ta) {
#pragma unroll
        for (int tb = 0; tb < RB; ++tb) {
            const int64_t n = (rtB0 + tb) * 32 + i;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = (rtA0 + ta) * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < g.M && n < g.N) Y[m * g.ldy + n] = __builtin_ldexpf(acc[ta][tb][r], g.eadj);
            }
        }
    }
}

template <int PA, int PB, int TM, int TN>
mx_status launch_scaled(ScaledArgs& g, int64_t batch, hipStream_t st) {
    constexpr int UA = (PA == 2) ? 2 * TM : TM, UB = (PB == 2) ? 2 * TN : TN;
    constexpr int smem = 2 * (UA + UB) * kUnitBytes;
    auto kern = gemm_scaled_kernel<PA, PB, TM, TN>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return MX_ERR_DEVICE;
        configured = true;
    }
    const int64_t tiles_m = ceil_div(g.M, 64 * TM), tiles_n = ceil_div(g.N, 64 * TN);
    if (tiles_m * tiles_n > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    g.tiles_n = (int32_t)tiles_n;
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, g);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int PA, int PB>
mx_status pick_tile(ScaledArgs& g, int64_t batch, hipStream_t st) {
    // 256 x 256 tiles move the fewest bytes per MAC; fall back to 256 x 128 when that would leave
    // most of the 256 compute units without a tile
    const int64_t big = ceil_div(g.M, 256) * ceil_div(g.N, 256) * batch;
    if (big >= 200) return launch_scaled<PA, PB, 4, 4>(g, batch, st);
    return launch_scaled<PA, PB, 4, 2>(g, batch, st);
}

}  // namespace

mx_status gemm_scaled(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, mx_format fa,
                      const void* B, mx_format fb, float* Y, int64_t ldy, int64_t batch_stride_y,
                      hipStream_t st) {
    const MatGeom ga = mat_geom(M, K, fa.mant_bits), gb = mat_geom(N, K, fb.mant_bits);
    ScaledArgs g;
    g.A = (const uint8_t*)A; g.B = (const uint8_t*)B; g.Y = Y; g.M = M; g.N = N;
    g.unitsA = ga.units; g.unitsB = gb.units; g.tilesA = ga.row_tiles; g.tilesB = gb.row_tiles;
    g.ksteps = ga.ksteps; g.fragA = ga.frag_bytes; g.fragB = gb.frag_bytes;
    g.matrixA = ga.matrix; g.matrixB = gb.matrix; g.ldy = ldy; g.batch_stride_y = batch_stride_y;
    // pieces are stored halved (2 bits in all), mantissa units are 2^-(w-2) each
    g.eadj = 2 - (fa.mant_bits - 2) - (fb.mant_bits - 2);
    g.tiles_n = 0;
    if (ga.pieces == 2 && gb.pieces == 1) return pick_tile<2, 1>(g, batch, st);
    if (ga.pieces == 1 && gb.pieces == 1) return pick_tile<1, 1>(g, batch, st);
    if (ga.pieces == 2 && gb.pieces == 2) return pick_tile<2, 2>(g, batch, st);
    return pick_tile<1, 2>(g, batch, st);
}

}  // namespace mx
