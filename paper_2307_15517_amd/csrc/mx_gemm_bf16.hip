// MXInt x MXInt product for blocks of 16 on the bfloat16 matrix cores of gfx950 (operands in
// MX_LAYOUT_MATRIX for block 16, see mx_bf16.h).
//
// Arithmetic (Section 3.2 of the paper: mantissa products summed per block, the two shared
// exponents applied once per block): the exponents were folded into the elements at packing time
// (element = mantissa * 2^exponent, exact in bfloat16), so one v_mfma_f32_32x32x16_bf16 takes one
// block of each operand per lane pair and adds the 16 exact products into the fp32 accumulator.
// Only the fp32 accumulation rounds.
//
// Structure: a workgroup of four waves (2 x 2) owns a (64*TM) x (64*TN) tile of Y.  Per K step of
// 32 the operand units are copied global -> LDS with 16-byte direct-to-LDS loads (the layout in
// HBM is the LDS image: the copy is linear and a fragment is one conflict-free 16-byte read per
// lane), S stages, one barrier per step, fragments double-buffered in registers, copies and LDS
// reads slotted between the MFMAs.
#include <type_traits>

#include "mx_bf16.h"
#include "mx_gemm.h"

namespace mx {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

struct BfArgs {
    const uint8_t* A;
    const uint8_t* B;
    float* Y;
    int64_t M, N;
    int64_t tilesA, tilesB;        // row tiles per matrix (for clamping)
    int64_t ksteps;
    int64_t matrixA, matrixB;
    int64_t ldy, batch_stride_y;
    int32_t tiles_m, tiles_n;      // workgroup tiles along M and N
    // quantized output (mx_gemm_q): the result leaves as a packed block-16 operand [M x N], blocks along N
    uint8_t* out;
    BfGeom go;
    const uint8_t* bias_mant;      // canonical MXInt bias [N] (one row), or null
    const uint8_t* bias_exps;
    int32_t wbias, bias_b;         // stored width and exponent bias of the bias format
    int32_t wo, bias_o, emax_o, rnd_o, brows_o;   // output format
};

// 16 bytes per lane from global memory straight into LDS: lane L's bytes land at lds_addr + 16*L.
// Inline assembly so that the compiler does not serialize every later LDS read behind the copy;
// completion is awaited explicitly with s_waitcnt vmcnt(n) before the barrier that publishes a stage.
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

// s_waitcnt vmcnt(n), every other counter left alone (gfx9 encoding: vmcnt = bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// S: LDS stages.  The stage of step ks is free once its fragments are in registers, i.e. from the
// barrier of step ks on, so the copy of step ks+S is issued during step ks.
// OCC: workgroups the register and LDS budget must leave room for on one compute unit.
// QOUT: instead of storing fp32, add the bias and quantize the tile to the output format
// (Section 3.2 of the paper: the emulated operator quantizes its result; Fig. 2b: the linear layer's
// bias is MXInt too), writing the packed operand the next product reads.
template <int TM, int TN, int S, int OCC, bool QOUT>
__global__ __launch_bounds__(256, OCC) void gemm_bf16_kernel(BfArgs g) {
    constexpr int UA = 2 * TM, UB = 2 * TN;            // units (row tiles) of the A / B tile per K step
    constexpr int NU = UA + UB;
    constexpr int STAGE = NU * kBfUnitBytes;
    constexpr int NLOAD = (2 * NU + 3) / 4;            // 1 KiB wave copies per wave per K step
    constexpr int RA = TM, RB = TN;                    // row tiles per wave: the wave tile is (32*RA) x (32*RB)
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroup i runs on XCD i % 8, each with its own L2: every XCD gets one contiguous range of
    // tiles, numbered with the M tile fastest, so that the tiles resident on an XCD share operand rows.
    const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n, per_xcd = (tiles + 7) / 8;
    const int64_t tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (tile >= tiles) return;
    const int64_t bm = tile % g.tiles_m, bn = tile / g.tiles_m;
    const int64_t bz = blockIdx.y;
    const uint8_t* Abase = g.A + bz * g.matrixA;
    const uint8_t* Bbase = g.B + bz * g.matrixB;

    // this wave's share of the global -> LDS copy: copy t moves KiB number (t % 2) of stage unit (t / 2)
    const uint8_t* src[NLOAD];
    int dst[NLOAD];
#pragma unroll
    for (int q = 0; q < NLOAD; ++q) {
        int t = q * 4 + wave;
        if (t >= 2 * NU) t = 2 * NU - 1;               // duplicate the last copy instead of branching
        const int n = t >> 1, part = t & 1;
        int64_t rt;
        const uint8_t* base;
        if (n < UA) {
            rt = bm * UA + n;
            rt = rt < g.tilesA ? rt : g.tilesA - 1;    // tiles past the matrix re-read its last row tile (never stored)
            base = Abase;
        } else {
            rt = bn * UB + (n - UA);
            rt = rt < g.tilesB ? rt : g.tilesB - 1;
            base = Bbase;
        }
        src[q] = base + rt * g.ksteps * kBfUnitBytes + part * 1024;
        dst[q] = n * kBfUnitBytes + part * 1024;
    }
    const uint32_t lane16 = lane * 16;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

    v16f acc[RA][RB];
#pragma unroll
    for (int ta = 0; ta < RA; ++ta)
#pragma unroll
        for (int tb = 0; tb < RB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ta][tb][r] = 0.f;

    // Copies are always issued in full, with the K step clamped to the last one, so that the number
    // of copies in flight is the same at every step and the vmcnt waits stay exact.
    auto issue_one = [&](int q, int64_t ks, int stage) {
        ks = ks < g.ksteps ? ks : g.ksteps - 1;
        copy16_to_lds(src[q] + ks * kBfUnitBytes, lane16, lds0 + stage * STAGE + dst[q]);
    };
    auto issue = [&](int64_t ks, int stage) {
#pragma unroll
        for (int q = 0; q < NLOAD; ++q) issue_one(q, ks, stage);
    };

    // fragment registers, two sets: the MFMAs of a K step run from one set while the LDS reads of
    // the next step fill the other.  [set][row tile][half of the K step]
    v4i fa[2][RA][2], fb[2][RB][2];
    auto read_unit = [&](int n, int stage, auto setc) {
        constexpr int set = decltype(setc)::value;
        const uint8_t* st = smem + stage * STAGE;
        if (n < RA) {
            const uint8_t* u = st + (wm * RA + n) * kBfUnitBytes + lane * 16;
            fa[set][n][0] = *reinterpret_cast<const v4i*>(u);
            fa[set][n][1] = *reinterpret_cast<const v4i*>(u + 1024);
        } else {
            const int t = n - RA;
            const uint8_t* u = st + (UA + wn * RB + t) * kBfUnitBytes + lane * 16;
            fb[set][t][0] = *reinterpret_cast<const v4i*>(u);
            fb[set][t][1] = *reinterpret_cast<const v4i*>(u + 1024);
        }
    };

    // Pipeline.  Queue of copies, oldest first, when step ks starts:  D(ks+1) ... D(ks+S-1).  Waiting
    // until only the newest S-2 steps' copies are outstanding means D(ks+1) has landed; the barrier
    // then publishes it and tells that every wave is done reading the stage of step ks (read into
    // registers during step ks-1), which the copy of step ks+S overwrites.
    if (g.ksteps > 0) {
#pragma unroll
        for (int st = 0; st < S; ++st) issue(st, st);
        wait_vmcnt<(S - 1) * NLOAD>();
        __syncthreads();
#pragma unroll
        for (int n = 0; n < RA + RB; ++n) read_unit(n, 0, std::integral_constant<int, 0>{});
    }
    constexpr int NM = 2 * RA * RB;                    // MFMAs per K step
    int cur = 0;                                       // stage of the current step: ks % S
    for (int64_t ks2 = 0; ks2 < g.ksteps / 2; ++ks2) {
        auto kstep = [&](auto jc) {
            constexpr int set = decltype(jc)::value;
            const int64_t ks = ks2 * 2 + set;
            const int nxt = cur + 1 == S ? 0 : cur + 1;
            // side work of this step, in issue order: LDS reads for step ks+1, copies for step ks+S
            constexpr int NAUX = (RA + RB) + NLOAD;
            auto aux = [&](int x) {
                if (x < RA + RB) { read_unit(x, nxt, std::integral_constant<int, set ^ 1>{}); return; }
                issue_one(x - (RA + RB), ks + S, cur);
            };
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<(S - 2) * NLOAD>();
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            // one half of the K step after the other: consecutive MFMAs never share an accumulator
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int tb = m % RB, ta = (m / RB) % RA, kf = m / (RA * RB);
                acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(v8bf, fa[set][ta][kf]), __builtin_bit_cast(v8bf, fb[set][tb][kf]), acc[ta][tb],
                    0, 0, 0);
#pragma unroll
                for (int x = m * NAUX / NM; x < (m + 1) * NAUX / NM; ++x) aux(x);
                __builtin_amdgcn_sched_barrier(0);        // pin the interleaving as written
            }
            cur = nxt;
        };
        kstep(std::integral_constant<int, 0>{});
        kstep(std::integral_constant<int, 1>{});
    }
    wait_vmcnt<0>();                                      // the clamped tail copies must not outlive the LDS

    const int64_t rtA0 = (bm * 2 + wm) * RA, rtB0 = (bn * 2 + wn) * RB;
    const int i = lane & 31, h = lane >> 5;
    if constexpr (QOUT) {
        // One row tile of the wave at a time: accumulators -> the wave's LDS tile, row-major; then lane
        // 32*h' + i' holds half h' of each 16-element block of row i' (what the layout's fragments hold),
        // completes the block maximum with its partner lane, quantizes and stores 16 bytes per fragment.
        constexpr int PITCH = 32 * RB + 4;               // floats; the skew spreads the rows over the banks
        static_assert(4 * 32 * PITCH * 4 + 64 * TN * 4 <= S * STAGE, "the turn-around tiles and the bias fit in the stages");
        __syncthreads();                                 // every wave is done reading the stages
        float* tile = reinterpret_cast<float*>(smem) + wave * (32 * PITCH);
        // the bias of the workgroup's columns, decoded once
        float* bias_lds = reinterpret_cast<float*>(smem) + 4 * 32 * PITCH;
        if (g.bias_mant != nullptr) {
            for (int c = threadIdx.x; c < 64 * TN; c += 256) {
                const int64_t n = bn * (64 * TN) + c;
                float bv = 0.f;
                if (n < g.N) {
                    const int64_t bit = n * g.wbias;
                    const int sh = (int)(bit & 7);
                    uint32_t code = g.bias_mant[bit >> 3];
                    if (sh + g.wbias > 8) code |= (uint32_t)g.bias_mant[(bit >> 3) + 1] << 8;
                    const int q = ((int)((code >> sh) << (32 - g.wbias))) >> (32 - g.wbias);
                    bv = __builtin_ldexpf((float)q, (int)g.bias_exps[n >> 4] - g.bias_b - (g.wbias - 2));
                }
                bias_lds[c] = bv;
            }
            __syncthreads();
        }
        uint8_t* obase = g.out + bz * g.go.matrix;
        const float qmax = (float)((1 << (g.wo - 1)) - 1);
#pragma unroll
        for (int ta = 0; ta < RA; ++ta) {
#pragma unroll
            for (int tb = 0; tb < RB; ++tb)
#pragma unroll
                for (int r = 0; r < 16; ++r) tile[(8 * (r >> 2) + 4 * h + (r & 3)) * PITCH + tb * 32 + i] = acc[ta][tb][r];
            __builtin_amdgcn_wave_barrier();
            const int64_t rt = rtA0 + ta, row = rt * 32 + i;
#pragma unroll
            for (int f = 0; f < 2 * RB; ++f) {
                const int64_t kf = rtB0 * 2 + f;          // block along N
                const int64_t col0 = kf * 16 + h * 8;
                const bool inside = row < g.M && col0 < g.N;
                const float4 t0 = *reinterpret_cast<const float4*>(tile + i * PITCH + f * 16 + h * 8);
                const float4 t1 = *reinterpret_cast<const float4*>(tile + i * PITCH + f * 16 + h * 8 + 4);
                float v[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
                if (!inside) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = 0.f;
                } else if (g.bias_mant != nullptr) {
                    const float4 b0 = *reinterpret_cast<const float4*>(bias_lds + wn * (32 * RB) + f * 16 + h * 8);
                    const float4 b1 = *reinterpret_cast<const float4*>(bias_lds + wn * (32 * RB) + f * 16 + h * 8 + 4);
                    v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
                    v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
                }
                uint32_t am = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t ab = __float_as_uint(v[e]) & 0x7fffffffu;
                    am = ab > am ? ab : am;
                }
                const uint32_t o = (uint32_t)__shfl_xor((int)am, 32, 64);
                am = o > am ? o : am;
                if (g.brows_o == 2) {                     // two-row blocks: the neighbouring lane holds the other row
                    const uint32_t o2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);
                    am = o2 > am ? o2 : am;
                }
                const int ef = (int)(am >> 23);
                int E = ef == 0 ? -127 : ef - 127;
                E = E < -g.bias_o ? -g.bias_o : E;
                E = E > g.emax_o ? g.emax_o : E;
                uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float sc = __builtin_ldexpf(v[e], (g.wo - 2) - E);
                    float r = g.rnd_o == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
                    r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
                    r += 0.0f;                           // -0.0 -> +0.0
                    out[e >> 1] |= bf16_of(r, E - (g.wo - 2)) << (16 * (e & 1));
                }
                if (rt < g.go.row_tiles && kf < g.go.ksteps * 2)
                    *reinterpret_cast<uint4*>(obase + bf_frag(g.go, rt, kf >> 1, (int)(kf & 1), lane)) =
                        make_uint4(out[0], out[1], out[2], out[3]);
                if (h == 0 && row < g.M && kf < g.go.nblk) obase[g.go.frag_bytes + row * g.go.nblk + kf] = (uint8_t)(E + g.bias_o);
            }
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }
    float* Y = g.Y + bz * g.batch_stride_y;
#pragma unroll
    for (int ta = 0; ta < RA; ++ta) {
#pragma unroll
        for (int tb = 0; tb < RB; ++tb) {
            const int64_t n = (rtB0 + tb) * 32 + i;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = (rtA0 + ta) * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                // written once and not read again by this kernel: a streaming store keeps the operands in the L2
                if (m < g.M && n < g.N) __builtin_nontemporal_store(acc[ta][tb][r], &Y[m * g.ldy + n]);
            }
        }
    }
}

template <int TM, int TN, int S, int OCC, bool QOUT>
mx_status launch_bf16(BfArgs& g, int64_t batch, hipStream_t st) {
    constexpr int smem = S * (2 * TM + 2 * TN) * kBfUnitBytes;
    static_assert(smem * OCC <= 160 * 1024, "LDS budget of one compute unit");
    auto kern = gemm_bf16_kernel<TM, TN, S, OCC, QOUT>;
    static std::atomic<uint64_t> done{0};
    if (!allow_dynamic_lds((const void*)kern, smem, done)) return MX_ERR_DEVICE;
    const int64_t tiles_m = ceil_div(g.M, 64 * TM), tiles_n = ceil_div(g.N, 64 * TN);
    if (tiles_m * tiles_n > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    g.tiles_m = (int32_t)tiles_m;
    g.tiles_n = (int32_t)tiles_n;
    dim3 grid((unsigned)(ceil_div(tiles_m * tiles_n, 8) * 8), (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, g);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

}  // namespace

// Tile 128 x 256, four waves.  With at least two tiles per compute unit two workgroups share one
// (three stages each), so that one workgroup's barrier and copy waits hide under the other's
// MFMAs; otherwise one workgroup per compute unit runs with four stages.
mx_status gemm_bf16(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, const void* B, float* Y,
                    int64_t ldy, int64_t batch_stride_y, hipStream_t st) {
    const BfGeom ga = bf_geom(M, K), gb = bf_geom(N, K);
    BfArgs g;
    g.A = (const uint8_t*)A; g.B = (const uint8_t*)B; g.Y = Y; g.M = M; g.N = N;
    g.tilesA = ga.row_tiles; g.tilesB = gb.row_tiles; g.ksteps = ga.ksteps;
    g.matrixA = ga.matrix; g.matrixB = gb.matrix; g.ldy = ldy; g.batch_stride_y = batch_stride_y;
    g.tiles_m = g.tiles_n = 0;
    g.out = nullptr; g.bias_mant = g.bias_exps = nullptr;
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 256) * batch;
    if (tiles >= 2 * 256) return launch_bf16<2, 4, 3, 2, false>(g, batch, st);
    return launch_bf16<2, 4, 4, 1, false>(g, batch, st);
}

// The same product with the bias added and the result quantized to `fo` (block 16, blocks along N),
// written as the packed operand [M x N] of the matrix layout.
mx_status gemm_bf16_q(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, const void* B,
                      const uint8_t* bias_mant, const uint8_t* bias_exps, mx_format fbias, mx_format fo, void* out,
                      hipStream_t st) {
    const BfGeom ga = bf_geom(M, K), gb = bf_geom(N, K);
    BfArgs g;
    g.A = (const uint8_t*)A; g.B = (const uint8_t*)B; g.Y = nullptr; g.M = M; g.N = N;
    g.tilesA = ga.row_tiles; g.tilesB = gb.row_tiles; g.ksteps = ga.ksteps;
    g.matrixA = ga.matrix; g.matrixB = gb.matrix; g.ldy = 0; g.batch_stride_y = 0;
    g.tiles_m = g.tiles_n = 0;
    g.out = (uint8_t*)out; g.go = bf_geom(M, N);
    g.bias_mant = bias_mant; g.bias_exps = bias_exps;
    g.wbias = fbias.mant_bits; g.bias_b = (1 << (fbias.exp_bits - 1)) - 1;
    g.wo = fo.mant_bits; g.bias_o = (1 << (fo.exp_bits - 1)) - 1;
    g.emax_o = ((1 << fo.exp_bits) - 1) - g.bias_o;
    g.rnd_o = fo.rounding; g.brows_o = fo.block_rows;
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 256) * batch;
    if (tiles >= 2 * 256) return launch_bf16<2, 4, 3, 2, true>(g, batch, st);
    return launch_bf16<2, 4, 4, 1, true>(g, batch, st);
}

}  // namespace mx
