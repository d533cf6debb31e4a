// MXInt x MXInt product on the block-scaled fp6 matrix cores of gfx950 (operands in
// MX_LAYOUT_MATRIX, see mx_matrix.h), for block sizes 32 and 64.
//
// Arithmetic (Section 3.2 of the paper: mantissa products summed per block, the two shared
// exponents applied once per block): every v_mfma_scale_f32_32x32x64_f8f6f4 takes two 32-element
// blocks per lane pair with their two exponent bytes and adds
//     (sum_k a_k*b_k) * 2^(Ea + Eb)
// into the fp32 accumulator; the mantissa pieces are exact in the 6-bit code, so the block sums
// are exact.  The accumulation over blocks rounds to fp32, and not quite as the integer path does:
// the instruction aligns the incoming accumulator to the largest single product of its two blocks and
// keeps 24 bits below that, so a block whose large products cancel can push out low bits of the
// running sum (bound: 1e-5 * sum_b |term_b| + 1e-6 * sum_k |product_k|; the first term alone when the
// exponent sums of an output's blocks span at most 24 - wa - wb binades, 12 for 8-bit by 4-bit operands).
// A mantissa wider than 4 bits takes two pieces (q = 16h + l), i.e. two MFMAs per operand pair.
//
// Structure: a workgroup of four waves (2 x 2) owns a (64*TM) x (64*TN) tile of Y.  Per K step of
// 64 the operand units are copied global -> LDS with 16-byte direct-to-LDS loads (the layout in
// HBM is the LDS image, so the copy is linear and the fragment reads are conflict-free b128
// reads), double buffered with one barrier per step.
#include <type_traits>

#include "mx_gemm.h"
#include "mx_matrix.h"

// From this many output tiles on, the product runs two workgroups per compute unit (three LDS stages each) instead of
// one workgroup with copy waves (five stages).
#ifndef MX_SCALED_TWO_PER_CU_TILES
#define MX_SCALED_TWO_PER_CU_TILES 512
#endif
// Matrix instructions at the end of a K step with no LDS read or copy issued between them.
#ifndef MX_SCALED_TAIL_MFMAS
#define MX_SCALED_TAIL_MFMAS 4
#endif

namespace mx {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v6i __attribute__((ext_vector_type(6)));
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
    int32_t tiles_m, tiles_n;      // workgroup tiles along M and N
    // quantized output (mx_gemm_q): the result leaves as a packed operand [M x N] of this layout, blocks along N
    uint8_t* out;
    MatGeom go;
    const uint8_t* bias_mant;      // canonical MXInt bias [N] (one row), or null
    const uint8_t* bias_exps;
    int32_t wbias, bias_b, blk_bias;   // stored width, exponent bias and block size of the bias format
    int32_t wo, bias_o, emax_o, rnd_o, brows_o, blk_o;   // output format
};

// `bytes` (16 or 4) per lane from global memory straight into LDS: lane L's bytes land at
// lds_addr + bytes*L.  Written as inline assembly so that the compiler does not serialize every
// later LDS read behind the copy (it cannot tell the stages apart); completion is awaited
// explicitly with s_waitcnt vmcnt(n) before the barrier that publishes a stage.
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
// Three consecutive KiB (one unit) with one setting of m0: the instruction's offset field moves the
// global address and the LDS address alike.
__device__ __forceinline__ void copy48_to_lds(const uint8_t* uniform_src, uint32_t lane_offset,
                                              uint32_t lds_addr) {
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, %1\n\t"
        "global_load_lds_dwordx4 %0, %1 offset:1024\n\t"
        "global_load_lds_dwordx4 %0, %1 offset:2048\n\t"
        :
        : "v"(lane_offset), "s"(uniform_src), "s"(lds_addr)
        : "memory", "m0");
}
__device__ __forceinline__ void copy4_to_lds(const uint8_t* uniform_src, uint32_t lane_offset,
                                             uint32_t lds_addr) {
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dword %0, %1\n\t"
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

// S: LDS stages.  The stage of step ks is free once its fragments are in registers, i.e. from
// the barrier of step ks on, so the copy of step ks+S is issued during step ks.
// OCC: workgroups the register and LDS budget must leave room for on one compute unit.
// QO: 0 = fp32 result; 1 / 2 = add the bias and quantize the tile to an output format of one / two
// mantissa pieces (Section 3.2 of the paper: the emulated operator quantizes its result; Fig. 2b: the
// linear layer's bias is MXInt too), writing the packed operand the next product reads.
// WS: 1 = eight waves, the four extra ones ("copy waves", one per SIMD next to a matrix wave) issue every
// global -> LDS copy and never touch the matrix cores.  A wave issues in order, so a matrix wave that has to
// wait for the copy path to take its copy also delays its next matrix instruction; with the copies in waves
// of their own the matrix waves only ever wait for the barrier.  For launches with one workgroup per compute
// unit (the second workgroup of the OCC = 2 form plays that part otherwise).
template <int PA, int PB, int TM, int TN, int S, int OCC, int QO, int WS>
__global__ __launch_bounds__(WS ? 512 : 256, WS ? 2 : OCC) void gemm_scaled_kernel(ScaledArgs g) {
    constexpr int kStages = S;
    static_assert(S >= 3 && S <= 5, "the scale copies of a group must have landed by its step 3");
    constexpr int UA = (PA == 2) ? 2 * TM : TM;        // units of the A tile per K step
    constexpr int UB = (PB == 2) ? 2 * TN : TN;
    constexpr int NU = UA + UB;
    constexpr int STAGE = NU * kUnitBytes;
    constexpr int NLOAD = (3 * NU + 3) / 4;            // 1 KiB wave copies per wave per K step
    // When the units divide among the four waves, a wave copies whole units (three KiB with one
    // address set-up); otherwise single KiB pieces.
    constexpr int CP = (NU % 4 == 0) ? 3 : 1;          // KiB per copy item
    constexpr int NI = NLOAD / CP;                     // copy items per wave per K step
    static_assert(NI * CP == NLOAD, "items cover the wave's copies");
    constexpr int RA = TM, RB = TN;                    // row tiles per wave: the wave tile is (32*RA) x (32*RB)
    constexpr int NT = 2 * TM + 2 * TN;                // row tiles of the workgroup tile (A then B)
    constexpr int NSC = (NT + 3) / 4;                  // 256-byte scale copies per wave per group of 4 steps
    constexpr int SCALES = NT * 256;                   // bytes of one scale slot
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];   // kStages stages, then 2 scale slots

    const int wave8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wave = wave8 & 3;                        // position among the matrix waves, or among the copy waves
    const bool copier = WS != 0 && wave8 >= 4;         // a copy wave
    const bool copies = WS == 0 || copier;             // this wave issues copies
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroup i runs on XCD i % 8, each with its own L2.  Give every XCD one contiguous range of tiles of
    // an order in which consecutive tiles form a compact block of the tile grid (below), so that the tiles
    // resident on an XCD at one time share rows of both operands in that L2.
    const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n, per_xcd = (tiles + 7) / 8;
    const int64_t tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (tile >= tiles) return;
    // bands of eight M tiles, N fastest across a band, M fastest inside it: a run of consecutive tiles is a
    // compact block of the tile grid
    const int64_t hm = g.tiles_m < 8 ? g.tiles_m : 8;
    const int64_t band = tile / (hm * g.tiles_n), rr = tile - band * hm * g.tiles_n;
    const int64_t hb = (g.tiles_m - band * hm) < hm ? (g.tiles_m - band * hm) : hm;
    const int64_t bn = rr / hb, bm = band * hm + (rr - bn * hb);
    const int64_t bz = blockIdx.y;
    const uint8_t* Abase = g.A + bz * g.matrixA;
    const uint8_t* Bbase = g.B + bz * g.matrixB;
    const int64_t groups = g.ksteps / 4;

    // this wave's share of the global -> LDS copy: item t moves KiB (t*CP % 3) .. of stage unit (t*CP / 3)
    const uint8_t* src[NI];
    int dst[NI];
#pragma unroll
    for (int q = 0; q < NI; ++q) {
        int t = (q * 4 + wave) * CP;
        if (t >= 3 * NU) t = 3 * NU - CP;              // duplicate the last item instead of branching
        const int n = t / 3, part = t - 3 * n;
        int64_t u;
        const uint8_t* base;
        if (n < UA) {
            u = bm * UA + n;
            u = u < g.unitsA ? u : g.unitsA - 1;       // tiles past the matrix re-read its last unit (never stored)
            base = Abase;
        } else {
            u = bn * UB + (n - UA);
            u = u < g.unitsB ? u : g.unitsB - 1;
            base = Bbase;
        }
        src[q] = base + u * g.ksteps * kUnitBytes + part * 1024;
        dst[q] = n * kUnitBytes + part * 1024;
    }
    // ... and of the scale copies: row tile t of the workgroup tile, 256 bytes per group of four K steps
    const uint8_t* ssrc[NSC];
    int sdst[NSC];
#pragma unroll
    for (int q = 0; q < NSC; ++q) {
        int t = q * 4 + wave;
        if (t >= NT) t = NT - 1;
        int64_t rt;
        const uint8_t* base;
        if (t < 2 * TM) {
            rt = bm * 2 * TM + t;
            rt = rt < g.tilesA ? rt : g.tilesA - 1;
            base = Abase + g.fragA;
        } else {
            rt = bn * 2 * TN + (t - 2 * TM);
            rt = rt < g.tilesB ? rt : g.tilesB - 1;
            base = Bbase + g.fragB;
        }
        ssrc[q] = base + rt * groups * 256;
        sdst[q] = kStages * STAGE + t * 256;
    }
    const uint32_t lane16 = lane * 16, lane4 = lane * 4;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

    v16f acc[RA][RB];
#pragma unroll
    for (int ta = 0; ta < RA; ++ta)
#pragma unroll
        for (int tb = 0; tb < RB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ta][tb][r] = 0.f;

    // Copies are always issued in full, with the K step / group clamped to the last one, so that
    // the number of copies in flight is the same at every step and the vmcnt waits stay exact.
    auto copy_item = [&](const uint8_t* from, uint32_t lds_addr) {
        if constexpr (CP == 3) copy48_to_lds(from, lane16, lds_addr);
        else copy16_to_lds(from, lane16, lds_addr);
    };
    auto issue = [&](int64_t ks, int stage) {
        ks = ks < g.ksteps ? ks : g.ksteps - 1;
#pragma unroll
        for (int q = 0; q < NI; ++q) copy_item(src[q] + ks * kUnitBytes, lds0 + stage * STAGE + dst[q]);
    };
    auto issue_scale_one = [&](int q, int64_t grp, int slot) {
        grp = grp < groups ? grp : groups - 1;
        copy4_to_lds(ssrc[q] + grp * 256, lane4, lds0 + slot * SCALES + sdst[q]);
    };

    // fragment registers, two sets: the MFMAs of a K step run from one set while the LDS reads of
    // the next step fill the other.
    struct Frag { int d[6]; };
    Frag fa[2][RA][PA], fb[2][RB][PB];
    auto load_unit = [&](const uint8_t* u, Frag& f0, Frag& f1) {     // u: unit base in LDS
        const uint4 l0 = *reinterpret_cast<const uint4*>(u + frag_lo(0, lane));
        const uint2 h0 = *reinterpret_cast<const uint2*>(u + frag_hi(0, lane));
        const uint4 l1 = *reinterpret_cast<const uint4*>(u + frag_lo(1, lane));
        // the two 8-byte parts are 512 bytes apart; read through an address the compiler cannot relate to the
        // first one, or it fuses them into one two-address read whose four result registers then have to be
        // copied into the two operand tuples
        typedef unsigned int u2v __attribute__((ext_vector_type(2)));
        typedef __attribute__((address_space(3))) const u2v lds_u2v;
        lds_u2v* u1 = (lds_u2v*)(u + frag_hi(1, lane));
        asm volatile("" : "+v"(u1));
        const u2v h1 = *u1;
        f0.d[0] = (int)l0.x; f0.d[1] = (int)l0.y; f0.d[2] = (int)l0.z; f0.d[3] = (int)l0.w;
        f0.d[4] = (int)h0.x; f0.d[5] = (int)h0.y;
        f1.d[0] = (int)l1.x; f1.d[1] = (int)l1.y; f1.d[2] = (int)l1.z; f1.d[3] = (int)l1.w;
        f1.d[4] = (int)h1.x; f1.d[5] = (int)h1.y;
    };
    auto operand = [](const Frag& f) {       // the fp6 forms read six of the eight operand dwords
        return v8i{f.d[0], f.d[1], f.d[2], f.d[3], f.d[4], f.d[5], 0, 0};
    };
    // the units this wave reads per K step: first those of A, then those of B
    constexpr int NUA = (PA == 2) ? RA : RA / 2, NUB = (PB == 2) ? RB : RB / 2;
    auto read_unit = [&](int n, int stage, auto setc) {
        constexpr int set = decltype(setc)::value;
        const uint8_t* st = smem + stage * STAGE;
        if (n < NUA) {
            if constexpr (PA == 2) load_unit(st + (wm * RA + n) * kUnitBytes, fa[set][n][0], fa[set][n][1]);
            else load_unit(st + (wm * NUA + n) * kUnitBytes, fa[set][2 * n][0], fa[set][2 * n + 1][0]);
        } else {
            const int t = n - NUA;
            if constexpr (PB == 2) load_unit(st + (UA + wn * RB + t) * kUnitBytes, fb[set][t][0], fb[set][t][1]);
            else load_unit(st + (UA + wn * NUB + t) * kUnitBytes, fb[set][2 * t][0], fb[set][2 * t + 1][0]);
        }
    };

    // scale dwords of the current group of four K steps, and the next group's (read during step 3)
    uint32_t scA[RA], scB[RB], nxA[RA], nxB[RB];
    auto read_scales = [&](int slot, uint32_t* a, uint32_t* b) {
        const uint32_t* sc = reinterpret_cast<const uint32_t*>(smem + kStages * STAGE + slot * SCALES) + lane;
#pragma unroll
        for (int t = 0; t < RA; ++t) a[t] = sc[(wm * RA + t) * 64];
#pragma unroll
        for (int t = 0; t < RB; ++t) b[t] = sc[(2 * TM + wn * RB + t) * 64];
    };

    // Pipeline.  Queue of copies, oldest first, when step ks starts:  D(ks+1) ... D(ks+S-1), with
    // the scale copies of the next group right ahead of the data copies issued at step 0 of a group.
    // Copies land in issue order, so once only the data copies of the newest S-2 steps are outstanding
    // (at step 3 of the group: those issued at steps 0, 1, 2 when S = 5) the scale copies have landed
    // too, and step 3 may read them; with more than five stages they could still be in flight there.
    // Waiting until only the newest S-2 steps' copies are outstanding means D(ks+1) has landed; the barrier then
    // publishes it and tells that every wave is done reading the stage of step ks (read into
    // registers during step ks-1), which the copy of step ks+S overwrites.
    // Inside a step the MFMAs (operands already in registers) are issued at once, and the LDS reads
    // for the next step, the copies for step ks+3 and the scale traffic are slotted between them so
    // that the matrix pipe never waits for them.
    if (g.ksteps > 0) {
        if (copies) {
            issue(0, 0);
#pragma unroll
            for (int q = 0; q < NSC; ++q) issue_scale_one(q, 0, 0);
#pragma unroll
            for (int st = 1; st < S; ++st) issue(st, st);
            wait_vmcnt<(S - 1) * NLOAD>();
        }
        __syncthreads();
        if (!copier) {
#pragma unroll
            for (int n = 0; n < NUA + NUB; ++n) read_unit(n, 0, std::integral_constant<int, 0>{});
            read_scales(0, nxA, nxB);
        }
    }
    constexpr int NM = PA * PB * RA * RB;              // MFMAs per K step
    int cur = 0;                                       // stage of the current step: ks % S
    // byte offset, inside a unit row, of the K step whose copies the current step issues (step ks + S,
    // clamped to the last one): carried from step to step instead of being derived from ks each time
    const uint32_t last_off = (uint32_t)((g.ksteps - 1) * kUnitBytes);
    uint32_t copy_off = (uint32_t)S * kUnitBytes;
    copy_off = copy_off < last_off ? copy_off : last_off;
    if (copier) {
        // the copy waves' loop: the same waits, barriers and copies, in the same order, as the WS = 0 form
        for (int64_t ks4 = 0; ks4 < groups; ++ks4) {
            auto cstep = [&](auto jc) {
                constexpr int j = decltype(jc)::value;
                wait_vmcnt<(S - 2) * NLOAD + (j == 1 ? NSC : 0)>();
                __syncthreads();
                if (j == 0) {
#pragma unroll
                    for (int q = 0; q < NSC; ++q) issue_scale_one(q, ks4 + 1, (int)((ks4 + 1) & 1));
                }
#pragma unroll
                for (int q = 0; q < NI; ++q) copy_item(src[q] + copy_off, lds0 + cur * STAGE + dst[q]);
                cur = cur + 1 == S ? 0 : cur + 1;
                copy_off = copy_off + kUnitBytes < last_off ? copy_off + kUnitBytes : last_off;
            };
            cstep(std::integral_constant<int, 0>{});
            cstep(std::integral_constant<int, 1>{});
            cstep(std::integral_constant<int, 2>{});
            cstep(std::integral_constant<int, 3>{});
        }
        wait_vmcnt<0>();                                  // the clamped tail copies must not outlive the LDS
        return;
    }
    for (int64_t ks4 = 0; ks4 < groups; ++ks4) {
#pragma unroll
        for (int t = 0; t < RA; ++t) scA[t] = nxA[t];
#pragma unroll
        for (int t = 0; t < RB; ++t) scB[t] = nxB[t];
        // one K step; j (stage, register set, byte of the scale dwords) must be a compile-time constant
        auto kstep = [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            constexpr int set = j & 1;
            const int64_t ks = ks4 * 4 + j;
            const int nxt = cur + 1 == S ? 0 : cur + 1;
            // side work of this step, in issue order: LDS reads for step ks+1, copies for step ks+S,
            // at j == 0 the scale copies of the next group, at j == 3 the read of those scales
            constexpr int NCP = WS ? 0 : NI, NSCP = WS ? 0 : NSC;      // copies issued by this wave
            constexpr int NAUX = (NUA + NUB) + NCP + (j == 0 ? NSCP : 0) + (j == 3 ? 1 : 0);
            constexpr int NSLOT = NM > MX_SCALED_TAIL_MFMAS ? NM - MX_SCALED_TAIL_MFMAS : 1;
            auto aux = [&](int x) {
                if (x < NUA + NUB) { read_unit(x, nxt, std::integral_constant<int, set ^ 1>{}); return; }
                x -= NUA + NUB;
                if (j == 0) {                             // the scale copies go ahead of the step's data copies
                    if (x < NSCP) { issue_scale_one(x, ks4 + 1, (int)((ks4 + 1) & 1)); return; }
                    x -= NSCP;
                }
                if (x < NCP) { copy_item(src[x] + copy_off, lds0 + cur * STAGE + dst[x]); return; }
                if (j == 3) read_scales((int)((ks4 + 1) & 1), nxA, nxB);
            };
            __builtin_amdgcn_sched_barrier(0);
            // newer than D(ks+1): the data copies of the last S-2 steps, and at j == 1 the scale copies
            // issued at the previous step, ahead of its data copies (at step 2 they are simply awaited too)
            if constexpr (WS == 0) wait_vmcnt<(S - 2) * NLOAD + (j == 1 ? NSC : 0)>();
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            // one piece pair after the other: consecutive MFMAs never share an accumulator
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int tb = m % RB, ta = (m / RB) % RA, pb = (m / (RA * RB)) % PB, pa = m / (RA * RB * PB);
                // piece 0 of a two-piece operand is the high one: scale byte + 4
                const int sa = (int)(scA[ta] + ((PA == 2 && pa == 0) ? 0x04040404u : 0u));
                const int sb = (int)(scB[tb] + ((PB == 2 && pb == 0) ? 0x04040404u : 0u));
                acc[ta][tb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                    operand(fa[set][ta][pa]), operand(fb[set][tb][pb]), acc[ta][tb], 2, 2, j, sa, j, sb);
                // the side work goes between the first NSLOT MFMAs: the step ends on MFMAs alone, so the LDS reads
                // have returned by the time the next step's barrier waits for them
                if (m < NSLOT) {
#pragma unroll
                    for (int x = m * NAUX / NSLOT; x < (m + 1) * NAUX / NSLOT; ++x) aux(x);
                }
                __builtin_amdgcn_sched_barrier(0);        // pin the interleaving as written
            }
            cur = nxt;
            copy_off = copy_off + kUnitBytes < last_off ? copy_off + kUnitBytes : last_off;
        };
        kstep(std::integral_constant<int, 0>{});
        kstep(std::integral_constant<int, 1>{});
        kstep(std::integral_constant<int, 2>{});
        kstep(std::integral_constant<int, 3>{});
    }
    if constexpr (WS == 0) wait_vmcnt<0>();               // the clamped tail copies must not outlive the LDS

    const int64_t rtA0 = (bm * 2 + wm) * RA, rtB0 = (bn * 2 + wn) * RB;
    const int i = lane & 31, h = lane >> 5;
    if constexpr (QO != 0) {
        // One row tile of the wave at a time: results -> the wave's LDS tile, row-major; then lane 32*h' + i'
        // holds the 32 consecutive elements of row i' that a fragment of the next product's left operand
        // gives it, and runs the quantizer of mx_quantize_pack on them.
        static_assert(RB % 2 == 0, "a wave covers whole K steps of the output");
        constexpr int PITCH = 32 * RB + 4;               // floats; the skew spreads the rows over the banks
        // LDS: four tiles of 32 x PITCH floats, then the bias of the 64*TN columns (the launch sizes the
        // allocation for whichever is larger, this or the stages)
        __syncthreads();                                 // every wave is done reading the stages
        float* tile = reinterpret_cast<float*>(smem) + wave * (32 * PITCH);
        float* bias_lds = reinterpret_cast<float*>(smem) + 4 * 32 * PITCH;
        if (g.bias_mant != nullptr) {                    // the bias of the workgroup's columns, decoded once
            for (int c = threadIdx.x; c < 64 * TN; c += 256) {
                const int64_t n = bn * (64 * TN) + c;
                float bv = 0.f;
                if (n < g.N) {
                    const int64_t bit = n * g.wbias;
                    const int sh = (int)(bit & 7);
                    uint32_t code = g.bias_mant[bit >> 3];
                    if (sh + g.wbias > 8) code |= (uint32_t)g.bias_mant[(bit >> 3) + 1] << 8;
                    const int q = ((int)((code >> sh) << (32 - g.wbias))) >> (32 - g.wbias);
                    bv = __builtin_ldexpf((float)q, (int)g.bias_exps[n / g.blk_bias] - g.bias_b - (g.wbias - 2));
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
                for (int r = 0; r < 16; ++r)
                    tile[(8 * (r >> 2) + 4 * h + (r & 3)) * PITCH + tb * 32 + i] = __builtin_ldexpf(acc[ta][tb][r], g.eadj);
            __builtin_amdgcn_wave_barrier();
            const int64_t rt = rtA0 + ta, row = rt * 32 + i;
#pragma unroll
            for (int ksl = 0; ksl < RB / 2; ++ksl) {
                const int64_t ks = rtB0 / 2 + ksl;        // K step of the output operand
                const int64_t col0 = ks * 64 + h * 32;
                const bool inside = row < g.M && col0 < g.N;
                float v[32];
#pragma unroll
                for (int q4 = 0; q4 < 8; ++q4) {
                    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (inside) {
                        t = *reinterpret_cast<const float4*>(tile + i * PITCH + ksl * 64 + h * 32 + 4 * q4);
                        if (g.bias_mant != nullptr) {
                            const float4 b = *reinterpret_cast<const float4*>(bias_lds + wn * (32 * RB) + ksl * 64 + h * 32 + 4 * q4);
                            t.x += b.x; t.y += b.y; t.z += b.z; t.w += b.w;
                        }
                    }
                    v[4 * q4] = t.x; v[4 * q4 + 1] = t.y; v[4 * q4 + 2] = t.z; v[4 * q4 + 3] = t.w;
                }
                uint32_t am = 0;
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    const uint32_t ab = __float_as_uint(v[e]) & 0x7fffffffu;
                    am = ab > am ? ab : am;
                }
                if (g.blk_o == 64) {                      // the two halves of a lane pair form one block
                    const uint32_t o = (uint32_t)__shfl_xor((int)am, 32, 64);
                    am = o > am ? o : am;
                }
                if (g.brows_o == 2) {                     // two-row blocks: the neighbouring lane holds the other row
                    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)am, 0xB1, 0xF, 0xF, true);
                    am = o > am ? o : am;
                }
                const int ef = (int)(am >> 23);
                int E = ef == 0 ? -127 : ef - 127;
                E = E < -g.bias_o ? -g.bias_o : E;
                E = E > g.emax_o ? g.emax_o : E;
                const int shift = (g.wo - 2) - E;
                v16f lo0, lo1, hi0, hi1;
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    const float sc = __builtin_ldexpf(v[e], shift);
                    float r = g.rnd_o == MX_RNE ? __builtin_rintf(sc) : __builtin_truncf(sc);
                    r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
                    float hi = 0.f, lo = r;
                    if (QO == 2) {
                        hi = __builtin_floorf(r * 0.0625f + 0.5f);      // h = floor((q + 8) / 16)
                        lo = r - 16.f * hi;
                    }
                    lo += 0.0f;                                          // -0.0 -> +0.0
                    if (e & 1) { lo1[e >> 1] = lo; hi1[e >> 1] = hi; }
                    else       { lo0[e >> 1] = lo; hi0[e >> 1] = hi; }
                }
                if (rt < g.go.row_tiles && ks < g.go.ksteps) {
                    const v6i fl = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(lo0, lo1, 2.0f);   // codes of piece / 2
                    uint8_t* unit = obase + mat_unit(g.go, QO == 2 ? rt : rt >> 1, ks);
                    const int lslot = QO == 2 ? 1 : (int)(rt & 1);
                    *reinterpret_cast<uint4*>(unit + frag_lo(lslot, lane)) =
                        make_uint4((uint32_t)fl[0], (uint32_t)fl[1], (uint32_t)fl[2], (uint32_t)fl[3]);
                    *reinterpret_cast<uint2*>(unit + frag_hi(lslot, lane)) = make_uint2((uint32_t)fl[4], (uint32_t)fl[5]);
                    if (QO == 2) {
                        const v6i fh = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(hi0, hi1, 2.0f);
                        *reinterpret_cast<uint4*>(unit + frag_lo(0, lane)) =
                            make_uint4((uint32_t)fh[0], (uint32_t)fh[1], (uint32_t)fh[2], (uint32_t)fh[3]);
                        *reinterpret_cast<uint2*>(unit + frag_hi(0, lane)) = make_uint2((uint32_t)fh[4], (uint32_t)fh[5]);
                    }
                    // the lane's scale byte of this K step (bytes of one dword come from different waves)
                    obase[g.go.frag_bytes + ((rt * (g.go.ksteps / 4) + (ks >> 2)) * 64 + lane) * 4 + (ks & 3)] =
                        inside ? (uint8_t)(E + 127) : (uint8_t)0;
                }
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
                if (m < g.M && n < g.N) __builtin_nontemporal_store(__builtin_ldexpf(acc[ta][tb][r], g.eadj), &Y[m * g.ldy + n]);
            }
        }
    }
}

template <int PA, int PB, int TM, int TN, int S, int OCC, int QO = 0, int WS = 0>
mx_status launch_scaled(ScaledArgs& g, int64_t batch, hipStream_t st) {
    static_assert(WS == 0 || (OCC == 1 && QO == 0), "copy waves: one workgroup per compute unit, fp32 result");
    constexpr int UA = (PA == 2) ? 2 * TM : TM, UB = (PB == 2) ? 2 * TN : TN;
    constexpr int pipe = S * (UA + UB) * kUnitBytes + 2 * (2 * TM + 2 * TN) * 256;
    constexpr int turn = QO == 0 ? 0 : 4 * 32 * (32 * TN + 4) * 4 + 64 * TN * 4;     // quantized ending
    constexpr int smem = pipe > turn ? pipe : turn;
    static_assert(smem * OCC <= 160 * 1024, "LDS budget of one compute unit");
    auto kern = gemm_scaled_kernel<PA, PB, TM, TN, S, OCC, QO, WS>;
    static std::atomic<uint64_t> done{0};
    if (!allow_dynamic_lds((const void*)kern, smem, done)) return MX_ERR_DEVICE;
    const int64_t tiles_m = ceil_div(g.M, 64 * TM), tiles_n = ceil_div(g.N, 64 * TN);
    if (tiles_m * tiles_n > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    if (g.ksteps * kUnitBytes > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;       // 32-bit offsets along K
    g.tiles_m = (int32_t)tiles_m;
    g.tiles_n = (int32_t)tiles_n;
    dim3 grid((unsigned)(ceil_div(tiles_m * tiles_n, 8) * 8), (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(WS ? 512 : 256), smem, st, g);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

// Tile 128 (M) x 256 (N): the left operand costs more bytes per element when it has two mantissa
// pieces, so the tile is wider along N.  When there are at least two tiles per compute unit and
// the stages are small enough, two workgroups share a compute unit (three stages each), so that
// one workgroup's barrier and copy waits hide under the other's MFMAs; otherwise one workgroup
// per compute unit runs with four copy waves beside its four matrix waves and five stages (the
// copies of a K step are requested four steps ahead).
template <int PA, int PB, int QO = 0>
mx_status pick_tile(ScaledArgs& g, int64_t batch, hipStream_t st) {
    const int64_t tiles = ceil_div(g.M, 128) * ceil_div(g.N, 256) * batch;
    if constexpr (PB == 1) {
        if (tiles >= MX_SCALED_TWO_PER_CU_TILES) return launch_scaled<PA, PB, 2, 4, 3, 2, QO>(g, batch, st);
        if constexpr (QO == 0) return launch_scaled<PA, PB, 2, 4, 5, 1, 0, 1>(g, batch, st);
        return launch_scaled<PA, PB, 2, 4, 4, 1, QO>(g, batch, st);
    } else {
        static_assert(QO == 0, "the quantized ending is built for one-piece right operands");
        return launch_scaled<PA, PB, 2, 4, 3, 1>(g, batch, st);
    }
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
    g.tiles_m = g.tiles_n = 0;
    g.out = nullptr; g.bias_mant = g.bias_exps = nullptr;
    if (ga.pieces == 2 && gb.pieces == 1) return pick_tile<2, 1>(g, batch, st);
    if (ga.pieces == 1 && gb.pieces == 1) return pick_tile<1, 1>(g, batch, st);
    if (ga.pieces == 2 && gb.pieces == 2) return pick_tile<2, 2>(g, batch, st);
    return pick_tile<1, 2>(g, batch, st);
}

// The same product with the bias added and the result quantized to `fo` (block 32 or 64, blocks along
// N), written as the packed operand [M x N] of this layout.  Right operands of up to 4 stored bits.
mx_status gemm_scaled_q(int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, mx_format fa,
                        const void* B, mx_format fb, const uint8_t* bias_mant, const uint8_t* bias_exps,
                        mx_format fbias, mx_format fo, void* out, hipStream_t st) {
    const MatGeom ga = mat_geom(M, K, fa.mant_bits), gb = mat_geom(N, K, fb.mant_bits);
    if (gb.pieces != 1) return MX_ERR_UNSUPPORTED;
    ScaledArgs g;
    g.A = (const uint8_t*)A; g.B = (const uint8_t*)B; g.Y = nullptr; g.M = M; g.N = N;
    g.unitsA = ga.units; g.unitsB = gb.units; g.tilesA = ga.row_tiles; g.tilesB = gb.row_tiles;
    g.ksteps = ga.ksteps; g.fragA = ga.frag_bytes; g.fragB = gb.frag_bytes;
    g.matrixA = ga.matrix; g.matrixB = gb.matrix; g.ldy = 0; g.batch_stride_y = 0;
    g.eadj = 2 - (fa.mant_bits - 2) - (fb.mant_bits - 2);
    g.tiles_m = g.tiles_n = 0;
    g.out = (uint8_t*)out; g.go = mat_geom(M, N, fo.mant_bits);
    g.bias_mant = bias_mant; g.bias_exps = bias_exps;
    g.wbias = fbias.mant_bits; g.bias_b = (1 << (fbias.exp_bits - 1)) - 1; g.blk_bias = fbias.block;
    g.wo = fo.mant_bits; g.bias_o = (1 << (fo.exp_bits - 1)) - 1;
    g.emax_o = ((1 << fo.exp_bits) - 1) - g.bias_o;
    g.rnd_o = fo.rounding; g.brows_o = fo.block_rows; g.blk_o = fo.block;
    const int po = mat_pieces(fo.mant_bits);
    if (ga.pieces == 2) return po == 2 ? pick_tile<2, 1, 2>(g, batch, st) : pick_tile<2, 1, 1>(g, batch, st);
    return po == 2 ? pick_tile<1, 1, 2>(g, batch, st) : pick_tile<1, 1, 1>(g, batch, st);
}

}  // namespace mx
