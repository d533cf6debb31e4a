// Decode-time linear layer in one launch (mx_linear, 1..8 activation rows, weights in the fragment layout).
//
// Arithmetic (Section 3.2 of the paper: quantize the input, then the MXInt dot-product operator -- exact
// integer block dots, the two shared exponents applied once per block; format of Section 4.1): the fp32
// activations are quantized with the arithmetic of mx_quantize on their way into on-chip memory, the block
// dots are taken with one int8 MFMA per block, each block's integer is scaled by
// 2^(Ea + Eb - (wa-2) - (wb-2)) and added into an fp32 accumulator.  mx_linear uses this kernel for three
// to eight rows; one and two rows go to the dot-product kernel of mx_gemv_dot.hip, which needs no exchange
// between workgroups.
//
// Work split: the path is bound by one pass over the packed weights, so every compute unit has to stream.
// The grid is (column groups of 32) x (K slices); a workgroup quantizes only its own slice of the
// activations (no workgroup repeats the whole row), keeps a ring of weight records in flight per wave and
// ends with 32 partial sums per row.  With more than one slice the partial sums go to the caller's workspace
// and the workgroup that arrives last at the column group's counter adds them in slice order, so the result
// does not depend on the order of arrival.
#include <type_traits>

#include "mx_decode.h"
#include "mx_frag.h"

#ifndef MX_DECODE_TARGET_WAVES
#define MX_DECODE_TARGET_WAVES 2560    // (column group, K slice) pairs aimed at: ten waves per compute unit
#endif
#ifndef MX_DECODE_WAVES
#define MX_DECODE_WAVES 4              // waves, i.e. column groups, per workgroup
#endif
#ifndef MX_DECODE_DEPTH
#define MX_DECODE_DEPTH 5              // weight records in flight per wave (narrow records)
#endif
#ifndef MX_DECODE_MIN_SLICE
#define MX_DECODE_MIN_SLICE 4          // records per wave at least
#endif

namespace mx {
namespace {

struct DecodeArgs {
    const float* x;
    int64_t x_stride;
    const uint8_t* B;        // packed weights [groups][chunks] records
    float* Y;
    int64_t ldy;
    uint32_t* counters;      // one per workgroup column: zero on entry, zero again on exit
    float* partial;          // [ksplit][M][32*groups]
    int32_t M, N, K;
    int32_t groups, quads, quads8, chunks, slice, ksplit;
    int32_t recordB;
    int32_t wa, bias, emax, rounding;
    int32_t eadj;            // -2*bias - (wa-2) - (wb-2)
};

// Grid: (workgroup columns) x (K slices); a workgroup of NW waves owns NW neighbouring column groups of 32
// and one K slice: its waves share the quantized activations of the slice (LDS), wave w streams the records of
// column group NW*column + w.
// Up to eight rows: one int8 MFMA per block with the activations as the 32-row operand (rows 8..31 of it are
// never looked at, so the lanes that would hold them may hold anything).
// D: weight records a wave keeps in flight.  It is sized so that a wave requests most of its slice before the
// activations are quantized: the weights stream while the workgroup prepares the other operand.
template <int WB, int B, int NW, int D>
__global__ __launch_bounds__(NW * 64, (D * (Piece<WB, B>::kDw + 1) + (B == 16 ? 92 : 112) <= 128 ? 4 : (D * (Piece<WB, B>::kDw + 1) + (B == 16 ? 92 : 112) <= 168 ? 3 : 2)))
void linear_splitk_kernel(DecodeArgs a) {
    constexpr int kDwB = Piece<WB, B>::kDw;
    constexpr int kHalfDw = B / 8;                       // int8 dwords of a half block
    constexpr int MP = 8;                                 // rows with a slot in LDS
    constexpr int MR = 4;                                 // accumulators per lane: rows 4h .. 4h+3
    constexpr int T = NW * 64;
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    __shared__ int is_last;

    const int gq = (int)(blockIdx.x % (unsigned)a.quads8), ks = (int)(blockIdx.x / (unsigned)a.quads8);
    if (gq >= a.quads) return;                            // whole workgroup, before any barrier
    const int c0 = ks * a.slice;
    const int nc = (a.chunks - c0 < a.slice) ? a.chunks - c0 : a.slice;     // records of this slice, >= 1
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 31, h = lane >> 5;
    const int gb = gq * NW + wave;                        // this wave's column group
    const bool wave_live = gb < a.groups;                 // wave-uniform

    // LDS: x8[nc*4 blocks][2 halves][8 rows][kHalfDw], xe[nc*4 blocks][8 rows] (Ea + eadj as int)
    uint32_t* x8 = lds;
    uint32_t* xe = x8 + MP * a.slice * 4 * 2 * kHalfDw;

    // ring of D records of this wave's column group; a record past the slice reads zeros without touching
    // memory, so no load sits under a condition and the waits stay exact
    const uint8_t* Bbase = a.B + ((int64_t)(wave_live ? gb : 0) * a.chunks + c0) * a.recordB;
    const BufRsrc rB = make_rsrc(Bbase, wave_live ? (uint32_t)(nc * a.recordB) : 0u);
    uint32_t pb[D][kDwB], eb[D];
    auto fetch = [&](int slot, int t) {
        const uint32_t off = (uint32_t)t * (uint32_t)a.recordB;
        buf_load_dwords<kDwB>(rB, off + lane * (kDwB * 4), pb[slot]);
        buf_load_dwords<1>(rB, off + 64 * (kDwB * 4) + i * 4, &eb[slot]);
    };

    // ---- activations of this slice: fp32 -> MXInt (the arithmetic of mx_quantize) -> int8 in LDS.
    // One item is four consecutive elements of a row; consecutive lanes take consecutive items, so a block is
    // B/4 neighbouring lanes and its maximum takes log2(B/4) DPP steps.  Loads return in the order of issue:
    // the first items are requested before the ring of weights.
    {
        const int ipr = nc * B;                            // items per row (slice elements / 4)
        const int n_it = a.M * ipr;
        const float qmax = (float)((1 << (a.wa - 1)) - 1);
        const int64_t k0 = (int64_t)c0 * 4 * B;
        constexpr int XU = 8;                              // items per thread requested before the weights
        constexpr float kMagic = 12582912.0f;              // 1.5 * 2^23: adding it rounds to an integer, ties to even
        // item -> (row, first element inside the slice), advanced without divisions
        int m_it = 0, e_it = 4 * (int)threadIdx.x;
        auto settle = [&]() {
            while (e_it >= 4 * ipr && m_it < a.M) { e_it -= 4 * ipr; ++m_it; }
        };
        settle();
        auto item_load = [&](int m, int e) -> float4 {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m < a.M && k0 + e < a.K) v = *reinterpret_cast<const float4*>(a.x + (int64_t)m * a.x_stride + k0 + e);   // K % 4 == 0
            return v;
        };
        auto item_store = [&](int m, int e, const float4& v) {
            float am = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(v.x), __builtin_fabsf(v.y)),
                                       __builtin_fmaxf(__builtin_fabsf(v.z), __builtin_fabsf(v.w)));
            uint32_t ab = __float_as_uint(am), o;
            o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)ab, 0xB1, 0xF, 0xF, true);  ab = o > ab ? o : ab;   // lane ^ 1
            o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)ab, 0x4E, 0xF, 0xF, true);  ab = o > ab ? o : ab;   // lane ^ 2
            if (B >= 32) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)ab, 0x141, 0xF, 0xF, true); ab = o > ab ? o : ab; }   // 7 - lane within 8
            if (B >= 64) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)ab, 0x140, 0xF, 0xF, true); ab = o > ab ? o : ab; }   // 15 - lane within 16
            if (m >= a.M) return;                          // after the cross-lane steps: every lane of a block takes part in them
            const int ef = (int)(ab >> 23);
            int E = ef == 0 ? -127 : ef - 127;
            E = E < -a.bias ? -a.bias : E;
            E = E > a.emax ? a.emax : E;
            const int shift = (a.wa - 2) - E;
            // round(x * 2^shift), clamped: the sum with kMagic holds the integer in its low mantissa bits (a
            // value beyond the clamp, however large, ends at the clamp as well), its low byte is the int8 code
            auto code = [&](float xx) -> uint32_t {
                float sc = __builtin_ldexpf(xx, shift);
                if (a.rounding != MX_RNE) sc = __builtin_truncf(sc);
                const float z = __builtin_fminf(__builtin_fmaxf(sc + kMagic, kMagic - qmax), kMagic + qmax);
                return __float_as_uint(z);
            };
            const uint32_t lo = __builtin_amdgcn_perm(code(v.y), code(v.x), 0x0C0C0400u);
            const uint32_t hi = __builtin_amdgcn_perm(code(v.w), code(v.z), 0x04000C0Cu);
            const uint32_t word = lo | hi;
            const int blk = e / B, p = e - blk * B;         // block of the slice, position inside it (B is a power of two)
            const int hh = p / (B / 2), d = (p - hh * (B / 2)) >> 2;
            const int ebyte = (k0 + e < a.K) ? E + a.bias : 0;
            x8[((blk * 2 + hh) * 8 + m) * kHalfDw + d] = word;
            if (p == 0) xe[blk * 8 + m] = (uint32_t)(ebyte + a.eadj - Unpack<WB, B>::kScaleLog2);
        };
        // every thread runs the same number of rounds (the DPP steps need whole blocks of lanes)
        const int rounds = (n_it + T - 1) / T;
        float4 xv[XU];
        int mm[XU], ee[XU];
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            mm[u] = m_it; ee[u] = e_it;
            xv[u] = item_load(m_it, e_it);
            e_it += 4 * T; settle();
        }
#pragma unroll
        for (int u = 0; u < D; ++u) fetch(u, u);
#pragma unroll
        for (int u = 0; u < XU; ++u)
            if (u < rounds) item_store(mm[u], ee[u], xv[u]);
        for (int r = XU; r < rounds; ++r) {
            const float4 v = item_load(m_it, e_it);
            item_store(m_it, e_it, v);
            e_it += 4 * T; settle();
        }
    }
    __syncthreads();

    float acc[MR];
#pragma unroll
    for (int r = 0; r < MR; ++r) acc[r] = 0.f;
    const int per_wave = wave_live ? nc : 0;
    for (int t0 = 0; t0 < per_wave; t0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int c = t0 + u;                             // record inside the slice
            const bool live = c < per_wave;                   // scalar condition: no load depends on it
            uint32_t fb[4][kHalfDw];
            uint32_t ebv = 0;
            if (live) {
#pragma unroll
                for (int j = 0; j < 4; ++j) Unpack<WB, B>::run(pb[u], j, fb[j]);
                ebv = eb[u];
            }
            fetch(u, c + D);                                  // the slot is free: refill it
            if (!live) continue;
            // the four blocks of the record: operands from LDS first, then the matrix instructions issued ahead
            // of the scaling of the block before, so that their latency is covered by vector work
            uint32_t fa[4][kHalfDw];
            int4 ea[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int blk = c * 4 + j;
                const uint32_t* xa = x8 + ((blk * 2 + h) * 8 + (i & 7)) * kHalfDw;
#pragma unroll
                for (int q = 0; q < kHalfDw; ++q) fa[j][q] = xa[q];
                ea[j] = *reinterpret_cast<const int4*>(xe + blk * 8 + 4 * h);
            }
            auto scale = [&](const v16i_t& d, int j) {
                const int ebj = (int)((ebv >> (8 * j)) & 0xFFu);
                acc[0] += __builtin_ldexpf((float)d[0], ea[j].x + ebj);
                acc[1] += __builtin_ldexpf((float)d[1], ea[j].y + ebj);
                acc[2] += __builtin_ldexpf((float)d[2], ea[j].z + ebj);
                acc[3] += __builtin_ldexpf((float)d[3], ea[j].w + ebj);
            };
            const v16i_t d0 = block_mfma<B>(fa[0], fb[0]);
            const v16i_t d1 = block_mfma<B>(fa[1], fb[1]);
            __builtin_amdgcn_sched_barrier(0);
            scale(d0, 0);
            __builtin_amdgcn_sched_barrier(0);
            const v16i_t d2 = block_mfma<B>(fa[2], fb[2]);
            __builtin_amdgcn_sched_barrier(0);
            scale(d1, 1);
            __builtin_amdgcn_sched_barrier(0);
            const v16i_t d3 = block_mfma<B>(fa[3], fb[3]);
            __builtin_amdgcn_sched_barrier(0);
            scale(d2, 2);
            scale(d3, 3);
        }
    }

    // ---- a wave's 32 sums per row: the result, or with several K slices this slice's partial sums.  The
    // partial sums are written and read with device-coherent accesses (they pass between workgroups that may
    // sit behind different L2 caches), so no cache has to be written back or invalidated as a whole.
    const int64_t np = (int64_t)a.groups * 32;
    const int64_t n = (int64_t)gb * 32 + i;
    // buffer accesses with the device-scope bit: written through / read at the level every compute unit shares
    constexpr int kDeviceScope = 0x10;
    const BufRsrc rP = make_rsrc(a.partial, (uint32_t)((int64_t)a.ksplit * a.M * np * 4));
    auto put = [&](int m, float s) {
        if (m >= a.M || !wave_live) return;
        if (a.ksplit == 1) { if (n < a.N) a.Y[(int64_t)m * a.ldy + n] = s; }
        else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(s), rP, (uint32_t)((((int64_t)ks * a.M + m) * np + n) * 4), 0, kDeviceScope);
    };
#pragma unroll
    for (int r = 0; r < 4; ++r) put(4 * h + r, acc[r]);
    if (a.ksplit == 1) return;

    // ---- the K slices of this workgroup column: whoever arrives last adds the partial sums in slice order.
    // Order: this thread's partial sums have been written through (the wait), then every thread's (the barrier),
    // then the arrival is counted; the last workgroup reads after it has seen every arrival.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(a.counters + gq, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = old == (uint32_t)(a.ksplit - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    // A thread owns up to OPT outputs of the workgroup's columns.  The loads of all of them, eight or sixteen slices at
    // a time, are requested before the first addition (one trip to memory for up to sixteen slices, not one per output
    // or per slice); the additions run in slice order whatever the order of arrival was.  A thread without an output
    // reads the first partial sum and drops it.
    const uint32_t kstride = (uint32_t)(a.M * np * 4);
    constexpr int OPT = (MP * NW * 32 + T - 1) / T;
    uint32_t off0[OPT];
    int64_t col_n[OPT];
    int row_m[OPT];
    float s[OPT];
#pragma unroll
    for (int o = 0; o < OPT; ++o) {
        const int t = (int)threadIdx.x + o * T;
        const int m = t / (NW * 32), col = t - m * (NW * 32);
        const int64_t nn = (int64_t)gq * (NW * 32) + col;
        const bool on = m < a.M && nn < np;
        row_m[o] = on ? m : -1;
        col_n[o] = nn;
        off0[o] = on ? (uint32_t)(((int64_t)m * np + nn) * 4) : 0u;
        s[o] = 0.f;
    }
    auto add_slices = [&](auto kbc) {                     // KB slices per trip
        constexpr int KB = decltype(kbc)::value;
        for (int k0 = 0; k0 < a.ksplit; k0 += KB) {
            uint32_t v[OPT][KB];
#pragma unroll
            for (int o = 0; o < OPT; ++o)
#pragma unroll
                for (int u = 0; u < KB; ++u) {
                    const int k = k0 + u < a.ksplit ? k0 + u : a.ksplit - 1;     // a repeated load instead of a branch
                    v[o][u] = __builtin_amdgcn_raw_buffer_load_b32(rP, off0[o] + (row_m[o] >= 0 ? (uint32_t)k * kstride : 0u), 0, kDeviceScope);
                }
#pragma unroll
            for (int o = 0; o < OPT; ++o)
#pragma unroll
                for (int u = 0; u < KB; ++u)
                    if (k0 + u < a.ksplit) s[o] += __uint_as_float(v[o][u]);
        }
    };
    if (a.ksplit <= 8) add_slices(std::integral_constant<int, 8>{});
    else add_slices(std::integral_constant<int, 16>{});
#pragma unroll
    for (int o = 0; o < OPT; ++o)
        if (row_m[o] >= 0 && col_n[o] < a.N) a.Y[(int64_t)row_m[o] * a.ldy + col_n[o]] = s[o];
    if (threadIdx.x == 0) __hip_atomic_store(a.counters + gq, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int B> constexpr int lds_per_chunk() { return (4 * 2 * 8 * (B / 8) + 4 * 8) * 4; }

template <int WB, int B>
mx_status launch_decode(const DecodeArgs& a, hipStream_t st) {
    // records in flight per wave: up to a whole slice, fewer when a record's lane piece is wide (the ring
    // lives in registers)
    constexpr int NW = MX_DECODE_WAVES;
    constexpr int kRegs = Piece<WB, B>::kDw + 1;
    constexpr int D = MX_DECODE_DEPTH * kRegs <= 96 ? MX_DECODE_DEPTH : (96 / kRegs < 2 ? 2 : 96 / kRegs);
    const size_t smem = (size_t)a.slice * lds_per_chunk<B>();
    auto kern = linear_splitk_kernel<WB, B, NW, D>;
    if (smem > 64 * 1024) return MX_ERR_UNSUPPORTED;          // the default limit of dynamic LDS; decode_plan stays below it
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.quads8 * a.ksplit)), dim3(NW * 64), smem, st, a);
    MX_HIP_LAUNCH_CHECK();
    return MX_OK;
}

template <int B>
mx_status dispatch_wb(const DecodeArgs& a, int wb, hipStream_t st) {
    switch (wb) {
        case 2: return launch_decode<2, B>(a, st);
        case 3: return launch_decode<3, B>(a, st);
        case 4: return launch_decode<4, B>(a, st);
        case 5: return launch_decode<5, B>(a, st);
        case 6: return launch_decode<6, B>(a, st);
        case 7: return launch_decode<7, B>(a, st);
        case 8: return launch_decode<8, B>(a, st);
    }
    return MX_ERR_BAD_ARG;
}

}  // namespace

// How mx_linear splits the weights of an M x K by N x K product over workgroups.  `ok` is false when the
// one-launch kernel does not take the shape (the caller then quantizes and multiplies in two launches).
DecodePlan decode_plan(int64_t M, int64_t K, int64_t N, int block, int wb) {
    DecodePlan p;
    p.ok = false; p.ksplit = 1; p.slice = 0; p.partial_floats = 0;
    const FragGeom gb = frag_geom(N, K, block, wb);
    if (M < 1 || M > 8 || K <= 0 || gb.groups > kDecodeMaxGroups || gb.chunks > (1 << 20)) return p;
    if ((gb.chunks + 1024) * (int64_t)gb.record >= (1LL << 31)) return p;       // 32-bit ring offsets
    const int64_t per_chunk = (int64_t)(4 * 2 * 8 * (block / 8) + 32) * 4;          // LDS bytes per record of a slice
    const int64_t lds_cap = (56 * 1024) / per_chunk;
    int64_t ksplit = (MX_DECODE_TARGET_WAVES + gb.groups / 2) / gb.groups;
    ksplit = ksplit < 1 ? 1 : ksplit;
    int64_t slice = ceil_div(gb.chunks, ksplit);
    slice = slice < MX_DECODE_MIN_SLICE ? MX_DECODE_MIN_SLICE : slice;
    slice = slice > lds_cap ? lds_cap : slice;
    slice = slice > gb.chunks ? gb.chunks : slice;
    ksplit = ceil_div(gb.chunks, slice);                                         // every slice holds a record
    if (ksplit > kDecodeMaxSplit) return p;
    p.ok = true; p.ksplit = (int32_t)ksplit; p.slice = (int32_t)slice;
    p.partial_floats = ksplit > 1 ? ksplit * M * gb.groups * 32 : 0;
    return p;
}

mx_status linear_decode(const float* x, int64_t M, int64_t K, int64_t row_stride, mx_format fx, void* workspace,
                        const void* B_packed, int64_t N, mx_format fb, float* Y, int64_t ldy, hipStream_t st) {
    const DecodePlan p = decode_plan(M, K, N, fb.block, fb.mant_bits);
    if (!p.ok) return MX_ERR_UNSUPPORTED;
    const FragGeom gb = frag_geom(N, K, fb.block, fb.mant_bits);
    DecodeArgs a;
    a.x = x; a.x_stride = row_stride; a.B = (const uint8_t*)B_packed; a.Y = Y; a.ldy = ldy;
    a.counters = reinterpret_cast<uint32_t*>(workspace);
    a.partial = reinterpret_cast<float*>((uint8_t*)workspace + kDecodeCounterBytes);
    a.M = (int32_t)M; a.N = (int32_t)N; a.K = (int32_t)K;
    a.groups = (int32_t)gb.groups;
    a.quads = (int32_t)ceil_div(gb.groups, MX_DECODE_WAVES); a.quads8 = (a.quads + 7) / 8 * 8;
    a.chunks = (int32_t)gb.chunks; a.slice = p.slice; a.ksplit = p.ksplit;
    a.recordB = gb.record;
    a.wa = fx.mant_bits;
    a.bias = (1 << (fx.exp_bits - 1)) - 1;
    a.emax = ((1 << fx.exp_bits) - 1) - a.bias;
    a.rounding = fx.rounding;
    a.eadj = -2 * a.bias - (fx.mant_bits - 2) - (fb.mant_bits - 2);
    if ((int64_t)a.quads8 * a.ksplit > 0x7fffffffLL) return MX_ERR_UNSUPPORTED;
    switch (fb.block) {
        case 16: return dispatch_wb<16>(a, fb.mant_bits, st);
        case 32: return dispatch_wb<32>(a, fb.mant_bits, st);
        case 64: return dispatch_wb<64>(a, fb.mant_bits, st);
    }
    return MX_ERR_UNSUPPORTED;
}

}  // namespace mx
