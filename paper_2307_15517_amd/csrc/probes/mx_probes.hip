// Roofline probes for the benchmark (not part of libmx): the simplest kernel of each kind, to tell what
// this GPU reaches where a kernel of the library is priced against a published peak.
//   mxp_read / mxp_write / mxp_copy   streaming passes over a buffer, 16 bytes per lane, grid-stride
//   mxp_mfma_fp6 / mxp_mfma_i8        a loop of independent matrix instructions on operands held in
//                                     registers (block-scaled 6-bit float form, and int8), nothing else
//                                     in the loop; every wave also reports shader cycles and the
//                                     constant 100 MHz counter over its loop, i.e. the clock it ran at
// All pointers are device pointers; every call only enqueues on `stream`.  Return 0, or 1 on a bad argument
// or a failed launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#define MXP_API extern "C" __attribute__((visibility("default")))

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kUnroll = 8;      // 16-byte accesses per lane in flight

__global__ __launch_bounds__(512) void read_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (size_t)gridDim.x * blockDim.x;
    uint32_t s = 0;
    for (size_t i = tid; i < n16; i += nt * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t j = i + u * nt;
            v[u] = j < n16 ? p[j] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) s += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (s == 0x12345678u) sink[0] = s;          // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(512) void write_kernel(uint4* __restrict__ p, size_t n16) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (size_t)gridDim.x * blockDim.x;
    const uint4 v = make_uint4((uint32_t)tid, 1u, 2u, 3u);
    for (size_t i = tid; i < n16; i += nt) p[i] = v;
}

__global__ __launch_bounds__(512) void copy_kernel(uint4* __restrict__ d, const uint4* __restrict__ p, size_t n16) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (size_t)gridDim.x * blockDim.x;
    for (size_t i = tid; i < n16; i += nt * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t j = i + u * nt;
            if (j < n16) v[u] = p[j];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t j = i + u * nt;
            if (j < n16) d[j] = v[u];
        }
    }
}

// out[wave] = {shader cycles of the loop, ticks of the 100 MHz counter over the loop}
struct Clock { uint64_t cycles, ticks; };

// 16 matrix instructions per iteration on 8 accumulators (two per accumulator, as a two-piece operand gives).
// a, b: 64 lanes x 4 fragments x 8 dwords each (the 6-bit form reads six of them).
__global__ __launch_bounds__(256, 2) void mfma_fp6_kernel(const uint32_t* a, const uint32_t* b, int iters, Clock* out,
                                                          float* sink) {
    const int lane = threadIdx.x & 63;
    v8i fa[4], fb[4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            fa[f][d] = d < 6 ? (int)a[(lane * 4 + f) * 8 + d] : 0;
            fb[f][d] = d < 6 ? (int)b[(lane * 4 + f) * 8 + d] : 0;
        }
    v16f acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    const int sc = 0x7f7f7f7f;                   // scale 2^0 in every byte
    const uint64_t c0 = __builtin_readcyclecounter(), t0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int t = m & 7;
            acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[(m >> 3) * 2 + (t >> 2)], fb[t & 3], acc[t], 2, 2, 0,
                                                                    sc, 0, sc);
        }
    }
    const uint64_t c1 = __builtin_readcyclecounter(), t1 = __builtin_amdgcn_s_memrealtime();
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    if (s == 12345.678f) sink[0] = s;
    if (lane == 0) {
        const int w = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
        out[w].cycles = c1 - c0;
        out[w].ticks = t1 - t0;
    }
}

// the same with v_mfma_i32_32x32x32_i8: 16 instructions per iteration on 8 accumulators.
// a, b: 64 lanes x 4 fragments x 4 dwords.
__global__ __launch_bounds__(256, 2) void mfma_i8_kernel(const uint32_t* a, const uint32_t* b, int iters, Clock* out,
                                                         float* sink) {
    const int lane = threadIdx.x & 63;
    v4i fa[4], fb[4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            fa[f][d] = (int)a[(lane * 4 + f) * 4 + d];
            fb[f][d] = (int)b[(lane * 4 + f) * 4 + d];
        }
    v16i acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0;
    const uint64_t c0 = __builtin_readcyclecounter(), t0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int t = m & 7;
            acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[(m >> 3) * 2 + (t >> 2)], fb[t & 3], acc[t], 0, 0, 0);
        }
    }
    const uint64_t c1 = __builtin_readcyclecounter(), t1 = __builtin_amdgcn_s_memrealtime();
    int s = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    if (s == 0x12345678) sink[0] = 1.f;
    if (lane == 0) {
        const int w = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
        out[w].cycles = c1 - c0;
        out[w].ticks = t1 - t0;
    }
}

int ok_launch() { return hipGetLastError() == hipSuccess ? 0 : 1; }

}  // namespace

// Workgroups of the streaming probes: eight of 512 threads per compute unit of a 256-unit GPU.
constexpr int kStreamGrid = 2048;
// Workgroups of the matrix probes: two of four waves per compute unit.
MXP_API int mxp_mfma_waves(void) { return 512 * 4; }

MXP_API int mxp_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || ((uintptr_t)src & 15) || bytes % 16) return 1;
    hipLaunchKernelGGL(read_kernel, dim3(kStreamGrid), dim3(512), 0, (hipStream_t)stream, (const uint4*)src, bytes / 16,
                       (uint32_t*)sink);
    return ok_launch();
}
MXP_API int mxp_write(void* dst, size_t bytes, void* stream) {
    if (!dst || ((uintptr_t)dst & 15) || bytes % 16) return 1;
    hipLaunchKernelGGL(write_kernel, dim3(kStreamGrid), dim3(512), 0, (hipStream_t)stream, (uint4*)dst, bytes / 16);
    return ok_launch();
}
MXP_API int mxp_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || (((uintptr_t)dst | (uintptr_t)src) & 15) || bytes % 16) return 1;
    hipLaunchKernelGGL(copy_kernel, dim3(kStreamGrid), dim3(512), 0, (hipStream_t)stream, (uint4*)dst, (const uint4*)src,
                       bytes / 16);
    return ok_launch();
}
// a, b: 64*4*8 dwords each; out: mxp_mfma_waves() records of two uint64; sink: 4 bytes.
// Operations per call: mxp_mfma_waves() * iters * 16 * 2*32*32*64.
MXP_API int mxp_mfma_fp6(const void* a, const void* b, int iters, void* out, void* sink, void* stream) {
    if (!a || !b || !out || !sink || iters < 0) return 1;
    hipLaunchKernelGGL(mfma_fp6_kernel, dim3(512), dim3(256), 0, (hipStream_t)stream, (const uint32_t*)a, (const uint32_t*)b,
                       iters, (Clock*)out, (float*)sink);
    return ok_launch();
}
// a, b: 64*4*4 dwords each.  Operations per call: mxp_mfma_waves() * iters * 16 * 2*32*32*32.
MXP_API int mxp_mfma_i8(const void* a, const void* b, int iters, void* out, void* sink, void* stream) {
    if (!a || !b || !out || !sink || iters < 0) return 1;
    hipLaunchKernelGGL(mfma_i8_kernel, dim3(512), dim3(256), 0, (hipStream_t)stream, (const uint32_t*)a, (const uint32_t*)b,
                       iters, (Clock*)out, (float*)sink);
    return ok_launch();
}
