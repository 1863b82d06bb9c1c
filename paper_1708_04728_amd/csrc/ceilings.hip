// Measuring aids, not part of the library: the rates this GPU sustains on the two resources the kernels are graded
// against (matrix-core issue, memory traffic), so that a kernel's distance from the published peaks can be split into
// "the machine does not reach the peak" and "the kernel does not reach the machine".  Built as a separate shared
// object (libdr_ceilings.so); bench.py --ceilings times these launches with HIP events.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Four waves per workgroup, each issuing `iters` rounds of four independent 32x32x16 bf16 matrix instructions on
// registers: nothing but matrix-core issue.  2 * 32 * 32 * 16 FLOP per instruction.
__global__ __launch_bounds__(256) void mfma_bf16_kernel(float* out, int iters, float a)
{
    f32x16 acc[4];
    bf16x8 va, vb;
    for (int i = 0; i < 8; ++i) { va[i] = (__bf16)a; vb[i] = (__bf16)(a + 1.f); }
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, vb, acc[i], 0, 0, 0);
    float s = 0.f;
    for (int i = 0; i < 4; ++i) s += acc[i][0];
    if (s == 12345.f) out[threadIdx.x] = s;          // keeps the loop alive; never true for the values used
}

// The two clocks a kernel can read: the shader clock (s_memtime) and the constant 100 MHz reference (s_memrealtime).
// Their ratio over a stretch of code is the frequency the compute units ran at during it.
__device__ __forceinline__ unsigned long long shader_ticks()
{
    unsigned long long t;
    asm volatile("s_memtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(t)::"memory");
    return t;
}
__device__ __forceinline__ unsigned long long reference_ticks()
{
    unsigned long long t;
    asm volatile("s_memrealtime %0\n s_waitcnt lgkmcnt(0)" : "=s"(t)::"memory");
    return t;
}

// The same instruction stream on operands that differ from lane to lane and from instruction to instruction (values
// in [-1, 1) from a hash of the lane's id), as a real layer's do: what the matrix cores sustain when the multipliers see
// changing data, and at which clock.  The first wave writes its shader-clock and reference-clock ticks to out[0], out[1].
__global__ __launch_bounds__(256) void mfma_bf16_data_kernel(float* out, int iters)
{
    f32x16 acc[4];
    bf16x8 va[4], vb[4];
    unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 8; ++e) {
            h = h * 1664525u + 1013904223u;
            va[i][e] = (__bf16)((float)(int)(h >> 8 & 0xFFFF) * (1.f / 32768.f) - 1.f);
            h = h * 1664525u + 1013904223u;
            vb[i][e] = (__bf16)((float)(int)(h >> 8 & 0xFFFF) * (1.f / 32768.f) - 1.f);
        }
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const unsigned long long s0 = shader_ticks(), r0 = reference_ticks();
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[i], vb[i], acc[i], 0, 0, 0);
    float s = 0.f;
    for (int i = 0; i < 4; ++i) s += acc[i][0];
    const unsigned long long s1 = shader_ticks(), r1 = reference_ticks();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = (float)(s1 - s0);
        out[1] = (float)(r1 - r0);
    }
    if (s == 12345.f) out[2 + threadIdx.x] = s;
}

// The same with the fp32 instruction (32x32x2: 2 * 32 * 32 * 2 FLOP each).
__global__ __launch_bounds__(256) void mfma_f32_kernel(float* out, int iters, float a)
{
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a + 1.f, acc[i], 0, 0, 0);
    float s = 0.f;
    for (int i = 0; i < 4; ++i) s += acc[i][0];
    if (s == 12345.f) out[threadIdx.x] = s;
}

// Plain copy, 16 bytes per lane, grid-stride: one read and one write of every byte.
__global__ __launch_bounds__(256) void copy16_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Reads of a buffer small enough to stay in the caches: every workgroup walks the whole buffer `passes` times.
__global__ __launch_bounds__(256) void read16_kernel(const u32x4* __restrict__ src, unsigned* sink, size_t n16, int passes)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int p = 0; p < passes; ++p)
        for (size_t i = threadIdx.x; i < n16; i += blockDim.x) {
            const u32x4 v = src[i];
            acc[0] ^= v[0]; acc[1] ^= v[1]; acc[2] ^= v[2]; acc[3] ^= v[3];
        }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[threadIdx.x] = acc[0];
}

int done() { return hipGetLastError() == hipSuccess ? 0 : 1; }

}  // namespace

extern "C" {

// out: at least 1 KiB of device memory.  FLOP of the launch = 2*32*32*16 * 4 * iters * 4 waves * blocks.
int drc_mfma_bf16(float* out, int iters, int blocks, void* stream)
{
    if (!out || iters < 1 || blocks < 1) return 2;
    hipLaunchKernelGGL(mfma_bf16_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters, 1.f);
    return done();
}

// The same count of FLOP on lane-varying operands; out[0], out[1] receive the first wave's shader-clock and
// 100 MHz reference-clock ticks over the loop (out: at least 2 KiB).
int drc_mfma_bf16_data(float* out, int iters, int blocks, void* stream)
{
    if (!out || iters < 1 || blocks < 1) return 2;
    hipLaunchKernelGGL(mfma_bf16_data_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
    return done();
}

// FLOP of the launch = 2*32*32*2 * 4 * iters * 4 waves * blocks.
int drc_mfma_f32(float* out, int iters, int blocks, void* stream)
{
    if (!out || iters < 1 || blocks < 1) return 2;
    hipLaunchKernelGGL(mfma_f32_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters, 1.f);
    return done();
}

// src, dst: device buffers of `bytes` bytes (a multiple of 16, 16-byte aligned, not overlapping).
int drc_copy16(const void* src, void* dst, size_t bytes, int blocks, void* stream)
{
    if (!src || !dst || bytes % 16 || ((uintptr_t)src | (uintptr_t)dst) % 16 || blocks < 1) return 2;
    hipLaunchKernelGGL(copy16_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, bytes / 16);
    return done();
}

// src: `bytes` bytes read `passes` times by each of `blocks` workgroups; sink: at least 1 KiB.
int drc_read16(const void* src, void* sink, size_t bytes, int passes, int blocks, void* stream)
{
    if (!src || !sink || bytes % 16 || (uintptr_t)src % 16 || passes < 1 || blocks < 1) return 2;
    hipLaunchKernelGGL(read16_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (unsigned*)sink, bytes / 16, passes);
    return done();
}

}  // extern "C"
