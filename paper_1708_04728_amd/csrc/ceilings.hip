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

// Plain 16-byte stores, grid-stride: what the memory side takes when nothing is read.
__global__ __launch_bounds__(256) void fill16_kernel(u32x4* __restrict__ dst, size_t n16)
{
    const u32x4 v = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = v;
}

// One k-step of the bf16 convolution kernels' inner loop in isolation: a wave multiplies 3 blocks of 32 filters by 2 blocks
// of 32 pixels (6 matrix instructions, 192 cycles of matrix work) from operands it reads out of LDS one k-step ahead
// (5 ds_read_b128 at the kernels' swizzled addresses, data in [-1, 1)).  MODE 0: the matrix instructions alone; 1: with the
// reads; 2: with the drain of the LDS counter and the workgroup barrier the kernels have every four k-steps; 3: with, behind
// that barrier, the next 96 x 128-byte filter slice requested from global memory straight into LDS and awaited one slice
// later (a two-stage ring, as in the kernels).  Every wave writes its shader-clock ticks per k-step to out[4 block + wave].
typedef __attribute__((address_space(3))) void* lds_ptr;
__device__ __forceinline__ u32x4 lds_read16(unsigned a)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=&v"(v) : "v"(a));
    return v;
}
__device__ __forceinline__ void defined_now(u32x4& v) { asm volatile("" : "+v"(v)); }
template <int N>
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }

template <int MODE>
__global__ __launch_bounds__(256) void kstep_kernel(float* out, int iters, const unsigned short* filt)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    for (int i = threadIdx.x; i < 72 * 1024 / 4; i += 256) {
        const unsigned h = (unsigned)i * 2654435761u + blockIdx.x;
        const unsigned lo = (h & 0x8000u) | (0x3d00u + ((h >> 3) & 0x1ffu)), hi = ((h >> 16) & 0x8000u) | (0x3d00u + ((h >> 19) & 0x1ffu));
        ((unsigned*)lds)[i] = lo | (hi << 16);
    }
    __syncthreads();
    const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, l32 = lane & 31;
    const unsigned a_rd = base + l32 * 128 + ((half << 4) ^ (((l32 >> 1) & 7) << 4));
    unsigned b_rd[2];
    for (int j = 0; j < 2; ++j) {
        const int row = wave * 64 + j * 32 + l32 + 59;
        b_rd[j] = base + 24576 + row * 128 + ((half << 4) ^ (((row >> 1) & 7) << 4));
    }
    f32x16 acc[3][2];
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    u32x4 fa[2][3], fb[2][2];
    auto fetch = [&](int sl, int ks, int stage) __attribute__((always_inline)) {
        const unsigned pa = (a_rd + stage * 12288) ^ (ks * 32);
        fa[sl][0] = lds_read16(pa); fa[sl][1] = lds_read16(pa + 4096); fa[sl][2] = lds_read16(pa + 8192);
        fb[sl][0] = lds_read16(b_rd[0] ^ (ks * 32)); fb[sl][1] = lds_read16(b_rd[1] ^ (ks * 32));
    };
    auto mul = [&](int sl) __attribute__((always_inline)) {
        for (int i = 0; i < 3; ++i) defined_now(fa[sl][i]);
        for (int j = 0; j < 2; ++j) defined_now(fb[sl][j]);
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[sl][i]), __builtin_bit_cast(bf16x8, fb[sl][j]), acc[i][j], 0, 0, 0);
    };
    fetch(0, 0, 0); fetch(1, 1, 0);
    lds_wait<0>();
    const unsigned long long t0 = shader_ticks();
    for (int it = 0; it < iters; ++it) {
        const int stage = it & 1;
        if constexpr (MODE == 0) {
            mul(0); mul(1); mul(0); mul(1);
        } else {
            fetch(1, 1, stage); lds_wait<5>(); mul(0);
            fetch(0, 2, stage); lds_wait<5>(); mul(1);
            fetch(1, 3, stage); lds_wait<5>(); mul(0);
            if constexpr (MODE >= 2) {
                if constexpr (MODE == 3) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                lds_wait<0>();
                __builtin_amdgcn_s_barrier();
            }
            if constexpr (MODE == 3) {
                const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)filt, 0, 96 * 1152, 0x00020000);
                const int lrow = wave * 8 + (lane >> 3), lc = (lane & 7) ^ ((lrow >> 1) & 7);
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr)(lds + stage * 12288 + i * 4096 + wave * 1024), 16, ((i * 32 + lrow) * 576 + lc * 8) * 2, ((it + 2) % 9) * 128, 0, 0);
            }
            fetch(0, 0, stage ^ 1); lds_wait<5>(); mul(1);
        }
    }
    lds_wait<0>();
    const unsigned long long t1 = shader_ticks();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float s = 0.f;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (lane == 0) out[blockIdx.x * 4 + wave] = (float)(t1 - t0) / (4.f * (float)iters);
    if (s == 123.456f) out[0] = s;
}

template <int MODE>
int launch_kstep(float* out, int iters, int blocks, const void* filt, hipStream_t st)
{
    if (hipFuncSetAttribute((const void*)kstep_kernel<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, 72 * 1024) != hipSuccess) return 1;
    hipLaunchKernelGGL(kstep_kernel<MODE>, dim3(blocks), dim3(256), 72 * 1024, st, out, iters, (const unsigned short*)filt);
    return hipGetLastError() == hipSuccess ? 0 : 1;
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

// dst: `bytes` bytes (a multiple of 16, 16-byte aligned).
int drc_fill16(void* dst, size_t bytes, int blocks, void* stream)
{
    if (!dst || bytes % 16 || (uintptr_t)dst % 16 || blocks < 1) return 2;
    hipLaunchKernelGGL(fill16_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst, bytes / 16);
    return done();
}

// One k-step in isolation (see kstep_kernel).  out: 4 * blocks floats (ticks per k-step of every wave); filt: at least
// 96 * 1152 + 4096 bytes of device memory (mode 3 reads it; any contents).  Each workgroup takes 72 KiB of LDS, so at most
// two share a compute unit.
int drc_kstep(int mode, float* out, int iters, int blocks, const void* filt, void* stream)
{
    if (!out || !filt || iters < 1 || blocks < 1 || mode < 0 || mode > 3) return 2;
    hipStream_t st = (hipStream_t)stream;
    return mode == 0 ? launch_kstep<0>(out, iters, blocks, filt, st) : mode == 1 ? launch_kstep<1>(out, iters, blocks, filt, st)
         : mode == 2 ? launch_kstep<2>(out, iters, blocks, filt, st) : launch_kstep<3>(out, iters, blocks, filt, st);
}

}  // extern "C"
