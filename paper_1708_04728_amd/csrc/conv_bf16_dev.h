// Device helpers shared by the bf16 convolution kernels that stream their operands into LDS with buffer loads:
// vector types, the out-of-range offset, the hand-made barrier and counter waits, loads that write LDS, LDS reads the
// compiler does not see, and small exact divisions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "dr_store.h"

namespace dr {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;
template <int V> using IC = std::integral_constant<int, V>;

constexpr int OOB = (int)0x80000000;

// Workgroup barrier between the slices.  A fence would make the compiler wait for every outstanding
// load that writes LDS (vmcnt(0)), which is exactly the prefetch this kernel keeps in flight, so the
// ordering is spelled out instead: the compiler may not move memory accesses across either side
// (the empty asm statements), this wave's own LDS reads have returned (lgkmcnt(0)), and the arrival of
// the operand loads is awaited by the caller with wait_vmcnt.
__device__ __forceinline__ void ring_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0); vmcnt and expcnt left at their maxima
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// One 16-byte buffer load per lane that writes LDS directly: lane l of the wave fills bytes
// [16 l, 16 l + 16) of the 1 KiB block at `lds` (wave-uniform); lanes whose voff lies outside the
// descriptor's range write zeros.  (Only the device pass may see the builtin: in the host pass it
// fails to type-check without a diagnostic and takes the kernel's launch stub with it.)
__device__ __forceinline__ void load_to_lds16(__amdgpu_buffer_rsrc_t r, unsigned char* lds, int voff, int soff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr)lds, 16, voff, soff, 0, 0);
#endif
}

// The same with 4 bytes per lane: lane l fills bytes [4 l, 4 l + 4) of the 256-byte block at `lds`.
__device__ __forceinline__ void load_to_lds4(__amdgpu_buffer_rsrc_t r, void* lds, int voff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr)lds, 4, voff, 0, 0, 0);
#endif
}

// LDS reads the compiler does not see (see the header): the data is valid after wait_lgkm + touch.
template <int OFF>
__device__ __forceinline__ u32x4 ds_read16(unsigned addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
__device__ __forceinline__ void wait_lgkm()
{
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void touch(u32x4& v) { asm volatile("" : "+v"(v)); }

// v / d for 0 <= v < 2^24 and 1 <= d <= 2^16, exact: (v * ceil(2^40 / d)) >> 40.  With m = (2^40 + e) / d,
// 0 <= e < d, the product is v / d + v e / (d 2^40) and the second term is below 2^-16 <= 1 / d.
__device__ __forceinline__ int div_small(int v, unsigned long long m)
{
    return (int)(((unsigned long long)(unsigned)v * m) >> 40);
}

// The persistent walk of the convolution kernels.  A launch has gn workgroups per filter block (grid of gn grid_m) and
// `tiles` pixel tiles per filter block.  Workgroup ids are dealt to the 8 dies in turn (id & 7); the renumbering b gives
// each die a contiguous range, so that the grid_m workgroups of one pixel tile (b / grid_m the same) and its neighbours share
// an L2.  Workgroup b keeps filter block b % grid_m and visits tiles nt0, nt0 + gn, ... for the tiles / gn whole rounds.
// The tiles left over (fewer than gn) go to the workgroups with the LOWEST ids among those of the same filter block: ids
// are handed out across dies and, within a die, across compute units before a unit gets its second workgroup, so the
// left-over round lands on as many different units of all dies as it has tiles -- not on the first dies' units only, which
// is what "tile nt0 + rounds gn if it exists" does and which makes the launch as long as if the round were full.
// (the host fills WalkArgs: the division by grid_m runs as a multiplication by magic_gm = ceil(2^32 / grid_m), exact for the
// workgroup counts of a launch, far below 2^16)
struct WalkArgs {
    int grid_m, gn, full, rem;            // filter blocks; workgroups per filter block; whole rounds tiles / gn; tiles left over
    unsigned magic_gm;
};
inline WalkArgs make_walk(int grid_m, int gn, int tiles)
{
    WalkArgs w;
    w.grid_m = grid_m; w.gn = gn; w.full = tiles / gn; w.rem = tiles - w.full * gn;
    w.magic_gm = grid_m > 1 ? (unsigned)((0x100000000ull + (unsigned)grid_m - 1) / (unsigned)grid_m) : 0u;
    return w;
}
struct TileWalk {
    int mt, nt0, gn, full, last, count;   // filter block; first tile; stride; whole rounds; the left-over tile; tiles of this workgroup
    __device__ __forceinline__ int tile(int t) const { return t < full ? nt0 + t * gn : last; }
};
__device__ __forceinline__ TileWalk tile_walk(const WalkArgs& k)
{
    const int G = k.gn * k.grid_m, die = (int)(blockIdx.x & 7), s = (int)(blockIdx.x >> 3), per = G >> 3, odd = G & 7;
    const int bid = die * per + min(die, odd) + s;
    TileWalk w;
    w.gn = k.gn; w.full = k.full;
    int u;                                              // workgroups of the same filter block with a lower id
    if (k.grid_m == 1) {
        w.mt = 0; w.nt0 = bid; u = (int)blockIdx.x;
    } else {
        w.nt0 = (int)__umulhi((unsigned)bid, k.magic_gm);
        w.mt = bid - w.nt0 * k.grid_m;
        u = 0;
        if (k.rem) {
            for (int x = 0; x < 8; ++x) {
                // die x holds ids x, x + 8, ...: renumbered first + s' for s' < len; those below this id: s' < s, and s' = s when x < die
                const int first = x * per + min(x, odd), len = per + (x < odd ? 1 : 0);
                const int L = min(len, s + (x < die ? 1 : 0));
                int r = w.mt - (first - (int)__umulhi((unsigned)first, k.magic_gm) * k.grid_m);   // the s' with (first + s') % grid_m == mt are r, r + grid_m, ...
                if (r < 0) r += k.grid_m;
                u += L > r ? (int)__umulhi((unsigned)(L - 1 - r), k.magic_gm) + 1 : 0;
            }
        }
    }
    w.last = k.full * k.gn + u;
    w.count = k.full + (u < k.rem ? 1 : 0);
    return w;
}

// bits lo..hi set (hi < lo: none); lo, hi in 0..15
__device__ __forceinline__ unsigned bit_range(int lo, int hi) { return hi >= lo ? (2u << hi) - (1u << lo) : 0u; }

// Bias + ReLU + bf16 store of a wave's TM x TN blocks of 32 filters x 32 pixels held in the matrix instruction's result
// layout (lane = pixel l32 of the block and half h; register v = filter 8 (v / 4) + 4 h + v % 4 of the block).  Two lanes
// that hold the same pixel exchange halves so that each ends up with 8 consecutive filters, 16 bytes of the pixel's
// channel run.  bias_rd: LDS address of the filter block's biases (128 floats) plus 32 h bytes; m_lane: first filter
// of the workgroup's block plus 8 h; nbase[j]: byte offset of the pixel's first channel written; n_ok[j]: the pixel
// exists.  Every lane issues all 2 TM TN stores (those without a destination with an offset outside the buffer), so the
// memory counter holds an exact number of them afterwards.
template <int TM, int TN>
__device__ __forceinline__ void store_blocks(const f32x16 (&acc)[TM][TN], unsigned bias_rd, int m_lane, int K, int relu,
                                             __amdgpu_buffer_rsrc_t ry, const int (&nbase)[TN], const bool (&n_ok)[TN])
{
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        u32x4 bv[2][2];
        bv[0][0] = ds_read16<0>(bias_rd + i * 128);
        bv[0][1] = ds_read16<16>(bias_rd + i * 128);
        bv[1][0] = ds_read16<64>(bias_rd + i * 128);
        bv[1][1] = ds_read16<80>(bias_rd + i * 128);
        wait_lgkm<0>();
        touch(bv[0][0]); touch(bv[0][1]); touch(bv[1][0]); touch(bv[1][1]);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][qp * 8 + e]),
                                                                     __float_as_uint(acc[i][j][qp * 8 + 4 + e]), false, false);
                    o[e] = __uint_as_float(sw[0]);
                    o[4 + e] = __uint_as_float(sw[1]);
                }
                const int mb = m_lane + i * 32 + qp * 16;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += __uint_as_float(bv[qp][e >> 2][e & 3]);
                if (relu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = fmaxf(o[e], 0.f);
                }
                u32x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
                const int voff = (n_ok[j] && mb < K) ? nbase[j] + mb * 2 : OOB;
#if defined(__HIP_DEVICE_COMPILE__)
                __builtin_amdgcn_raw_buffer_store_b128(pk, ry, voff, 0, 0);
#endif
            }
        }
    }
}

// The first half of store_blocks without the store: bias + ReLU + bf16 pack of a wave's TM x TN blocks, returned as
// hk[j][2 i + qp] = the 8 consecutive filters 32 i + 16 qp + 8 h .. of pixel l32 of pixel block j.  That is the layout of
// the matrix instruction's SECOND operand for a contraction over those filters (k-step 2 i + qp holds filters
// 16 (2 i + qp) .. + 15, a lane of half h the 8 from 8 h on, for the pixel of its column): a 1x1 convolution on the
// layer's output can multiply straight from these registers.
template <int TM, int TN>
__device__ __forceinline__ void pack_blocks(const f32x16 (&acc)[TM][TN], unsigned bias_rd, int relu, u32x4 (&hk)[TN][2 * TM])
{
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        u32x4 bv[2][2];
        bv[0][0] = ds_read16<0>(bias_rd + i * 128);
        bv[0][1] = ds_read16<16>(bias_rd + i * 128);
        bv[1][0] = ds_read16<64>(bias_rd + i * 128);
        bv[1][1] = ds_read16<80>(bias_rd + i * 128);
        wait_lgkm<0>();
        touch(bv[0][0]); touch(bv[0][1]); touch(bv[1][0]); touch(bv[1][1]);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][qp * 8 + e]),
                                                                     __float_as_uint(acc[i][j][qp * 8 + 4 + e]), false, false);
                    o[e] = __uint_as_float(sw[0]);
                    o[4 + e] = __uint_as_float(sw[1]);
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += __uint_as_float(bv[qp][e >> 2][e & 3]);
                if (relu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = fmaxf(o[e], 0.f);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) hk[j][2 * i + qp][e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
            }
        }
    }
}

}  // namespace
}  // namespace dr
