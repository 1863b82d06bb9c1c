// bf16 convolution forward (Eq. (7): Y_j = (W * X)_j + B_j): bf16 storage, fp32 accumulation on the
// gfx950 matrix cores, channels-last (NHWC) activations and KRSC filters.
//
//   D[m][n] = sum_k A[m][k] * B[k][n]     m = output channel, n = (image, p, q), k = (r, s, c)
//
// v_mfma_f32_32x32x16_bf16 wants, per lane, 8 consecutive k of one row of A and of one column of B.
// With the channel index innermost in memory for both the filters (KRSC) and the activations
// (NHWC), 8 consecutive k of one tap are 16 contiguous bytes: every global load is a 16-byte buffer
// load that lands in LDS unchanged, and every MFMA operand is one 16-byte LDS read.  (In NCHW the
// contraction index is strided by H*W elements and each operand would need a transpose.)
//
// A workgroup (256 threads, 4 wave64) owns a BM x BN tile and walks k tap by tap, BK channels per
// slice; the slice position only moves a wave-uniform scalar offset (the buffer instructions' scalar
// operand), the zero-padding test is redone once per tap, and a ragged channel tail is masked by
// pushing the lane's offset out of the buffer.  Register prefetch one slice ahead, double-buffered
// LDS, one LDS-only barrier per slice.  Vector-ALU work does not overlap with MFMA on this GPU, so
// the loop is kept free of address arithmetic.  The store adds bias (+ residual), applies ReLU,
// rounds to bf16 (nearest even) and writes 4 consecutive output channels (8 bytes) per lane.
//
// Shapes the fast kernel cannot take (C not a multiple of 8: the 3-channel network input) run in a
// plain gather kernel at the end of this file.
#include <type_traits>

#include "dr_internal.h"

namespace dr {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int NT = 256;

struct KArgs {
    const uint16_t* x;
    const uint16_t* w;
    const float* bias;
    const uint16_t* res;
    uint16_t* y;
    ConvGeom g;
    int grid_m, grid_n;
    int x_bytes, w_bytes;
    unsigned magic_rs, magic_s, magic_c;   // ceil(2^32 / d) for d = R*S, S, C (gather mode: k < 65536)
};

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float bf16_to_f32(uint32_t u16) { return __uint_as_float(u16 << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// GATHER = false: the fast path described above (KRSC filters, C % 8 == 0).
// GATHER = true:  any C and either filter order; k runs in the filters' own memory order, every
//                 operand element is fetched by its own 2-byte buffer load after decoding (c, r, s),
//                 eight of them are packed into the 16-byte LDS chunk.  Meant for the 3-channel
//                 network input, where Kg = 147 is a handful of slices.
template <int BM, int BN, int WGM, int WGN, int BK, bool GATHER>
__global__ __launch_bounds__(NT) void conv_bf16_nhwc_kernel(const KArgs a)
{
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CH = BK / 8;                    // 16-byte chunks per row of a slice
    constexpr int LDT = BK + 8;                   // padded LDS row (bf16 elements)
    static_assert(WGM * WGN == 4 && TM >= 1 && TN >= 1, "bad tiling");
    static_assert(BK % 16 == 0, "BK");
    constexpr int A_CH = BM * CH, B_CH = BN * CH;
    constexpr int A_PER = (A_CH + NT - 1) / NT, B_PER = (B_CH + NT - 1) / NT;

    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDT];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDT];

    const ConvGeom& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int half = lane >> 5, l32 = lane & 31;

    int bid = blockIdx.x;
    const int nblk = a.grid_m * a.grid_n;
    if (nblk % 8 == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);   // contiguous tile range per XCD
    const int m0 = (bid % a.grid_m) * BM;
    const int n0 = (bid / a.grid_m) * BN;
    const int PQ = g.P * g.Q;

    constexpr int OOB = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, a.w_bytes, 0x00020000);

    // ---- per-lane constants: which row / chunk of the A and B slices this lane moves
    int va[A_PER], a_c8[A_PER];        // byte offset of (row, chunk) in the filter tensor; first channel of the chunk
    int b_ih0[B_PER], b_iw0[B_PER], b_base[B_PER], b_c8[B_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int f = tid + i * NT;
        const int gm = m0 + f / CH;
        a_c8[i] = (f % CH) * 8;
        va[i] = ((A_CH % NT == 0 || f < A_CH) && gm < g.K) ? (gm * g.Kg + a_c8[i]) * 2 : OOB;
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
        const int f = tid + i * NT;
        const int ng = n0 + f / CH;
        b_c8[i] = (f % CH) * 8;
        b_ih0[i] = b_iw0[i] = -(1 << 30);
        b_base[i] = 0;
        if ((B_CH % NT == 0 || f < B_CH) && ng < g.Ng) {
            const int img = ng / PQ, pix = ng - img * PQ;
            const int p = pix / g.Q, q = pix - p * g.Q;
            b_ih0[i] = p * g.sh - g.ph;
            b_iw0[i] = q * g.sw - g.pw;
            b_base[i] = (((img * g.H + b_ih0[i]) * g.W + b_iw0[i]) * g.C + b_c8[i]) * 2;
        }
    }

    u32x4 ra[A_PER], rb[B_PER];
    int ld_c0 = 0, ld_r = 0, ld_s = 0;          // wave-uniform position of the next slice to load
    int vb[B_PER];                               // per-lane offsets of the current tap (OOB when padded away)
    auto tap_offsets = [&]() {
        // the tap's own offset goes into the per-lane part: the hardware range-checks the per-lane
        // offset alone, and b_base may be negative while the tap is in the padding
        const int tap_off = (ld_r * g.W + ld_s) * g.C * 2;
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const bool ok = (unsigned)(b_ih0[i] + ld_r) < (unsigned)g.H && (unsigned)(b_iw0[i] + ld_s) < (unsigned)g.W;
            vb[i] = ok ? b_base[i] + tap_off : OOB;
        }
    };
    const bool ragged_c = (g.C % BK) != 0;
    int ld_k0 = 0;                               // gather mode: first k of the next slice
    auto load_u16 = [&](__amdgpu_buffer_rsrc_t r, int off) -> unsigned {
        return (unsigned)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
    };
    auto divm = [](int v, int d, unsigned magic) { return d == 1 ? v : (int)__umulhi((unsigned)v, magic); };
    auto load_slice = [&]() {
        if constexpr (GATHER) {
            const int RS = g.R * g.S;
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                unsigned e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = ld_k0 + a_c8[i] + j;
                    e[j] = load_u16(rw, (k < g.Kg && va[i] != OOB) ? va[i] + (ld_k0 + j) * 2 : OOB);
                }
                ra[i] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                // decode the chunk's first k in the filters' order, then step element by element
                const int k = ld_k0 + b_c8[i];
                int c, r, sx;
                if (g.w_krsc) {
                    const int t = divm(k, g.C, a.magic_c);                   // k / C
                    c = k - t * g.C;
                    r = divm(t, g.S, a.magic_s);
                    sx = t - r * g.S;
                } else {
                    c = divm(k, RS, a.magic_rs);                             // k / (R*S)
                    const int t = k - c * RS;
                    r = divm(t, g.S, a.magic_s);
                    sx = t - r * g.S;
                }
                unsigned e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool ok = k + j < g.Kg && (unsigned)(b_ih0[i] + r) < (unsigned)g.H && (unsigned)(b_iw0[i] + sx) < (unsigned)g.W;
                    // b_base holds the offset of x[img][ih0][iw0][chunk's first channel]; remove that channel again
                    e[j] = load_u16(rx, ok ? b_base[i] - b_c8[i] * 2 + ((r * g.W + sx) * g.C + c) * 2 : OOB);
                    if (g.w_krsc) { if (++c == g.C) { c = 0; if (++sx == g.S) { sx = 0; ++r; } } }
                    else { if (++sx == g.S) { sx = 0; if (++r == g.R) { r = 0; ++c; } } }
                }
                rb[i] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
            ld_k0 += BK;
            return;
        }
        if (ld_c0 == 0) tap_offsets();
        const int tap = ld_r * g.S + ld_s;
        const int sa = (tap * g.C + ld_c0) * 2;
        const int sb = ld_c0 * 2;
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int off = (ragged_c && ld_c0 + a_c8[i] >= g.C) ? OOB : va[i];
            ra[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, off, sa, 0));
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int off = (ragged_c && ld_c0 + b_c8[i] >= g.C) ? OOB : vb[i];
            rb[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, off, sb, 0));
        }
        ld_c0 += BK;
        if (ld_c0 >= g.C) { ld_c0 = 0; if (++ld_s == g.S) { ld_s = 0; ++ld_r; } }
    };
    auto store_slice = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int f = tid + i * NT;
            if (A_CH % NT == 0 || f < A_CH) *reinterpret_cast<u32x4*>(&As[buf][(f / CH) * LDT + (f % CH) * 8]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int f = tid + i * NT;
            if (B_CH % NT == 0 || f < B_CH) *reinterpret_cast<u32x4*>(&Bs[buf][(f / CH) * LDT + (f % CH) * 8]) = rb[i];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nslices = GATHER ? (g.Kg + BK - 1) / BK : g.R * g.S * ((g.C + BK - 1) / BK);
    load_slice();
    store_slice(0);
    if (1 < nslices) load_slice();
    lds_barrier();

    for (int it = 0; it < nslices; ++it) {
        const int buf = it & 1;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm * WM + i * 32 + l32) * LDT + ks * 16 + half * 8]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(wn * WN + j * 32 + l32) * LDT + ks * 16 + half * 8]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (it + 1 < nslices) {
            store_slice(buf ^ 1);
            if (it + 2 < nslices) load_slice();
        }
        lds_barrier();
    }

    // ---- store.  Register v of a 32x32 tile: row 8*(v/4) + 4*half + v%4, column l32; a lane therefore
    // owns 4 consecutive output channels of one pixel per group of 4 registers.
    const bool vec_ok = ((g.y_ctot | g.y_coff) & 3) == 0 && (g.res_ctot & 3) == 0;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + l32;
        if (n >= g.Ng) continue;
        uint16_t* yb = a.y + (size_t)n * g.y_ctot + g.y_coff;
        const uint16_t* rbp = a.res ? a.res + (size_t)n * g.res_ctot : nullptr;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int mb = m0 + wm * WM + i * 32 + q4 * 8 + half * 4;
                if (mb >= g.K) continue;
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = acc[i][j][q4 * 4 + e];
                if (vec_ok && mb + 3 < g.K) {
                    if (a.bias) {
                        const f32x4 bv = *reinterpret_cast<const f32x4*>(a.bias + mb);
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] += bv[e];
                    }
                    if (rbp) {
                        const u32x2 rv = *reinterpret_cast<const u32x2*>(rbp + mb);
                        o[0] += bf16_to_f32(rv.x & 0xFFFFu); o[1] += __uint_as_float(rv.x & 0xFFFF0000u);
                        o[2] += bf16_to_f32(rv.y & 0xFFFFu); o[3] += __uint_as_float(rv.y & 0xFFFF0000u);
                    }
                    if (g.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = fmaxf(o[e], 0.f);
                    }
                    u32x2 pk;
                    pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
                    pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
                    *reinterpret_cast<u32x2*>(yb + mb) = pk;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int m = mb + e;
                        if (m < g.K) {
                            float v = o[e] + (a.bias ? a.bias[m] : 0.f);
                            if (rbp) v += bf16_to_f32(rbp[m]);
                            if (g.relu) v = fmaxf(v, 0.f);
                            yb[m] = (uint16_t)f32_to_bf16(v);
                        }
                    }
                }
            }
    }
}

// ---- any shape, either activation layout, KCRS filters: one output element per thread -------------
// Used where the matrix-core kernel does not apply (3 input channels).  x strides are passed in
// elements so that NCHW and NHWC share the code.
struct GArgs {
    const uint16_t* x;
    const uint16_t* w;
    const float* bias;
    const uint16_t* res;
    uint16_t* y;
    ConvGeom g;
    long xs_n, xs_c, xs_h, xs_w;     // input strides
    long ys_n, ys_c, ys_p, ys_q;     // output strides
    long rs_n, rs_c, rs_p, rs_q;     // residual strides
    int w_krsc;
};

__global__ __launch_bounds__(256) void conv_bf16_gather_kernel(const GArgs a)
{
    const ConvGeom& g = a.g;
    const long total = (long)g.Ng * g.K;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        // lanes along the output channel for NHWC stores; (n, m) decode is layout independent
        const int m = (int)(i % g.K);
        const int n = (int)(i / g.K);
        const int img = n / (g.P * g.Q), pix = n - img * (g.P * g.Q);
        const int p = pix / g.Q, q = pix - p * g.Q;
        float acc = a.bias ? a.bias[m] : 0.f;
        for (int c = 0; c < g.C; ++c)
            for (int r = 0; r < g.R; ++r) {
                const int ih = p * g.sh + r - g.ph;
                if ((unsigned)ih >= (unsigned)g.H) continue;
                for (int s = 0; s < g.S; ++s) {
                    const int iw = q * g.sw + s - g.pw;
                    if ((unsigned)iw >= (unsigned)g.W) continue;
                    const long wi = a.w_krsc ? (((long)m * g.R + r) * g.S + s) * g.C + c : (((long)m * g.C + c) * g.R + r) * g.S + s;
                    acc = fmaf(bf16_to_f32(a.w[wi]), bf16_to_f32(a.x[img * a.xs_n + c * a.xs_c + ih * a.xs_h + iw * a.xs_w]), acc);
                }
            }
        if (a.res) acc += bf16_to_f32(a.res[img * a.rs_n + m * a.rs_c + p * a.rs_p + q * a.rs_q]);
        if (g.relu) acc = fmaxf(acc, 0.f);
        a.y[img * a.ys_n + (g.y_coff + m) * a.ys_c + p * a.ys_p + q * a.ys_q] = (uint16_t)f32_to_bf16(acc);
    }
}

template <int BM, int BN, int WGM, int WGN, int BK, bool GATHER = false>
int launch_tile(const KArgs& base, hipStream_t st)
{
    KArgs a = base;
    a.grid_m = (a.g.K + BM - 1) / BM;
    a.grid_n = (a.g.Ng + BN - 1) / BN;
    hipLaunchKernelGGL((conv_bf16_nhwc_kernel<BM, BN, WGM, WGN, BK, GATHER>), dim3((unsigned)(a.grid_m * a.grid_n)), dim3(NT), 0, st, a);
    return check_launch("conv_bf16");
}

}  // namespace

int launch_conv_bf16(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias,
                     const uint16_t* residual, uint16_t* y, hipStream_t st)
{
    TraceScope trace("conv_bf16", &g, g.Ng, st);
    // several taps at stride 1 on few channels: the input patch of a tile is loaded once for all taps (conv_bf16_patch.hip)
    if (!residual && conv_bf16_patch_eligible(g, x, w, y)) return launch_conv_bf16_patch(g, x, w, bias, y, st);
    if (!residual && conv_bf16_rows_eligible(g, x, w, y)) return launch_conv_bf16_rows(g, x, w, bias, y, st);
    if (conv_bf16_dma_eligible(g, x, w)) return launch_conv_bf16_dma(g, x, w, bias, residual, y, st);
    const size_t xb = (size_t)g.N * g.C * g.H * g.W * 2, wb = (size_t)g.K * g.Kg * 2;
    if (g.nhwc && g.w_krsc && g.C % 8 == 0 && xb < (1ull << 31) && wb < (1ull << 31)) {
        KArgs a;
        a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.g = g;
        a.grid_m = a.grid_n = 0;
        a.x_bytes = (int)xb; a.w_bytes = (int)wb;
        a.magic_rs = a.magic_s = a.magic_c = 0;
        const bool deep = g.C % 64 == 0 || g.C > 64;
        if (g.K <= 32) return deep ? launch_tile<32, 128, 1, 4, 64>(a, st) : launch_tile<32, 128, 1, 4, 32>(a, st);
        if (g.K <= 64 || (g.K + 63) / 64 * 64 < (g.K + 127) / 128 * 128)
            return deep ? launch_tile<64, 128, 2, 2, 64>(a, st) : launch_tile<64, 128, 2, 2, 32>(a, st);
        return deep ? launch_tile<128, 128, 2, 2, 64>(a, st) : launch_tile<128, 128, 2, 2, 32>(a, st);
    }
    if (g.nhwc && g.Kg < 65536 && xb < (1ull << 31) && wb < (1ull << 31)) {
        KArgs a;
        a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.g = g;
        a.grid_m = a.grid_n = 0;
        a.x_bytes = (int)xb; a.w_bytes = (int)wb;
        auto magic = [](int d) { return (unsigned)((0x100000000ull + d - 1) / d); };
        a.magic_rs = magic(g.R * g.S); a.magic_s = magic(g.S); a.magic_c = magic(g.C);
        return g.K <= 32 ? launch_tile<32, 128, 1, 4, 32, true>(a, st) : launch_tile<64, 128, 2, 2, 32, true>(a, st);
    }
    GArgs a;
    a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.g = g; a.w_krsc = g.w_krsc;
    const long PQ = (long)g.P * g.Q, HW = (long)g.H * g.W;
    if (g.nhwc) {
        a.xs_n = HW * g.C; a.xs_c = 1; a.xs_h = (long)g.W * g.C; a.xs_w = g.C;
        a.ys_n = PQ * g.y_ctot; a.ys_c = 1; a.ys_p = (long)g.Q * g.y_ctot; a.ys_q = g.y_ctot;
        a.rs_n = PQ * g.res_ctot; a.rs_c = 1; a.rs_p = (long)g.Q * g.res_ctot; a.rs_q = g.res_ctot;
    } else {
        a.xs_n = HW * g.C; a.xs_c = HW; a.xs_h = g.W; a.xs_w = 1;
        a.ys_n = PQ * g.y_ctot; a.ys_c = PQ; a.ys_p = g.Q; a.ys_q = 1;
        a.rs_n = PQ * g.res_ctot; a.rs_c = PQ; a.rs_p = g.Q; a.rs_q = 1;
    }
    const long total = (long)g.Ng * g.K;
    const unsigned grid = (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
    hipLaunchKernelGGL(conv_bf16_gather_kernel, dim3(grid), dim3(256), 0, st, a);
    return check_launch("conv_bf16_gather");
}

}  // namespace dr
