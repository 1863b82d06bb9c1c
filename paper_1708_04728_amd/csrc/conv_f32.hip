// fp32 convolution forward (Eq. (7): Y_j = (W * X)_j + B_j) as an implicit GEMM on the gfx950
// matrix cores.
//
//   D[m][n] = sum_k A[m][k] * B[k][n]     m = output channel        (M  = K filters)
//                                         n = (image, p, q)         (Ng = N*P*Q)
//                                         k = (c, r, s)             (Kg = C*R*S)
//   A = the KCRS weight tensor viewed as an M x Kg row-major matrix (no copy),
//   B = the im2col matrix, never materialised: each element is gathered from NCHW x on the fly.
//
// A workgroup of 256 threads (4 wave64) owns a BM x BN tile of D and walks Kg in slices of
// BK = 16.  Both operand slices are staged in LDS with the GEMM-k index contiguous per row
// (rows padded to 20 floats so that 128-bit LDS accesses of consecutive rows fall in distinct
// banks).  v_mfma_f32_32x32x2_f32 consumes two k per instruction, one from lanes 0-31 and one
// from lanes 32-63; the kernel gives lane half g the slice's k in [8g, 8g+8) so that every lane
// fetches its eight A (or B) values of a slice with two 128-bit LDS reads.  Global loads for slice
// i+1 are issued before the MFMAs of slice i (register prefetch, two LDS buffers, one barrier per
// slice).  With lanes running along n, both the gather from x and the store to NCHW y are
// coalesced.  Bias, the optional residual sum and ReLU are applied in the store.
#include "dr_internal.h"

namespace dr {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;        // k per LDS slice
constexpr int LDT = BK + 4;   // padded row length (floats) of both LDS tiles
constexpr int NT = 256;       // threads per workgroup

struct KArgs {
    const float* x;
    const float* w;
    const float* bias;
    const float* res;
    float* y;
    ConvGeom g;
    int grid_m, grid_n;
};

// FR, FS: compile-time filter size (0 = taken from the geometry at run time).
template <int BM, int BN, int WGM, int WGN, int FR, int FS>
__global__ __launch_bounds__(NT) void conv_f32_kernel(const KArgs a)
{
    constexpr int WM = BM / WGM, WN = BN / WGN;   // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA tiles per wave
    static_assert(WGM * WGN == 4 && TM >= 1 && TN >= 1, "bad tiling");
    constexpr int A_F4 = BM * (BK / 4);           // float4 groups in an A slice
    constexpr int B_F4 = BN * (BK / 4);
    constexpr int A_PER = (A_F4 + NT - 1) / NT;
    constexpr int B_PER = B_F4 / NT;
    static_assert(B_F4 % NT == 0, "BN must be a multiple of 64");

    __shared__ __attribute__((aligned(16))) float As[2][BM * LDT];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * LDT];

    const ConvGeom& g = a.g;
    const int R = FR ? FR : g.R, S = FS ? FS : g.S;
    const int RS = R * S;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int half = lane >> 5, l32 = lane & 31;

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs; the remap
    // gives each XCD a contiguous range of tiles (m fastest), so the tiles that share an input
    // region share an L2.
    int bid = blockIdx.x;
    const int nblk = a.grid_m * a.grid_n;
    if (nblk % 8 == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int m0 = (bid % a.grid_m) * BM;
    const int n0 = (bid / a.grid_m) * BN;

    const int HW = g.H * g.W, PQ = g.P * g.Q;

    // ---- per-thread gather state for B: one fixed n, B_PER groups of 4 consecutive k per slice
    const int bn = tid % BN;
    const int bkq0 = tid / BN;                   // first k-group; next ones at +NT/BN
    constexpr int BKQ_STEP = NT / BN;
    const int ng = n0 + bn;
    const bool n_ok = ng < g.Ng;
    int ih0 = 0, iw0 = 0;
    const float* xb = a.x;
    if (n_ok) {
        const int img = ng / PQ, pix = ng - img * PQ;
        const int p = pix / g.Q, q = pix - p * g.Q;
        ih0 = p * g.sh - g.ph;
        iw0 = q * g.sw - g.pw;
        xb = a.x + (size_t)img * g.C * HW;
    }
    const bool vecA = (g.Kg & 3) == 0;

    f32x4 ra[A_PER], rb[B_PER];

    auto load_slice = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int f = tid + i * NT;
            const int m = f >> 2, kq = f & 3;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            const int gm = m0 + m, gk = k0 + kq * 4;
            if ((A_F4 % NT == 0 || f < A_F4) && gm < g.K) {
                const float* src = a.w + (size_t)gm * g.Kg + gk;
                if (vecA) {
                    if (gk < g.Kg) v = *reinterpret_cast<const f32x4*>(src);
                } else {
                    if (gk + 0 < g.Kg) v.x = src[0];
                    if (gk + 1 < g.Kg) v.y = src[1];
                    if (gk + 2 < g.Kg) v.z = src[2];
                    if (gk + 3 < g.Kg) v.w = src[3];
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int gk = k0 + (bkq0 + i * BKQ_STEP) * 4;
            int c = gk / RS;
            int rs = gk - c * RS;
            int r = rs / S;
            int s = rs - r * S;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ih = ih0 + r, iw = iw0 + s;
                const bool ok = n_ok && (gk + j < g.Kg) && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
                v[j] = ok ? xb[(size_t)c * HW + ih * g.W + iw] : 0.f;
                if (++s == S) { s = 0; if (++r == R) { r = 0; ++c; } }
            }
            rb[i] = f32x4{v[0], v[1], v[2], v[3]};
        }
    };

    auto store_slice = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int f = tid + i * NT;
            if (A_F4 % NT == 0 || f < A_F4)
                *reinterpret_cast<f32x4*>(&As[buf][(f >> 2) * LDT + (f & 3) * 4]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i)
            *reinterpret_cast<f32x4*>(&Bs[buf][bn * LDT + (bkq0 + i * BKQ_STEP) * 4]) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nslices = (g.Kg + BK - 1) / BK;
    load_slice(0);
    store_slice(0);
    __syncthreads();

    for (int it = 0; it < nslices; ++it) {
        const int buf = it & 1;
        if (it + 1 < nslices) load_slice((it + 1) * BK);

        f32x4 fa[TM][2], fb[TN][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float* p = &As[buf][(wm * WM + i * 32 + l32) * LDT + half * 8];
            fa[i][0] = *reinterpret_cast<const f32x4*>(p);
            fa[i][1] = *reinterpret_cast<const f32x4*>(p + 4);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const float* p = &Bs[buf][(wn * WN + j * 32 + l32) * LDT + half * 8];
            fb[j][0] = *reinterpret_cast<const f32x4*>(p);
            fb[j][1] = *reinterpret_cast<const f32x4*>(p + 4);
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][kk >> 2][kk & 3], fb[j][kk >> 2][kk & 3],
                                                                     acc[i][j], 0, 0, 0);

        if (it + 1 < nslices) store_slice(buf ^ 1);
        __syncthreads();
    }

    // ---- store: accumulator register v of a 32x32 tile holds row 8*(v/4) + 4*half + v%4, column l32
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + l32;
        if (n >= g.Ng) continue;
        const int img = n / PQ, pix = n - img * PQ;
        float* yb = a.y + ((size_t)img * g.y_ctot + g.y_coff) * PQ + pix;
        const float* rbase = a.res ? a.res + (size_t)img * g.res_ctot * PQ + pix : nullptr;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                if (m < g.K) {
                    float o = acc[i][j][v] + (a.bias ? a.bias[m] : 0.f);
                    if (rbase) o += rbase[(size_t)m * PQ];
                    if (g.relu) o = fmaxf(o, 0.f);
                    yb[(size_t)m * PQ] = o;
                }
            }
    }
}

template <int BM, int BN, int WGM, int WGN>
int launch_tile(const KArgs& base, hipStream_t st)
{
    KArgs a = base;
    a.grid_m = (a.g.K + BM - 1) / BM;
    a.grid_n = (a.g.Ng + BN - 1) / BN;
    const dim3 grid((unsigned)(a.grid_m * a.grid_n)), block(NT);
    const int R = a.g.R, S = a.g.S;
#define DR_LAUNCH(FR, FS) hipLaunchKernelGGL((conv_f32_kernel<BM, BN, WGM, WGN, FR, FS>), grid, block, 0, st, a)
    if (R == 1 && S == 1) DR_LAUNCH(1, 1);
    else if (R == 3 && S == 3) DR_LAUNCH(3, 3);
    else if (R == 5 && S == 5) DR_LAUNCH(5, 5);
    else if (R == 7 && S == 7) DR_LAUNCH(7, 7);
    else if (R == 11 && S == 11) DR_LAUNCH(11, 11);
    else DR_LAUNCH(0, 0);
#undef DR_LAUNCH
    return check_launch("conv_f32");
}

}  // namespace

int launch_conv_f32(const ConvGeom& g, const float* x, const float* w, const float* bias, const float* residual,
                    float* y, hipStream_t st)
{
    TraceScope trace("conv_f32", &g, g.Ng, st);
    KArgs a;
    a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.g = g;
    a.grid_m = a.grid_n = 0;
    // Tile choice: the tile height that pads M (the filter count) least, taller tiles on ties;
    // narrower tiles along n when the grid would otherwise leave compute units idle.
    int best = 128, pad_best = (g.K + 127) / 128 * 128;
    for (int bm : {64, 32}) {
        const int padded = (g.K + bm - 1) / bm * bm;
        if (padded < pad_best) { best = bm; pad_best = padded; }
    }
    if (best == 32) return launch_tile<32, 256, 1, 4>(a, st);
    if (best == 64) return launch_tile<64, 128, 1, 4>(a, st);
    const long tiles128 = (long)((g.K + 127) / 128) * ((g.Ng + 127) / 128);
    if (tiles128 < 512) return launch_tile<128, 64, 2, 2>(a, st);
    return launch_tile<128, 128, 2, 2>(a, st);
}

}  // namespace dr
