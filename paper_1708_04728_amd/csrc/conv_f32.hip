// fp32 convolution forward (Eq. (7): Y_j = (W * X)_j + B_j) as an implicit GEMM on the gfx950
// matrix cores.
//
//   D[m][n] = sum_k A[m][k] * B[k][n]     m = output channel        (M  = K filters)
//                                         n = (image, p, q)         (Ng = N*P*Q)
//                                         k = (c, r, s)             (Kg = C*R*S)
//   A = the KCRS weight tensor viewed as an M x Kg matrix (no copy),
//   B = the im2col matrix, never materialised: each element is gathered from NCHW x on the fly.
//
// A workgroup of 256 threads (4 wave64) owns a BM x BN tile of D and walks Kg in slices of BK.
// Both operand slices are staged in LDS with the slice's k index contiguous per row (rows padded by
// 4 floats so that 128-bit LDS accesses of consecutive rows fall in distinct banks).
// v_mfma_f32_32x32x2_f32 consumes two k per instruction, one from lanes 0-31 and one from lanes
// 32-63; the kernel gives lane half g the slice's k in [g*BK/2, (g+1)*BK/2), so every lane fetches
// its A (or B) values of a slice with BK/8 128-bit LDS reads.  Global loads run PF slices ahead of
// the MFMAs in registers (PF register sets), LDS is double buffered, one barrier per slice.  With
// lanes running along n, both the gather from x and the store to NCHW y are coalesced.  Bias, the
// optional residual sum and ReLU are applied in the store.
//
// On this GPU fp32 MFMA and ordinary vector-ALU instructions do not overlap (measured: their times
// add), so every address computation in the loop costs matrix throughput.  Two slice orders exist:
//   CF = true  ("channel fastest": filters given in KRSC order, C % BK == 0): a slice is BK
//        consecutive channels of one filter tap (r, s).  All per-lane offsets are loop invariants;
//        the slice only moves a wave-uniform scalar offset, which rides in the buffer instructions'
//        scalar operand, and the padding test is redone once per tap.  Almost no vector-ALU work
//        per slice, and the filter rows are read with 16-byte loads.
//   CF = false (filters in KCRS order, any shape): k runs in KCRS order.  The workgroup first writes a
//        table k -> (offset of x[0][c][r][s], r, s) to LDS (contractions of up to KTAB elements, which
//        covers the small-channel first layers this path is for); an element's k is the same for a
//        whole wave, so its table entry arrives by one broadcast LDS read and the lane adds its
//        pixel's base offset; with padding it also tests the (r, s) bits of two per-lane masks of
//        valid window rows and columns.  Longer contractions decode (c, r, s) per element.
//        Without padding and with a filter width S that rounds up to a multiple of 4 cheaply (11 -> 12,
//        7 -> 8), k instead runs over (c, r, groups of 4 taps): the four activations of a group are
//        neighbours in memory and arrive by one 16-byte load per lane (consecutive pixels at stride 4
//        read consecutive 16-byte pieces), the taps added by the rounding count as zeros on both sides.
//        That quarter of the load instructions is what the first layer of AlexNet was limited by.
//
// A layer with fewer tiles than the device has compute units (one image, or a few) leaves most of the
// matrix cores idle while each workgroup walks the whole contraction alone.  Given scratch memory, the
// launcher then cuts the contraction into `splits` ranges of slices: blockIdx.y picks the range, the
// workgroup stores its raw partial sums to part[split][m][n], and conv_f32_reduce_kernel adds the
// ranges in a fixed order and applies bias, residual and ReLU.  No atomics: the result does not
// depend on the order in which workgroups finish.
#include <algorithm>
#include <type_traits>

#include "dr_internal.h"

namespace dr {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NT = 256;       // threads per workgroup
constexpr int KTAB = 512;     // CF = false: contraction elements (or groups of 4 taps) whose table entries fit the 4 KB LDS table

struct KArgs {
    const float* x;
    const float* w;
    const float* bias;
    const float* res;
    float* y;
    ConvGeom g;
    int grid_m, grid_n;
    int x_bytes, w_bytes;   // sizes of the x and w tensors (both < 2 GiB, checked by the launcher)
    int w_krsc;             // filters are in KRSC order (else KCRS)
    int row_groups;         // CF = false: k runs over (c, r, groups of 4 taps), see the header
    // Stacked convolution (Eq. (12): several filter banks on one input) whose filter ranges go to different tensors:
    // filter m < split_end[0] goes to destination 0, m < split_end[1] to destination 1, ... (unused ends hold INT_MAX).
    // Element (img, m, pix) of destination d lies at y_seg[d][(img * ctot_seg[d] + m) * P * Q + pix] (the host has
    // folded the destination's channel offset and the range's first filter into y_seg).  nsplit <= 1: everything to y.
    int nsplit;
    int split_end[3];
    float* y_seg[4];
    int ctot_seg[4];
    float* part;            // partial sums [splits][K][Ng] of a split contraction, or NULL
    int splits, slices_per_split;
};

template <int V> using IC = std::integral_constant<int, V>;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global load (its fence covers all address spaces), which would serialise the register prefetch
// with the MFMAs; global memory needs no ordering inside this kernel.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, int voff, int soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}

// BM x BN: workgroup tile; WGM x WGN: wave grid (4 waves); BK: k per LDS slice; PF: prefetch distance
// in slices; CF: slice order (see above); FR, FS: compile-time filter size for CF = false (0 = taken
// from the geometry at run time); SPLIT: the workgroup takes range blockIdx.y of the contraction and
// stores raw partial sums.
template <int BM, int BN, int WGM, int WGN, int BK, int PF, bool CF, int FR, int FS, bool SPLIT>
__global__ __launch_bounds__(NT) void conv_f32_kernel(const KArgs a)
{
    constexpr int WM = BM / WGM, WN = BN / WGN;   // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA tiles per wave
    constexpr int LDT = BK + 4;                   // padded LDS row (floats)
    constexpr int KQ = BK / 4;                    // float4 groups per row
    constexpr int HK = BK / 2;                    // k per lane half
    static_assert(WGM * WGN == 4 && TM >= 1 && TN >= 1, "bad tiling");
    static_assert(BK == 16 || BK == 32, "BK");
    static_assert(PF == 1 || PF == 2, "PF");
    constexpr int A_F4 = BM * KQ;                 // float4 groups in an A slice
    constexpr int B_F4 = BN * KQ;
    constexpr int A_PER = (A_F4 + NT - 1) / NT;
    constexpr int B_PER = B_F4 / NT;
    static_assert(B_F4 % NT == 0, "BN * BK must be a multiple of 1024");
    static_assert(BN <= NT && NT % BN == 0, "one n per thread");

    __shared__ __attribute__((aligned(16))) float As[2][BM * LDT];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * LDT];
    __shared__ __attribute__((aligned(16))) int ktab[CF ? 4 : 2 * KTAB];   // CF = false: {byte offset, r | s << 8} per k

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

    // Global reads go through buffer descriptors: a lane whose element lies outside the tensor (zero
    // padding, ragged M / n / k tails) gets its offset moved beyond num_records and the hardware
    // returns 0 for it without touching memory, so the gather needs no branches.
    constexpr int OOB = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, a.w_bytes, 0x00020000);

    // ---- per-thread gather state for B: one fixed n, B_PER groups of 4 consecutive k per slice
    constexpr int BKQ_STEP = NT / BN;             // k-groups covered by one pass of the workgroup
    const int bn = tid % BN;
    const int bkq0 = tid / BN;
    const int ng = n0 + bn;
    const bool n_ok = ng < g.Ng;
    int ih0 = -(1 << 30), iw0 = -(1 << 30);      // fails every bounds test when n is out of range
    int xoff0 = 0;                                // element offset of x[img][0][ih0][iw0]
    if (n_ok) {
        const int img = ng / PQ, pix = ng - img * PQ;
        const int p = pix / g.Q, q = pix - p * g.Q;
        ih0 = p * g.sh - g.ph;
        iw0 = q * g.sw - g.pw;
        xoff0 = img * g.C * HW + ih0 * g.W + iw0;
    }
    // ---- CF = false: the k table and this lane's masks of window rows / columns inside the image
    const bool rg = !CF && a.row_groups;
    const int S4 = (S + 3) & ~3;
    const int kg_eff = rg ? g.C * R * S4 : g.Kg;     // contraction length including the taps added by rounding S up
    const int ktab_n = (kg_eff + BK - 1) / BK * BK;
    const bool use_tab = !CF && !rg && ktab_n <= KTAB && R <= 31 && S <= 31;
    const bool nopad = g.ph == 0 && g.pw == 0;      // then every window lies inside the image
    unsigned rowmask = 0, colmask = 0;
    if constexpr (!CF) {
        if (use_tab) {
            for (int k = tid; k < ktab_n; k += NT) {
                int off = OOB, rs_bits = 31;          // beyond the contraction: the load returns 0 (mask bit 31 is never set)
                if (k < g.Kg) {
                    const int c = k / RS, rs = k - c * RS, r = rs / S, s_ = rs - r * S;
                    off = (c * HW + r * g.W + s_) * 4;
                    rs_bits = r | (s_ << 8);
                }
                ktab[2 * k] = off;
                ktab[2 * k + 1] = rs_bits;
            }
            if (n_ok) {
                for (int r = 0; r < R; ++r) rowmask |= ((unsigned)(ih0 + r) < (unsigned)g.H ? 1u : 0u) << r;
                for (int s_ = 0; s_ < S; ++s_) colmask |= ((unsigned)(iw0 + s_) < (unsigned)g.W ? 1u : 0u) << s_;
            }
            lds_barrier();                            // the table is complete before the first slice is gathered
        }
        if (rg) {
            // per group of 4 taps: {byte offset of x[0][c][r][s0], element offset of w[0][c][r][s0] | taps that exist << 24}
            for (int gq = tid; gq < ktab_n / 4; gq += NT) {
                int xo = OOB, meta = 0;
                const int kk = gq * 4;
                if (kk < kg_eff) {
                    const int c = kk / (R * S4), rem = kk - c * R * S4, r = rem / S4, s0 = rem - r * S4;
                    xo = (c * HW + r * g.W + s0) * 4;
                    meta = ((c * R + r) * S + s0) | (min(4, S - s0) << 24);
                }
                ktab[2 * gq] = xo;
                ktab[2 * gq + 1] = meta;
            }
            lds_barrier();
        }
    }
    const int bbase = n_ok ? xoff0 * 4 : OOB;        // (table path) byte offset of this lane's window origin

    // ---- per-thread state for A: rows f / KQ of the slice, byte offset of the row start
    const bool vecA = (g.Kg & 3) == 0;
    int arow[A_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int f = tid + i * NT;
        const int gm = m0 + f / KQ;
        arow[i] = ((A_F4 % NT == 0 || f < A_F4) && gm < g.K) ? gm * g.Kg * 4 : OOB;
    }

    f32x4 ra[PF][A_PER], rb[PF][B_PER];

    // ---- CF = true: loader state.  Slices are visited tap by tap, BK channels at a time.
    int ld_c0 = 0, ld_r = 0, ld_s = 0;            // wave-uniform position of the next slice to load
    int vb[CF ? B_PER : 1][4];                    // per-lane byte offsets of the 4 channels of a group
    int va[CF ? A_PER : 1];                       // per-lane byte offset of a float4 of the filter row
    if constexpr (CF) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) va[i] = arow[i] + ((tid + i * NT) % KQ) * 16;
    }
    auto tap_offsets = [&]() {   // padding test of tap (ld_r, ld_s) for this lane's pixel
        const bool ok = (unsigned)(ih0 + ld_r) < (unsigned)g.H && (unsigned)(iw0 + ld_s) < (unsigned)g.W;
        const int base = ok ? (xoff0 + ld_r * g.W + ld_s) * 4 : OOB;
#pragma unroll
        for (int i = 0; i < B_PER; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) vb[CF ? i : 0][j] = base + ((bkq0 + i * BKQ_STEP) * 4 + j) * HW * 4;
    };

    // this workgroup's range of slices: [s_begin, s_begin + nslices)
    const int nslices_all = CF ? RS * (g.C / BK) : (kg_eff + BK - 1) / BK;
    const int s_begin = SPLIT ? (int)blockIdx.y * a.slices_per_split : 0;
    const int nslices = SPLIT ? min(a.slices_per_split, nslices_all - s_begin) : nslices_all;
    if constexpr (CF && SPLIT) {
        if (s_begin) {
            const int per_tap = g.C / BK, tap = s_begin / per_tap;
            ld_c0 = (s_begin - tap * per_tap) * BK;
            ld_r = tap / S;
            ld_s = tap - ld_r * S;
            if (ld_c0) tap_offsets();   // load_slice computes them itself at the first slice of a tap
        }
    }

    auto load_slice = [&](int it, auto set_c) {
        constexpr int SET = decltype(set_c)::value;
        if constexpr (CF) {
            if (ld_c0 == 0) tap_offsets();
            const int sa = ((ld_r * S + ld_s) * g.C + ld_c0) * 4;   // scalar parts of the addresses
            const int sb = ld_c0 * HW * 4;
#pragma unroll
            for (int i = 0; i < A_PER; ++i)
                ra[SET][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, va[i], sa, 0));
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = buf_load(rx, vb[i][j], sb);
                rb[SET][i] = v;
            }
            ld_c0 += BK;
            if (ld_c0 == g.C) { ld_c0 = 0; if (++ld_s == S) { ld_s = 0; ++ld_r; } }
        } else {
            const int k0 = (s_begin + it) * BK;
            if (rg) {
#pragma unroll
                for (int i = 0; i < A_PER; ++i) {
                    const int meta = ktab[2 * (k0 / 4 + (tid + i * NT) % KQ) + 1];
                    const int ao = meta & 0xFFFFFF, nt = meta >> 24;
                    f32x4 v;
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = buf_load(rw, j < nt ? arow[i] + (ao + j) * 4 : OOB, 0);
                    ra[SET][i] = v;
                }
#pragma unroll
                for (int i = 0; i < B_PER; ++i) {
                    const int gq = k0 / 4 + bkq0 + i * BKQ_STEP;              // the same for the whole wave
                    const int xo = ktab[2 * gq], nt = ktab[2 * gq + 1] >> 24;
                    const int vo = bbase + xo;
                    f32x4 v;
                    if ((unsigned)vo < (unsigned)a.x_bytes && (unsigned)vo + 16u > (unsigned)a.x_bytes) {
                        // the tensor's last few elements: one by one, each checked against the end
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = buf_load(rx, vo + 4 * j, 0);
                    } else {
                        v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, vo, 0, 0));
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = j < nt ? v[j] : 0.f;
                    rb[SET][i] = v;
                }
                return;
            }
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int gk = k0 + ((tid + i * NT) % KQ) * 4;
                const int off = arow[i] + gk * 4;
                if (vecA) {
                    ra[SET][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, gk < g.Kg ? off : OOB, 0, 0));
                } else {
                    f32x4 v;
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = buf_load(rw, gk + j < g.Kg ? off + 4 * j : OOB, 0);
                    ra[SET][i] = v;
                }
            }
            if (use_tab) {
#pragma unroll
                for (int i = 0; i < B_PER; ++i) {
                    const int gk = k0 + (bkq0 + i * BKQ_STEP) * 4;            // the same for the whole wave
                    typedef int i32x4 __attribute__((ext_vector_type(4)));
                    const i32x4 e01 = *reinterpret_cast<const i32x4*>(&ktab[2 * gk]);
                    const i32x4 e23 = *reinterpret_cast<const i32x4*>(&ktab[2 * gk + 4]);
                    const int off[4] = {e01[0], e01[2], e23[0], e23[2]}, rsb[4] = {e01[1], e01[3], e23[1], e23[3]};
                    f32x4 v;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        int vo = bbase + off[j];
                        if (!nopad) {
                            const bool ok = ((rowmask >> (rsb[j] & 255)) & (colmask >> (rsb[j] >> 8)) & 1u) != 0;
                            vo = ok ? vo : OOB;
                        }
                        v[j] = buf_load(rx, vo, 0);
                    }
                    rb[SET][i] = v;
                }
            } else {
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int gk = k0 + (bkq0 + i * BKQ_STEP) * 4;
                int c = gk / RS;
                int rs = gk - c * RS;
                int r = rs / S;
                int s = rs - r * S;
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool ok = (gk + j < g.Kg) && (unsigned)(ih0 + r) < (unsigned)g.H && (unsigned)(iw0 + s) < (unsigned)g.W;
                    v[j] = buf_load(rx, ok ? (xoff0 + c * HW + r * g.W + s) * 4 : OOB, 0);
                    if (++s == S) { s = 0; if (++r == R) { r = 0; ++c; } }
                }
                rb[SET][i] = v;
            }
            }
        }
    };

    auto store_slice = [&](int buf, auto set_c) {
        constexpr int SET = decltype(set_c)::value;
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int f = tid + i * NT;
            if (A_F4 % NT == 0 || f < A_F4)
                *reinterpret_cast<f32x4*>(&As[buf][(f / KQ) * LDT + (f % KQ) * 4]) = ra[SET][i];
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i)
            *reinterpret_cast<f32x4*>(&Bs[buf][bn * LDT + (bkq0 + i * BKQ_STEP) * 4]) = rb[SET][i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // One slice: MFMAs on LDS buffer it&1; then register set SET (slice it+1, loaded PF slices ago)
    // moves to the other LDS buffer and is refilled with slice it+1+PF.
    auto slice_step = [&](int it, auto set_c) {
        const int buf = it & 1;
        f32x4 fa[TM][HK / 4], fb[TN][HK / 4];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float* p = &As[buf][(wm * WM + i * 32 + l32) * LDT + half * HK];
#pragma unroll
            for (int h = 0; h < HK / 4; ++h) fa[i][h] = *reinterpret_cast<const f32x4*>(p + 4 * h);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const float* p = &Bs[buf][(wn * WN + j * 32 + l32) * LDT + half * HK];
#pragma unroll
            for (int h = 0; h < HK / 4; ++h) fb[j][h] = *reinterpret_cast<const f32x4*>(p + 4 * h);
        }
#pragma unroll
        for (int kk = 0; kk < HK; ++kk)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][kk >> 2][kk & 3], fb[j][kk >> 2][kk & 3],
                                                                     acc[i][j], 0, 0, 0);
        if (it + 1 < nslices) {
            store_slice(buf ^ 1, set_c);
            if (it + 1 + PF < nslices) load_slice(it + 1 + PF, set_c);
        }
        lds_barrier();
    };

    load_slice(0, IC<0>{});
    store_slice(0, IC<0>{});
    if (1 < nslices) load_slice(1, IC<0>{});
    if (PF == 2 && 2 < nslices) load_slice(2, IC<PF - 1>{});
    lds_barrier();

    for (int it = 0; it < nslices; it += PF) {
        slice_step(it, IC<0>{});
        if (PF == 2 && it + 1 < nslices) slice_step(it + 1, IC<PF - 1>{});
    }

    // ---- store: accumulator register v of a 32x32 tile holds row 8*(v/4) + 4*half + v%4, column l32
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + l32;
        if (n >= g.Ng) continue;
        const int img = n / PQ, pix = n - img * PQ;
        float* yb = a.y + ((size_t)img * g.y_ctot + g.y_coff) * PQ + pix;
        const float* rbase = a.res ? a.res + (size_t)img * g.res_ctot * PQ + pix : nullptr;
        if constexpr (SPLIT) {
            float* pb = a.part + (size_t)blockIdx.y * g.K * g.Ng + n;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * WM + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                    if (m < g.K) pb[(size_t)m * g.Ng] = acc[i][j][v];
                }
            continue;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                if (m < g.K) {
                    float o = acc[i][j][v] + (a.bias ? a.bias[m] : 0.f);
                    if (rbase) o += rbase[(size_t)m * PQ];
                    if (g.relu) o = fmaxf(o, 0.f);
                    if (a.nsplit > 1) {
                        const bool s1 = m >= a.split_end[0], s2 = m >= a.split_end[1], s3 = m >= a.split_end[2];
                        float* base = s3 ? a.y_seg[3] : s2 ? a.y_seg[2] : s1 ? a.y_seg[1] : a.y_seg[0];
                        const int ct = s3 ? a.ctot_seg[3] : s2 ? a.ctot_seg[2] : s1 ? a.ctot_seg[1] : a.ctot_seg[0];
                        base[((size_t)img * ct + m) * PQ + pix] = o;
                        continue;
                    }
                    yb[(size_t)m * PQ] = o;
                }
            }
    }
}

// y = bias + residual + sum over the ranges of a split contraction, ReLU: one thread per output element,
// consecutive threads along n (these layers are small: what counts is the number of loads in flight).
__global__ __launch_bounds__(256) void conv_f32_reduce_kernel(const float* __restrict__ part, int splits, ConvGeom g,
                                                              const float* __restrict__ bias, const float* __restrict__ res,
                                                              float* __restrict__ y)
{
    const size_t total = (size_t)g.K * g.Ng;
    const int PQ = g.P * g.Q;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int m = (int)(i / g.Ng), n = (int)(i - (size_t)m * g.Ng);
        float sum = 0.f;
#pragma unroll 4
        for (int s = 0; s < splits; ++s) sum += part[s * total + i];   // unrolled: four loads in flight, the order of the sum unchanged
        const int img = n / PQ, pix = n - img * PQ;
        float o = sum + (bias ? bias[m] : 0.f);
        if (res) o += res[((size_t)img * g.res_ctot + m) * PQ + pix];
        if (g.relu) o = fmaxf(o, 0.f);
        y[((size_t)img * g.y_ctot + g.y_coff + m) * PQ + pix] = o;
    }
}

// How a layer's contraction is cut when scratch memory is there: enough ranges to give the device about two
// workgroups per compute unit, each at least two slices long; 1 = not cut (the layer's tiles reach half
// of the compute units, or it is too shallow).
inline int split_plan(int tiles, int nslices, int* slices_per_split)
{
    const int cus = device_cus();
    *slices_per_split = nslices;
    if (2 * tiles > cus || nslices < 4) return 1;   // measured: no gain once half the compute units have a tile
    const int want = (2 * cus + tiles - 1) / tiles;
    int per = (nslices + want - 1) / want;
    if (per < 2) per = 2;
    *slices_per_split = per;
    return (nslices + per - 1) / per;
}

// Slices of the contraction, and whether a KCRS layer takes the groups-of-4-taps order (no padding, a filter width
// that rounding up to a multiple of 4 lengthens by at most a quarter, a table that fits LDS).
template <int BK>
int contraction_slices(const ConvGeom& g, int* row_groups)
{
    *row_groups = 0;
    if (g.w_krsc) return g.R * g.S * (g.C / BK);
    const int S4 = (g.S + 3) & ~3;
    const long kg4 = (long)g.C * g.R * S4;
    if (g.ph == 0 && g.pw == 0 && S4 * 4 <= g.S * 5 && (kg4 + BK - 1) / BK * BK <= 4 * KTAB) {
        *row_groups = 1;
        return (int)((kg4 + BK - 1) / BK);
    }
    return (g.Kg + BK - 1) / BK;
}

template <int BM, int BN, int BK>
size_t split_bytes(const ConvGeom& g)
{
    int rgm;
    const int nslices = contraction_slices<BK>(g, &rgm);
    int per;
    const int splits = split_plan(((g.K + BM - 1) / BM) * ((g.Ng + BN - 1) / BN), nslices, &per);
    return splits > 1 ? (size_t)splits * g.K * g.Ng * sizeof(float) : 0;
}

template <int BM, int BN, int WGM, int WGN, int BK, int PF>
int launch_tile(const KArgs& base, void* ws, size_t ws_bytes, hipStream_t st)
{
    KArgs a = base;
    a.grid_m = (a.g.K + BM - 1) / BM;
    a.grid_n = (a.g.Ng + BN - 1) / BN;
    a.part = nullptr;
    a.splits = 1;
    const int nslices = contraction_slices<BK>(a.g, &a.row_groups);
    a.slices_per_split = nslices;
    if (ws && a.nsplit <= 1) {
        int per;
        const int splits = split_plan(a.grid_m * a.grid_n, nslices, &per);
        if (splits > 1 && (size_t)splits * a.g.K * a.g.Ng * sizeof(float) <= ws_bytes && ((uintptr_t)ws & 15) == 0) {
            a.part = (float*)ws;
            a.splits = splits;
            a.slices_per_split = per;
        }
    }
    const dim3 grid((unsigned)(a.grid_m * a.grid_n), (unsigned)a.splits), block(NT);
    const int R = a.g.R, S = a.g.S;
#define DR_LAUNCH(CF, FR, FS)                                                                                              \
    do {                                                                                                                   \
        if (a.part) hipLaunchKernelGGL((conv_f32_kernel<BM, BN, WGM, WGN, BK, PF, CF, FR, FS, true>), grid, block, 0, st, a);   \
        else hipLaunchKernelGGL((conv_f32_kernel<BM, BN, WGM, WGN, BK, PF, CF, FR, FS, false>), grid, block, 0, st, a);         \
    } while (0)
    if (a.w_krsc) DR_LAUNCH(true, 0, 0);
    else if (R == 1 && S == 1) DR_LAUNCH(false, 1, 1);
    else if (R == 3 && S == 3) DR_LAUNCH(false, 3, 3);
    else if (R == 5 && S == 5) DR_LAUNCH(false, 5, 5);
    else if (R == 7 && S == 7) DR_LAUNCH(false, 7, 7);
    else if (R == 11 && S == 11) DR_LAUNCH(false, 11, 11);
    else DR_LAUNCH(false, 0, 0);
#undef DR_LAUNCH
    const int rc = check_launch("conv_f32");
    if (rc != DR_OK) return rc;
    if (a.part) {
        const ConvGeom& g = a.g;
        const size_t threads = (size_t)g.K * g.Ng;
        const unsigned blocks = (unsigned)std::min<size_t>((threads + 255) / 256, (size_t)device_cus() * 8);
        hipLaunchKernelGGL(conv_f32_reduce_kernel, dim3(blocks), dim3(256), 0, st, a.part, a.splits, g, a.bias, a.res, a.y);
        return check_launch("conv_f32 (sum of the split contraction)");
    }
    return DR_OK;
}

}  // namespace

size_t conv_f32_scratch_bytes(const ConvGeom& g)
{
    const bool rows32 = (g.K + 31) / 32 * 32 < (g.K + 63) / 64 * 64;
    if (g.w_krsc && g.C % 32 == 0) return rows32 ? split_bytes<32, 128, 32>(g) : split_bytes<64, 64, 32>(g);
    return rows32 ? split_bytes<32, 128, 16>(g) : split_bytes<64, 64, 16>(g);
}

int launch_conv_f32(const ConvGeom& g, const float* x, const float* w, const float* bias, const float* residual,
                    float* y, hipStream_t st, void* ws, size_t ws_bytes, const ConvSplit* split)
{
    TraceScope trace("conv_f32", &g, g.Ng, st);
    KArgs a;
    a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.g = g;
    a.grid_m = a.grid_n = 0;
    a.nsplit = 0;
    for (int d = 0; d < 4; ++d) { a.y_seg[d] = nullptr; a.ctot_seg[d] = 0; if (d < 3) a.split_end[d] = 0x7FFFFFFF; }
    if (split && split->n > 1) {
        a.nsplit = split->n;
        const long PQ = (long)g.P * g.Q;
        int start = 0;
        for (int d = 0; d < split->n && d < 4; ++d) {
            const ConvDest& s = split->dst[d];
            a.y_seg[d] = (float*)s.y + ((long)s.c_offset - start) * PQ;
            a.ctot_seg[d] = s.ctot;
            start += s.k;
            if (d < 3 && d + 1 < split->n) a.split_end[d] = start;
        }
    }
    const size_t xb = (size_t)g.N * g.C * g.H * g.W * 4, wb = (size_t)g.K * g.Kg * 4;
    if (xb >= (1ull << 31) || wb >= (1ull << 31))
        return fail(DR_ERR_UNSUPPORTED, "conv_f32: input (%zu bytes) or filter tensor (%zu bytes) is 2 GiB or larger", xb, wb);
    a.x_bytes = (int)xb; a.w_bytes = (int)wb;
    a.w_krsc = g.w_krsc;
    // Tile choice (from sweeps on the inception / streamline shapes): 32-row tiles when they pad the
    // filter count less than 64-row tiles (16, 32, 96 filters ...), else 64 x 64 tiles; both give the
    // grid several workgroups per compute unit, which matters more here than operand reuse.  The
    // deepest slice the channel count allows, two slices of prefetch.
    const bool rows32 = (g.K + 31) / 32 * 32 < (g.K + 63) / 64 * 64;
    if (g.w_krsc && g.C % 32 == 0)      // (32-deep slices with the groups-of-4-taps order: measured 10 % slower)
        return rows32 ? launch_tile<32, 128, 1, 4, 32, 2>(a, ws, ws_bytes, st) : launch_tile<64, 64, 2, 2, 32, 2>(a, ws, ws_bytes, st);
    return rows32 ? launch_tile<32, 128, 1, 4, 16, 2>(a, ws, ws_bytes, st) : launch_tile<64, 64, 2, 2, 16, 2>(a, ws, ws_bytes, st);
}

}  // namespace dr
