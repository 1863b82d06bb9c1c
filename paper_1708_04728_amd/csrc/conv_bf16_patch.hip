// bf16 convolution forward (Eq. (7)) for filters of several taps at stride 1 on maps with few channels per pixel: the
// input patch of a tile is brought into LDS ONCE and every tap multiplies from there.
//
// The streaming kernel (conv_bf16_dma.hip) fetches, for every tap (r, s) of the filter, the 128 bytes of each of the
// tile's pixels again: nine times for a 3x3 filter.  Counters show what that costs: the path that carries global memory
// into LDS (address unit, vector cache, the fabric from L2) is busy 60-70 % of a launch while the matrix cores are busy a
// third of it.  Here a tile is TH whole output rows of one image (TH Q <= 256 pixels), its input patch the TH + R - 1 input
// rows around them with pad_w zero columns on either side (row pitch PW = W + 2 pad_w pixels), one LDS row of 128 bytes per
// patch pixel and block of 64 channels.  Output pixel (dp, q) of the tile reads, for tap (r, s), patch pixel
// (dp + r) PW + q + s: the same per-lane base for every tap, plus a wave-uniform offset.  Per tile and 64 channels the
// loads are then (TH + R - 1) PW input rows once plus the filter slices, instead of R S TH Q input rows plus the filter
// slices -- for 3x3 on 56 x 56 x 64 with 96 filters per workgroup a third of the bytes per multiply-add.  Where it takes
// fewer tiles per image a tile is a run of HALF rows instead (PArgs): nine half rows of a 56 x 56 map are 252 outputs over
// at most five output rows, 13 tiles per image instead of 14; a lane's patch pixel then depends on whether its tile starts in
// mid-row and is set at the top of every tile.
//
// Everything else is the streaming kernel's: filters go through a two-stage ring of 64-deep slices, one tap and channel
// block per slice, in (r, s, c) order (the same order of accumulation: results are bit-identical); LDS rows are swizzled
// by (row >> 1) & 7; out-of-image patch pixels and filters beyond the last are loaded from offsets outside the buffer
// (zeros); the store is the one every lane issues (exact count in the memory counter).  Workgroups are persistent over
// tiles of one block of 32 TM filters; the next tile's patch and first filter slices are requested before the current
// tile's store.
#include "dr_internal.h"
#include "dr_store.h"
#include "conv_bf16_dev.h"

namespace dr {
namespace {

constexpr int PATCH_ROWS = 352;          // LDS rows of 128 bytes the patch of a tile of whole rows may take (patch pixels x 64-channel blocks): the rule
constexpr int PATCH_CAP = 416;           // ... and what the kernel holds (a tile of half rows covers one input row more: 7 x 58 on 56 x 56 maps)
constexpr int PATCH_BN = 256;            // pixel rows of a tile in the matrix instructions (TH Q of them carry outputs)

struct PArgs {
    const uint16_t* x;
    const uint16_t* w;
    const float* bias;
    uint16_t* y;
    ConvGeom g;
    int grid_m, tiles, tiles_per_img;    // filter blocks; pixel tiles in all, per image
    WalkArgs wk;                         // the persistent walk over them (tile_walk)
    int x_bytes, w_bytes, y_bytes;
    int c8, cblks;                       // C / 8, C / 64
    // A tile is TH consecutive SEGMENTS of one image: a segment is an output row (sh = 0) or half of one (sh = 1, QS = Q / 2
    // outputs), numbered row by row.  Half rows fill the 256 pixel rows of a tile better on some maps (56 x 56: 9 half rows =
    // 252 outputs and 13 tiles per image, against 4 rows = 224 outputs and 14 tiles).
    int TH, THQ, QS, sh, segs;           // segments per tile, outputs per tile (TH QS), outputs per segment, log2 segments per row, segments per image
    int PW, PPN, PPB;                    // patch row pitch (pixels), patch pixels, 32-row load passes per channel block
    unsigned magic_pw, magic_qs;         // ceil(2^32 / PW), ceil(2^32 / QS)
};

// TM: 32-filter blocks per workgroup (all four waves share them); a wave owns 64 of the tile's 256 pixel rows.
// FX: 0 = any filter; 33 = a 3x3 filter on 64 channels, known at compile time: the nine slices of a tile are unrolled, their
// filter offsets are constants and the patch addresses of the nine taps are computed once per workgroup.
template <int TM, int OCC, int FX>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
void conv_bf16_patch_kernel(const PArgs a)
{
    constexpr bool FIXED = FX == 33;
    constexpr int TN = 2, BM = TM * 32, A_PER = TM, A_BYTES = BM * 128, NS = 2, E = 2 * TM * TN;
    static_assert(TM >= 1 && TM <= 4 && A_PER + E < 63, "bad configuration");

    __shared__ __attribute__((aligned(1024))) unsigned char aring[NS * A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char patch[PATCH_CAP * 128];
    __shared__ __attribute__((aligned(1024))) float bias_lds[128];
    const unsigned aring_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)aring;
    const unsigned patch_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)patch;

    const ConvGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    // loader: this lane fetches row lrow of every 32-row pass, logical chunk lc (chunk j of row r lives at chunk j ^ ((r >> 1) & 7))
    const int lrow = wave * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((lrow >> 1) & 7);
    // reader of the filter tile: LDS byte offset of this lane's chunk for k-step 0; k-step ks flips bits 5..6
    const unsigned a_rd = aring_lds + l32 * 128 + ((half << 4) ^ (((l32 >> 1) & 7) << 4));
    // reader of the patch: the pixel this lane holds in block j is output col[j] of segment seg[j] of the tile (rows beyond the
    // tile's outputs multiply pixel 0 again; nothing of them is stored); row0[j]: its patch pixel for tap (0, 0), set per tile
    int nl[TN], seg[TN], col[TN], row0[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        nl[j] = wave * 64 + j * 32 + l32;
        const int nn = nl[j] < a.THQ ? nl[j] : 0;
        seg[j] = (int)__umulhi((unsigned)nn, a.magic_qs);
        col[j] = nn - seg[j] * a.QS;
    }
    // tile tt: image, first segment; the patch starts pad_h input rows above output row (first segment >> sh)
    auto tile_origin = [&](int tt, int& img, int& s0) __attribute__((always_inline)) {
        img = tt / a.tiles_per_img;
        s0 = (tt - img * a.tiles_per_img) * a.TH;
    };

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, a.w_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rbias = __builtin_amdgcn_make_buffer_rsrc((void*)a.bias, 0, a.bias ? g.K * 4 : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc((void*)a.y, 0, a.y_bytes, 0x00020000);

    // ---- persistent walk (tile_walk)
    const TileWalk walk = tile_walk(a.wk);
    const int mt = walk.mt, my_tiles = walk.count;
    const int R_ = FIXED ? 3 : g.R, S_ = FIXED ? 3 : g.S, CB_ = FIXED ? 1 : a.cblks;
    const int nslices = R_ * S_ * CB_;                  // slice sl = (tap, channel block), channel block fastest

    if (my_tiles == 0) return;                          // (whole workgroup, before anything is in flight; the launcher leaves no such workgroup)

    int a_voff[A_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int m = mt * BM + i * 32 + lrow;
        a_voff[i] = m < g.K ? (m * g.Kg + lc * 8) * 2 : OOB;
    }
    if (wave * 64 < BM) {
        const int ml = wave * 64 + lane, m = mt * BM + ml;
        load_to_lds4(rbias, bias_lds + wave * 64, (ml < BM && m < g.K) ? m * 4 : OOB);
    }
    const int m_lane = mt * BM + half * 8;
    const unsigned bias_rd = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)bias_lds + (half * 8) * 4;

    // ---- loaders
    int ld_i = 0;                                      // the next filter slice to load (the same cycle for every tile)
    auto issue_a = [&](int stage) __attribute__((always_inline)) {
        unsigned char* sa = aring + stage * A_BYTES + wave * 1024;
        const int soff = ld_i * 128;                   // slice (tap, cb) starts (tap C + 64 cb) elements into a filter's row
#pragma unroll
        for (int i = 0; i < A_PER; ++i) load_to_lds16(rw, sa + i * 4096, a_voff[i], soff);
        if (++ld_i == nslices) ld_i = 0;
    };
    auto issue_patch = [&](int tt) __attribute__((always_inline)) {
        int img, s0;
        tile_origin(tt, img, s0);
        const int p0 = s0 >> a.sh;
        for (int cb = 0; cb < CB_; ++cb)
            for (int pb = 0; pb < a.PPB; ++pb) {
                const int pp = pb * 32 + lrow;                                  // patch pixel this lane fetches
                const int prow = (int)__umulhi((unsigned)pp, a.magic_pw), pcol = pp - prow * a.PW;
                const int ih = p0 - g.ph + prow, iw = pcol - g.pw;
                const bool ok = pp < a.PPN && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
                const int voff = ok ? (((img * g.H + ih) * g.W + iw) * g.C + cb * 64 + lc * 8) * 2 : OOB;
                load_to_lds16(rx, patch + ((cb * a.PPB + pb) * 32 + wave * 8) * 128, voff, 0);
            }
    };

    // ---- operands: two register slots (k-step ks of a slice in slot ks & 1), each k-step fetched one step ahead of the
    // matrix cores: a step of this wave tile is 2 TM matrix instructions, long enough to cover the LDS latency
    f32x16 acc[TM][TN];
    u32x4 fa[2][TM], fb[2][TN];
    unsigned b_cur[TN], b_nxt[TN];                     // LDS address of this lane's patch chunk for k-step 0 of the current / next slice
    auto b_setup = [&](int r, int s, int cb, unsigned* out) __attribute__((always_inline)) {
        const int tap = r * a.PW + s + cb * a.PPB * 32;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int row = row0[j] + tap;
            out[j] = patch_lds + row * 128 + ((half << 4) ^ (((row >> 1) & 7) << 4));
        }
    };
    auto fetch = [&](int stage, const unsigned* b, auto ks_c) __attribute__((always_inline)) {
        constexpr int KS = decltype(ks_c)::value, SL = KS & 1;
        const unsigned pa = (a_rd + stage * A_BYTES) ^ (KS * 32);
        fa[SL][0] = ds_read16<0>(pa);
        if constexpr (TM > 1) fa[SL][1] = ds_read16<4096>(pa);
        if constexpr (TM > 2) fa[SL][2] = ds_read16<8192>(pa);
        if constexpr (TM > 3) fa[SL][3] = ds_read16<12288>(pa);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[SL][j] = ds_read16<0>(b[j] ^ (KS * 32));
    };
    auto multiply = [&](auto ks_c, auto pending_c) __attribute__((always_inline)) {
        constexpr int SL = decltype(ks_c)::value & 1;
        wait_lgkm<decltype(pending_c)::value>();
#pragma unroll
        for (int i = 0; i < TM; ++i) touch(fa[SL][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) touch(fb[SL][j]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[SL][i]),
                                                                    __builtin_bit_cast(bf16x8, fb[SL][j]), acc[i][j], 0, 0, 0);
    };

    // bias + ReLU + bf16 store of the tile's outputs; every lane issues all E stores (see the streaming kernel's epilogue)
    auto epilogue = [&](int tt) __attribute__((always_inline)) {
        int img, s0;
        tile_origin(tt, img, s0);
        const int segs_left = a.segs - s0;                                // segments of the image from this tile on
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
                const bool n_ok = nl[j] < a.THQ && seg[j] < segs_left;
                const int gs = s0 + seg[j], pr = gs >> a.sh;              // the segment within the image, its output row
                const int nbase = (((img * g.P + pr) * g.Q + (gs - (pr << a.sh)) * a.QS + col[j]) * g.y_ctot + g.y_coff) * 2;
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
                    if (g.relu) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = fmaxf(o[e], 0.f);
                    }
                    u32x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
                    const int voff = (n_ok && mb < g.K) ? nbase + mb * 2 : OOB;
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_raw_buffer_store_b128(pk, ry, voff, 0, 0);
#endif
                }
            }
        }
    };

    // ---- pipeline.  Filter slice k lives in ring stage k & 1.  Memory operations of a wave, in issue order, around a tile
    // boundary: ... filter slices of tile t | patch of tile t + 1, its filter slices 0 and 1 | the E stores of tile t | filter
    // slice 2 of tile t + 1 ...  Loads return in order, so "at most n operations outstanding" with n the number issued after
    // the awaited load means that load has landed; the stores only ever make such a wait longer.
    unsigned b_tap[FIXED ? 9 : 1][TN];                  // FIXED: this lane's patch address for each of the nine taps
    issue_patch(walk.tile(0));
    issue_a(0);
    if (nslices > 1) issue_a(1);
    int gi = 0;
    for (int t = 0; t < my_tiles; ++t) {
        const int tt = walk.tile(t);
        {
            // where this lane's pixels lie in the tile's patch (with half rows that depends on whether the tile starts in mid-row)
            int img, s0;
            tile_origin(tt, img, s0);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int gs = s0 + seg[j], pr = gs >> a.sh;
                row0[j] = (pr - (s0 >> a.sh)) * a.PW + (gs - (pr << a.sh)) * a.QS + col[j];
            }
            if constexpr (FIXED) {
#pragma unroll
                for (int tp = 0; tp < 9; ++tp) b_setup(tp / 3, tp % 3, 0, b_tap[tp]);
            }
        }
        // the patch and the first filter slice have landed: behind them are filter slice 1 and, from the second tile on, the stores
        if (nslices > 1) {
            if (t > 0) wait_vmcnt<A_PER + E>();
            else wait_vmcnt<A_PER>();
        } else {
            if (t > 0) wait_vmcnt<E>();
            else wait_vmcnt<0>();
        }
        ring_barrier();
        int r = 0, s = 0, cb = 0;
        if constexpr (FIXED) { b_cur[0] = b_tap[0][0]; b_cur[1] = b_tap[0][1]; }
        else b_setup(0, 0, 0, b_cur);
        fetch(gi & 1, b_cur, IC<0>{});
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
#pragma unroll
        for (int sl = 0; sl < nslices; ++sl, ++gi) {
            const int stage = gi & 1;
            const bool more = sl + 1 < nslices;          // (wave-uniform) the tile has another slice
            if (more) {
                if constexpr (FIXED) { b_nxt[0] = b_tap[sl + 1 < 9 ? sl + 1 : 0][0]; b_nxt[1] = b_tap[sl + 1 < 9 ? sl + 1 : 0][1]; }
                else {
                    if (++cb == CB_) { cb = 0; if (++s == S_) { s = 0; ++r; } }
                    b_setup(r, s, cb, b_nxt);
                }
            }
            constexpr int PEND = TM + TN;                // the reads of the step just requested may be pending
            fetch(stage, b_cur, IC<1>{});
            multiply(IC<0>{}, IC<PEND>{});
            fetch(stage, b_cur, IC<2>{});
            multiply(IC<1>{}, IC<PEND>{});
            fetch(stage, b_cur, IC<3>{});
            multiply(IC<2>{}, IC<PEND>{});
            // (the matrix instructions stay on one path through the loop: in two arms of a branch the compiler gives them two
            // register sets and copies all accumulators between them)
            if (more) {
                // filter slice gi + 1 has landed: nothing was issued behind it but, right after a tile boundary, the stores
                if (sl == 0 && t > 0) wait_vmcnt<E>();
                else wait_vmcnt<0>();
                ring_barrier();                          // ... and everybody has read slice gi out of its stage (its last step has arrived too)
                if (sl + 2 < nslices) issue_a(stage);
                fetch(stage ^ 1, b_nxt, IC<0>{});
#pragma unroll
                for (int j = 0; j < TN; ++j) b_cur[j] = b_nxt[j];
            } else {
                wait_lgkm<0>();
            }
            multiply(IC<3>{}, IC<PEND>{});
        }
        if (t + 1 < my_tiles) {
            ring_barrier();                              // everybody has read the patch and both filter stages for the last time
            issue_patch(walk.tile(t + 1));
            issue_a(gi & 1);
            if (nslices > 1) issue_a((gi & 1) ^ 1);
        }
        epilogue(tt);
    }
    wait_lgkm<0>();
}

template <int TM, int FX>
int launch_patch(PArgs a, hipStream_t st)
{
    constexpr int BM = TM * 32, OCC = 2;
    static_assert(OCC * (2 * BM * 128 + PATCH_CAP * 128 + 1024) <= 160 * 1024, "two workgroups per compute unit must fit LDS");
    a.grid_m = (a.g.K + BM - 1) / BM;
    int gn = device_cus() * OCC / a.grid_m;
    if (gn < 1) gn = 1;
    if (gn > a.tiles) gn = a.tiles;
    a.wk = make_walk(a.grid_m, gn, a.tiles);
    hipLaunchKernelGGL((conv_bf16_patch_kernel<TM, OCC, FX>), dim3((unsigned)(gn * a.grid_m)), dim3(256), 0, st, a);
    return check_launch("conv_bf16_patch");
}

// Output rows per tile: as many as fit 256 pixel rows and the patch's LDS; 0 when the layer is not for this kernel.
int patch_rows_per_tile(const ConvGeom& g)
{
    if (!g.nhwc || !g.w_krsc || g.C % 64 != 0 || g.K % 8 != 0 || g.sh != 1 || g.sw != 1 || g.R * g.S < 2 || g.R > 7 || g.S > 7) return 0;
    if (g.Q < 2 || g.Q > PATCH_BN || g.W + 2 * g.pw < 2 || g.res_ctot) return 0;
    const int PW = g.W + 2 * g.pw, cblks = g.C / 64;
    int th = PATCH_BN / g.Q;
    if (th > g.P) th = g.P;
    while (th >= 1 && cblks * (((th + g.R - 1) * PW + 31) / 32 * 32) > PATCH_ROWS) --th;
    // worth it when most of the 256 pixel rows carry outputs (whole maps smaller than that are left to the streaming kernel)
    return th >= 1 && th * g.Q * 4 >= PATCH_BN * 3 ? th : 0;
}

}  // namespace

bool conv_bf16_patch_eligible(const ConvGeom& g, const void* x, const void* w, const void* y)
{
    const double xb = (double)g.N * g.C * g.H * g.W * 2.0, wb = (double)g.K * g.Kg * 2.0, yb = (double)g.Ng * g.y_ctot * 2.0;
    if (xb >= 2147483648.0 || wb >= 2147483648.0 || yb >= 2147483648.0 || g.Ng >= (1 << 24)) return false;
    if (((uintptr_t)x & 15) || ((uintptr_t)w & 15) || ((uintptr_t)y & 15) || g.y_ctot % 8 != 0 || g.y_coff % 8 != 0) return false;
    return patch_rows_per_tile(g) > 0;
}

int launch_conv_bf16_patch(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, uint16_t* y, hipStream_t st, int tm)
{
    PArgs a{};
    a.x = x; a.w = w; a.bias = bias; a.y = y; a.g = g;
    a.x_bytes = (int)((size_t)g.N * g.C * g.H * g.W * 2);
    a.w_bytes = (int)((size_t)g.K * g.Kg * 2);
    a.y_bytes = (int)((size_t)g.Ng * g.y_ctot * 2);
    a.c8 = g.C / 8; a.cblks = g.C / 64;
    a.TH = patch_rows_per_tile(g);
    if (a.TH < 1) return fail(DR_ERR_UNSUPPORTED, "conv_bf16_patch: layer not eligible");
    a.PW = g.W + 2 * g.pw;
    a.QS = g.Q; a.sh = 0; a.segs = g.P;
    a.tiles_per_img = (g.P + a.TH - 1) / a.TH;
    int patch_rows = a.TH + g.R - 1;
    if (g.Q % 2 == 0 && g.Q / 2 >= 2) {
        // tiles of half rows where that takes fewer tiles per image: th2 half rows span at most th2 / 2 + 1 output rows
        int th2 = PATCH_BN / (g.Q / 2);
        if (th2 > 2 * g.P) th2 = 2 * g.P;
        while (th2 >= 1 && a.cblks * (((th2 / 2 + 1 + g.R - 1) * a.PW + 31) / 32 * 32) > PATCH_CAP) --th2;
        if (th2 >= 1 && (2 * g.P + th2 - 1) / th2 < a.tiles_per_img) {
            a.TH = th2; a.QS = g.Q / 2; a.sh = 1; a.segs = 2 * g.P;
            a.tiles_per_img = (2 * g.P + th2 - 1) / th2;
            patch_rows = th2 / 2 + 1 + g.R - 1;
        }
    }
    a.THQ = a.TH * a.QS;
    a.tiles = g.N * a.tiles_per_img;
    a.PPN = patch_rows * a.PW;
    a.PPB = (a.PPN + 31) / 32;
    a.magic_pw = (unsigned)((0x100000000ull + a.PW - 1) / a.PW);
    a.magic_qs = (unsigned)((0x100000000ull + a.QS - 1) / a.QS);
    // 96 filters per workgroup when that wastes fewer padded filter rows than 64
    const int pad96 = (g.K + 95) / 96 * 96, pad64 = (g.K + 63) / 64 * 64;
    if (tm == 0) tm = pad96 <= pad64 ? 3 : 2;
    // (unrolled for 3x3 on 64 channels: a workgroup that has its compute unit to itself -- while its neighbour stores, or in
    // the last, partly filled round -- takes 12 % less time per tile with 96-filter blocks, the whole layer 4-5 %)
    if (g.R == 3 && g.S == 3 && g.C == 64) return tm == 3 ? launch_patch<3, 33>(a, st) : launch_patch<2, 33>(a, st);
    return tm == 3 ? launch_patch<3, 0>(a, st) : launch_patch<2, 0>(a, st);
}

}  // namespace dr
