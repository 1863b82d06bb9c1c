// bf16 convolution forward (Eq. (7)) for filters of several taps at stride 1 on maps of any size with up to 64 channels
// (a multiple of 16): the patch kernel's idea -- bring the input patch of a tile into LDS once, multiply every tap from
// there -- without its two restrictions (64-channel blocks, tiles inside one image).
//
// Rows of all images as one stack.  The batch's output rows are numbered g = n P + p, and a tile is TH consecutive rows
// of that stack (TH Q <= 256 outputs), wherever the image borders fall: on 28 x 28 maps 9 rows (252 of the 256 pixel
// rows of the matrix instructions carry outputs; whole rows of one image would leave 7 x 28 = 196), on 14 x 14 maps 18
// rows, on 7 x 7 maps 36.  The patch holds, for every image the tile touches, the input rows around the tile's share of
// that image, each image with its own R - 1 extra rows: output row g0 + dp, in image img0 + io, reads for filter row r
// the patch row dp + io (R - 1) + r.  Rows are PW = W + 2 pad_w pixels wide with the zero columns in place.
//
// A patch pixel is C / 8 chunks of 16 bytes plus ONE chunk of padding: the pitch in chunks is odd, and 32 lanes that
// read the same chunk of 32 consecutive pixels then fall on different LDS banks whatever C is (measured: every odd pitch
// reads at the rate of a contiguous read, pitch 2, 4, 8 and 16 at 1.4, 1.3, 2.5 and 5 times that).  No swizzle, so the
// address of a k-step is the lane's base plus a wave-uniform offset.
//
// The contraction runs over k-steps of 16 channels in filter order (r, s, c) -- the order of the filter's memory, so
// a 64-deep filter slice is 128 consecutive bytes of each filter's row whatever C is, and the order of accumulation (and
// every bit of the result) is the streaming kernel's.  The last slice of a row is filled up with zeros.  The patch
// offset of each k-step comes from three counters on the scalar unit.
//
// Pipeline, ring of filter slices, stores and waits are the patch kernel's (conv_bf16_patch.hip).
#include <atomic>
#include "dr_internal.h"
#include "dr_store.h"
#include "conv_bf16_dev.h"

namespace dr {
namespace {

constexpr int ROWS_BN = 256;             // pixel rows of a tile in the matrix instructions (TH Q of them carry outputs)

struct RArgs {
    const uint16_t* x;
    const uint16_t* w;
    const float* bias;
    uint16_t* y;
    ConvGeom g;
    int grid_m, tiles;                   // filter blocks, pixel tiles
    WalkArgs wk;                         // the persistent walk over them (tile_walk)
    int x_bytes, w_bytes, y_bytes;
    int TH, THQ;                         // stacked output rows per tile, outputs per tile
    int PW, NP, CCH, J;                  // patch row pitch (pixels); chunks per patch pixel (C / 8 + 1); C / 8; k-steps per tap
    int PR;                              // rows of an image as the patch sees it: with its padding, H + 2 pad_h (packed input: hp)
    int rows_max, passes;                // patch rows of a tile (the most any tile needs); 4 KiB load passes
    int U, nslices, tail_chunks;         // k-steps; filter slices; 16-byte chunks of a filter's row in the last slice
    int Kg;                              // elements of a filter's row in memory
    int taps_per_row;                    // taps the k-steps walk along a patch row before the next filter row
    int tap_skip, row_skip;              // bytes from behind a tap's last k-step to the next tap / on top of that to the next filter row
    int row_mul, D;                      // patch row of output row dp in image img0 + io, filter row 0: row_mul dp + io D
    int row_chunks, px_chunks;           // chunks per patch row; chunks from one output pixel's window to the next one's
    int packed, wp;                      // input is the padded 4-channel copy xp[N][PR][wp][4] (see launch_conv_bf16_rows_stem)
    unsigned magic_np, magic_pw, magic_q, magic_p, magic_pr, magic_rc;   // ceil(2^32 / d) for d = NP, PW, Q, P, PR, row_chunks
    // a 1x1 convolution on the layer's output, in the same kernel (TAIL): filters w2[K2][K], bias2, ReLU flag; g.y_ctot and
    // g.y_coff then describe ITS destination and the layer's own output is never written
    const uint16_t* w2;
    const float* bias2;
    int K2, relu2, w2_bytes;
};

// TM: 32-filter blocks per workgroup (all four waves share them); a wave owns 64 of the tile's 256 pixel rows.
// TAIL: the workgroup holds ALL the layer's filters (K <= 32 TM) and a 1x1 convolution with at most 32 TM filters follows:
// the tile's results -- bias, ReLU, rounded to bf16 as the stored tensor would be -- stay in registers, which already are
// the second operand of a contraction over the layer's filters (pack_blocks), the 1x1 filters wait in LDS, and 2 TM k-steps
// later the tile of the 1x1 convolution's output is stored instead.  The intermediate tensor is neither written nor read.
template <int TM, int OCC, bool TAIL = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
void conv_bf16_rows_kernel(const RArgs a)
{
    constexpr int TN = 2, BM = TM * 32, A_PER = TM, A_BYTES = BM * 128, NS = 2, E = 2 * TM * TN;
    static_assert(TM >= 1 && TM <= 4 && A_PER + E < 63, "bad configuration");

    __shared__ __attribute__((aligned(1024))) unsigned char aring[NS * A_BYTES];
    __shared__ __attribute__((aligned(1024))) float bias_lds[128];
    __shared__ __attribute__((aligned(1024))) unsigned char w2s[TAIL ? BM * 128 : 16];   // 1x1 filters: rows of 64 k, swizzled like the ring
    __shared__ __attribute__((aligned(16))) float bias2_lds[TAIL ? 128 : 4];
    extern __shared__ __attribute__((aligned(1024))) unsigned char patch[];
    const unsigned aring_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)aring;
    const unsigned patch_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)patch;

    const ConvGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    // filter loader: this lane fetches row lrow of every 32-row pass, logical chunk lc (chunk j of row r lives at chunk j ^ ((r >> 1) & 7))
    const int lrow = wave * 8 + (lane >> 3);
    const int lc = (lane & 7) ^ ((lrow >> 1) & 7);
    // reader of the filter tile: LDS byte offset of this lane's chunk for k-step 0; k-step ks flips bits 5..6
    const unsigned a_rd = aring_lds + l32 * 128 + ((half << 4) ^ (((l32 >> 1) & 7) << 4));
    // the two pixels of the tile this lane multiplies: row of the tile and column (rows beyond the tile's outputs multiply
    // pixel 0 again; nothing of them is stored)
    int nl[TN], dp[TN], qq[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        nl[j] = wave * 64 + j * 32 + l32;
        const int nn = nl[j] < a.THQ ? nl[j] : 0;
        dp[j] = (int)__umulhi((unsigned)nn, a.magic_q);
        qq[j] = nn - dp[j] * g.Q;
    }

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, a.w_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rbias = __builtin_amdgcn_make_buffer_rsrc((void*)a.bias, 0, a.bias ? g.K * 4 : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc((void*)a.y, 0, a.y_bytes, 0x00020000);

    // ---- persistent walk (tile_walk)
    const TileWalk walk = tile_walk(a.wk);
    const int mt = walk.mt, my_tiles = walk.count;
    const int nslices = a.nslices;

    if (my_tiles == 0) return;                          // (whole workgroup, before anything is in flight; the launcher leaves no such workgroup)

    int a_voff[A_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int m = mt * BM + i * 32 + lrow;
        a_voff[i] = m < g.K ? (m * a.Kg + lc * 8) * 2 : OOB;
    }
    if (wave * 64 < BM) {
        const int ml = wave * 64 + lane, m = mt * BM + ml;
        load_to_lds4(rbias, bias_lds + wave * 64, (ml < BM && m < g.K) ? m * 4 : OOB);
    }
    const int m_lane = mt * BM + half * 8;
    const unsigned bias_rd = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)bias_lds + (half * 8) * 4;
    if constexpr (TAIL) {
        // the 1x1 filters and their biases, once per workgroup (older than every other load, so the first wait covers them)
        const __amdgpu_buffer_rsrc_t rw2 = __builtin_amdgcn_make_buffer_rsrc((void*)a.w2, 0, a.w2_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rb2 = __builtin_amdgcn_make_buffer_rsrc((void*)a.bias2, 0, a.bias2 ? a.K2 * 4 : 0, 0x00020000);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m2 = i * 32 + lrow;
            load_to_lds16(rw2, w2s + i * 4096 + wave * 1024, (m2 < a.K2 && lc * 8 < g.K) ? (m2 * g.K + lc * 8) * 2 : OOB, 0);
        }
        if (wave * 64 < BM) load_to_lds4(rb2, bias2_lds + wave * 64, wave * 64 + lane < a.K2 ? (wave * 64 + lane) * 4 : OOB);
    }

    // ---- loaders
    int ld_i = 0;                                      // the next filter slice to load (the same cycle for every tile)
    auto issue_a = [&](int stage) __attribute__((always_inline)) {
        unsigned char* sa = aring + stage * A_BYTES + wave * 1024;
        const int soff = ld_i * 128;                   // slice ld_i starts 64 ld_i elements into a filter's row
        const bool cut = ld_i == nslices - 1 && lc >= a.tail_chunks;     // behind the end of the row: zeros
#pragma unroll
        for (int i = 0; i < A_PER; ++i) load_to_lds16(rw, sa + i * 4096, cut ? OOB : a_voff[i], soff);
        if (++ld_i == nslices) ld_i = 0;
    };
    // patch of the tile that starts at row p0 of image img0: chunk c of patch pixel pp goes to chunk pp NP + c; the lanes
    // on the padding chunk, on pixels outside the image (or behind the last image) and behind the patch fetch zeros
    auto issue_patch = [&](int img0, int p0) __attribute__((always_inline)) {
        if (a.packed) {
            // rows of the padded copy as they are: chunk cc of patch row prow is pixel pair cc of row row_mul p0 + prow
            for (int pass = 0; pass < a.passes; ++pass) {
                const int p = pass * 256 + tid;
                const int prow = (int)__umulhi((unsigned)p, a.magic_rc), cc = p - prow * a.row_chunks;
                const int pr = a.row_mul * p0 + prow;
                const int io = (int)__umulhi((unsigned)pr, a.magic_pr), img = img0 + io;
                const bool ok = prow < a.rows_max && img < g.N;
                const int voff = ok ? ((img * a.PR + (pr - io * a.PR)) * a.wp * 4 + cc * 8) * 2 : OOB;
                load_to_lds16(rx, patch + pass * 4096 + wave * 1024, voff, 0);
            }
            return;
        }
        for (int pass = 0; pass < a.passes; ++pass) {
            const int p = pass * 256 + tid;
            const int pp = (int)__umulhi((unsigned)p, a.magic_np), c = p - pp * a.NP;
            const int prow = (int)__umulhi((unsigned)pp, a.magic_pw), pcol = pp - prow * a.PW;
            const int pr = p0 + prow;
            const int io = (int)__umulhi((unsigned)pr, a.magic_pr);
            const int ih = pr - io * a.PR - g.ph, iw = pcol - g.pw, img = img0 + io;
            const bool ok = c < a.CCH && prow < a.rows_max && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W && img < g.N;
            const int voff = ok ? (((img * g.H + ih) * g.W + iw) * g.C + c * 8) * 2 : OOB;
            load_to_lds16(rx, patch + pass * 4096 + wave * 1024, voff, 0);
        }
    };

    // ---- operands: two register slots (k-step ks of a slice in slot ks & 1), each k-step fetched one step ahead of the
    // matrix cores
    f32x16 acc[TM][TN];
    u32x4 fa[2][TM], fb[2][TN];
    unsigned pb[TN];                                   // LDS address of this lane's chunk of tap (0, 0), channels 0..15, per pixel
    // patch offset of the k-steps in order: channels of a tap (32 bytes a step), next tap (the padding chunk), next filter row
    int ku = 0, kj = 0, ks_ = 0, koff = 0;
    auto next_off = [&]() __attribute__((always_inline)) {
        const int ret = ku < a.U ? koff : 0;            // (behind the last k-step the filters are zeros: any pixel will do)
        ++ku;
        koff += 32;
        if (++kj == a.J) {
            kj = 0;
            koff += a.tap_skip;
            if (++ks_ == a.taps_per_row) { ks_ = 0; koff += a.row_skip; }
        }
        return ret;
    };
    auto fetch = [&](int stage, int boff, auto ks_c) __attribute__((always_inline)) {
        constexpr int KS = decltype(ks_c)::value, SL = KS & 1;
        const unsigned pa = (a_rd + stage * A_BYTES) ^ (KS * 32);
        fa[SL][0] = ds_read16<0>(pa);
        if constexpr (TM > 1) fa[SL][1] = ds_read16<4096>(pa);
        if constexpr (TM > 2) fa[SL][2] = ds_read16<8192>(pa);
        if constexpr (TM > 3) fa[SL][3] = ds_read16<12288>(pa);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[SL][j] = ds_read16<0>(pb[j] + (unsigned)boff);
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

    // ---- pipeline.  Filter slice k lives in ring stage k & 1.  Memory operations of a wave, in issue order, around a tile
    // boundary: ... filter slices of tile t | patch of tile t + 1, its filter slices 0 and 1 | the E stores of tile t | filter
    // slice 2 of tile t + 1 ...  Loads return in order, so "at most n operations outstanding" with n the number issued after
    // the awaited load means that load has landed; the stores only ever make such a wait longer.
    auto tile_origin = [&](int tt, int& img0, int& p0) __attribute__((always_inline)) {
        const int g0 = tt * a.TH;
        img0 = (int)__umulhi((unsigned)g0, a.magic_p);
        p0 = g0 - img0 * g.P;
    };
    int img0, p0;
    tile_origin(walk.tile(0), img0, p0);
    issue_patch(img0, p0);
    issue_a(0);
    if (nslices > 1) issue_a(1);
    int gi = 0;
    for (int t = 0; t < my_tiles; ++t) {
        const int tt = walk.tile(t);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int io = (int)__umulhi((unsigned)(p0 + dp[j]), a.magic_p);
            pb[j] = patch_lds + (unsigned)((a.row_mul * dp[j] + io * a.D) * a.row_chunks + qq[j] * a.px_chunks + half) * 16u;
        }
        ku = 0; kj = 0; ks_ = 0; koff = 0;
        // the patch and the first filter slice have landed: behind them are filter slice 1 and, from the second tile on, the stores
        if (nslices > 1) {
            if (t > 0) wait_vmcnt<A_PER + E>();
            else wait_vmcnt<A_PER>();
        } else {
            if (t > 0) wait_vmcnt<E>();
            else wait_vmcnt<0>();
        }
        ring_barrier();
        fetch(gi & 1, next_off(), IC<0>{});
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        for (int sl = 0; sl < nslices; ++sl, ++gi) {
            const int stage = gi & 1;
            const bool more = sl + 1 < nslices;          // (wave-uniform) the tile has another slice
            constexpr int PEND = TM + TN;                // the reads of the step just requested may be pending
            fetch(stage, next_off(), IC<1>{});
            multiply(IC<0>{}, IC<PEND>{});
            fetch(stage, next_off(), IC<2>{});
            multiply(IC<1>{}, IC<PEND>{});
            fetch(stage, next_off(), IC<3>{});
            multiply(IC<2>{}, IC<PEND>{});
            // (the matrix instructions stay on one path through the loop: in two arms of a branch the compiler gives them two
            // register sets and copies all accumulators between them)
            if (more) {
                // filter slice gi + 1 has landed: nothing was issued behind it but, right after a tile boundary, the stores
                if (sl == 0 && t > 0) wait_vmcnt<E>();
                else wait_vmcnt<0>();
                ring_barrier();                          // ... and everybody has read slice gi out of its stage (its last step has arrived too)
                if (sl + 2 < nslices) issue_a(stage);
                fetch(stage ^ 1, next_off(), IC<0>{});
            } else {
                wait_lgkm<0>();
            }
            multiply(IC<3>{}, IC<PEND>{});
        }
        const int nfirst = tt * a.THQ;                   // (a tile is TH whole rows of the stack: its outputs are consecutive)
        if (t + 1 < my_tiles) {
            ring_barrier();                              // everybody has read the patch and both filter stages for the last time
            tile_origin(walk.tile(t + 1), img0, p0);
            issue_patch(img0, p0);
            issue_a(gi & 1);
            if (nslices > 1) issue_a((gi & 1) ^ 1);
        }
        int nbase[TN];
        bool n_ok[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            n_ok[j] = nl[j] < a.THQ && nfirst + nl[j] < g.Ng;
            nbase[j] = ((nfirst + nl[j]) * g.y_ctot + g.y_coff) * 2;
        }
        if constexpr (TAIL) {
            u32x4 hk[TN][2 * TM];
            pack_blocks<TM, TN>(acc, bias_rd, g.relu, hk);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
            const unsigned w2_rd = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)w2s + l32 * 128 +
                                   ((half << 4) ^ (((l32 >> 1) & 7) << 4));
#pragma unroll
            for (int ks = 0; ks < 2 * TM; ++ks) {
                // k-step ks of the 1x1 filters: chunk 2 ks + h of a row, i.e. bits 5.. of the unswizzled offset
                u32x4 f2[TM];
#pragma unroll
                for (int i = 0; i < TM; ++i) f2[i] = ds_read16<0>((w2_rd + i * 4096) ^ (ks * 32));
                wait_lgkm<0>();
#pragma unroll
                for (int i = 0; i < TM; ++i) touch(f2[i]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f2[i]),
                                                                            __builtin_bit_cast(bf16x8, hk[j][ks]), acc[i][j], 0, 0, 0);
            }
            const unsigned bias2_rd = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)bias2_lds + (half * 8) * 4;
            store_blocks<TM, TN>(acc, bias2_rd, half * 8, a.K2, a.relu2, ry, nbase, n_ok);
        } else {
            store_blocks<TM, TN>(acc, bias_rd, m_lane, g.K, g.relu, ry, nbase, n_ok);
        }
    }
    wait_lgkm<0>();
}

constexpr int LDS_PER_CU = 160 * 1024;

template <int TM, int OCC, bool TAIL = false>
int launch_rows(RArgs a, int patch_bytes, hipStream_t st)
{
    constexpr int BM = TM * 32;
    a.grid_m = (a.g.K + BM - 1) / BM;
    int gn = device_cus() * OCC / a.grid_m;
    if (gn < 1) gn = 1;
    if (gn > a.tiles) gn = a.tiles;
    // the kernel's dynamic LDS limit, once per device (benign race: every thread stores the same value)
    constexpr int MAX_DEV = 64;
    static std::atomic<bool> sized[MAX_DEV];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return fail(DR_ERR_HIP, "conv_bf16_rows: no current device");
    if (!sized[dev].load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute((const void*)conv_bf16_rows_kernel<TM, OCC, TAIL>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_PER_CU / 2) != hipSuccess)
            return fail(DR_ERR_HIP, "conv_bf16_rows: cannot size the patch");
        sized[dev].store(true, std::memory_order_relaxed);
    }
    a.wk = make_walk(a.grid_m, gn, a.tiles);
    hipLaunchKernelGGL((conv_bf16_rows_kernel<TM, OCC, TAIL>), dim3((unsigned)(gn * a.grid_m)), dim3(256), (size_t)patch_bytes, st, a);
    return check_launch("conv_bf16_rows");
}

struct RowsPlan {
    int tm, occ, TH, rows_max, NP, patch_bytes;
};

// Filter block, rows per tile and patch size; false when the layer is not for this kernel.
bool rows_plan(const ConvGeom& g, RowsPlan& pl)
{
    if (!g.nhwc || !g.w_krsc || g.C % 16 != 0 || g.C > 64 || g.K % 8 != 0 || g.sh != 1 || g.sw != 1 || g.R * g.S < 2 || g.R > 7 || g.S > 7) return false;
    if (g.P < 2 || g.Q < 2 || g.Q > ROWS_BN || g.P > 32768 || (double)g.N * g.P * g.P >= 4294967296.0 || g.res_ctot) return false;
    const int pad96 = (g.K + 95) / 96 * 96, pad64 = (g.K + 63) / 64 * 64;
    pl.tm = pad96 <= pad64 ? 3 : 2;
    pl.NP = g.C / 8 + 1;
    const int PW = g.W + 2 * g.pw;
    // two workgroups per compute unit: ring, biases and 1 KiB to spare taken off each half
    const int budget = LDS_PER_CU / 2 - (2 * pl.tm * 32 * 128 + 512 + 1024);
    long long stack = (long long)g.N * g.P;
    int th = ROWS_BN / g.Q;
    if (th > stack) th = (int)stack;
    for (; th >= 1; --th) {
        int segs = (th + g.P - 2) / g.P + 1;             // images a tile of th stacked rows can touch
        if (segs > g.N) segs = g.N;
        pl.rows_max = th + (g.R - 1) * segs;
        pl.patch_bytes = (pl.rows_max * PW * pl.NP * 16 + 4095) / 4096 * 4096;
        if (pl.patch_bytes <= budget) break;
    }
    pl.TH = th;
    // worth it when most of the 256 pixel rows carry outputs and there are tiles for a quarter of the compute units at least
    // (layers with fewer go to the streaming kernel and its smaller tiles)
    if (th < 1 || th * g.Q * 4 < ROWS_BN * 3) return false;
    const long long tiles = (stack + th - 1) / th, blocks = (g.K + pl.tm * 32 - 1) / (pl.tm * 32);
    if (tiles * blocks * 4 < device_cus()) return false;
    // a third (fourth) workgroup per compute unit where LDS and registers (64-filter blocks) have room and there are tiles for it
    const int per_wg = 2 * pl.tm * 32 * 128 + 512 + 1024 + pl.patch_bytes;
    pl.occ = 2;
    if (3 * per_wg <= LDS_PER_CU && tiles * blocks > 2 * device_cus()) pl.occ = 3;
    if (pl.tm == 2 && 4 * per_wg <= LDS_PER_CU && tiles * blocks > 3 * device_cus()) pl.occ = 4;
    return true;
}

unsigned magic(int d) { return (unsigned)((0x100000000ull + (unsigned)d - 1) / (unsigned)d); }

// Rows per tile, patch rows and bytes for the padded 4-channel copy; false when the layer is not for this kernel.
// (tail: a 1x1 convolution of K2 filters follows in the same kernel, see the kernel's TAIL)
bool stem_plan(const ConvGeom& g, int hp, int wp, RowsPlan& pl, const RowsTail* tail = nullptr)
{
    if (tail && (g.K > 64 || tail->K2 > 64 || tail->K2 < 8 || tail->K2 % 8 != 0 || !tail->w2 || ((uintptr_t)tail->w2 & 15))) return false;
    const int extra = tail ? 64 * 128 + 512 : 0;         // the 1x1 filters and biases in LDS
    if (!g.nhwc || g.C > 4 || g.R > 8 || g.S > 8 || g.sw % 2 != 0 || g.sw > 8 || g.sh < 1 || g.K % 8 != 0 || g.res_ctot) return false;
    if (g.P < 2 || g.Q < 2 || g.Q > ROWS_BN || wp % 8 != 0 || hp < (g.P - 1) * g.sh + 8 || wp < (g.Q - 1) * g.sw + 8) return false;
    if (hp > 32768 || (double)g.N * hp * hp >= 4294967296.0 || (double)g.N * g.P * g.P >= 4294967296.0) return false;
    const int pad96 = (g.K + 95) / 96 * 96, pad64 = (g.K + 63) / 64 * 64;
    pl.tm = pad96 <= pad64 ? 3 : 2;
    pl.NP = 0;
    if (tail) pl.tm = 2;
    const int budget = LDS_PER_CU / 2 - (2 * pl.tm * 32 * 128 + 512 + 1024) - extra;
    const long long stack = (long long)g.N * g.P;
    int th = ROWS_BN / g.Q;
    if (th > stack) th = (int)stack;
    for (; th >= 1; --th) {
        int segs = g.P % th == 0 ? 1 : (th + g.P - 2) / g.P + 1;
        if (segs > g.N) segs = g.N;
        pl.rows_max = g.sh * (th - 1) + (segs - 1) * (hp - g.sh * g.P) + 8;
        pl.patch_bytes = (pl.rows_max * (wp / 2) * 16 + 4095) / 4096 * 4096;
        if (pl.patch_bytes <= budget) break;
    }
    pl.TH = th;
    if (th < 1 || th * g.Q * 4 < ROWS_BN * 3) return false;
    const long long tiles = (stack + th - 1) / th, blocks = (g.K + pl.tm * 32 - 1) / (pl.tm * 32);
    if (tiles * blocks * 4 < device_cus()) return false;
    const int per_wg = 2 * pl.tm * 32 * 128 + 512 + 1024 + pl.patch_bytes + extra;
    pl.occ = 2;
    if (3 * per_wg <= LDS_PER_CU && tiles * blocks > 2 * device_cus()) pl.occ = 3;
    if (pl.tm == 2 && !tail && 4 * per_wg <= LDS_PER_CU && tiles * blocks > 3 * device_cus()) pl.occ = 4;
    return true;
}

}  // namespace

bool conv_bf16_rows_eligible(const ConvGeom& g, const void* x, const void* w, const void* y)
{
    const double xb = (double)g.N * g.C * g.H * g.W * 2.0, wb = (double)g.K * g.Kg * 2.0, yb = (double)g.Ng * g.y_ctot * 2.0;
    if (xb >= 2147483648.0 || wb >= 2147483648.0 || yb >= 2147483648.0 || g.Ng >= (1 << 24)) return false;
    if (((uintptr_t)x & 15) || ((uintptr_t)w & 15) || ((uintptr_t)y & 15) || g.y_ctot % 8 != 0 || g.y_coff % 8 != 0) return false;
    RowsPlan pl;
    return rows_plan(g, pl);
}

int launch_conv_bf16_rows(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, uint16_t* y, hipStream_t st)
{
    RowsPlan pl;
    if (!rows_plan(g, pl)) return fail(DR_ERR_UNSUPPORTED, "conv_bf16_rows: layer not eligible");
    RArgs a{};
    a.x = x; a.w = w; a.bias = bias; a.y = y; a.g = g;
    a.x_bytes = (int)((size_t)g.N * g.C * g.H * g.W * 2);
    a.w_bytes = (int)((size_t)g.K * g.Kg * 2);
    a.y_bytes = (int)((size_t)g.Ng * g.y_ctot * 2);
    a.TH = pl.TH;
    a.THQ = pl.TH * g.Q;
    a.tiles = (int)(((long long)g.N * g.P + pl.TH - 1) / pl.TH);
    a.PW = g.W + 2 * g.pw;
    a.NP = pl.NP; a.CCH = g.C / 8; a.J = g.C / 16;
    a.PR = g.P + g.R - 1;
    a.rows_max = pl.rows_max;
    a.passes = pl.patch_bytes / 4096;
    a.U = g.Kg / 16;
    a.nslices = (a.U + 3) / 4;
    a.tail_chunks = g.Kg / 8 - 8 * (a.nslices - 1);
    a.Kg = g.Kg;
    a.taps_per_row = g.S;
    a.tap_skip = 16;                                     // over the padding chunk
    a.row_skip = (a.PW - g.S) * a.NP * 16;
    a.row_mul = 1; a.D = g.R - 1;
    a.row_chunks = a.PW * a.NP; a.px_chunks = a.NP;
    a.packed = 0; a.wp = 0;
    a.magic_np = magic(a.NP); a.magic_pw = magic(a.PW); a.magic_q = magic(g.Q); a.magic_p = magic(g.P); a.magic_pr = magic(a.PR);
    a.magic_rc = magic(a.row_chunks);
    if (pl.tm == 3) return pl.occ == 3 ? launch_rows<3, 3>(a, pl.patch_bytes, st) : launch_rows<3, 2>(a, pl.patch_bytes, st);
    return pl.occ == 4 ? launch_rows<2, 4>(a, pl.patch_bytes, st) : pl.occ == 3 ? launch_rows<2, 3>(a, pl.patch_bytes, st) : launch_rows<2, 2>(a, pl.patch_bytes, st);
}

// The network's first layer (3 channels): the input is the padded 4-channel copy xp[N][hp][wp][4] (one pixel is 8 bytes, a
// 16-byte chunk a pixel pair; wp a multiple of 8, the padding in place) and the filters are wp8[K][8][8][4] with zeros
// beyond R, S, C, as for the streaming kernel's form of this layer.  A window row is 8 taps x 4 channels = two k-steps of
// consecutive chunks, so the patch needs neither a pixel pitch nor padding chunks: its rows are the copy's rows as they
// are, the window of output pixel q starts stride_w / 2 chunks after that of pixel q - 1 (lanes read consecutive chunks),
// and the k-steps walk two chunks along a row and then one row down.  Per tile the loads are the rows under the tile once
// (10 rows of 116 chunks for two output rows of 112 at stride 2) instead of 128 bytes per output pixel and slice.
//
// tail (may be NULL): a 1x1 convolution on the layer's output (stride 1, no padding, K2 <= 64 filters over the layer's
// K <= 64) computed in the same kernel; g.y_ctot / g.y_coff and y then describe the 1x1 convolution's destination.
bool conv_bf16_rows_stem_eligible(const ConvGeom& g, int hp, int wp, const void* xp, const void* y, const RowsTail* tail)
{
    const double xb = (double)g.N * hp * wp * 8.0, yb = (double)g.Ng * g.y_ctot * 2.0;
    if (xb >= 2147483648.0 || yb >= 2147483648.0 || g.Ng >= (1 << 24)) return false;
    if (((uintptr_t)xp & 15) || ((uintptr_t)y & 15) || g.y_ctot % 8 != 0 || g.y_coff % 8 != 0) return false;
    RowsPlan pl;
    return stem_plan(g, hp, wp, pl, tail);
}

int launch_conv_bf16_rows_stem(const ConvGeom& g, const uint16_t* xp, int hp, int wp, const uint16_t* wp8, const float* bias, uint16_t* y,
                               hipStream_t st, const RowsTail* tail)
{
    // (with a tail the trace gets two records: this layer with its input and filters as bytes, the 1x1 convolution -- no
    // time of its own -- with its filters and its output)
    const long long in_bytes = (long long)g.N * g.C * g.H * g.W * 2 + (long long)g.K * g.Kg * 2;
    TraceScope trace("conv_bf16", &g, g.Ng, st, tail ? in_bytes : 0);
    RowsPlan pl;
    if (!stem_plan(g, hp, wp, pl, tail)) return fail(DR_ERR_UNSUPPORTED, "conv_bf16_rows: layer not eligible");
    RArgs a{};
    a.x = xp; a.w = wp8; a.bias = bias; a.y = y; a.g = g;
    a.x_bytes = (int)((size_t)g.N * hp * wp * 8);
    a.w_bytes = (int)((size_t)g.K * 256 * 2);
    a.y_bytes = (int)((size_t)g.Ng * g.y_ctot * 2);
    a.TH = pl.TH;
    a.THQ = pl.TH * g.Q;
    a.tiles = (int)(((long long)g.N * g.P + pl.TH - 1) / pl.TH);
    a.PW = wp; a.NP = 1; a.CCH = 1; a.J = 2;
    a.PR = hp;
    a.rows_max = pl.rows_max;
    a.passes = pl.patch_bytes / 4096;
    a.U = 16; a.nslices = 4; a.tail_chunks = 8;
    a.Kg = 256;
    a.taps_per_row = 1;
    a.row_chunks = wp / 2; a.px_chunks = g.sw / 2;
    a.tap_skip = a.row_chunks * 16 - 64;                 // from behind a window row's 64 bytes to the next row's window
    a.row_skip = 0;
    a.row_mul = g.sh; a.D = hp - g.sh * g.P;
    a.packed = 1; a.wp = wp;
    a.magic_np = magic(1 + 1); a.magic_pw = magic(wp); a.magic_q = magic(g.Q); a.magic_p = magic(g.P); a.magic_pr = magic(hp);
    a.magic_rc = magic(a.row_chunks);
    if (tail) {
        a.w2 = tail->w2; a.bias2 = tail->bias2; a.K2 = tail->K2; a.relu2 = tail->relu2;
        a.w2_bytes = tail->K2 * g.K * 2;
        const int rc = pl.occ == 3 ? launch_rows<2, 3, true>(a, pl.patch_bytes, st) : launch_rows<2, 2, true>(a, pl.patch_bytes, st);
        if (rc == DR_OK) {
            ConvGeom g2 = g;
            g2.C = g.K; g2.K = tail->K2; g2.R = g2.S = 1; g2.sh = g2.sw = 1; g2.ph = g2.pw = 0; g2.H = g.P; g2.W = g.Q; g2.Kg = g.K;
            g2.relu = tail->relu2; g2.c_logical = 0;
            TraceScope second("conv_bf16", &g2, g.Ng, st, (long long)g.Ng * tail->K2 * 2 + (long long)tail->K2 * g.K * 2);
        }
        return rc;
    }
    if (pl.tm == 3) return pl.occ == 3 ? launch_rows<3, 3>(a, pl.patch_bytes, st) : launch_rows<3, 2>(a, pl.patch_bytes, st);
    return pl.occ == 4 ? launch_rows<2, 4>(a, pl.patch_bytes, st) : pl.occ == 3 ? launch_rows<2, 3>(a, pl.patch_bytes, st) : launch_rows<2, 2>(a, pl.patch_bytes, st);
}

}  // namespace dr
