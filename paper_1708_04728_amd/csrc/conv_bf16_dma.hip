// bf16 convolution forward (Eq. (7): Y_j = (W * X)_j + B_j), the main kernel: channels-last (NHWC)
// activations, KRSC filters, fp32 accumulation on the gfx950 matrix cores, operands streamed from
// global memory straight into LDS.
//
//   D[m][n] = sum_k A[m][k] * B[k][n]     m = output channel, n = (image, p, q), k = (r, s, c)
//
// Contraction order.  For a fixed filter row r the S*C values (s, c) of the filters are contiguous in
// KRSC memory, and so are the S*C activations x[img][ih0 + r][iw0 .. iw0 + S - 1][0 .. C - 1] that they
// multiply.  The kernel walks k as R such runs, 64 elements (eight 16-byte chunks) per slice; a chunk
// never straddles a pixel because C is a multiple of 8.  Lanes whose chunk lies in the zero padding,
// beyond the end of the run, or in a row / filter beyond the tensor get a buffer offset outside
// the descriptor's range: the hardware then delivers zeros, so the loop has no branches.
//   TAP = true  (C % 64 == 0): a slice lies inside one tap, the padding test is wave-uniform per
//        tap and is hoisted out of the slice loop; only a scalar offset moves from slice to slice.
//   TAP = false: the tap of a lane's chunk differs from lane to lane; it is looked up per slice in
//        per-row validity bit masks (a few vector-ALU instructions per load).  When a row's run is not a
//        multiple of 64 elements, the last slice of every row would be partly empty (S * C = 80: 2
//        slices for 1.25); with `flat` set the slices instead run on into the next filter row - the
//        filters of row r + 1 follow those of row r in KRSC memory, and a lane whose chunk has
//        wrapped takes the next row's address and verdict - so that only the tile's last slice is
//        ragged (5x5 filters on 16 channels: 7 slices instead of 10, on 32 channels 13 instead of 15).
//
// Data movement.  Every operand chunk is fetched by a 16-byte buffer load that writes LDS directly
// (no register staging): lane l of a wave fills slot l of a 1 KiB block, i.e. 8 rows x 8 chunks of a
// 128-byte-per-row tile.  Which chunk of its row a lane fetches is permuted (chunk ^ ((row >> 1) & 7))
// so that the MFMA operand reads (32 rows x one 16-byte chunk per half-wave) hit all 64 banks evenly.
// The tiles live in a ring of NS stages; loads run NS - 1 slices ahead of the matrix cores, across
// tile boundaries: a workgroup is persistent, keeps one block of output channels and walks pixel
// tiles nt, nt + stride, ... so that the store of one tile overlaps the loads of the next.  One barrier
// per slice.  The compiler makes every LDS read it knows of wait for ALL outstanding loads that write
// LDS, which would empty the ring once per slice; the operand reads are therefore issued as inline
// assembly with their own lgkmcnt waits, and the bias is copied from LDS into registers once.
//
// Store.  Accumulator register v of a 32x32 tile holds row 8 (v / 4) + 4 half + v % 4 of column
// lane % 32.  One v_permlane32_swap per register pair gives every lane 8 consecutive output channels
// of its pixel; bias, residual and ReLU are applied in fp32, the result is rounded to bf16 (nearest
// even) once and written as one 16-byte store.
#include <type_traits>

#include "dr_internal.h"
#include "dr_store.h"
#include "conv_bf16_dev.h"

namespace dr {
namespace {

struct DArgs {
    const uint16_t* x;
    const uint16_t* w;
    const float* bias;
    const uint16_t* res;
    uint16_t* y;
    ConvGeom g;
    int grid_m, grid_n;       // tiles along m (channel blocks) and along n (pixel tiles)
    WalkArgs wk;              // the persistent walk over them (tile_walk)
    int x_bytes, w_bytes;
    int c8;                   // C / 8: chunks per tap
    int run_chunks;           // S * C / 8: chunks per filter row
    int slices_per_run;       // ceil(run_chunks / 8)
    int slices_per_tile;      // slices of one tile's contraction: R * slices_per_run, fewer when `flat`
    int flat;                 // TAP = false only: slices run on from one filter row into the next (see the header)
    unsigned magic_c8;        // ceil(2^32 / c8)
    unsigned long long m_pq, m_q;   // ceil(2^40 / (P*Q)), ceil(2^40 / Q)
    int vec_ok;               // 16-byte stores / bias / residual accesses are aligned
    int exact_store;          // every lane issues each of a tile's stores (lanes without an output store out of range): see the epilogue
    int y_bytes;              // bytes of the output tensor (exact_store only: below 2^31)
    int pointwise;            // 1x1 filter, stride 1, no padding
    int step_img, step_p, step_q;   // the pixels one pass of loads covers (8 per wave) as (images, rows, columns) of the output
    int stem_hp, stem_wp;     // rows / pixels per row of the padded 4-channel input copy (0: ordinary input)
    // Stacked convolution (several filter banks on one input, Eq. (12)) whose channel ranges go to different
    // tensors: channel m < split_end[0] goes to destination 0, m < split_end[1] to destination 1, ...
    // (unused ends hold INT_MAX).  y_seg[d] is offset by the host so that channel m of pixel n lands at
    // y_seg[d][n * ctot_seg[d] + m]; every range starts at a multiple of 8.  nsplit <= 1: everything goes to y.
    int nsplit;
    int split_end[3];
    uint16_t* y_seg[4];
    int ctot_seg[4];
    // Block kernel (FUSE): the convolution's output never leaves the compute unit; what is stored is
    // maxpool3x3s2(lrn5(relu(conv))), f_PP x f_QQ pixels per image, at channel f_coff of a tensor with f_ctot channels.
    // A workgroup owns all filters of a patch of FUSE_SIDE x FUSE_SIDE convolution pixels (f_ty x f_tx patches per image).
    int f_ty, f_tx, f_PP, f_QQ, f_ctot, f_coff, f_b075;
    float f_a_over_n, f_beta, f_k;
    uint16_t* f_y;
};

// Block kernel: pooled outputs per patch side, and the convolution pixels they need (3x3 windows at stride 2)
constexpr int FUSE_POOLED = 7, FUSE_SIDE = 2 * FUSE_POOLED + 1, FUSE_PIXELS = FUSE_SIDE * FUSE_SIDE;
constexpr int FUSE_PITCH = 400;     // bytes per staged pixel: 192 channels of bf16 + 16, so that 16 consecutive pixels cover every bank

// A workgroup is WGM x WGN waves (4 or 8), each with a tile of TM x TN blocks of 32 x 32.  OCC: workgroups per
// compute unit the register allocation must leave room for (512 / (OCC * waves / 4) registers per lane).
// KB: contraction elements per slice, 64 (LDS rows of 128 bytes, 8 chunks) or 32 (rows of 64 bytes, 4 chunks).  Half-depth
// slices halve a stage, so that a wider tile keeps a ring of three or four stages at two workgroups per compute unit.
// FUSE: the block kernel (Sec. 3.1, the streamlined block's original form in one pass): one patch of FUSE_SIDE x FUSE_SIDE
// convolution pixels x all filters per workgroup; bias + ReLU, then the tile is laid down in LDS as bf16 (the precision
// the layer-by-layer form stores it in), normalised across channels in place, and pooled from there.
template <int TM, int TN, int WGM, int WGN, int NS, bool TAP, int OCC, int KB = 64, bool FUSE = false>
__global__ __launch_bounds__(WGM * WGN * 64) __attribute__((amdgpu_waves_per_eu(OCC * WGM * WGN / 4, OCC * WGM * WGN / 4)))
void conv_bf16_dma_kernel(const DArgs a)
{
    constexpr int RB = KB * 2, CPR = KB / 8, RPB = 1024 / RB;            // bytes and chunks per LDS row; rows per 1 KiB load block
    constexpr int WAVES = WGM * WGN, RP = WAVES * RPB;                   // rows one pass of loads covers
    constexpr int WM = TM * 32, WN = TN * 32, BM = WGM * WM, BN = WGN * WN;
    // loads per lane and slice; a filter block that is not a whole number of passes is padded (the extra rows fetch nothing)
    constexpr int A_PER = (BM + RP - 1) / RP, B_PER = BN / RP, L = A_PER + B_PER;
    constexpr int A_BYTES = A_PER * RP * RB, STAGE = A_BYTES + BN * RB, PASS = RP * RB;
    constexpr int KSTEPS = KB / 16;                                      // matrix-instruction steps per slice
    static_assert((KB == 64 || KB == 32) && (WAVES == 4 || WAVES == 8) && (BM % RP == 0 || KB == 32) && BN % RP == 0 && NS >= 2 &&
                  (NS - 1) * L < 63 && BM <= 256, "bad configuration");
    static_assert(!FUSE || (BN >= FUSE_PIXELS && BM * 2 + 16 <= FUSE_PITCH && FUSE_PIXELS * FUSE_PITCH <= NS * STAGE && KB == 64), "block kernel tile");

    __shared__ __attribute__((aligned(1024))) unsigned char ring[NS * STAGE];
    __shared__ __attribute__((aligned(1024))) float bias_lds[256];
    const unsigned ring_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;

    const ConvGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int half = lane >> 5, l32 = lane & 31;
    const int PQ = g.P * g.Q;

    // Chunk j of row r is stored at chunk j ^ swz(r): 16 consecutive rows then cover every bank once, for the loads'
    // writes as for the operand reads.  (Rows of 128 bytes: two rows per 256 bytes; rows of 64 bytes: four.)
    auto swz = [](int r) { return KB == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3); };
    // loader: this lane fetches row lrow of every RP-row group, logical chunk lc of the slice
    const int lrow = wave * RPB + lane / CPR;
    const int lc = (lane % CPR) ^ swz(lrow);
    // reader: LDS byte offset of this lane's operand chunk for k-step 0; k-step ks flips bits 5 (and 6)
    const int lane_x = (half << 4) ^ (swz(l32) << 4);
    const unsigned a_rd = ring_lds + (wm * WM + l32) * RB + lane_x;
    const unsigned b_rd = ring_lds + A_BYTES + (wn * WN + l32) * RB + lane_x;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, a.w_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rbias = __builtin_amdgcn_make_buffer_rsrc((void*)a.bias, 0, a.bias ? g.K * 4 : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc((void*)a.y, 0, a.exact_store ? a.y_bytes : 0, 0x00020000);

    // ---- persistent walk (tile_walk)
    const TileWalk walk = tile_walk(a.wk);
    const int mt = walk.mt, my_tiles = walk.count;
    const int nslices = a.slices_per_tile;
    const int total = my_tiles * nslices;

    // ---- per-lane constants of the channel block: filter offsets for the loader, bias for the store
    int a_voff[A_PER];            // byte offset of (filter m, chunk lc) or OOB
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int ml = i * RP + lrow, m = mt * BM + ml;
        a_voff[i] = (ml < BM && m < g.K) ? (m * g.Kg + lc * 8) * 2 : OOB;
    }
    // The bias of the channel block travels like the operands, ahead of them: 4 bytes per lane straight
    // into LDS (zeros beyond the last filter and without a bias), so that nothing in the prologue waits
    // for a load of its own.  After the first barrier every lane copies its share into registers.
    if (wave * 64 < BM) {
        const int ml = wave * 64 + lane, m = mt * BM + ml;
        load_to_lds4(rbias, bias_lds + wave * 64, (ml < BM && m < g.K) ? m * 4 : OOB);
    }
    // after the store's lane exchange a lane owns channels mb .. mb + 7, mb = m_lane + 32 i + 16 qp
    const int m_lane = mt * BM + wm * WM + half * 8;
    const unsigned bias_rd = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)bias_lds + (wm * WM + half * 8) * 4;

    // ---- loader state of the pixel tile being fetched
    int b_base[B_PER];            // byte offset of x[img][ih0][iw0][lc * 8] (may lie outside the tensor)
    unsigned b_mask[B_PER];       // bits 0..15: tap s is OUTSIDE the image row; bits 16..31: filter row r is inside
    unsigned b_cur[B_PER];        // TAP: offset of the current tap or OOB;  else: b_mask with the current row's verdict
    int ld_t = 0, ld_nt = walk.tile(0), ld_r = 0, ld_j0 = 0, ld_s = 0, ld_c = 0;   // wave-uniform cursor of the next slice to load
    int ld_fresh = 1;             // TAP = false: the cursor has entered a new filter row (its verdicts are due)

    // Per-lane state of pixel tile nt.  A 1x1 filter at stride 1 without padding reads input pixel n for
    // output pixel n: no decoding.  Otherwise the first fetched pixel is decoded into (image, p, q) by
    // exact division and the others follow by stepping RP pixels at a time (RP = step_img P Q + step_p Q +
    // step_q, so each coordinate wraps at most once per step).
    auto tile_setup = [&](int nt) __attribute__((always_inline)) {
        const int n_first = nt * BN + lrow;
        if constexpr (FUSE) {
            // row t of the tile is pixel (t / SIDE, t % SIDE) of patch (ty, tx) of image img; patches overlap by one row / column
            const int per_img = a.f_ty * a.f_tx;
            const int img = nt / per_img, rem = nt - img * per_img, ty = rem / a.f_tx, tx = rem - ty * a.f_tx;
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int t = lrow + i * RP, dy = t / FUSE_SIDE, dx = t - dy * FUSE_SIDE;
                const int p = ty * (FUSE_SIDE - 1) + dy, q = tx * (FUSE_SIDE - 1) + dx;
                const bool valid = t < FUSE_PIXELS && p < g.P && q < g.Q && img < g.N;
                const int ih0 = p * g.sh - g.ph, iw0 = q * g.sw - g.pw;
                b_base[i] = valid ? (((img * g.H + ih0) * g.W + iw0) * g.C + lc * 8) * 2 : 0;
                const unsigned wv = bit_range(max(0, -iw0), min(g.S - 1, g.W - 1 - iw0));
                const unsigned hv = valid ? bit_range(max(0, -ih0), min(g.R - 1, g.H - 1 - ih0)) : 0u;
                b_mask[i] = (~wv & 0xFFFFu) | (hv << 16);
            }
            return;
        }
        if (a.pointwise) {
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int n = n_first + i * RP;
                b_base[i] = (n * g.C + lc * 8) * 2;
                b_mask[i] = n < g.Ng ? 0x1FFFEu : 0xFFFFu;
            }
            return;
        }
        int img = div_small(n_first < g.Ng ? n_first : 0, a.m_pq);
        int pix = (n_first < g.Ng ? n_first : 0) - img * PQ;
        int p = div_small(pix, a.m_q), q = pix - p * g.Q;
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int n = n_first + i * RP;
            if (a.stem_wp) {
                // packed small-channel input (see launch_conv_bf16_stem): chunk lc of a slice is pixel pair lc & 3 of
                // window row lc >> 2; nothing is ever outside the padded copy
                b_base[i] = ((img * a.stem_hp + p * g.sh + (lc >> 2)) * a.stem_wp + q * g.sw + 2 * (lc & 3)) * 8;
                b_mask[i] = n < g.Ng ? 0xFFFFFEu : 0xFFFFu;          // (every "filter row", at most 8, is inside)
            } else {
                const int ih0 = p * g.sh - g.ph, iw0 = q * g.sw - g.pw;
                b_base[i] = (((img * g.H + ih0) * g.W + iw0) * g.C + lc * 8) * 2;
                const unsigned wv = bit_range(max(0, -iw0), min(g.S - 1, g.W - 1 - iw0));
                const unsigned hv = n < g.Ng ? bit_range(max(0, -ih0), min(g.R - 1, g.H - 1 - ih0)) : 0u;   // no row of a pixel beyond the tensor
                b_mask[i] = (~wv & 0xFFFFu) | (hv << 16);
            }
            q += a.step_q;
            if (q >= g.Q) { q -= g.Q; ++p; }
            p += a.step_p;
            if (p >= g.P) { p -= g.P; ++img; }
            img += a.step_img;
        }
    };
    auto row_setup = [&]() __attribute__((always_inline)) {      // TAP = false: verdict of filter row ld_r for every fetched pixel
#pragma unroll
        for (int i = 0; i < B_PER; ++i) b_cur[i] = ((b_mask[i] >> (16 + ld_r)) & 1u) ? (b_mask[i] | 0xFFFF0000u) : 0xFFFFFFFFu;
    };
    auto tap_setup = [&]() __attribute__((always_inline)) {      // TAP = true: offsets of tap (ld_r, ld_s)
        const int tap_off = (ld_r * g.W + ld_s) * g.C * 2;
        const unsigned want = 1u << (16 + ld_r), sel = want | (1u << ld_s);
#pragma unroll
        for (int i = 0; i < B_PER; ++i) b_cur[i] = (b_mask[i] & sel) == want ? (unsigned)(b_base[i] + tap_off) : (unsigned)OOB;
    };

    auto issue_slice = [&](int stage) __attribute__((always_inline)) {
        unsigned char* sa = ring + stage * STAGE + wave * 1024;
        unsigned char* sb = sa + A_BYTES;
        if constexpr (TAP) {
            if (ld_c == 0) tap_setup();
            const int soff_a = ((ld_r * g.S + ld_s) * a.c8 + ld_c) * 16;
            const int soff_b = ld_c * 16;
#pragma unroll
            for (int i = 0; i < A_PER; ++i)
                load_to_lds16(rw, sa + i * PASS, a_voff[i], soff_a);
#pragma unroll
            for (int i = 0; i < B_PER; ++i)
                load_to_lds16(rx, sb + i * PASS, (int)b_cur[i], soff_b);
            ld_c += CPR;
            if (ld_c == a.c8) {
                ld_c = 0;
                if (++ld_s == g.S) {
                    ld_s = 0;
                    if (++ld_r == g.R) { ld_r = 0; ld_nt = walk.tile(++ld_t); tile_setup(ld_nt); }
                }
            }
        } else {
            if (ld_fresh) { row_setup(); ld_fresh = 0; }
            const int jl0 = ld_j0 + lc;                                            // this lane's chunk within the run of row ld_r
            const bool straddle = a.flat && ld_j0 + CPR > a.run_chunks;           // (wave-uniform) the slice runs on into row ld_r + 1
            const int soff_a = (ld_r * a.run_chunks + ld_j0) * 16;                // filter rows follow one another in memory
            const int run_off = ld_r * g.W * g.C * 2 + ld_j0 * 16;
            if (!straddle) {
                const int s = a.c8 == 1 ? jl0 : (int)__umulhi((unsigned)jl0, a.magic_c8);   // its tap: jl0 / (C / 8), at most 15
                const int sh = 31 - s;
                const bool a_ok = jl0 < a.run_chunks;
#pragma unroll
                for (int i = 0; i < A_PER; ++i)
                    load_to_lds16(rw, sa + i * PASS, a_ok ? a_voff[i] : OOB, soff_a);
#pragma unroll
                for (int i = 0; i < B_PER; ++i) {
                    const unsigned off = ((b_cur[i] << sh) & 0x80000000u) | (unsigned)(b_base[i] + run_off);
                    load_to_lds16(rx, sb + i * PASS, (int)off, 0);
                }
            } else {
                const bool wrap = jl0 >= a.run_chunks;                            // this lane's chunk belongs to row ld_r + 1
                const int jl = wrap ? jl0 - a.run_chunks : jl0;
                const int s = a.c8 == 1 ? jl : (int)__umulhi((unsigned)jl, a.magic_c8);
                const int sh = 31 - s;
                const bool more = ld_r + 1 < g.R;                                 // (wave-uniform) there is a next row
                const bool a_ok = !wrap || more;
                const int off_l = run_off + (wrap ? (g.W * g.C - a.run_chunks * 8) * 2 : 0);
                const int next_bit = (17 + ld_r) & 31;
#pragma unroll
                for (int i = 0; i < A_PER; ++i)
                    load_to_lds16(rw, sa + i * PASS, a_ok ? a_voff[i] : OOB, soff_a);
#pragma unroll
                for (int i = 0; i < B_PER; ++i) {
                    const unsigned nxt = (more && ((b_mask[i] >> next_bit) & 1u)) ? (b_mask[i] | 0xFFFF0000u) : 0xFFFFFFFFu;
                    const unsigned vm = wrap ? nxt : b_cur[i];
                    const unsigned off = ((vm << sh) & 0x80000000u) | (unsigned)(b_base[i] + off_l);
                    load_to_lds16(rx, sb + i * PASS, (int)off, 0);
                }
            }
            ld_j0 += CPR;
            if (ld_j0 >= a.run_chunks) {
                ld_j0 = a.flat ? ld_j0 - a.run_chunks : 0;
                ld_fresh = 1;
                if (++ld_r == g.R) { ld_r = 0; ld_j0 = 0; ld_nt = walk.tile(++ld_t); tile_setup(ld_nt); }
            }
        }
    };

    f32x16 acc[TM][TN];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    };

    // One slice = 4 k-steps of 16.  The operands of a k-step go from LDS into one of four register slots
    // (slot = step % 4) three steps before the matrix cores use them, across slice boundaries, so that
    // the LDS latency hides behind about three steps of MFMAs.  LDS reads return in order: "at most the
    // reads of two steps outstanding" means the oldest of three steps in flight has arrived.
    // (Half-depth slices: two k-steps per slice, two slots, each k-step fetched one step before its use -- a step of a
    // wide wave tile is long enough to cover the LDS latency.)
    constexpr int SLOTS = KB == 64 ? 4 : 2;
    u32x4 fa[SLOTS][TM], fb[SLOTS][TN];
    auto fetch_step = [&](int stage, auto ks_c) __attribute__((always_inline)) {     // k-step KS of a stage -> slot KS
        constexpr int KS = decltype(ks_c)::value;
        static_assert(KS < KSTEPS && KS < SLOTS, "k-step");
        const unsigned pa = (a_rd + stage * STAGE) ^ (KS * 32), pb = (b_rd + stage * STAGE) ^ (KS * 32);
        constexpr int BLK = 32 * RB;                                       // one 32-row block of an operand
        fa[KS][0] = ds_read16<0>(pa);
        if constexpr (TM > 1) fa[KS][1] = ds_read16<BLK>(pa);
        if constexpr (TM > 2) fa[KS][2] = ds_read16<2 * BLK>(pa);
        if constexpr (TM > 3) fa[KS][3] = ds_read16<3 * BLK>(pa);
        if constexpr (TM > 4) fa[KS][4] = ds_read16<4 * BLK>(pa);
        if constexpr (TM > 5) fa[KS][5] = ds_read16<5 * BLK>(pa);
        fb[KS][0] = ds_read16<0>(pb);
        if constexpr (TN > 1) fb[KS][1] = ds_read16<BLK>(pb);
        if constexpr (TN > 2) fb[KS][2] = ds_read16<2 * BLK>(pb);
        if constexpr (TN > 3) fb[KS][3] = ds_read16<3 * BLK>(pb);
    };
    auto multiply_step = [&](auto ks_c) __attribute__((always_inline)) {              // waits for slot KS, multiplies it
        constexpr int KS = decltype(ks_c)::value;
        wait_lgkm<(SLOTS - 2) * (TM + TN) + (SLOTS == 2 ? TM + TN : 0)>();            // the reads of the younger steps may be pending
#pragma unroll
        for (int i = 0; i < TM; ++i) touch(fa[KS][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) touch(fb[KS][j]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[KS][i]),
                                                                    __builtin_bit_cast(bf16x8, fb[KS][j]), acc[i][j], 0, 0, 0);
    };

    auto epilogue = [&](int nt) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            // this lane's 16 bias values of block row i, from LDS: read and awaited before the first branch
            u32x4 bv[2][2];
            bv[0][0] = ds_read16<0>(bias_rd + i * 128);
            bv[0][1] = ds_read16<16>(bias_rd + i * 128);
            bv[1][0] = ds_read16<64>(bias_rd + i * 128);
            bv[1][1] = ds_read16<80>(bias_rd + i * 128);
            wait_lgkm<0>();
            touch(bv[0][0]); touch(bv[0][1]); touch(bv[1][0]); touch(bv[1][1]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = nt * BN + wn * WN + j * 32 + l32;
                uint16_t* yb = a.y + (size_t)n * g.y_ctot + g.y_coff;     // (replaced per channel group in a stacked convolution)
                const uint16_t* rb = a.res + (size_t)n * g.res_ctot;
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    // registers 8 qp .. 8 qp + 3 hold channels +0..3 (lower half-wave) / +4..7 (upper);
                    // registers 8 qp + 4 .. 8 qp + 7 hold channels +8..11 / +12..15
                    float o[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][qp * 8 + e]),
                                                                         __float_as_uint(acc[i][j][qp * 8 + 4 + e]), false, false);
                        o[e] = __uint_as_float(sw[0]);
                        o[4 + e] = __uint_as_float(sw[1]);
                    }
                    const int mb = m_lane + i * 32 + qp * 16;     // first of this lane's 8 channels
                    if (n >= g.Ng || mb >= g.K) continue;
                    if (a.nsplit > 1) {                           // (wave-uniform) pick this lane's destination
                        const bool s1 = mb >= a.split_end[0], s2 = mb >= a.split_end[1], s3 = mb >= a.split_end[2];
                        uint16_t* base = s3 ? a.y_seg[3] : s2 ? a.y_seg[2] : s1 ? a.y_seg[1] : a.y_seg[0];
                        const int ct = s3 ? a.ctot_seg[3] : s2 ? a.ctot_seg[2] : s1 ? a.ctot_seg[1] : a.ctot_seg[0];
                        yb = base + (size_t)n * ct;
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] += __uint_as_float(bv[qp][e >> 2][e & 3]);
                    if (a.vec_ok && mb + 7 < g.K) {
                        if (a.res) {
                            const u32x4 rv = *reinterpret_cast<const u32x4*>(rb + mb);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                o[2 * e] += __uint_as_float(rv[e] << 16);
                                o[2 * e + 1] += __uint_as_float(rv[e] & 0xFFFF0000u);
                            }
                        }
                        if (g.relu) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) o[e] = fmaxf(o[e], 0.f);
                        }
                        u32x4 pk;
#pragma unroll
                        for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
                        *reinterpret_cast<u32x4*>(yb + mb) = pk;
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int m = mb + e;
                            if (m < g.K) {
                                float v = o[e];
                                if (a.res) v += __uint_as_float((uint32_t)rb[m] << 16);
                                if (g.relu) v = fmaxf(v, 0.f);
                                yb[m] = (uint16_t)f32_to_bf16(v);
                            }
                        }
                    }
                }
            }
        }
    };

    // The same store for the common case (one destination, no residual, aligned, filters a multiple of 8, output below 2 GiB) as
    // buffer stores that EVERY lane issues: a lane without an output (beyond the last pixel or filter) stores at an offset
    // outside the tensor, which the hardware drops.  A tile then leaves exactly E = 2 TM TN store instructions per wave in
    // the memory counter, and the waits for the operand loads of the next slices can allow for them (stores and loads share
    // one counter; an unknown number of stores would force those waits to let every store drain first).
    constexpr int E = 2 * TM * TN;
    auto epilogue_exact = [&](int nt) __attribute__((always_inline)) {
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
                const int n = nt * BN + wn * WN + j * 32 + l32;
                const int nbase = (n * g.y_ctot + g.y_coff) * 2;
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
                    const int mb = m_lane + i * 32 + qp * 16;     // first of this lane's 8 channels
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] += __uint_as_float(bv[qp][e >> 2][e & 3]);
                    if (g.relu) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = fmaxf(o[e], 0.f);
                    }
                    u32x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
                    const int voff = (n < g.Ng && mb < g.K) ? nbase + mb * 2 : OOB;
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_raw_buffer_store_b128(pk, ry, voff, 0, 0);
#endif
                }
            }
        }
    };

    // ---- block kernel: what follows the contraction.  (a) bias + ReLU, rounded to bf16, into LDS as [pixel][channel] (the ring
    // is free: every load has landed and, after the barrier, every operand read has returned); (b) across-channel
    // normalisation in place: an item is 8 channels of a pixel, its window's two channels on either side come from the
    // neighbouring items; results wait in registers until everybody has read; (c) 3x3 stride-2 maxima of the normalised
    // pixels, clipped at the image's last row / column, 16 bytes per store.
    auto epilogue_block = [&](int nt) __attribute__((always_inline)) {
        constexpr int NTH = WAVES * 64;
        unsigned char* stage_lds = ring;
        const int groups = (g.K + 7) >> 3;                       // 16-byte channel groups per pixel
        ring_barrier();
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
                const int t = wn * WN + j * 32 + l32;            // pixel row of the tile
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
                    const int ml = wm * WM + half * 8 + i * 32 + qp * 16;     // first of this lane's 8 channels
                    u32x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        pk[e] = pack_bf16x2(fmaxf(o[2 * e] + __uint_as_float(bv[qp][(2 * e) >> 2][(2 * e) & 3]), 0.f),
                                            fmaxf(o[2 * e + 1] + __uint_as_float(bv[qp][(2 * e + 1) >> 2][(2 * e + 1) & 3]), 0.f));
                    if (t < FUSE_PIXELS && ml < g.K) *reinterpret_cast<u32x4*>(stage_lds + t * FUSE_PITCH + ml * 2) = pk;
                }
            }
        }
        __syncthreads();
        // (b) normalisation, window of 5 channels: y_c = x_c (k + alpha / n (x_{c-2}^2 + ... + x_{c+2}^2))^-beta
        constexpr int ITEMS_MAX = FUSE_PIXELS * 24, PER = (ITEMS_MAX + NTH - 1) / NTH;
        u32x4 keep[PER];
        const int items = FUSE_PIXELS * groups;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int it = tid + u * NTH;
            keep[u] = u32x4{0u, 0u, 0u, 0u};
            if (it < items) {
                const int t = it / groups, gc = it - t * groups;
                const unsigned char* src = stage_lds + t * FUSE_PITCH + gc * 16;
                const u32x4 m = *reinterpret_cast<const u32x4*>(src);
                const uint32_t lft = gc > 0 ? *reinterpret_cast<const uint32_t*>(src - 4) : 0u;
                const uint32_t rgt = gc < groups - 1 ? *reinterpret_cast<const uint32_t*>(src + 16) : 0u;
                float v[12];                                     // channels c0 - 2 .. c0 + 9
                v[0] = __uint_as_float(lft << 16); v[1] = __uint_as_float(lft & 0xFFFF0000u);
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[2 + 2 * e] = __uint_as_float(m[e] << 16); v[3 + 2 * e] = __uint_as_float(m[e] & 0xFFFF0000u); }
                v[10] = __uint_as_float(rgt << 16); v[11] = __uint_as_float(rgt & 0xFFFF0000u);
                // channels beyond the last filter do not exist (a ragged last group holds whatever the padded filter rows gave: zeros)
                float sq[12];
#pragma unroll
                for (int e = 0; e < 12; ++e) sq[e] = v[e] * v[e];
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float ss = ((sq[e] + sq[e + 1]) + sq[e + 2]) + (sq[e + 3] + sq[e + 4]);
                    o[e] = v[e + 2] * pow_neg_beta(fmaf(a.f_a_over_n, ss, a.f_k), a.f_beta, a.f_b075 != 0);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) keep[u][e] = pack_bf16x2(o[2 * e], o[2 * e + 1]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int it = tid + u * NTH;
            if (it < items) {
                const int t = it / groups, gc = it - t * groups;
                *reinterpret_cast<u32x4*>(stage_lds + t * FUSE_PITCH + gc * 16) = keep[u];
            }
        }
        __syncthreads();
        // (c) pooling
        const int per_img = a.f_ty * a.f_tx;
        const int img = nt / per_img, rem = nt - img * per_img, ty = rem / a.f_tx, tx = rem - ty * a.f_tx;
        const int pitems = FUSE_POOLED * FUSE_POOLED * groups;
        for (int it = tid; it < pitems; it += NTH) {
            const int pp = it / groups, gc = it - pp * groups;
            const int pa = pp / FUSE_POOLED, pb = pp - pa * FUSE_POOLED;
            const int oy = ty * FUSE_POOLED + pa, ox = tx * FUSE_POOLED + pb;            // pooled pixel in the image
            if (oy >= a.f_PP || ox >= a.f_QQ) continue;
            float best[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
#pragma unroll
            for (int wy = 0; wy < 3; ++wy)
#pragma unroll
                for (int wx = 0; wx < 3; ++wx) {
                    const int dy = 2 * pa + wy, dx = 2 * pb + wx;
                    if (ty * (FUSE_SIDE - 1) + dy < g.P && tx * (FUSE_SIDE - 1) + dx < g.Q) {
                        const u32x4 m = *reinterpret_cast<const u32x4*>(stage_lds + (dy * FUSE_SIDE + dx) * FUSE_PITCH + gc * 16);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            best[2 * e] = fmaxf(best[2 * e], __uint_as_float(m[e] << 16));
                            best[2 * e + 1] = fmaxf(best[2 * e + 1], __uint_as_float(m[e] & 0xFFFF0000u));
                        }
                    }
                }
            uint16_t* dst = a.f_y + ((size_t)(img * a.f_PP + oy) * a.f_QQ + ox) * a.f_ctot + a.f_coff + gc * 8;
            if (gc * 8 + 7 < g.K) {
                u32x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(best[2 * e], best[2 * e + 1]);
                *reinterpret_cast<u32x4*>(dst) = pk;
            } else {
                for (int e = 0; e < 8; ++e)
                    if (gc * 8 + e < g.K) dst[e] = f32_to_bf16(best[e]);
            }
        }
    };

    // ---- pipeline.  Slice k lives in ring stage k % NS.  Iteration gi multiplies slice gi; after its first
    // k-step the workgroup meets: slice gi + 1 has landed and slice gi has been read completely, so the
    // loads of slice gi + NS go out into the stage slice gi leaves, and the remaining three k-steps
    // already fetch the first three k-steps of slice gi + 1.
    tile_setup(ld_nt);
    int issued = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (issued < total) { issue_slice(s); ++issued; }
    if (NS - 1 < total) wait_vmcnt<(NS - 1) * L>();     // the bias and slice 0 have landed (this wave's part)
    else wait_vmcnt<0>();
    ring_barrier();
    fetch_step(0, IC<0>{});
    if constexpr (KB == 64) {
        fetch_step(0, IC<1>{});
        fetch_step(0, IC<2>{});
    }

    // Slices multiplied since the last tile's stores went out.  For NS - 1 slices after a tile with exact stores its E stores are
    // younger than the slice being awaited, like the NS - 2 slices of loads behind it: the wait allows for them.
    constexpr bool ALLOW_STORES = (NS - 2) * L + E <= 63;
    const bool exact = ALLOW_STORES && a.exact_store;
    int since_epi = NS;
    auto wait_next_slice = [&](int gi_) __attribute__((always_inline)) {      // this wave's loads of slice gi_ + 1 have landed
        if (gi_ + NS - 1 < total) {
            if (since_epi <= NS - 1) wait_vmcnt<ALLOW_STORES ? (NS - 2) * L + E : 0>();
            else wait_vmcnt<(NS - 2) * L>();
        } else wait_vmcnt<0>();
    };
    int gi = 0, stage = 0;
    for (int t = 0; t < my_tiles; ++t) {
        zero_acc();
        for (int sl = 0; sl < nslices; ++sl, ++gi) {
            const int next_stage = stage + 1 == NS ? 0 : stage + 1;
            ++since_epi;
            if constexpr (KB == 32) {
                // two k-steps per slice: the second step's operands leave LDS while the first multiplies; the workgroup then
                // meets (slice gi + 1 has landed, slice gi has been read completely), the loads of slice gi + NS go out into
                // the stage slice gi leaves, and the first step of slice gi + 1 is fetched while the second multiplies
                fetch_step(stage, IC<1>{});
                multiply_step(IC<0>{});
                if (gi + 1 < total) {
                    wait_next_slice(gi);
                    ring_barrier();
                    if (issued < total) { issue_slice(stage); ++issued; }
                }
                fetch_step(next_stage, IC<0>{});      // (after the last slice: reads nobody uses)
                multiply_step(IC<1>{});
            } else {
            multiply_step(IC<0>{});
            fetch_step(stage, IC<3>{});
            // With three or more stages a slice's loads have a whole further iteration to land, and the waves of the
            // workgroup take turns: wave w sends its loads after k-step w (slot), so that the four bursts do not queue up
            // behind one another in the compute unit's address path while every wave waits.
            int slot = -1;
            if (gi + 1 < total) {
                // this wave's loads of slice gi + 1 have landed once at most the NS - 2 slices behind it are pending
                wait_next_slice(gi);
                ring_barrier();
                if (issued < total) {
                    slot = NS >= 3 ? (wave & 3) : 0;
                    ++issued;
                    if (slot == 0) issue_slice(stage);
                }
            }
            multiply_step(IC<1>{});
            if (NS >= 3 && slot == 1) issue_slice(stage);
            fetch_step(next_stage, IC<0>{});      // (after the last slice: reads nobody uses)
            multiply_step(IC<2>{});
            if (NS >= 3 && slot == 2) issue_slice(stage);
            fetch_step(next_stage, IC<1>{});
            multiply_step(IC<3>{});
            if (NS >= 3 && slot == 3) issue_slice(stage);
            fetch_step(next_stage, IC<2>{});
            }
            stage = next_stage;
        }
        if constexpr (FUSE) epilogue_block(walk.tile(t));     // (one tile per workgroup: see launch_block)
        else if (exact) { epilogue_exact(walk.tile(t)); since_epi = 0; }
        else epilogue(walk.tile(t));
    }
    wait_lgkm<0>();
}

template <int TM, int TN, int WGM, int WGN, int NS, int OCC, int KB = 64, bool FUSE = false>
int launch_cfg(DArgs a, hipStream_t st)
{
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, NTH = WGM * WGN * 64, CPR = KB / 8, RP = WGM * WGN * (512 / KB);
    constexpr int LDS = NS * ((BM + RP - 1) / RP * RP + BN) * KB * 2 + 1024;
    // slices of KB contraction elements: whole taps when the channel count allows, else runs of a filter row's S * C values
    // that go on into the next row when that saves slices (see the kernel's header)
    a.slices_per_run = (a.run_chunks + CPR - 1) / CPR;
    a.slices_per_tile = a.g.R * a.slices_per_run;
    a.flat = 0;
    if (a.stem_wp) {
        a.slices_per_tile = a.g.R;                    // (launch_conv_bf16_stem: one "filter row" per slice)
    } else if (a.g.C % KB != 0 && a.run_chunks >= CPR && (a.g.R * a.run_chunks + CPR - 1) / CPR < a.slices_per_tile) {
        a.flat = 1;                                   // slices that run on across filter rows save at least one slice per tile
        a.slices_per_tile = (a.g.R * a.run_chunks + CPR - 1) / CPR;
    }
    a.step_img = RP / (a.g.P * a.g.Q);
    a.step_p = (RP % (a.g.P * a.g.Q)) / a.g.Q;
    a.step_q = RP % a.g.Q;
    static_assert(LDS <= 160 * 1024, "LDS ring too large");
    a.grid_m = (a.g.K + BM - 1) / BM;
    if (!FUSE) a.grid_n = (a.g.Ng + BN - 1) / BN;      // (block kernel: the caller has counted the patches)
    // workgroups per channel block: what the device holds at once, at most one per pixel tile (a layer
    // with fewer tiles than that runs in a single round)
    static_assert(OCC * LDS <= 160 * 1024, "the ring does not fit OCC times");
    int gn = device_cus() * OCC / a.grid_m;
    if (gn < 1) gn = 1;
    if (gn > a.grid_n) gn = a.grid_n;
    if (FUSE) gn = a.grid_n;                           // one patch per workgroup: its epilogue needs the whole ring
    const unsigned G = (unsigned)(gn * a.grid_m);
    a.wk = make_walk(a.grid_m, gn, a.grid_n);
    if (a.g.C % KB == 0)
        hipLaunchKernelGGL((conv_bf16_dma_kernel<TM, TN, WGM, WGN, NS, true, OCC, KB, FUSE>), dim3(G), dim3(NTH), 0, st, a);
    else
        hipLaunchKernelGGL((conv_bf16_dma_kernel<TM, TN, WGM, WGN, NS, false, OCC, KB, FUSE>), dim3(G), dim3(NTH), 0, st, a);
    return check_launch("conv_bf16");
}

// Tile choice, from sweeps over the ResNet / GoogLeNet layer shapes at batch 128.  The kernel is limited by
// instruction issue and by how fast a compute unit's vector memory path feeds LDS, not by the matrix
// cores: two workgroups of 64, 96 or 128 filters x 128 pixels per compute unit beat one large tile.  Among
// them, the cost of a tile grows with its filter count (measured: about 0.44 + filters / 32) and the
// number of rounds is tiles / resident workgroups, rounded up while it is small (a persistent workgroup
// walks a whole number of tiles).
thread_local int t_shared_device = 0;

inline float tile_rounds(int K, int Ng, int bm, int bn)
{
    const float r = (float)((K + bm - 1) / bm) * (float)((Ng + bn - 1) / bn) / (float)(device_cus() * 2);
    return r <= 1.f ? 1.f : (r < 3.f ? ceilf(r) : r);
}
int launch_auto(DArgs a, hipStream_t st)
{
    const int K = a.g.K, Ng = a.g.Ng;
    // a layer whose 64 x 64 tiles all fit the device at two workgroups per compute unit: twice the
    // workgroups of the 128-pixel tiles and a ring of four stages, for layers that would leave compute
    // units idle (the 7 x 7 maps, the narrow reducers of the 14 x 14 maps); also taken for K <= 32,
    // where padding the filter block to 64 costs less than one more kernel variant between the others
    // (not while other streams of the same caller keep the device busy: measured slower there)
    if (!t_shared_device && ((K + 63) / 64) * ((Ng + 63) / 64) <= 2 * device_cus()) return launch_cfg<1, 1, 2, 2, 4, 2>(a, st);   // 64 x 64 tiles
    if (K <= 32) {
        // fewer 256-pixel tiles than compute units: halve the tiles
        if ((Ng + 255) / 256 < device_cus()) return launch_cfg<1, 1, 1, 4, 2, 3>(a, st);   // 32 x 128 tiles
        return launch_cfg<1, 2, 1, 4, 2, 2>(a, st);                                        // 32 x 256 tiles
    }
    // several taps and 97..128 filters on enough pixels for one round of 256-pixel tiles: one workgroup holds all filters of
    // its pixels (128 x 64 per wave, half-depth slices so that three stages fit), so every pixel row is fetched once per tap
    // instead of twice (GoogLeNet 3a's 3x3 96 -> 128 on 28 x 28: 41 -> 34 us against 64 x 128 and 128 x 128 tiles)
    if (a.g.R * a.g.S > 1 && K > 96 && K <= 128 && (Ng + 255) / 256 >= device_cus() && (Ng + 255) / 256 <= 2 * device_cus())
        return launch_cfg<4, 2, 1, 4, 3, 2, 32>(a, st);                          // 128 x 256 tiles
    const float c64 = tile_rounds(K, Ng, 64, 128) * (0.44f + 2.f), c96 = tile_rounds(K, Ng, 96, 128) * (0.44f + 3.f);
    const float r128 = tile_rounds(K, Ng, 128, 128), c128 = r128 * (0.44f + 4.f);   // pays only when it saves a round
    if (r128 <= 1.f && c128 < c64 && c128 < c96) return launch_cfg<2, 2, 2, 2, 2, 2>(a, st);   // 128 x 128 tiles, 64 x 64 per wave
    if (c96 < c64) return launch_cfg<3, 1, 1, 4, 2, 2>(a, st);                  // 96 x 128 tiles
    return launch_cfg<2, 1, 1, 4, 3, 2>(a, st);                                 // 64 x 128 tiles
}

}  // namespace

SharedDeviceScope::SharedDeviceScope(bool on) : on_(on) { if (on_) ++t_shared_device; }
SharedDeviceScope::~SharedDeviceScope() { if (on_) --t_shared_device; }

bool conv_bf16_dma_eligible(const ConvGeom& g, const void* x, const void* w)
{
    const size_t xb = (size_t)g.N * g.C * g.H * g.W * 2, wb = (size_t)g.K * g.Kg * 2;
    return g.nhwc && g.w_krsc && g.C % 8 == 0 && g.S <= 9 && g.R <= 16 && g.Ng < (1 << 24) && (long)g.P * g.Q <= 65536 && xb < (1ull << 31) &&
           wb < (1ull << 31) && aligned16(x) && aligned16(w);
}

static DArgs base_args(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, const uint16_t* residual, uint16_t* y)
{
    DArgs a{};
    a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.g = g;
    a.grid_m = a.grid_n = 0;
    a.x_bytes = (int)((size_t)g.N * g.C * g.H * g.W * 2);
    a.w_bytes = (int)((size_t)g.K * g.Kg * 2);
    a.c8 = g.C / 8;
    a.run_chunks = g.S * a.c8;
    a.slices_per_run = 0;                             // (the slice plan depends on the slice depth: launch_cfg)
    a.magic_c8 = (unsigned)((0x100000000ull + a.c8 - 1) / a.c8);
    a.m_pq = ((1ull << 40) + (unsigned)(g.P * g.Q) - 1) / (unsigned)(g.P * g.Q);
    a.m_q = ((1ull << 40) + (unsigned)g.Q - 1) / (unsigned)g.Q;
    a.pointwise = g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0;
    a.stem_hp = a.stem_wp = 0;
    a.slices_per_tile = 0; a.flat = 0;
    a.vec_ok = g.y_ctot % 8 == 0 && g.y_coff % 8 == 0 && aligned16(y) && (!residual || (g.res_ctot % 8 == 0 && aligned16(residual)));
    a.nsplit = 0;
    for (int d = 0; d < 4; ++d) { a.y_seg[d] = nullptr; a.ctot_seg[d] = 0; if (d < 3) a.split_end[d] = 0x7FFFFFFF; }
    // stores that every lane issues (see the kernel's epilogue): one destination, no residual, whole aligned channel groups, and
    // byte offsets into the output that fit the buffer instruction's 31 bits
    const double ybytes = (double)g.Ng * g.y_ctot * 2.0;
    a.exact_store = y && a.vec_ok && !residual && g.K % 8 == 0 && ybytes < 2147483648.0;
    a.y_bytes = a.exact_store ? (int)ybytes : 0;
    return a;
}

// The block kernel: y = maxpool3x3s2(lrn5(relu(conv(x) + bias))), ceil-mode pooling without padding, for layers the
// streaming kernel takes with at most 192 filters.  One workgroup of eight waves per patch of 15 x 15 convolution pixels
// (7 x 7 pooled ones) x all filters; neighbouring patches share one row / column of convolution pixels, which both compute.
bool conv_bf16_block_eligible(const ConvGeom& g, const void* x, const void* w, const dr_pool& p, const dr_lrn& l)
{
    return conv_bf16_dma_eligible(g, x, w) && g.K <= 192 && g.K % 8 == 0 && l.local_size == 5 && p.kh == 3 && p.kw == 3 && p.stride_h == 2 &&
           p.stride_w == 2 && p.pad_h == 0 && p.pad_w == 0 && g.P >= 1 && g.Q >= 1;
}

int launch_conv_bf16_block(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, const dr_lrn& l, int PP, int QQ,
                           uint16_t* y, int y_ctot, int y_coff, hipStream_t st)
{
    DArgs a = base_args(g, x, w, bias, nullptr, nullptr);
    a.f_ty = (PP + FUSE_POOLED - 1) / FUSE_POOLED;
    a.f_tx = (QQ + FUSE_POOLED - 1) / FUSE_POOLED;
    a.f_PP = PP; a.f_QQ = QQ; a.f_ctot = y_ctot; a.f_coff = y_coff;
    a.f_a_over_n = l.alpha / (float)l.local_size; a.f_beta = l.beta; a.f_k = l.k; a.f_b075 = l.beta == 0.75f;
    a.f_y = y;
    const long tiles = (long)g.N * a.f_ty * a.f_tx;
    if (tiles >= (1l << 24)) return fail(DR_ERR_UNSUPPORTED, "conv + lrn + maxpool: more than 2^24 patches");
    a.grid_n = (int)tiles;
    return launch_cfg<3, 2, 2, 4, 2, 1, 64, true>(a, st);       // 192 filters x 256 pixel rows, eight waves of 96 x 64
}

int launch_conv_bf16_dma(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias,
                         const uint16_t* residual, uint16_t* y, hipStream_t st, const ConvSplit* split)
{
    DArgs a = base_args(g, x, w, bias, residual, y);
    a.nsplit = 0;
    if (split && split->n > 1) {
        a.nsplit = split->n;
        a.exact_store = 0;                            // (several destinations: the ordinary store)
        int start = 0;
        for (int d = 0; d < 4; ++d) {
            if (d < split->n) {
                const ConvDest& s = split->dst[d];
                a.y_seg[d] = (uint16_t*)s.y + s.c_offset - start;
                a.ctot_seg[d] = s.ctot;
                a.vec_ok = a.vec_ok && s.ctot % 8 == 0 && s.c_offset % 8 == 0 && aligned16(s.y);
                start += s.k;
                if (d < 3) a.split_end[d] = d + 1 < split->n ? start : 0x7FFFFFFF;
            } else {
                a.y_seg[d] = nullptr;
                a.ctot_seg[d] = 0;
                if (d < 3) a.split_end[d] = 0x7FFFFFFF;
            }
        }
    }
    return launch_auto(a, st);
}

// Convolution of an input with at most 4 channels (the 3-channel network input), even column stride,
// filters of at most 8x8 taps.  The caller has copied the input into xp[N][hp][wp][4]: zero padding laid
// out physically (the original pixel (y, x) sits at (y + pad_h, x + pad_w)), channels padded to 4,
// hp >= (P-1) stride_h + 8, wp >= (Q-1) stride_w + 8 and a multiple of 8; and the filters into
// wp8[K][8][8][4] with zeros beyond R, S, C.  One pixel is 8 bytes, so a 16-byte chunk is a pixel pair
// and, with an even stride, every window starts on a chunk.  A slice of 64 contraction elements is
// two window rows of 8 taps x 4 channels: 4 slices per tile, no padding tests, all loads aligned.  The
// streaming kernel runs it as a 4-"tap" convolution over 64 "channels" whose per-lane chunk offsets
// come from the stem branch of its tile setup.
int launch_conv_bf16_stem(const ConvGeom& real, const uint16_t* xp, int hp, int wp, const uint16_t* wp8, const float* bias,
                          uint16_t* y, hipStream_t st)
{
    TraceScope trace("conv_bf16", &real, real.Ng, st);
    ConvGeom g = real;
    g.C = 64; g.R = 4; g.S = 1; g.Kg = 256;
    g.W = wp / 8;                 // so that one "tap row" of W * C * 2 bytes is two rows of the padded copy
    g.ph = g.pw = 0;
    g.w_krsc = 1; g.nhwc = 1;
    DArgs a;
    a.x = xp; a.w = wp8; a.bias = bias; a.res = nullptr; a.y = y; a.g = g;
    a.grid_m = a.grid_n = 0;
    a.x_bytes = (int)((size_t)real.N * hp * wp * 8);
    a.w_bytes = (int)((size_t)real.K * 256 * 2);
    a.c8 = 8; a.run_chunks = 8; a.slices_per_run = 1; a.magic_c8 = (unsigned)((0x100000000ull + 7) / 8);
    a.m_pq = ((1ull << 40) + (unsigned)(g.P * g.Q) - 1) / (unsigned)(g.P * g.Q);
    a.m_q = ((1ull << 40) + (unsigned)g.Q - 1) / (unsigned)g.Q;
    a.pointwise = 0;
    a.slices_per_tile = 4; a.flat = 0;
    a.stem_hp = hp; a.stem_wp = wp;
    a.nsplit = 0;
    a.vec_ok = g.y_ctot % 8 == 0 && g.y_coff % 8 == 0 && aligned16(y);
    const double ybytes = (double)g.Ng * g.y_ctot * 2.0;
    a.exact_store = a.vec_ok && g.K % 8 == 0 && ybytes < 2147483648.0;
    a.y_bytes = a.exact_store ? (int)ybytes : 0;
    return launch_auto(a, st);
}

bool conv_bf16_stem_eligible(const ConvGeom& g)
{
    return g.nhwc && g.C <= 4 && g.R <= 8 && g.S <= 8 && g.sw % 2 == 0 && g.Ng < (1 << 24) && (long)g.P * g.Q <= 65536;
}

}  // namespace dr
