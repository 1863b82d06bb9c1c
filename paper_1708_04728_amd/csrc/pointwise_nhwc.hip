// Bandwidth-bound layers for channels-last (NHWC) tensors: max/avg pooling, across-channel LRN,
// concat, BatchNorm(+Scale).  The c values of a pixel are contiguous, so one lane owns one 16-byte
// group of channels (8 bf16 or 4 fp32) of one pixel and consecutive lanes walk the channel axis:
// every access is a coalesced 16-byte vector, window neighbours are whole vectors, and the
// cross-channel LRN window is completed with wavefront shuffles from the neighbouring lanes.
#include <type_traits>
#include <utility>

#include "dr_internal.h"
#include "dr_store.h"

namespace dr {
namespace {

// ---- pooling ------------------------------------------------------------------------------------------
// V = elements per lane (a 16-byte vector, or 1 when C is not a multiple of the vector width).
// A workgroup of BX x BY threads: BX (a power of two >= C / V, at most 256) lanes walk the channel
// groups of a pixel, the BY rows of the workgroup take consecutive output pixels of one output row
// (n, p); no per-element division.
template <typename T, int V, bool AVG>
__global__ __launch_bounds__(256) void pool_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int H, int W, int P,
                                                        int Q, int qgroups, int bx_log2, dr_pool p)
{
    const int CV = C / V;
    const int bx = 1 << bx_log2, by = 256 >> bx_log2;
    const int tx = threadIdx.x & (bx - 1), ty = threadIdx.x >> bx_log2;
    const unsigned row = blockIdx.x / (unsigned)qgroups;          // n * P + p
    const int qg = (int)(blockIdx.x - row * (unsigned)qgroups);
    const unsigned n = row / (unsigned)P;
    const int pp = (int)(row - n * (unsigned)P);
    const int q = qg * by + ty;
    if (q >= Q) return;
    const int h0 = pp * p.stride_h - p.pad_h, w0 = q * p.stride_w - p.pad_w;
    const int ha = max(h0, 0), hb = min(h0 + p.kh, H);
    const int wa = max(w0, 0), wb = min(w0 + p.kw, W);
    const T* xb = x + (size_t)n * H * W * C;
    T* yb = y + ((size_t)row * Q + q) * C;
    for (int cv = tx; cv < CV; cv += bx) {
        float m[V];
#pragma unroll
        for (int j = 0; j < V; ++j) m[j] = AVG ? 0.f : -INFINITY;
        if (hb - ha == 3 && wb - wa == 3) {
            // a full 3x3 window (every window of the workloads but the edge ones): nine independent loads
            const T* src = xb + ((size_t)ha * W + wa) * C + cv * V;
            float v[9][V];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    if constexpr (V == 1) v[r * 3 + c][0] = Store<T>::ld(src + ((size_t)r * W + c) * C);
                    else Store<T>::ldv(src + ((size_t)r * W + c) * C, v[r * 3 + c]);
                }
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int j = 0; j < V; ++j) m[j] = AVG ? m[j] + v[t][j] : fmaxf(m[j], v[t][j]);
        } else {
            // any window: walk its rows, up to 8 independent loads in flight per row segment
            for (int h = ha; h < hb; ++h)
                for (int w = wa; w < wb; w += 8) {
                    const T* src = xb + ((size_t)h * W + w) * C + cv * V;
                    float v[8][V];
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        if (w + t < wb) {
                            if constexpr (V == 1) v[t][0] = Store<T>::ld(src + (size_t)t * C);
                            else Store<T>::ldv(src + (size_t)t * C, v[t]);
                        } else {
#pragma unroll
                            for (int j = 0; j < V; ++j) v[t][j] = AVG ? 0.f : -INFINITY;
                        }
                    }
#pragma unroll
                    for (int t = 0; t < 8; ++t)
#pragma unroll
                        for (int j = 0; j < V; ++j) m[j] = AVG ? m[j] + v[t][j] : fmaxf(m[j], v[t][j]);
                }
        }
        if (AVG) {
#pragma unroll
            for (int j = 0; j < V; ++j) m[j] /= (float)(p.kh * p.kw);
        }
        if constexpr (V == 1) Store<T>::st(yb + cv, m[0]);
        else Store<T>::stv(yb + cv * V, m);
    }
}

// Average over the whole image (the 7x7 pooling in front of the classifier): 32 channel vectors x 8 pixel
// groups per workgroup; a thread sums every 8th pixel with up to 8 loads in flight, the 8 partial sums
// of a channel vector meet in LDS.
template <typename T>
__global__ __launch_bounds__(256) void global_avgpool_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int HW, int cgroups)
{
    constexpr int V = Store<T>::VN;
    __shared__ float part[8][32][V + 1];
    const int CV = C / V;
    const int n = blockIdx.x / cgroups, cg = blockIdx.x - n * cgroups;
    const int cl = threadIdx.x & 31, pg = threadIdx.x >> 5;
    const int cv = cg * 32 + cl;
    float s[V];
#pragma unroll
    for (int j = 0; j < V; ++j) s[j] = 0.f;
    if (cv < CV) {
        const T* xb = x + (size_t)n * HW * C + (size_t)cv * V;
        for (int p0 = pg; p0 < HW; p0 += 64) {
            float v[8][V];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (p0 + 8 * t < HW) Store<T>::ldv(xb + (size_t)(p0 + 8 * t) * C, v[t]);
                else {
#pragma unroll
                    for (int j = 0; j < V; ++j) v[t][j] = 0.f;
                }
            }
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int j = 0; j < V; ++j) s[j] += v[t][j];
        }
    }
#pragma unroll
    for (int j = 0; j < V; ++j) part[pg][cl][j] = s[j];
    __syncthreads();
    if (pg == 0 && cv < CV) {
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float a = 0.f;
#pragma unroll
            for (int g = 0; g < 8; ++g) a += part[g][cl][j];
            o[j] = a / (float)HW;
        }
        Store<T>::stv(y + (size_t)n * C + (size_t)cv * V, o);
    }
}

// 3x3 max-pooling, the window of every pooling layer of the networks here: separable.  A thread owns
// one output column q and one channel group and walks down a strip of PR output rows; per input row
// it takes the maximum of the row's three window pixels (three 16-byte loads), and an output is the
// maximum of three such row maxima, two of which are kept in registers from the previous outputs.
// Loads per output: 3 (PR + 2) / PR at stride 1 instead of 9.  Pixels outside the input never win.
template <typename T, int V>
__global__ __launch_bounds__(256) void maxpool3_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int H, int W, int P,
                                                            int Q, int PR, int pstrips, int qgroups, int bx_log2, int stride, int pad)
{
    const int CV = C / V;
    const int bx = 1 << bx_log2, by = 256 >> bx_log2;
    const int tx = threadIdx.x & (bx - 1), ty = threadIdx.x >> bx_log2;
    const unsigned qg = blockIdx.x % (unsigned)qgroups, t = blockIdx.x / (unsigned)qgroups;
    const unsigned strip = t % (unsigned)pstrips, n = t / (unsigned)pstrips;
    const int q = (int)qg * by + ty;
    if (q >= Q) return;
    const int p0 = (int)strip * PR, p1 = min(p0 + PR, P);
    const int w0 = q * stride - pad;
    const T* xb = x + (size_t)n * H * W * C;
    for (int cv = tx; cv < CV; cv += bx) {
        auto row_max = [&](int h, float* m) {
#pragma unroll
            for (int j = 0; j < V; ++j) m[j] = -INFINITY;
            if ((unsigned)h >= (unsigned)H) return;
            const T* src = xb + ((size_t)h * W + w0) * C + cv * V;
            float v[3][V];
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                if ((unsigned)(w0 + c) < (unsigned)W) {
                    if constexpr (V == 1) v[c][0] = Store<T>::ld(src + (size_t)c * C);
                    else Store<T>::ldv(src + (size_t)c * C, v[c]);
                } else {
#pragma unroll
                    for (int j = 0; j < V; ++j) v[c][j] = -INFINITY;
                }
            }
#pragma unroll
            for (int j = 0; j < V; ++j) m[j] = fmaxf(fmaxf(v[0][j], v[1][j]), v[2][j]);
        };
        float r0[V], r1[V], r2[V];
        int hb = p0 * stride - pad;                 // first input row of the current window
        row_max(hb, r0);
        row_max(hb + 1, r1);
        for (int p = p0; p < p1; ++p, hb += stride) {
            row_max(hb + 2, r2);
            float o[V];
#pragma unroll
            for (int j = 0; j < V; ++j) o[j] = fmaxf(fmaxf(r0[j], r1[j]), r2[j]);
            T* dst = y + (((size_t)n * P + p) * Q + q) * C + cv * V;
            if constexpr (V == 1) Store<T>::st(dst, o[0]);
            else Store<T>::stv(dst, o);
            if (stride == 1) {
#pragma unroll
                for (int j = 0; j < V; ++j) { r0[j] = r1[j]; r1[j] = r2[j]; }
            } else if (stride == 2) {
#pragma unroll
                for (int j = 0; j < V; ++j) r0[j] = r2[j];
                if (p + 1 < p1) row_max(hb + 3, r1);
            } else if (p + 1 < p1) {
                row_max(hb + stride, r0);
                row_max(hb + stride + 1, r1);
            }
        }
    }
}

// The same for strides 1 and 2 with 16-byte vectors, all loads first: a thread fetches the 3 x NR input
// vectors its strip of PR outputs needs (NR = (PR - 1) STRIDE + 3 rows) before it uses any of them, so
// that it waits for memory once instead of once per input row.
template <typename T> struct NegInfWord;
template <> struct NegInfWord<float> { static constexpr uint32_t v = 0xFF800000u; };
template <> struct NegInfWord<uint16_t> { static constexpr uint32_t v = 0xFF80FF80u; };
template <typename T> __device__ __forceinline__ void unpack16(const uint4& r, float* v);
template <> __device__ __forceinline__ void unpack16<float>(const uint4& r, float* v)
{
    v[0] = __uint_as_float(r.x); v[1] = __uint_as_float(r.y); v[2] = __uint_as_float(r.z); v[3] = __uint_as_float(r.w);
}
template <> __device__ __forceinline__ void unpack16<uint16_t>(const uint4& r, float* v)
{
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}

template <typename T, int PR, int STRIDE>
__global__ __launch_bounds__(256) void maxpool3_front_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int H, int W, int P,
                                                             int Q, int pstrips, int pgroups, unsigned cv_magic, unsigned qcv_magic, int pad,
                                                             unsigned blocks)
{
    constexpr int V = Store<T>::VN, NR = (PR - 1) * STRIDE + 3;
    const int CV = C / V, QCV = Q * CV;
    // Workgroups go to the device's 8 dies in turn (workgroup b to die b % 8), each die with an L2 of its own.  The
    // workgroups are renumbered so that a die works on one contiguous eighth of the tensor: the rows two neighbouring
    // strips share and the columns two neighbouring workgroups share are then fetched into one L2 instead of two.
    // (The launcher rounds the grid up to a multiple of 8; the surplus workgroups leave here.)
    const unsigned block = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (block >= blocks) return;
    // a thread owns one (strip of output rows, output column, channel vector) item of one image; the items are numbered
    // strip by strip, column by column, which within a row is also their order in memory (channels-last): consecutive
    // lanes touch consecutive 16-byte pieces whatever the channel count, and no lane idles except in an image's last
    // workgroup.  (The magic numbers are ceil(2^32 / divisor); the launcher checks that the divisions are exact.)
    const unsigned pg = block % (unsigned)pgroups, n = block / (unsigned)pgroups;
    const int item = (int)pg * 256 + (int)threadIdx.x;
    if (item >= pstrips * QCV) return;
    // (a divisor of 1 has no 32-bit magic number: ceil(2^32 / 1) does not fit)
    const int strip = QCV == 1 ? item : (int)__umulhi((unsigned)item, qcv_magic);
    const int pair = item - strip * QCV;
    const int q = CV == 1 ? pair : (int)__umulhi((unsigned)pair, cv_magic);
    const int cv = pair - q * CV;
    const int p0 = (int)strip * PR;
    const int w0 = q * STRIDE - pad, h0 = p0 * STRIDE - pad;
    const T* xb = x + (size_t)n * H * W * C;
    constexpr uint32_t NEG = NegInfWord<T>::v;
    uint4 raw[NR][3];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            raw[r][c] = make_uint4(NEG, NEG, NEG, NEG);
            if ((unsigned)(h0 + r) < (unsigned)H && (unsigned)(w0 + c) < (unsigned)W)
                raw[r][c] = *reinterpret_cast<const uint4*>(xb + ((size_t)(h0 + r) * W + (w0 + c)) * C + cv * V);
        }
    float rm[NR][V];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        float a[V], b[V], c[V];
        unpack16<T>(raw[r][0], a);
        unpack16<T>(raw[r][1], b);
        unpack16<T>(raw[r][2], c);
#pragma unroll
        for (int j = 0; j < V; ++j) rm[r][j] = fmaxf(fmaxf(a[j], b[j]), c[j]);
    }
#pragma unroll
    for (int i = 0; i < PR; ++i) {
        if (p0 + i >= P) break;
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) o[j] = fmaxf(fmaxf(rm[i * STRIDE][j], rm[i * STRIDE + 1][j]), rm[i * STRIDE + 2][j]);
        Store<T>::stv(y + (((size_t)n * P + p0 + i) * Q + q) * C + cv * V, o);
    }
}

template <typename T>
int pool_launch(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, bool avg, hipStream_t st)
{
    constexpr int VN = Store<T>::VN;
    if (tensor_elems(yd) == 0) return DR_OK;
    const bool vec = xd.c % VN == 0 && aligned16(x) && aligned16(y);
    const int cv = vec ? xd.c / VN : xd.c;
    int bx_log2 = 0;
    while ((1 << bx_log2) < cv && bx_log2 < 8) ++bx_log2;
    const int by = 256 >> bx_log2;
    const int qgroups = (yd.w + by - 1) / by;
    if ((double)yd.n * yd.h * qgroups >= 2147483648.0) return fail(DR_ERR_UNSUPPORTED, "pooling: tensor too large");
    if (!avg && p.kh == 3 && p.kw == 3 && p.stride_h == p.stride_w && p.pad_h == p.pad_w) {
        // strips of 4 output rows (best in sweeps over the pooling layers of the networks here), 2 while the
        // launch would otherwise have fewer than ~2048 workgroups
        const long per_strip = (long)yd.n * qgroups;
        const double qcv_d = (double)yd.w * cv;
        if (vec && (p.stride_h == 1 || p.stride_h == 2) && qcv_d * qcv_d * yd.h < 4294967296.0) {   // (the kernel's divisions are exact then)
            const int qcv = yd.w * cv;
            const unsigned cv_magic = (unsigned)((0x100000000ull + cv - 1) / cv), qcv_magic = (unsigned)((0x100000000ull + qcv - 1) / qcv);
            // workgroups per image for `strips_` strips
            auto groups_for = [&](int strips_) { return (int)(((long)strips_ * qcv + 255) / 256); };
            // strips of 7 rows for the 14 x 14 and 7 x 7 stride-1 layers (measured 10 % faster there than strips of 4)
            const bool seven = p.stride_h == 1 && yd.h % 7 == 0 && yd.h <= 14;
            const int PRF = p.stride_h == 1 ? (seven ? 7 : 4) : 2, strips = (yd.h + PRF - 1) / PRF;
            const int pgroups = groups_for(strips);
            const unsigned blocks = (unsigned)((long)yd.n * pgroups);
            const dim3 gf((blocks + 7) / 8 * 8);        // a multiple of 8: see the kernel's renumbering
            if (seven)
                hipLaunchKernelGGL((maxpool3_front_kernel<T, 7, 1>), gf, dim3(256), 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w,
                                   strips, pgroups, cv_magic, qcv_magic, p.pad_h, blocks);
            else if (p.stride_h == 1)
                hipLaunchKernelGGL((maxpool3_front_kernel<T, 4, 1>), gf, dim3(256), 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w,
                                   strips, pgroups, cv_magic, qcv_magic, p.pad_h, blocks);
            else
                hipLaunchKernelGGL((maxpool3_front_kernel<T, 2, 2>), gf, dim3(256), 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w,
                                   strips, pgroups, cv_magic, qcv_magic, p.pad_h, blocks);
            return check_launch("maxpool");
        }
        int PR = 4;
        while (PR > 2 && per_strip * ((yd.h + PR - 1) / PR) < 2048) PR >>= 1;
        const int pstrips = (yd.h + PR - 1) / PR;
        const dim3 g3((unsigned)(per_strip * pstrips));
        if (vec)
            hipLaunchKernelGGL((maxpool3_nhwc_kernel<T, VN>), g3, dim3(256), 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w, PR,
                               pstrips, qgroups, bx_log2, p.stride_h, p.pad_h);
        else
            hipLaunchKernelGGL((maxpool3_nhwc_kernel<T, 1>), g3, dim3(256), 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w, PR,
                               pstrips, qgroups, bx_log2, p.stride_h, p.pad_h);
        return check_launch("maxpool");
    }
    if (avg && vec && yd.h == 1 && yd.w == 1 && p.kh == xd.h && p.kw == xd.w && p.pad_h == 0 && p.pad_w == 0) {
        const int cgroups = (cv + 31) / 32;
        hipLaunchKernelGGL((global_avgpool_nhwc_kernel<T>), dim3((unsigned)(yd.n * cgroups)), dim3(256), 0, st, (const T*)x, (T*)y, xd.c,
                           xd.h * xd.w, cgroups);
        return check_launch("avgpool");
    }
    const dim3 grid((unsigned)(yd.n * yd.h * qgroups)), block(256);
#define DR_POOL(V, AVG) hipLaunchKernelGGL((pool_nhwc_kernel<T, V, AVG>), grid, block, 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w, qgroups, bx_log2, p)
    if (vec) { if (avg) DR_POOL(VN, true); else DR_POOL(VN, false); }
    else { if (avg) DR_POOL(1, true); else DR_POOL(1, false); }
#undef DR_POOL
    return check_launch(avg ? "avgpool" : "maxpool");
}

// ---- LRN -------------------------------------------------------------------------------------------------
// Window of 5 channels.  A pixel occupies LPP = C / V consecutive lanes of one wave (PPW pixels per
// wave, the remaining lanes idle), so the two channels on either side of a lane's vector live in the
// neighbouring lanes and arrive by shuffle; the first / last lane of a pixel sees zeros instead.
template <typename T, int V>
__global__ __launch_bounds__(256) void lrn5_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int LPP, int PPW,
                                                        size_t pixels, float a_over_n, float beta, float k, int b075)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const int sub = lane / LPP, cv = lane - sub * LPP;       // pixel slot within the wave, vector within the pixel
    const bool lane_on = sub < PPW;
    for (size_t pw = wave; pw * PPW < pixels; pw += nwaves) {
        const size_t pix = pw * PPW + sub;
        const bool on = lane_on && pix < pixels;
        float v[V];
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = 0.f;
        if (on) Store<T>::ldv(x + pix * C + (size_t)cv * V, v);
        float sq[V + 4];                                     // squares of channels c0-2 .. c0+V+1
#pragma unroll
        for (int j = 0; j < V; ++j) sq[j + 2] = v[j] * v[j];
        // every lane takes part in the shuffles (idle lanes carry zeros)
        const float l0 = __shfl_up(sq[V], 1, 64), l1 = __shfl_up(sq[V + 1], 1, 64);       // neighbour's last two
        const float r0 = __shfl_down(sq[2], 1, 64), r1 = __shfl_down(sq[3], 1, 64);       // neighbour's first two
        const bool has_l = cv > 0 && lane > 0, has_r = cv < LPP - 1 && lane < 63;
        sq[0] = has_l ? l0 : 0.f; sq[1] = has_l ? l1 : 0.f;
        sq[V + 2] = has_r ? r0 : 0.f; sq[V + 3] = has_r ? r1 : 0.f;
        if (on) {
            float o[V];
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float ss = ((sq[j] + sq[j + 1]) + sq[j + 2]) + (sq[j + 3] + sq[j + 4]);
                o[j] = v[j] * pow_neg_beta(fmaf(a_over_n, ss, k), beta, b075);
            }
            Store<T>::stv(y + pix * C + (size_t)cv * V, o);
        }
    }
}

// Any window length / channel count: every output re-reads its window (served by the caches).
template <typename T>
__global__ __launch_bounds__(256) void lrn_generic_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y, int C, size_t total,
                                                               int nl, float a_over_n, float beta, float k)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int c = (int)(i % C);
        const size_t base = i - c;
        float ss = 0.f;
        for (int cc = c - nl / 2; cc < c - nl / 2 + nl; ++cc)
            if (cc >= 0 && cc < C) {
                const float v = Store<T>::ld(x + base + cc);
                ss = fmaf(v, v, ss);
            }
        Store<T>::st(y + i, Store<T>::ld(x + i) * powf(fmaf(a_over_n, ss, k), -beta));
    }
}

template <typename T>
int lrn_launch(const dr_tensor& d, const void* x, void* y, const dr_lrn& p, hipStream_t st)
{
    constexpr int VN = Store<T>::VN;
    const float a_over_n = p.alpha / (float)p.local_size;
    const size_t pixels = (size_t)d.n * d.h * d.w;
    const int lpp = d.c / VN;
    if (p.local_size == 5 && d.c % VN == 0 && lpp >= 1 && lpp <= 64 && aligned16(x) && aligned16(y)) {
        const int ppw = 64 / lpp;
        const size_t waves = (pixels + ppw - 1) / ppw;
        hipLaunchKernelGGL((lrn5_nhwc_kernel<T, VN>), dim3(blocks_for(waves, 4, 256 * 64)), dim3(256), 0, st, (const T*)x, (T*)y,
                           d.c, lpp, ppw, pixels, a_over_n, p.beta, p.k, (int)(p.beta == 0.75f));
        return check_launch("lrn");
    }
    const size_t total = pixels * d.c;
    hipLaunchKernelGGL((lrn_generic_nhwc_kernel<T>), dim3(blocks_for(total, 256, 256 * 32)), dim3(256), 0, st, (const T*)x, (T*)y,
                       d.c, total, p.local_size, a_over_n, p.beta, p.k);
    return check_launch("lrn");
}

// ---- LRN and 3x3 max-pooling in one pass (the non-tensor tail of a conv - ReLU - LRN - pool block, Sec. 3.1) ------
// Same decomposition as maxpool3_front_kernel: a thread owns one output column, one 16-byte channel group and
// a strip of PR output rows, and fetches its 3 x NR input vectors first.  The lanes of a pixel are
// consecutive lanes of one wave (at most 64 channel groups), so the two channels on either side of a
// lane's vector arrive by shuffle, as in lrn5_nhwc_kernel.
//   LRN_FIRST: y = maxpool(lrn(x)): every fetched vector is normalised (a pixel of the input is normalised
//              by each of the up to 4 threads whose windows hold it), pixels outside the input never win;
//   else:      y = lrn(maxpool(x)): the pooled vector is normalised.
// The intermediate tensor is never rounded to the storage type.
// f(integral_constant<int, LO>{}), ..., f(integral_constant<int, HI - 1>{})
template <int LO, typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F& f, std::integer_sequence<int, Is...>) { (f(std::integral_constant<int, LO + Is>{}), ...); }
template <int LO, int HI, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (HI > LO) static_for_impl<LO>(f, std::make_integer_sequence<int, HI - LO>{});
}

template <typename T, int PR, int STRIDE, bool LRN_FIRST>
__global__ __launch_bounds__(256) void pool_lrn_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int H, int W, int P, int Q,
                                                       int pstrips, int qgroups, int bx_log2, int pad, float a_over_n, float beta, float k,
                                                       int b075)
{
    constexpr int V = Store<T>::VN, NR = (PR - 1) * STRIDE + 3;
    const int CV = C / V;
    const int bx = 1 << bx_log2, by = 256 >> bx_log2;
    const int cv = threadIdx.x & (bx - 1), ty = threadIdx.x >> bx_log2;
    const unsigned qg = blockIdx.x % (unsigned)qgroups, t = blockIdx.x / (unsigned)qgroups;
    const unsigned strip = t % (unsigned)pstrips, n = t / (unsigned)pstrips;
    const int q = (int)qg * by + ty;
    const bool on = q < Q && cv < CV;                     // idle lanes still take part in the shuffles, with zeros
    const bool has_l = cv > 0, has_r = cv < CV - 1;
    const int p0 = (int)strip * PR;
    const int w0 = q * STRIDE - pad, h0 = p0 * STRIDE - pad;
    const T* xb = x + (size_t)n * H * W * C;
    constexpr uint32_t NEG = NegInfWord<T>::v;

    auto lrn_vec = [&](const float* v, float* o) __attribute__((always_inline)) {
        float sq[V + 4];
#pragma unroll
        for (int j = 0; j < V; ++j) sq[j + 2] = v[j] * v[j];
        const float l0 = __shfl_up(sq[V], 1, 64), l1 = __shfl_up(sq[V + 1], 1, 64);
        const float r0 = __shfl_down(sq[2], 1, 64), r1 = __shfl_down(sq[3], 1, 64);
        sq[0] = has_l ? l0 : 0.f; sq[1] = has_l ? l1 : 0.f;
        sq[V + 2] = has_r ? r0 : 0.f; sq[V + 3] = has_r ? r1 : 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float ss = ((sq[j] + sq[j + 1]) + sq[j + 2]) + (sq[j + 3] + sq[j + 4]);
            o[j] = v[j] * pow_neg_beta(fmaf(a_over_n, ss, k), beta, b075);
        }
    };

    uint4 raw[NR][3];
    bool ok[NR][3];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            ok[r][c] = on && (unsigned)(h0 + r) < (unsigned)H && (unsigned)(w0 + c) < (unsigned)W;
            raw[r][c] = make_uint4(NEG, NEG, NEG, NEG);
            if (ok[r][c]) raw[r][c] = *reinterpret_cast<const uint4*>(xb + ((size_t)(h0 + r) * W + (w0 + c)) * C + cv * V);
        }
    float rm[NR][V];
    // (one instantiation per window pixel: the body with its shuffles is too large for the loop unroller)
    static_for<0, NR * 3>([&](auto rc_c) __attribute__((always_inline)) {
        constexpr int r = decltype(rc_c)::value / 3, c = decltype(rc_c)::value % 3;
        if constexpr (c == 0) {
#pragma unroll
            for (int j = 0; j < V; ++j) rm[r][j] = -INFINITY;
        }
        float v[V];
        unpack16<T>(raw[r][c], v);
        if constexpr (LRN_FIRST) {
            // whether a window pixel exists is the same for every lane of the pixel, so the lanes agree
            // on what they exchange; a missing pixel is normalised as zeros and then discarded
            float z[V], o[V];
#pragma unroll
            for (int j = 0; j < V; ++j) z[j] = ok[r][c] ? v[j] : 0.f;
            lrn_vec(z, o);
#pragma unroll
            for (int j = 0; j < V; ++j) rm[r][j] = fmaxf(rm[r][j], ok[r][c] ? o[j] : -INFINITY);
            __builtin_amdgcn_sched_barrier(0);     // one pixel at a time: interleaving all of them needs > 256 registers
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) rm[r][j] = fmaxf(rm[r][j], v[j]);
        }
    });
#pragma unroll
    for (int i = 0; i < PR; ++i) {
        const bool row_on = p0 + i < P;                    // (the same for the whole workgroup)
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) o[j] = fmaxf(fmaxf(rm[i * STRIDE][j], rm[i * STRIDE + 1][j]), rm[i * STRIDE + 2][j]);
        if constexpr (!LRN_FIRST) {
            float z[V], res[V];
#pragma unroll
            for (int j = 0; j < V; ++j) z[j] = (on && row_on) ? o[j] : 0.f;
            lrn_vec(z, res);
#pragma unroll
            for (int j = 0; j < V; ++j) o[j] = res[j];
        }
        if (on && row_on) Store<T>::stv(y + (((size_t)n * P + p0 + i) * Q + q) * C + cv * V, o);
    }
}

// y = maxpool(lrn(x)) through LDS: a workgroup normalises the input patch of a TP x TQ tile of outputs once
// (pixel by pixel, the lanes of a pixel exchanging their edge channels by shuffle), keeps it in LDS as fp32,
// and then takes the 3x3 maxima from there.  An input pixel is normalised once per tile that holds it
// (1.2 - 1.5 times on average) instead of once per window.  PH x PW = patch size, LP = lanes per pixel (a
// power of two >= C / V).
template <typename T, int STRIDE, int TP, int TQ>
__global__ __launch_bounds__(256) void lrn_pool_lds_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int H, int W, int P, int Q,
                                                           int ptiles, int qtiles, int lp_log2, int pad, float a_over_n, float beta, float k,
                                                           int b075)
{
    constexpr int V = Store<T>::VN, PH = (TP - 1) * STRIDE + 3, PW = (TQ - 1) * STRIDE + 3;
    extern __shared__ __attribute__((aligned(16))) float patch[];       // [PH * PW][C]
    const int CV = C / V;
    const int lp = 1 << lp_log2, slots = 256 >> lp_log2;
    const int cv = threadIdx.x & (lp - 1), slot = threadIdx.x >> lp_log2;
    const unsigned qt = blockIdx.x % (unsigned)qtiles, t = blockIdx.x / (unsigned)qtiles;
    const unsigned pt = t % (unsigned)ptiles, n = t / (unsigned)ptiles;
    const int p0 = (int)pt * TP, q0 = (int)qt * TQ;
    const int h0 = p0 * STRIDE - pad, w0 = q0 * STRIDE - pad;
    const bool lane_on = cv < CV, has_l = cv > 0, has_r = cv < CV - 1;
    const T* xb = x + (size_t)n * H * W * C;

    // ---- normalise the patch, NB pixels per thread at a time with their loads issued together (every lane
    // runs every iteration: the shuffles need whole waves)
    constexpr int NB = 6;
    for (int pp0 = 0; pp0 < PH * PW; pp0 += NB * slots) {
        uint4 raw[NB];
        bool px_on[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int pp = pp0 + u * slots + slot;
            const int pr = pp / PW, pc = pp - pr * PW;
            const int h = h0 + pr, w = w0 + pc;
            px_on[u] = pp < PH * PW && (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
            raw[u] = make_uint4(0u, 0u, 0u, 0u);
            if (px_on[u] && lane_on) raw[u] = *reinterpret_cast<const uint4*>(xb + ((size_t)h * W + w) * C + cv * V);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int pp = pp0 + u * slots + slot;
            float v[V];
            unpack16<T>(raw[u], v);
            float sq[V + 4];
#pragma unroll
            for (int j = 0; j < V; ++j) sq[j + 2] = v[j] * v[j];
            const float l0 = __shfl_up(sq[V], 1, 64), l1 = __shfl_up(sq[V + 1], 1, 64);
            const float r0 = __shfl_down(sq[2], 1, 64), r1 = __shfl_down(sq[3], 1, 64);
            sq[0] = has_l ? l0 : 0.f; sq[1] = has_l ? l1 : 0.f;
            sq[V + 2] = has_r ? r0 : 0.f; sq[V + 3] = has_r ? r1 : 0.f;
            if (pp < PH * PW && lane_on) {
                float o[V];
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    const float ss = ((sq[j] + sq[j + 1]) + sq[j + 2]) + (sq[j + 3] + sq[j + 4]);
                    o[j] = px_on[u] ? v[j] * pow_neg_beta(fmaf(a_over_n, ss, k), beta, b075) : -INFINITY;   // outside the input: never wins
                }
                float* dst = patch + (size_t)pp * C + cv * V;
#pragma unroll
                for (int j = 0; j < V; j += 4) *reinterpret_cast<float4*>(dst + j) = make_float4(o[j], o[j + 1], o[j + 2], o[j + 3]);
            }
        }
    }
    __syncthreads();
    // ---- 3x3 maxima from LDS
    for (int item = threadIdx.x; item < TP * TQ * CV; item += 256) {
        const int op = item / CV, c = item - op * CV;
        const int i = op / TQ, j = op - i * TQ;
        const int p = p0 + i, q = q0 + j;
        if (p >= P || q >= Q) continue;
        float m[V];
#pragma unroll
        for (int e = 0; e < V; ++e) m[e] = -INFINITY;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const float* src = patch + (size_t)((i * STRIDE + r) * PW + j * STRIDE + s) * C + c * V;
#pragma unroll
                for (int e = 0; e < V; e += 4) {
                    const float4 f = *reinterpret_cast<const float4*>(src + e);
                    m[e] = fmaxf(m[e], f.x); m[e + 1] = fmaxf(m[e + 1], f.y); m[e + 2] = fmaxf(m[e + 2], f.z); m[e + 3] = fmaxf(m[e + 3], f.w);
                }
            }
        Store<T>::stv(y + (((size_t)n * P + p) * Q + q) * C + c * V, m);
    }
}

template <typename T>
int pool_lrn_launch(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, const dr_lrn& l, bool lrn_first,
                    hipStream_t st)
{
    constexpr int VN = Store<T>::VN;
    if (tensor_elems(yd) == 0) return DR_OK;
    const int cv = xd.c / VN;
    int bx_log2 = 0;
    while ((1 << bx_log2) < cv) ++bx_log2;
    const int by = 256 >> bx_log2;
    const int qgroups = (yd.w + by - 1) / by;
    const int PRF = p.stride_h == 1 ? 4 : 2, strips = (yd.h + PRF - 1) / PRF;
    if ((double)yd.n * strips * qgroups >= 2147483648.0) return fail(DR_ERR_UNSUPPORTED, "lrn + pooling: tensor too large");
    if (lrn_first) {
        // through LDS where the fp32 patch of a tile fits 64 KB (two workgroups per compute unit)
        constexpr int TP1 = 4, TQ1 = 8, TP2 = 2, TQ2 = 8;
        const int s = p.stride_h;
        const int ph = s == 1 ? TP1 + 2 : (TP2 - 1) * 2 + 3, pw = s == 1 ? TQ1 + 2 : (TQ2 - 1) * 2 + 3;
        const size_t lds = (size_t)ph * pw * xd.c * sizeof(float);
        if (lds <= 64 * 1024) {
            const int tp = s == 1 ? TP1 : TP2, tq = s == 1 ? TQ1 : TQ2;
            const int ptiles = (yd.h + tp - 1) / tp, qtiles = (yd.w + tq - 1) / tq;
            const dim3 g2((unsigned)((long)yd.n * ptiles * qtiles));
            const float aon = l.alpha / (float)l.local_size;
            if (s == 1)
                hipLaunchKernelGGL((lrn_pool_lds_kernel<T, 1, TP1, TQ1>), g2, dim3(256), lds, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h,
                                   yd.w, ptiles, qtiles, bx_log2, p.pad_h, aon, l.beta, l.k, (int)(l.beta == 0.75f));
            else
                hipLaunchKernelGGL((lrn_pool_lds_kernel<T, 2, TP2, TQ2>), g2, dim3(256), lds, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h,
                                   yd.w, ptiles, qtiles, bx_log2, p.pad_h, aon, l.beta, l.k, (int)(l.beta == 0.75f));
            return check_launch("lrn_maxpool");
        }
    }
    const dim3 grid((unsigned)((long)yd.n * qgroups * strips));
    const float a_over_n = l.alpha / (float)l.local_size;
    const int b075 = (int)(l.beta == 0.75f);
#define DR_PL(PR, S, F) hipLaunchKernelGGL((pool_lrn_kernel<T, PR, S, F>), grid, dim3(256), 0, st, (const T*)x, (T*)y, xd.c, xd.h, xd.w, yd.h, yd.w, \
                                           strips, qgroups, bx_log2, p.pad_h, a_over_n, l.beta, l.k, b075)
    if (p.stride_h == 1) { if (lrn_first) DR_PL(4, 1, true); else DR_PL(4, 1, false); }
    else { if (lrn_first) DR_PL(2, 2, true); else DR_PL(2, 2, false); }
#undef DR_PL
    return check_launch(lrn_first ? "lrn_maxpool" : "maxpool_lrn");
}

// ---- concat ----------------------------------------------------------------------------------------------
struct ConcatArgs {
    const void* src[DR_MAX_BRANCHES];
    int c[DR_MAX_BRANCHES];       // channels of each input, in units of V
    int c_off[DR_MAX_BRANCHES];   // first output channel of each input, in units of V
    int nb;
};

// One lane per 16-byte group of the output pixel: the group's position picks the input it comes from.
template <typename T, int V>
__global__ __launch_bounds__(256) void concat_nhwc_kernel(ConcatArgs a, T* __restrict__ y, int CyV, size_t total)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int cv = (int)(i % CyV);
        const size_t pix = i / CyV;
        int b = 0;
#pragma unroll
        for (int j = 1; j < DR_MAX_BRANCHES; ++j)
            if (j < a.nb && cv >= a.c_off[j]) b = j;
        const T* src = (const T*)a.src[b] + (pix * a.c[b] + (cv - a.c_off[b])) * V;
        if constexpr (V == 1) y[i] = *src;
        else *reinterpret_cast<uint4*>(y + i * V) = *reinterpret_cast<const uint4*>(src);
    }
}

template <typename T>
int concat_launch(const dr_tensor& yd, int nb, const ConcatSeg* segs, void* y, hipStream_t st)
{
    constexpr int VN = Store<T>::VN;
    bool vec = aligned16(y) && yd.c % VN == 0;
    for (int i = 0; i < nb; ++i) vec = vec && aligned16(segs[i].src) && segs[i].c % VN == 0 && segs[i].c_off % VN == 0;
    const int v = vec ? VN : 1;
    ConcatArgs a;
    a.nb = nb;
    for (int i = 0; i < DR_MAX_BRANCHES; ++i) { a.src[i] = nullptr; a.c[i] = 0; a.c_off[i] = 0; }
    for (int i = 0; i < nb; ++i) { a.src[i] = segs[i].src; a.c[i] = segs[i].c / v; a.c_off[i] = segs[i].c_off / v; }
    const size_t total = (size_t)yd.n * yd.h * yd.w * (yd.c / v);
    if (total == 0) return DR_OK;
    const dim3 grid(blocks_for(total, 256, 256 * 64)), block(256);
    if (vec) hipLaunchKernelGGL((concat_nhwc_kernel<T, VN>), grid, block, 0, st, a, (T*)y, yd.c / v, total);
    else hipLaunchKernelGGL((concat_nhwc_kernel<T, 1>), grid, block, 0, st, a, (T*)y, yd.c, total);
    return check_launch("concat");
}

// ---- BatchNorm + Scale ----------------------------------------------------------------------------------
// BX (power of two >= C / V) lanes own one channel group each and keep its scale and shift in
// registers; the BY rows of the workgroup stride over the pixels.
template <typename T, int V>
__global__ __launch_bounds__(256) void bn_nhwc_kernel(const T* x, T* y, int C, size_t pixels, int bx_log2,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      const float* __restrict__ mean, const float* __restrict__ var, float eps,
                                                      int relu)
{
    const int CV = C / V;
    const int bx = 1 << bx_log2, by = 256 >> bx_log2;
    const int tx = threadIdx.x & (bx - 1), ty = threadIdx.x >> bx_log2;
    for (int cv = tx; cv < CV; cv += bx) {
        float sc[V], mu[V], sh[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int c = cv * V + j;
            sc[j] = 1.0f / sqrtf(var[c] + eps);
            mu[j] = mean[c];
            sh[j] = beta[c];
        }
        float ga[V];
#pragma unroll
        for (int j = 0; j < V; ++j) ga[j] = gamma[cv * V + j];
        for (size_t pix = (size_t)blockIdx.x * by + ty; pix < pixels; pix += (size_t)gridDim.x * by) {
            float v[V];
            const size_t off = pix * C + (size_t)cv * V;
            if constexpr (V == 1) v[0] = Store<T>::ld(x + off);
            else Store<T>::ldv(x + off, v);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                v[j] = ga[j] * ((v[j] - mu[j]) * sc[j]) + sh[j];
                if (relu) v[j] = fmaxf(v[j], 0.f);
            }
            if constexpr (V == 1) Store<T>::st(y + off, v[0]);
            else Store<T>::stv(y + off, v);
        }
    }
}

template <typename T>
int bn_launch(const dr_tensor& d, const void* x, void* y, const float* gamma, const float* beta, const float* mean,
              const float* var, float eps, int relu, hipStream_t st)
{
    constexpr int VN = Store<T>::VN;
    if (tensor_elems(d) == 0) return DR_OK;
    const bool vec = d.c % VN == 0 && aligned16(x) && aligned16(y);
    const int cv = vec ? d.c / VN : d.c;
    int bx_log2 = 0;
    while ((1 << bx_log2) < cv && bx_log2 < 8) ++bx_log2;
    const int by = 256 >> bx_log2;
    const size_t pixels = (size_t)d.n * d.h * d.w;
    const dim3 grid(blocks_for(pixels, by * 4, 256 * 32)), block(256);
    if (vec) hipLaunchKernelGGL((bn_nhwc_kernel<T, VN>), grid, block, 0, st, (const T*)x, (T*)y, d.c, pixels, bx_log2, gamma, beta, mean, var, eps, relu);
    else hipLaunchKernelGGL((bn_nhwc_kernel<T, 1>), grid, block, 0, st, (const T*)x, (T*)y, d.c, pixels, bx_log2, gamma, beta, mean, var, eps, relu);
    return check_launch("bn");
}

}  // namespace

namespace {

// ---- channel padding (bf16): lets a convolution whose channel count is not a multiple of 8 (the 3-channel
// network input) run in the matrix-core kernels, which fetch 16-byte channel groups ---------------------
// y[pix][0 .. Cp) = x[pix][0 .. C), zeros beyond; one thread per 16-byte group of y.
__global__ __launch_bounds__(256) void pad_channels_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ y, size_t groups,
                                                           int C, int Cp)
{
    const int gp = Cp / 8;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < groups; i += (size_t)gridDim.x * blockDim.x) {
        const size_t pix = i / gp;
        const int c0 = (int)(i - pix * gp) * 8;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = c0 + 2 * e < C ? x[pix * C + c0 + 2 * e] : 0u;
            const uint32_t hi = c0 + 2 * e + 1 < C ? x[pix * C + c0 + 2 * e + 1] : 0u;
            w[e] = lo | (hi << 16);
        }
        *reinterpret_cast<uint4*>(y + i * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// y[k][r][s][0 .. Cp) = w[k][c][r][s] (KCRS) or w[k][r][s][c] (KRSC), zeros beyond C
__global__ __launch_bounds__(256) void pad_filters_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ y, int K, int C, int RS,
                                                          int Cp, int krsc)
{
    const size_t total = (size_t)K * RS * Cp;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % Cp);
        const size_t t = i / Cp;
        const int rs = (int)(t % RS);
        const size_t k = t / RS;
        y[i] = c < C ? (krsc ? w[(k * RS + rs) * C + c] : w[(k * C + c) * RS + rs]) : (uint16_t)0;
    }
}

// xp[n][yy][xx][0..3] = x[n][yy - pad_h][xx - pad_w][0..C) where that pixel exists, else 0: one thread per pixel of xp
__global__ __launch_bounds__(256) void stem_pack_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ xp, int C, int H, int W,
                                                        int pad_h, int pad_w, int hp, int wp, size_t total)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int xx = (int)(i % wp);
        const size_t t = i / wp;
        const int yy = (int)(t % hp);
        const size_t n = t / hp;
        const int yi = yy - pad_h, xi = xx - pad_w;
        uint32_t e[4] = {0u, 0u, 0u, 0u};
        if ((unsigned)yi < (unsigned)H && (unsigned)xi < (unsigned)W) {
            const uint16_t* src = x + ((n * H + yi) * W + xi) * C;
#pragma unroll
            for (int c = 0; c < 4; ++c) e[c] = c < C ? src[c] : 0u;
        }
        *reinterpret_cast<uint2*>(xp + i * 4) = make_uint2(e[0] | (e[1] << 16), e[2] | (e[3] << 16));
    }
}

// The same copy, a workgroup per PACK_ROWS rows of xp: the input rows are fetched whole with 16-byte loads into LDS
// (an input row of W * C bf16 values must be a multiple of 16 bytes, x 16-byte aligned) and the pixels are picked
// out of LDS; two pixels of xp per thread and 16-byte store.  A quarter of the load instructions of the kernel above.
constexpr int PACK_ROWS = 4;
__global__ __launch_bounds__(256) void stem_pack_rows_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ xp, int C, int H, int W,
                                                             int pad_h, int pad_w, int hp, int wp)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char pack_lds[];
    const int row_bytes = W * C * 2, chunks = row_bytes >> 4, pairs = wp >> 1;
    const int groups = (hp + PACK_ROWS - 1) / PACK_ROWS;
    const int n = blockIdx.x / groups, yy0 = (blockIdx.x - n * groups) * PACK_ROWS;
    for (int i = threadIdx.x; i < PACK_ROWS * chunks; i += blockDim.x) {
        const int r = i / chunks, ch = i - r * chunks, yi = yy0 + r - pad_h;
        if (yy0 + r < hp && (unsigned)yi < (unsigned)H)
            *reinterpret_cast<uint4*>(pack_lds + r * row_bytes + ch * 16) =
                *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(x) + ((size_t)n * H + yi) * row_bytes + ch * 16);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < PACK_ROWS * pairs; i += blockDim.x) {
        const int r = i / pairs, pr = i - r * pairs, yy = yy0 + r, yi = yy - pad_h;
        if (yy >= hp) continue;
        uint32_t e[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        if ((unsigned)yi < (unsigned)H) {
            const uint16_t* row = reinterpret_cast<const uint16_t*>(pack_lds + r * row_bytes);
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int xi = 2 * pr + k - pad_w;
                if ((unsigned)xi < (unsigned)W) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) e[4 * k + c] = c < C ? row[xi * C + c] : 0u;
                }
            }
        }
        *reinterpret_cast<uint4*>(xp + (((size_t)n * hp + yy) * wp + 2 * pr) * 4) =
            make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

// wp8[k][r][s][c] (8 x 8 x 4 per filter) = w[k][c][r][s] (KCRS) or w[k][r][s][c] (KRSC) inside R x S x C, else 0
__global__ __launch_bounds__(256) void stem_filters_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ y, int K, int C, int R,
                                                           int S, int krsc)
{
    const int total = K * 256;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int c = i & 3, s = (i >> 2) & 7, r = (i >> 5) & 7, k = i >> 8;
        uint16_t v = 0;
        if (c < C && r < R && s < S) v = krsc ? w[((k * R + r) * S + s) * C + c] : w[((k * C + c) * R + r) * S + s];
        y[i] = v;
    }
}

}  // namespace

int launch_stem_pack_bf16(const void* x, void* xp, int N, int C, int H, int W, int pad_h, int pad_w, int hp, int wp, hipStream_t st)
{
    TraceScope trace("conv_pad", nullptr, (long long)((size_t)N * hp * wp * 4), st);
    const size_t total = (size_t)N * hp * wp;
    if (total == 0) return DR_OK;
    const size_t row_bytes = (size_t)W * C * 2;
    const size_t groups = (size_t)N * ((hp + PACK_ROWS - 1) / PACK_ROWS);
    if (row_bytes % 16 == 0 && PACK_ROWS * row_bytes <= 48 * 1024 && aligned16(x) && aligned16(xp) && wp % 2 == 0 && groups < (1u << 31)) {
        hipLaunchKernelGGL(stem_pack_rows_kernel, dim3((unsigned)groups), dim3(256), PACK_ROWS * row_bytes, st, (const uint16_t*)x,
                           (uint16_t*)xp, C, H, W, pad_h, pad_w, hp, wp);
        return check_launch("stem_pack");
    }
    hipLaunchKernelGGL(stem_pack_kernel, dim3(blocks_for(total, 256, 256 * 64)), dim3(256), 0, st, (const uint16_t*)x, (uint16_t*)xp, C, H, W,
                       pad_h, pad_w, hp, wp, total);
    return check_launch("stem_pack");
}

int launch_stem_filters_bf16(const void* w, void* wp8, int K, int C, int R, int S, int krsc, hipStream_t st)
{
    TraceScope trace("conv_pad", nullptr, (long long)K * 256, st);
    if (K == 0) return DR_OK;
    hipLaunchKernelGGL(stem_filters_kernel, dim3(blocks_for((size_t)K * 256, 256, 1024)), dim3(256), 0, st, (const uint16_t*)w, (uint16_t*)wp8, K, C,
                       R, S, krsc);
    return check_launch("stem_filters");
}

int launch_pad_channels_bf16(const void* x, void* y, size_t pixels, int C, int Cp, hipStream_t st)
{
    TraceScope trace("conv_pad", nullptr, (long long)(pixels * Cp), st);
    const size_t groups = pixels * (Cp / 8);
    if (groups == 0) return DR_OK;
    hipLaunchKernelGGL(pad_channels_kernel, dim3(blocks_for(groups, 256, 256 * 64)), dim3(256), 0, st, (const uint16_t*)x, (uint16_t*)y, groups, C, Cp);
    return check_launch("pad_channels");
}

int launch_pad_filters_bf16(const void* w, void* y, int K, int C, int RS, int Cp, int krsc, hipStream_t st)
{
    TraceScope trace("conv_pad", nullptr, (long long)((size_t)K * RS * Cp), st);
    const size_t total = (size_t)K * RS * Cp;
    if (total == 0) return DR_OK;
    hipLaunchKernelGGL(pad_filters_kernel, dim3(blocks_for(total, 256, 4096)), dim3(256), 0, st, (const uint16_t*)w, (uint16_t*)y, K, C, RS, Cp, krsc);
    return check_launch("pad_filters");
}

int launch_pool_nhwc(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, bool avg, hipStream_t st)
{
    return xd.dtype == DR_BF16 ? pool_launch<uint16_t>(xd, x, yd, y, p, avg, st) : pool_launch<float>(xd, x, yd, y, p, avg, st);
}

int launch_lrn_nhwc(const dr_tensor& d, const void* x, void* y, const dr_lrn& p, hipStream_t st)
{
    return d.dtype == DR_BF16 ? lrn_launch<uint16_t>(d, x, y, p, st) : lrn_launch<float>(d, x, y, p, st);
}

bool pool_lrn_nhwc_supported(const dr_tensor& xd, const void* x, const void* y, const dr_pool& p, const dr_lrn& l)
{
    const int vn = xd.dtype == DR_BF16 ? 8 : 4;
    return xd.layout == DR_NHWC && xd.c % vn == 0 && xd.c / vn <= 64 && aligned16(x) && aligned16(y) && p.kh == 3 && p.kw == 3 &&
           p.stride_h == p.stride_w && (p.stride_h == 1 || p.stride_h == 2) && p.pad_h == p.pad_w && p.pad_h <= 1 && l.local_size == 5;
}

int launch_pool_lrn_nhwc(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, const dr_lrn& l, bool lrn_first,
                         hipStream_t st)
{
    TraceScope trace(lrn_first ? "lrn_maxpool" : "maxpool_lrn", nullptr, (long long)tensor_elems(yd), st,
                     (long long)(tensor_bytes(xd) + tensor_bytes(yd)));
    return xd.dtype == DR_BF16 ? pool_lrn_launch<uint16_t>(xd, x, yd, y, p, l, lrn_first, st)
                               : pool_lrn_launch<float>(xd, x, yd, y, p, l, lrn_first, st);
}

int launch_concat_nhwc(const dr_tensor& yd, int nb, const ConcatSeg* segs, void* y, hipStream_t st)
{
    return yd.dtype == DR_BF16 ? concat_launch<uint16_t>(yd, nb, segs, y, st) : concat_launch<float>(yd, nb, segs, y, st);
}

int launch_bn_nhwc(const dr_tensor& d, const void* x, void* y, const float* gamma, const float* beta, const float* mean,
                   const float* var, float eps, int relu, hipStream_t st)
{
    return d.dtype == DR_BF16 ? bn_launch<uint16_t>(d, x, y, gamma, beta, mean, var, eps, relu, st)
                              : bn_launch<float>(d, x, y, gamma, beta, mean, var, eps, relu, st);
}

}  // namespace dr
