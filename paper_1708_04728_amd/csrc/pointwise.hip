// Bandwidth-bound layers: ReLU, across-channel LRN, max/avg pooling, concat, BatchNorm(+Scale),
// residual add, plus the small classifier tail (inner product, softmax).  NCHW; fp32 or bf16 storage,
// fp32 arithmetic.  Every kernel reads each input element once from HBM (neighbouring windows are
// served by the caches) and writes each output once, with 16-byte accesses where the shape allows.
#include "dr_internal.h"
#include "dr_store.h"

namespace dr {
namespace {

// ---- ReLU / add+ReLU -----------------------------------------------------------------------------
// ADD = false: y = max(a, 0);  ADD = true: y = max(a + b, 0).
template <typename T, bool ADD>
__global__ __launch_bounds__(256) void relu_kernel(const T* a, const T* b, T* y,
                                                   size_t nvec, size_t count)
{
    constexpr int VN = Store<T>::VN;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        float v[VN], u[VN];
        Store<T>::ldv(a + i * VN, v);
        if constexpr (ADD) Store<T>::ldv(b + i * VN, u);
#pragma unroll
        for (int j = 0; j < VN; ++j) v[j] = fmaxf(ADD ? v[j] + u[j] : v[j], 0.f);
        Store<T>::stv(y + i * VN, v);
    }
    // scalar tail (and the whole tensor when the pointers are not 16-byte aligned: nvec = 0)
    for (size_t i = nvec * VN + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        float v = Store<T>::ld(a + i);
        if (ADD) v += Store<T>::ld(b + i);
        Store<T>::st(y + i, fmaxf(v, 0.f));
    }
}

template <typename T, bool ADD>
int relu_launch(const void* a, const void* b, void* y, size_t count, hipStream_t st)
{
    if (count == 0) return DR_OK;
    constexpr int VN = Store<T>::VN;
    const bool vec = aligned16(a) && aligned16(y) && (!ADD || aligned16(b));
    const size_t nvec = vec ? count / VN : 0;
    const unsigned grid = blocks_for(nvec ? nvec : count, 256, 256 * 16);
    hipLaunchKernelGGL((relu_kernel<T, ADD>), dim3(grid), dim3(256), 0, st, (const T*)a, (const T*)b, (T*)y, nvec, count);
    return check_launch(ADD ? "add_relu" : "relu");
}

// ---- LRN ---------------------------------------------------------------------------------------------
// (s^-beta: pow_neg_beta in dr_store.h)

// One thread owns V adjacent pixels (one 16-byte vector, or one element when V == 1) of one image and a
// run of CH channels.  It first issues all CH + NL - 1 loads of the run and its halo (independent, so
// they overlap in the memory system), then slides the window of NL channels over the registers.
template <typename T, int V, int NL, int CH>
__global__ __launch_bounds__(256) void lrn_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int HW, int HWv,
                                                  int nruns, float a_over_n, float beta, float k, int b075)
{
    const int pv = blockIdx.x * blockDim.x + threadIdx.x;
    if (pv >= HWv) return;
    const int n = blockIdx.y / nruns, run = blockIdx.y - n * nruns;
    const int c0 = run * CH;
    constexpr int LO = NL / 2;                    // window of channel c = [c - LO, c - LO + NL)
    const T* xb = x + (size_t)n * C * HW + (size_t)pv * V;
    T* yb = y + (size_t)n * C * HW + (size_t)pv * V;

    float v[CH + NL - 1][V];                      // channels c0 - LO .. c0 + CH + NL - 2 - LO
#pragma unroll
    for (int i = 0; i < CH + NL - 1; ++i) {
        const int c = c0 - LO + i;
        if (c >= 0 && c < C) {
            if constexpr (V == 1) v[i][0] = Store<T>::ld(xb + (size_t)c * HW);
            else Store<T>::ldv(xb + (size_t)c * HW, v[i]);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) v[i][j] = 0.f;
        }
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        if (c0 + i >= C) break;
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float ss = 0.f;
#pragma unroll
            for (int w = 0; w < NL; ++w) ss = fmaf(v[i + w][j], v[i + w][j], ss);
            o[j] = v[i + LO][j] * pow_neg_beta(fmaf(a_over_n, ss, k), beta, b075);
        }
        if constexpr (V == 1) Store<T>::st(yb + (size_t)(c0 + i) * HW, o[0]);
        else Store<T>::stv(yb + (size_t)(c0 + i) * HW, o);
    }
}

// Any window length: every output re-reads its window (served by the caches).
template <typename T>
__global__ __launch_bounds__(256) void lrn_generic_kernel(const T* __restrict__ x, T* __restrict__ y, int C, int HW,
                                                          size_t total, int nl, float a_over_n, float beta, float k)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int pix = (int)(i % HW);
        const size_t nc = i / HW;
        const int c = (int)(nc % C);
        const size_t n = nc / C;
        float ss = 0.f;
        for (int cc = c - nl / 2; cc < c - nl / 2 + nl; ++cc)
            if (cc >= 0 && cc < C) {
                const float v = Store<T>::ld(x + (n * C + cc) * HW + pix);
                ss = fmaf(v, v, ss);
            }
        Store<T>::st(y + i, Store<T>::ld(x + i) * powf(fmaf(a_over_n, ss, k), -beta));
    }
}

template <typename T>
int lrn_launch(const void* x, void* y, int N, int C, int HW, const dr_lrn& p, hipStream_t st)
{
    const float a_over_n = p.alpha / (float)p.local_size;
    if (p.local_size != 5) {
        const size_t total = (size_t)N * C * HW;
        hipLaunchKernelGGL((lrn_generic_kernel<T>), dim3(blocks_for(total, 256, 256 * 32)), dim3(256), 0, st, (const T*)x,
                           (T*)y, C, HW, total, p.local_size, a_over_n, p.beta, p.k);
        return check_launch("lrn");
    }
    constexpr int VN = Store<T>::VN;
    constexpr int CH = 64 / VN;                   // channels per run: (CH + 4) * VN registers of window
    const bool vec = (HW % VN == 0) && aligned16(x) && aligned16(y);
    const int HWv = vec ? HW / VN : HW;
    const int nruns = (C + CH - 1) / CH;
    if ((long)N * nruns > 65535) return fail(DR_ERR_UNSUPPORTED, "lrn: batch %d x %d channel runs exceeds the grid limit", N, nruns);
    const dim3 grid((HWv + 255) / 256, (unsigned)(N * (vec ? nruns : (C + 15) / 16)));
    const int b075 = p.beta == 0.75f;
    if (vec && (long)N * HWv * nruns < 65536 && (long)N * ((C + 3) / 4) <= 65535) {
        // small tensor: shorter runs (more halo re-reads, served by the caches) to put more waves to work
        const int nr4 = (C + 3) / 4;
        hipLaunchKernelGGL((lrn_kernel<T, VN, 5, 4>), dim3((HWv + 255) / 256, (unsigned)(N * nr4)), dim3(256), 0, st, (const T*)x,
                           (T*)y, C, HW, HWv, nr4, a_over_n, p.beta, p.k, b075);
        return check_launch("lrn");
    }
    if (vec)
        hipLaunchKernelGGL((lrn_kernel<T, VN, 5, CH>), grid, dim3(256), 0, st, (const T*)x, (T*)y, C, HW, HWv, nruns, a_over_n,
                           p.beta, p.k, b075);
    else
        hipLaunchKernelGGL((lrn_kernel<T, 1, 5, 16>), grid, dim3(256), 0, st, (const T*)x, (T*)y, C, HW, HWv, (C + 15) / 16,
                           a_over_n, p.beta, p.k, b075);
    return check_launch("lrn");
}

// ---- pooling --------------------------------------------------------------------------------------------
// A workgroup computes PR output rows of one (n, c) plane.  The input rows those windows touch are one
// contiguous range of the plane: it is copied to LDS with coalesced loads (every input element is
// fetched from global memory once, all loads of a workgroup in flight together), then each thread
// reduces its windows out of LDS.  AVG = false: maximum over the window clipped to the input
// (padding never wins);  AVG = true: mean over the full window (no padding allowed).
constexpr int POOL_LDS_BYTES = 32 * 1024;

template <typename T, bool AVG>
__global__ __launch_bounds__(256) void pool_kernel(const T* __restrict__ x, T* __restrict__ y, int H, int W, int P, int Q,
                                                   int PR, int pgroups, float inv_q, dr_pool p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char pool_lds[];   // (PR - 1) * stride + kh rows of W elements
    T* tile = reinterpret_cast<T*>(pool_lds);
    const unsigned plane = blockIdx.x / (unsigned)pgroups;
    const int p0 = (int)(blockIdx.x - plane * (unsigned)pgroups) * PR;
    const int p1 = min(p0 + PR, P);
    const int h_lo = max(p0 * p.stride_h - p.pad_h, 0);
    const int h_hi = min((p1 - 1) * p.stride_h - p.pad_h + p.kh, H);      // exclusive
    const T* src = x + (size_t)plane * H * W + (size_t)h_lo * W;
    const int count = (h_hi - h_lo) * W;
    for (int base = 0; base < count; base += 256 * 8) {      // 8 independent loads in flight per thread
        T r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = base + j * 256 + threadIdx.x;
            r[j] = i < count ? src[i] : T(0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = base + j * 256 + threadIdx.x;
            if (i < count) tile[i] = r[j];
        }
    }
    __syncthreads();
    T* yb = y + ((size_t)plane * P + p0) * Q;
    const int outs = (p1 - p0) * Q;
    for (int i = threadIdx.x; i < outs; i += 256) {
        int pr = (int)(((float)i + 0.5f) * inv_q);                          // i / Q for i < 2^20
        int q = i - pr * Q;
        if (q < 0) { --pr; q += Q; } else if (q >= Q) { ++pr; q -= Q; }
        const int h0 = (p0 + pr) * p.stride_h - p.pad_h, w0 = q * p.stride_w - p.pad_w;
        const int ha = max(h0, 0), hb = min(h0 + p.kh, H);
        const int wa = max(w0, 0), wb = min(w0 + p.kw, W);
        float m = AVG ? 0.f : -INFINITY;
        if (p.kh == 3 && p.kw == 3 && hb - ha == 3 && wb - wa == 3) {
            // whole 3x3 window inside the input (all but the edge windows): straight-line code
            const T* t = &tile[(ha - h_lo) * W + wa];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    const float v = Store<T>::ld(t + r * W + c);
                    m = AVG ? m + v : fmaxf(m, v);
                }
        } else {
            for (int h = ha; h < hb; ++h)
                for (int w = wa; w < wb; ++w) {
                    const float v = Store<T>::ld(&tile[(h - h_lo) * W + w]);
                    m = AVG ? m + v : fmaxf(m, v);
                }
        }
        if (AVG) m /= (float)(p.kh * p.kw);
        Store<T>::st(yb + i, m);
    }
}

template <typename T, bool AVG>
int pool_launch(const void* x, void* y, int NC, int H, int W, int P, int Q, const dr_pool& p, hipStream_t st)
{
    if ((size_t)NC * P * Q == 0) return DR_OK;
    // output rows per workgroup: as many as fit the LDS tile, at most ~4 outputs per thread
    const int rows_fit = (int)(POOL_LDS_BYTES / sizeof(T)) / W;
    if (rows_fit < p.kh) return fail(DR_ERR_UNSUPPORTED, "pooling: rows of %d elements do not fit the LDS tile", W);
    int PR = (rows_fit - p.kh) / p.stride_h + 1;
    const int cap = (1024 + Q - 1) / Q;
    if (PR > cap) PR = cap;
    if (PR > P) PR = P;
    const int pgroups = (P + PR - 1) / PR;
    if ((double)NC * pgroups >= 2147483648.0 || (double)PR * Q >= 1048576.0) return fail(DR_ERR_UNSUPPORTED, "pooling: tensor too large");
    const size_t lds = (size_t)((PR - 1) * p.stride_h + p.kh) * W * sizeof(T);
    hipLaunchKernelGGL((pool_kernel<T, AVG>), dim3((unsigned)(NC * pgroups)), dim3(256), lds, st, (const T*)x, (T*)y, H, W, P, Q, PR,
                       pgroups, 1.0f / (float)Q, p);
    return check_launch(AVG ? "avgpool" : "maxpool");
}

// ---- concat ----------------------------------------------------------------------------------------------
struct ConcatArgs {
    const void* src[DR_MAX_BRANCHES];
    int c[DR_MAX_BRANCHES];
    int c_off[DR_MAX_BRANCHES];
};

// blockIdx.z = branch, blockIdx.y = image; within an image a branch is one contiguous run of c*HW
// elements in both the source and the destination.
template <typename T, int V>
__global__ __launch_bounds__(256) void concat_kernel(ConcatArgs a, T* __restrict__ y, int Cy, int HW)
{
    const int b = blockIdx.z, n = blockIdx.y;
    const size_t run = (size_t)a.c[b] * HW;
    const T* src = (const T*)a.src[b] + (size_t)n * run;
    T* dst = y + ((size_t)n * Cy + a.c_off[b]) * HW;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i * V < run; i += stride) {
        if constexpr (V == 1) dst[i] = src[i];
        else *reinterpret_cast<uint4*>(dst + i * V) = *reinterpret_cast<const uint4*>(src + i * V);
    }
}

template <typename T>
int concat_launch(int nb, const ConcatSeg* segs, void* y, int N, int Cy, int HW, hipStream_t st)
{
    constexpr int VN = Store<T>::VN;
    ConcatArgs a;
    bool vec = aligned16(y) && ((size_t)Cy * HW % VN == 0);
    int cmax = 0;
    for (int i = 0; i < nb; ++i) {
        a.src[i] = segs[i].src; a.c[i] = segs[i].c; a.c_off[i] = segs[i].c_off;
        vec = vec && aligned16(segs[i].src) && ((size_t)segs[i].c * HW % VN == 0) && ((size_t)segs[i].c_off * HW % VN == 0);
        if (segs[i].c > cmax) cmax = segs[i].c;
    }
    if (N == 0 || cmax == 0 || HW == 0) return DR_OK;
    if (N > 65535) return fail(DR_ERR_UNSUPPORTED, "concat: batch %d exceeds 65535", N);
    const size_t items = (size_t)cmax * HW / (vec ? VN : 1);
    const dim3 grid(blocks_for(items, 256 * 4, 4096), (unsigned)N, (unsigned)nb);
    if (vec) hipLaunchKernelGGL((concat_kernel<T, VN>), grid, dim3(256), 0, st, a, (T*)y, Cy, HW);
    else hipLaunchKernelGGL((concat_kernel<T, 1>), grid, dim3(256), 0, st, a, (T*)y, Cy, HW);
    return check_launch("concat");
}

// ---- filter repack KCRS -> KRSC -----------------------------------------------------------------
// One thread per output element (lanes along c: coalesced writes; the strided reads hit the caches).
template <typename T>
__global__ __launch_bounds__(256) void pack_filters_kernel(const T* __restrict__ src, T* __restrict__ dst, int C, int RS,
                                                           size_t total)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int c = (int)(i % C);
        const size_t t = i / C;
        const int rs = (int)(t % RS);
        const size_t k = t / RS;
        dst[i] = src[(k * C + c) * RS + rs];
    }
}

// ---- BatchNorm + Scale ------------------------------------------------------------------------------
// blockIdx.y walks the (n, c) planes, so the four per-channel parameters are wave-uniform.
template <typename T, int V>
__global__ __launch_bounds__(256) void bn_kernel(const T* x, T* y, int NC, int C, int HW,
                                                 const float* __restrict__ gamma, const float* __restrict__ beta,
                                                 const float* __restrict__ mean, const float* __restrict__ var, float eps,
                                                 int relu)
{
    for (int plane = blockIdx.y; plane < NC; plane += gridDim.y) {
        const int c = plane % C;
        const float mu = mean[c];
        const float inv = 1.0f / sqrtf(var[c] + eps);
        const float ga = gamma[c], be = beta[c];
        const T* xb = x + (size_t)plane * HW;
        T* yb = y + (size_t)plane * HW;
        for (int i = blockIdx.x * blockDim.x + threadIdx.x; i * V < HW; i += gridDim.x * blockDim.x) {
            float v[V];
            if constexpr (V == 1) v[0] = Store<T>::ld(xb + i);
            else Store<T>::ldv(xb + (size_t)i * V, v);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                v[j] = ga * ((v[j] - mu) * inv) + be;
                if (relu) v[j] = fmaxf(v[j], 0.f);
            }
            if constexpr (V == 1) Store<T>::st(yb + i, v[0]);
            else Store<T>::stv(yb + (size_t)i * V, v);
        }
    }
}

template <typename T>
int bn_launch(const void* x, void* y, int N, int C, int HW, const float* gamma, const float* beta, const float* mean,
              const float* var, float eps, int relu, hipStream_t st)
{
    if ((size_t)N * C * HW == 0) return DR_OK;
    constexpr int VN = Store<T>::VN;
    const bool vec = (HW % VN == 0) && aligned16(x) && aligned16(y);
    const int items = vec ? HW / VN : HW;
    const dim3 grid(blocks_for(items, 256, 64), (unsigned)((size_t)N * C < 32768 ? N * C : 32768));
    if (vec)
        hipLaunchKernelGGL((bn_kernel<T, VN>), grid, dim3(256), 0, st, (const T*)x, (T*)y, N * C, C, HW, gamma, beta, mean, var, eps,
                           relu);
    else
        hipLaunchKernelGGL((bn_kernel<T, 1>), grid, dim3(256), 0, st, (const T*)x, (T*)y, N * C, C, HW, gamma, beta, mean, var, eps,
                           relu);
    return check_launch("bn");
}

// ---- inner product ---------------------------------------------------------------------------------
// One wave per output unit o and a slice of the batch: lanes stride over the inputs (coalesced
// reads of the weight row and of the activation row), then a butterfly reduction.
template <typename T>
__global__ __launch_bounds__(64) void fc_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                const float* __restrict__ bias, T* __restrict__ y, int N, int I, int O)
{
    const int o = blockIdx.x, lane = threadIdx.x;
    const float b = bias ? bias[o] : 0.f;
    const T* wr = w + (size_t)o * I;
    for (int n = blockIdx.y; n < N; n += gridDim.y) {
        const T* xr = x + (size_t)n * I;
        float acc = 0.f;
        for (int i = lane; i < I; i += 64) acc = fmaf(Store<T>::ld(wr + i), Store<T>::ld(xr + i), acc);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) Store<T>::st(y + (size_t)n * O + o, acc + b);
    }
}

// ---- softmax ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void softmax_kernel(const T* __restrict__ x, float* __restrict__ y, int O)
{
    __shared__ float red[4];
    const T* xb = x + (size_t)blockIdx.x * O;
    float* yb = y + (size_t)blockIdx.x * O;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float m = -INFINITY;
    for (int i = threadIdx.x; i < O; i += 256) m = fmaxf(m, Store<T>::ld(xb + i));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.f;
    for (int i = threadIdx.x; i < O; i += 256) s += expf(Store<T>::ld(xb + i) - m);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    s = (red[0] + red[1]) + (red[2] + red[3]);
    for (int i = threadIdx.x; i < O; i += 256) yb[i] = expf(Store<T>::ld(xb + i) - m) / s;
}

}  // namespace

#define DR_BY_DTYPE(dtype, call_f32, call_bf16) ((dtype) == DR_BF16 ? (call_bf16) : (call_f32))

int launch_pack_filters(int dtype, const void* w_kcrs, void* w_krsc, int K, int C, int RS, hipStream_t st)
{
    const size_t total = (size_t)K * C * RS;
    TraceScope trace("pack_filters", nullptr, (long long)total, st);
    if (dtype == DR_BF16)
        hipLaunchKernelGGL((pack_filters_kernel<uint16_t>), dim3(blocks_for(total, 256, 4096)), dim3(256), 0, st,
                           (const uint16_t*)w_kcrs, (uint16_t*)w_krsc, C, RS, total);
    else
        hipLaunchKernelGGL((pack_filters_kernel<float>), dim3(blocks_for(total, 256, 4096)), dim3(256), 0, st,
                           (const float*)w_kcrs, (float*)w_krsc, C, RS, total);
    return check_launch("pack_filters");
}

int launch_relu(int dtype, const void* x, void* y, size_t count, hipStream_t st)
{
    TraceScope trace("relu", nullptr, (long long)(count), st, 2ll * count * elem_size(dtype));
    return DR_BY_DTYPE(dtype, (relu_launch<float, false>(x, nullptr, y, count, st)),
                       (relu_launch<uint16_t, false>(x, nullptr, y, count, st)));
}

int launch_add_relu(int dtype, const void* a, const void* b, void* y, size_t count, hipStream_t st)
{
    TraceScope trace("add_relu", nullptr, (long long)(count), st, 3ll * count * elem_size(dtype));
    return DR_BY_DTYPE(dtype, (relu_launch<float, true>(a, b, y, count, st)), (relu_launch<uint16_t, true>(a, b, y, count, st)));
}

int launch_lrn(const dr_tensor& d, const void* x, void* y, const dr_lrn& p, hipStream_t st)
{
    TraceScope trace("lrn", nullptr, (long long)tensor_elems(d), st, 2ll * tensor_bytes(d));
    if (tensor_elems(d) == 0) return DR_OK;
    if (d.layout == DR_NHWC) return launch_lrn_nhwc(d, x, y, p, st);
    return DR_BY_DTYPE(d.dtype, lrn_launch<float>(x, y, d.n, d.c, d.h * d.w, p, st), lrn_launch<uint16_t>(x, y, d.n, d.c, d.h * d.w, p, st));
}

int launch_maxpool(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, hipStream_t st)
{
    TraceScope trace("maxpool", nullptr, (long long)tensor_elems(yd), st, (long long)(tensor_bytes(xd) + tensor_bytes(yd)));
    if (xd.layout == DR_NHWC) return launch_pool_nhwc(xd, x, yd, y, p, false, st);
    return DR_BY_DTYPE(xd.dtype, (pool_launch<float, false>(x, y, xd.n * xd.c, xd.h, xd.w, yd.h, yd.w, p, st)),
                       (pool_launch<uint16_t, false>(x, y, xd.n * xd.c, xd.h, xd.w, yd.h, yd.w, p, st)));
}

int launch_avgpool(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, hipStream_t st)
{
    TraceScope trace("avgpool", nullptr, (long long)tensor_elems(yd), st, (long long)(tensor_bytes(xd) + tensor_bytes(yd)));
    if (xd.layout == DR_NHWC) return launch_pool_nhwc(xd, x, yd, y, p, true, st);
    return DR_BY_DTYPE(xd.dtype, (pool_launch<float, true>(x, y, xd.n * xd.c, xd.h, xd.w, yd.h, yd.w, p, st)),
                       (pool_launch<uint16_t, true>(x, y, xd.n * xd.c, xd.h, xd.w, yd.h, yd.w, p, st)));
}

int launch_concat(const dr_tensor& yd, int nb, const ConcatSeg* segs, void* y, hipStream_t st)
{
    TraceScope trace("concat", nullptr, (long long)tensor_elems(yd), st, 2ll * tensor_bytes(yd));
    if (yd.layout == DR_NHWC) return launch_concat_nhwc(yd, nb, segs, y, st);
    return DR_BY_DTYPE(yd.dtype, concat_launch<float>(nb, segs, y, yd.n, yd.c, yd.h * yd.w, st),
                       concat_launch<uint16_t>(nb, segs, y, yd.n, yd.c, yd.h * yd.w, st));
}

int launch_bn(const dr_tensor& d, const void* x, void* y, const float* gamma, const float* beta, const float* mean,
              const float* var, float eps, int relu, hipStream_t st)
{
    TraceScope trace("bn", nullptr, (long long)tensor_elems(d), st, 2ll * tensor_bytes(d));
    if (d.layout == DR_NHWC) return launch_bn_nhwc(d, x, y, gamma, beta, mean, var, eps, relu, st);
    return DR_BY_DTYPE(d.dtype, bn_launch<float>(x, y, d.n, d.c, d.h * d.w, gamma, beta, mean, var, eps, relu, st),
                       bn_launch<uint16_t>(x, y, d.n, d.c, d.h * d.w, gamma, beta, mean, var, eps, relu, st));
}

int launch_fc(int dtype, const void* x, const void* w, const float* bias, void* y, int N, int I, int O, hipStream_t st)
{
    TraceScope trace("fc", nullptr, (long long)((size_t)N * O), st);
    if (N == 0 || O == 0) return DR_OK;
    if (dtype == DR_BF16) {
        // an inner product is a 1x1 convolution over a one-pixel image: y[n][o] = sum_i w[o][i] x[n][i] runs on
        // the matrix cores through the streaming convolution kernel when its layout conditions hold
        ConvGeom g;
        g.N = N; g.C = I; g.H = g.W = 1; g.K = O; g.R = g.S = 1; g.sh = g.sw = 1; g.ph = g.pw = 0; g.P = g.Q = 1;
        g.Kg = I; g.Ng = N; g.y_ctot = O; g.y_coff = 0; g.relu = 0; g.res_ctot = 0; g.w_krsc = 1; g.nhwc = 1; g.c_logical = 0;
        if (conv_bf16_dma_eligible(g, x, w))
            return launch_conv_bf16_dma(g, (const uint16_t*)x, (const uint16_t*)w, bias, nullptr, (uint16_t*)y, st);
    }
    const dim3 grid((unsigned)O, (unsigned)(N < 8 ? N : 8));
    if (dtype == DR_BF16)
        hipLaunchKernelGGL((fc_kernel<uint16_t>), grid, dim3(64), 0, st, (const uint16_t*)x, (const uint16_t*)w, bias, (uint16_t*)y, N, I, O);
    else
        hipLaunchKernelGGL((fc_kernel<float>), grid, dim3(64), 0, st, (const float*)x, (const float*)w, bias, (float*)y, N, I, O);
    return check_launch("fc");
}

int launch_softmax(int dtype, const void* x, float* y, int N, int O, hipStream_t st)
{
    TraceScope trace("softmax", nullptr, (long long)((size_t)N * O), st, (long long)((size_t)N * O * (elem_size(dtype) + 4)));
    if (N == 0 || O == 0) return DR_OK;
    if (dtype == DR_BF16) hipLaunchKernelGGL((softmax_kernel<uint16_t>), dim3(N), dim3(256), 0, st, (const uint16_t*)x, y, O);
    else hipLaunchKernelGGL((softmax_kernel<float>), dim3(N), dim3(256), 0, st, (const float*)x, y, O);
    return check_launch("softmax");
}

}  // namespace dr
