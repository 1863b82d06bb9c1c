// Layer-wise regression of a slim layer (Sec. 3.1: the optimisation goal below Eq. (4), Lemma 1): the slim
// layer f~(W, b; X) = max(conv(X; W, b), 0) is fitted to the feature map Y of the block it replaces by
// gradient descent on L(W, b) = sum || Y - f~(W, b; X) ||^2.  fp32, NCHW tensors, KCRS filters.
//
//   regression_loss_grad   dz = 2 (f - y) where f > 0 else 0,  L = sum (f - y)^2
//   conv_wgrad             dw[k][c,r,s] = sum_{n,p,q} dz[n,k,p,q] x[n,c,p*sh+r-ph,q*sw+s-pw],  db[k] = sum dz[n,k,p,q]
//                          (db is column C*R*S of the same GEMM: the gathered operand is 1 there)
//   sgd_step               w -= lr * dw
//
// The weight gradient is a GEMM  D[m][n] = sum_l A[m][l] B[l][n]  with m = filter, n = (c, r, s) and the
// contraction over l = (image, p, q): A is dz (for one image and filter the (p, q) run is contiguous), B is
// gathered from x.  A workgroup owns a 64 x 64 tile of D for a range of images, stages 32 l at a time in LDS
// (l contiguous per row, rows padded by 4 floats) and multiplies with v_mfma_f32_32x32x2_f32, each lane half
// taking 16 consecutive l of the slice so that an operand is four 128-bit LDS reads.  The ranges of images
// give enough workgroups to fill the device; their partial sums go to workspace and are added in a fixed
// order by a second kernel, so the result does not depend on scheduling.
#include "dr_internal.h"

namespace dr {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int OOB = (int)0x80000000;

// grid of a grid-stride kernel: at most 4096 workgroups (the loss kernel leaves one partial sum per workgroup)
inline unsigned blocks_for_train(size_t count)
{
    const size_t b = (count + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, int voff, int soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}

// sum over the 256 threads of a workgroup, in a fixed order (wave shuffles, then the 4 wave sums through LDS)
__device__ __forceinline__ float block_sum(float v, float* red)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    const float s = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return s;
}

__global__ __launch_bounds__(256) void regression_loss_grad_kernel(const float* __restrict__ f, const float* __restrict__ y,
                                                                   float* __restrict__ dz, size_t nvec, size_t count, float* __restrict__ partial)
{
    __shared__ float red[4];
    float acc = 0.f;
    // 16-byte vectors where the three pointers allow it (nvec = 0 otherwise), then the scalar tail
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) {
        const f32x4 fv = reinterpret_cast<const f32x4*>(f)[i], yv = reinterpret_cast<const f32x4*>(y)[i];
        f32x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float d = fv[j] - yv[j];
            acc += d * d;
            o[j] = fv[j] > 0.f ? 2.f * d : 0.f;
        }
        reinterpret_cast<f32x4*>(dz)[i] = o;
    }
    for (size_t i = nvec * 4 + (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) {
        const float fi = f[i], d = fi - y[i];
        acc += d * d;
        dz[i] = fi > 0.f ? 2.f * d : 0.f;
    }
    const float s = block_sum(acc, red);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// out[0] = sum of partial[0..n): thread t adds the entries t, t + 256, ... in double, the 256 sums are then added
// in a fixed tree, so the value does not depend on scheduling
__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ partial, int n, float* __restrict__ out)
{
    __shared__ double red[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += (double)partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int d = 128; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = (float)red[0];
}

struct WArgs {
    const float* x;
    const float* dz;
    float* out;            // the partial sums [splits][K][CRS + 1] (splits > 1), else unused
    float* dw;             // splits == 1: the results themselves
    float* db;             // (may be NULL)
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int CRS, grid_m, grid_n, splits, imgs_per_split;    // the GEMM has CRS + 1 columns: column CRS is db
    int x_bytes, dz_bytes;
};

constexpr int BM = 64, BN = 64, BL = 32, LDT = BL + 4;

__global__ __launch_bounds__(256) void conv_wgrad_f32_kernel(const WArgs a)
{
    __shared__ __attribute__((aligned(16))) float As[BM * LDT];
    __shared__ __attribute__((aligned(16))) float Bs[BN * LDT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, half = lane >> 5, l32 = lane & 31;
    int bid = blockIdx.x;
    const int mt = bid % a.grid_m; bid /= a.grid_m;
    const int nt = bid % a.grid_n, sp = bid / a.grid_n;
    const int m0 = mt * BM, n0 = nt * BN;
    const int img_lo = sp * a.imgs_per_split, img_hi = min(a.N, img_lo + a.imgs_per_split);
    const int PQ = a.P * a.Q, HW = a.H * a.W;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc((void*)a.dz, 0, a.dz_bytes, 0x00020000);

    // loader: this thread fetches l = tid % 32 of the slice for rows tid / 32 + 8 i of both tiles
    const int ll = tid & 31, row0 = tid >> 5;
    int a_off[8];                 // dz: element offset of (image 0, filter m0 + row, pq 0) or OOB
    int b_off[8], b_r[8], b_s[8]; // x: element offset of (image 0, c, r - ph, s - pw) and the tap, or OOB
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int m = m0 + row0 + 8 * i;
        a_off[i] = m < a.K ? m * PQ : OOB;
        const int n = n0 + row0 + 8 * i;
        if (n < a.CRS) {
            const int c = n / (a.R * a.S), rs = n - c * a.R * a.S, r = rs / a.S, s = rs - r * a.S;
            b_off[i] = c * HW + (r - a.ph) * a.W + (s - a.pw);
            b_r[i] = r - a.ph; b_s[i] = s - a.pw;
        } else {
            b_off[i] = OOB; b_r[i] = n == a.CRS ? 1 : 0; b_s[i] = 0;      // b_r = 1: the column of ones (bias gradient)
        }
    }
    const int slices_per_img = (PQ + BL - 1) / BL;
    const int total = (img_hi - img_lo) * slices_per_img;

    float ra[8], rb[8];
    auto fetch = [&](int sl) __attribute__((always_inline)) {
        const int img = img_lo + sl / slices_per_img, pq = (sl % slices_per_img) * BL + ll;
        const bool l_on = pq < PQ;
        const int p = pq / a.Q, q = pq - p * a.Q;
        const int ih0 = p * a.sh, iw0 = q * a.sw;
        const int xo = ih0 * a.W + iw0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ao = (l_on && a_off[i] != OOB) ? (a_off[i] + pq) * 4 : OOB;
            ra[i] = buf_load(rz, ao, img * a.K * PQ * 4);
            const bool in = l_on && b_off[i] != OOB && (unsigned)(ih0 + b_r[i]) < (unsigned)a.H && (unsigned)(iw0 + b_s[i]) < (unsigned)a.W;
            rb[i] = buf_load(rx, in ? (b_off[i] + xo) * 4 : OOB, img * a.C * HW * 4);
            if (b_off[i] == OOB && b_r[i] == 1 && l_on) rb[i] = 1.f;
        }
    };

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    if (total > 0) fetch(0);
    for (int sl = 0; sl < total; ++sl) {
        __syncthreads();                                   // the previous slice has been read by every wave
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            As[(row0 + 8 * i) * LDT + ll] = ra[i];
            Bs[(row0 + 8 * i) * LDT + ll] = rb[i];
        }
        __syncthreads();
        if (sl + 1 < total) fetch(sl + 1);                 // in flight during the multiplications
        const float* ap = As + (wm * 32 + l32) * LDT + half * 16;
        const float* bp = Bs + (wn * 32 + l32) * LDT + half * 16;
        f32x4 av[4], bv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            av[j] = *reinterpret_cast<const f32x4*>(ap + 4 * j);
            bv[j] = *reinterpret_cast<const f32x4*>(bp + 4 * j);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[j >> 2][j & 3], bv[j >> 2][j & 3], acc, 0, 0, 0);
    }
    // register v holds row 8 (v / 4) + 4 half + v % 4 of column lane % 32
    const int CRS1 = a.CRS + 1;
    float* out = a.out + (size_t)sp * a.K * CRS1;
    const int n = n0 + wn * 32 + l32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (m >= a.K || n > a.CRS) continue;
        if (a.splits > 1) out[(size_t)m * CRS1 + n] = acc[v];
        else if (n < a.CRS) a.dw[(size_t)m * a.CRS + n] = acc[v];
        else if (a.db) a.db[m] = acc[v];
    }
}

// element i of the [K][CRS + 1] result = sum over the splits, in split order; column CRS goes to db
__global__ __launch_bounds__(256) void sum_splits_kernel(const float* __restrict__ part, int splits, int K, int CRS, float* __restrict__ dw,
                                                         float* __restrict__ db)
{
    const size_t count = (size_t)K * (CRS + 1);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) {
        float s = 0.f;
        for (int sp = 0; sp < splits; ++sp) s += part[(size_t)sp * count + i];
        const size_t m = i / (CRS + 1);
        const int n = (int)(i - m * (CRS + 1));
        if (n < CRS) dw[m * CRS + n] = s;
        else if (db) db[m] = s;
    }
}

__global__ __launch_bounds__(256) void sgd_step_kernel(float* __restrict__ w, const float* __restrict__ dw, float lr, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) w[i] = w[i] - lr * dw[i];
}

int wgrad_splits(int N, int K, int CRS, int* imgs_per_split)
{
    if (N < 1) { *imgs_per_split = 1; return 1; }
    const int tiles = ((K + BM - 1) / BM) * ((CRS + 1 + BN - 1) / BN);
    int want = (1024 + tiles - 1) / tiles;                  // about four workgroups per compute unit
    if (want > N) want = N;
    if (want < 1) want = 1;
    *imgs_per_split = (N + want - 1) / want;
    return (N + *imgs_per_split - 1) / *imgs_per_split;
}

}  // namespace

size_t regression_loss_workspace_bytes() { return 4096 * sizeof(float); }

int launch_regression_loss_grad(const float* f, const float* y, float* dz, size_t count, float* loss, void* ws, hipStream_t st)
{
    TraceScope trace("loss_grad", nullptr, (long long)count, st, 3ll * count * 4);
    const bool vec = (((uintptr_t)f | (uintptr_t)y | (uintptr_t)dz) & 15) == 0;
    const size_t nvec = vec ? count / 4 : 0;
    const unsigned grid = blocks_for_train(nvec ? nvec : count);
    hipLaunchKernelGGL(regression_loss_grad_kernel, dim3(grid), dim3(256), 0, st, f, y, dz, nvec, count, (float*)ws);
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, (const float*)ws, (int)grid, loss);
    return check_launch("regression_loss_grad");
}

size_t conv_wgrad_workspace_bytes(const ConvGeom& g)
{
    int ips = 0;
    const int splits = wgrad_splits(g.N, g.K, g.Kg, &ips);
    return splits > 1 ? (size_t)splits * g.K * (g.Kg + 1) * sizeof(float) : 0;
}

int launch_conv_wgrad_f32(const ConvGeom& g, const float* x, const float* dz, float* dw, float* db, void* ws, hipStream_t st)
{
    WArgs a;
    a.x = x; a.dz = dz;
    a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.K = g.K; a.R = g.R; a.S = g.S;
    a.sh = g.sh; a.sw = g.sw; a.ph = g.ph; a.pw = g.pw; a.P = g.P; a.Q = g.Q;
    a.CRS = g.Kg;
    a.grid_m = (g.K + BM - 1) / BM;
    a.grid_n = (g.Kg + 1 + BN - 1) / BN;
    a.splits = wgrad_splits(g.N, g.K, g.Kg, &a.imgs_per_split);
    a.x_bytes = (int)((size_t)g.N * g.C * g.H * g.W * 4);
    a.dz_bytes = (int)((size_t)g.N * g.K * g.P * g.Q * 4);
    a.out = (float*)ws; a.dw = dw; a.db = db;
    {
        ConvGeom t = g;
        TraceScope trace("conv_wgrad_f32", &t, g.Ng, st);
        hipLaunchKernelGGL(conv_wgrad_f32_kernel, dim3((unsigned)(a.grid_m * a.grid_n * a.splits)), dim3(256), 0, st, a);
    }
    if (const int rc = check_launch("conv_wgrad")) return rc;
    if (a.splits > 1) {
        const size_t count = (size_t)g.K * (g.Kg + 1);
        TraceScope trace("wgrad_sum", nullptr, (long long)count, st, (long long)((a.splits + 1) * count * 4));
        hipLaunchKernelGGL(sum_splits_kernel, dim3(blocks_for_train(count)), dim3(256), 0, st, (const float*)ws, a.splits, g.K, g.Kg, dw, db);
    }
    return check_launch("conv_wgrad");
}

int launch_sgd_step(float* w, const float* dw, float lr, size_t count, hipStream_t st)
{
    if (count == 0) return DR_OK;
    TraceScope trace("sgd_step", nullptr, (long long)count, st, 3ll * count * 4);
    hipLaunchKernelGGL(sgd_step_kernel, dim3(blocks_for_train(count)), dim3(256), 0, st, w, dw, lr, count);
    return check_launch("sgd_step");
}

}  // namespace dr
