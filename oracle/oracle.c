/*
 * CPU oracle for the CNN-block forward pass (original and slim forms).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain nested loops, every tensor and every
 * intermediate in fp64, NCHW layout, no blocking / fusion / reordering beyond
 * what each layer's definition states.  Shares no code with the HIP library and
 * must never be called from the product path.  OpenMP only distributes whole
 * output planes over threads; each output value is still one plain loop nest.
 *
 * Each function cites the passage of the paper that defines the operation.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* Output size of a convolution along one axis (floor rule). */
int orc_conv_out_size(int in, int filt, int stride, int pad)
{
    if (in + 2 * pad < filt) return 0;
    return (in + 2 * pad - filt) / stride + 1;
}

/* Output size of a pooling layer along one axis: ceil rule, and the last window must start
 * inside the input or its left padding (never entirely in the right padding).
 * Sec. 3.1 only names "p nearby regions"; the ceil rule is the one under which a 3x3 stride-2
 * pool maps 56 -> 28 and 112 -> 56 as the GoogLeNet blocks of Fig. 3 / Table 4 need. */
int orc_pool_out_size(int in, int win, int stride, int pad)
{
    int span = in + 2 * pad - win;
    if (span < 0) return 0;
    int out = (span + stride - 1) / stride + 1;
    if (pad > 0 && (out - 1) * stride >= in + pad) out -= 1;
    return out;
}

/* Convolution layer, Sec. 3.1 proof of Lemma 2, Eq. (7): Y_j = (W * X)_j + B_j, j = output channel.
 * '*' is cross-correlation (no filter flip) with zero padding:
 *   y[n,k,p,q] = b[k] + sum_{c,r,s} w[k,c,r,s] * x[n,c,p*sh+r-ph,q*sw+s-pw].
 * b may be NULL (zero bias).  relu != 0 applies max(.,0) to the result. */
void orc_conv2d(const double *x, int N, int C, int H, int W,
                const double *w, const double *b, int K, int R, int S,
                int sh, int sw, int ph, int pw, int relu, double *y)
{
    const int P = orc_conv_out_size(H, R, sh, ph), Q = orc_conv_out_size(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = b ? b[k] : 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r) {
                            const int ih = p * sh + r - ph;
                            if (ih < 0 || ih >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int iw = q * sw + s - pw;
                                if (iw < 0 || iw >= W) continue;
                                acc += w[(((size_t)k * C + c) * R + r) * S + s] *
                                       x[(((size_t)n * C + c) * H + ih) * W + iw];
                            }
                        }
                    if (relu && acc < 0.0) acc = 0.0;
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
}

/* ReLU (a non-tensor layer of Fig. 2; kept by streamline slimming, Sec. 3.1 Example). */
void orc_relu(const double *x, size_t count, double *y)
{
    for (size_t i = 0; i < count; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

/* Across-channel LRN, Sec. 3.1 Eq. (3) (parameters kappa, rho, alpha [, beta]):
 *   y[n,c,h,w] = x[n,c,h,w] / (k + alpha/n_local * sum_{c'} x[n,c',h,w]^2)^beta,
 * c' over the window of n_local channels centred on c, clipped to [0,C); the divisor stays n_local. */
void orc_lrn(const double *x, int N, int C, int H, int W,
             int n_local, double alpha, double beta, double k, double *y)
{
    const int half = n_local / 2;
    const size_t HW = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t i = 0; i < HW; ++i) {
                double ss = 0.0;
                for (int cc = c - half; cc <= c - half + n_local - 1; ++cc) {
                    if (cc < 0 || cc >= C) continue;
                    const double v = x[((size_t)n * C + cc) * HW + i];
                    ss += v * v;
                }
                const double scale = k + alpha / (double)n_local * ss;
                y[((size_t)n * C + c) * HW + i] = x[((size_t)n * C + c) * HW + i] / pow(scale, beta);
            }
}

/* Max-pooling f_pooling(p), Sec. 3.1 Eq. (3): maximum over the part of the kh x kw window that
 * lies inside the input (padding never wins: it acts as -infinity). */
void orc_maxpool(const double *x, int N, int C, int H, int W,
                 int kh, int kw, int sh, int sw, int ph, int pw, double *y)
{
    const int P = orc_pool_out_size(H, kh, sh, ph), Q = orc_pool_out_size(W, kw, sw, pw);
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < (long)N * C; ++nc)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                double m = -INFINITY;
                for (int r = 0; r < kh; ++r) {
                    const int ih = p * sh + r - ph;
                    if (ih < 0 || ih >= H) continue;
                    for (int s = 0; s < kw; ++s) {
                        const int iw = q * sw + s - pw;
                        if (iw < 0 || iw >= W) continue;
                        const double v = x[((size_t)nc * H + ih) * W + iw];
                        if (v > m) m = v;
                    }
                }
                y[((size_t)nc * P + p) * Q + q] = m;
            }
}

/* Average pooling (the 7x7 pool of GoogLeNet's "loss3" row, Table 4): mean over a k x k window,
 * stride `stride`, no padding, floor output size. */
void orc_avgpool(const double *x, int N, int C, int H, int W, int k, int stride, double *y)
{
    const int P = orc_conv_out_size(H, k, stride, 0), Q = orc_conv_out_size(W, k, stride, 0);
    for (long nc = 0; nc < (long)N * C; ++nc)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                double s = 0.0;
                for (int r = 0; r < k; ++r)
                    for (int t = 0; t < k; ++t)
                        s += x[((size_t)nc * H + p * stride + r) * W + q * stride + t];
                y[((size_t)nc * P + p) * Q + q] = s / (double)(k * k);
            }
}

/* Channel concatenation, Sec. 3.2 Eq. (11): Y_LR = [Y_left; Y_right].  Copies x (N x Cx x HW) into
 * channels [c_off, c_off+Cx) of y (N x Cy x HW). */
void orc_concat_into(const double *x, int N, int Cx, size_t HW, double *y, int Cy, int c_off)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Cx; ++c)
            for (size_t i = 0; i < HW; ++i)
                y[((size_t)n * Cy + c_off + c) * HW + i] = x[((size_t)n * Cx + c) * HW + i];
}

/* BatchNorm followed by Scale at inference, Sec. 3.1 Eq. (8) read with m = 1 (mu, sigma^2 are the
 * running statistics themselves) and eps added under the root:
 *   y_j = gamma_j * (x_j - mu_j) / sqrt(var_j + eps) + beta_j. */
void orc_bn(const double *x, int N, int C, size_t HW, const double *gamma, const double *beta,
            const double *mean, const double *var, double eps, double *y)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                y[o] = gamma[c] * ((x[o] - mean[c]) / sqrt(var[c] + eps)) + beta[c];
            }
}

/* Closed-form merge of conv + BatchNorm + Scale into one conv, Lemma 2 Eq. (6) with m = 1:
 *   eta_j = gamma_j / sqrt(var_j + eps);  W~_j = eta_j W_j;  B~_j = eta_j B_j + beta_j - eta_j mu_j.
 * crs = C*R*S weights per output channel. */
void orc_fold_bn(int K, size_t crs, const double *w, const double *b, const double *gamma,
                 const double *beta, const double *mean, const double *var, double eps,
                 double *w_out, double *b_out)
{
    for (int j = 0; j < K; ++j) {
        const double eta = gamma[j] / sqrt(var[j] + eps);
        for (size_t i = 0; i < crs; ++i) w_out[j * crs + i] = eta * w[j * crs + i];
        b_out[j] = eta * (b ? b[j] : 0.0) + beta[j] - eta * mean[j];
    }
}

/* Residual merge of a ResNet bottleneck (Sec. 4.2): y = max(a + b, 0). */
void orc_add_relu(const double *a, const double *b, size_t count, double *y)
{
    for (size_t i = 0; i < count; ++i) {
        const double s = a[i] + b[i];
        y[i] = s > 0.0 ? s : 0.0;
    }
}

/* Inner-product (fully connected) tensor layer, Sec. 1: y[n,o] = b[o] + sum_i w[o,i] x[n,i]. */
void orc_fc(const double *x, int N, int I, const double *w, const double *b, int O, double *y)
{
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o) {
            double acc = b ? b[o] : 0.0;
            for (int i = 0; i < I; ++i) acc += w[(size_t)o * I + i] * x[(size_t)n * I + i];
            y[(size_t)n * O + o] = acc;
        }
}

/* Softmax over the class axis (a non-tensor layer of Fig. 2): exp(x - max) / sum exp(x - max). */
void orc_softmax(const double *x, int N, int O, double *y)
{
    for (int n = 0; n < N; ++n) {
        double m = -INFINITY, s = 0.0;
        for (int o = 0; o < O; ++o) if (x[(size_t)n * O + o] > m) m = x[(size_t)n * O + o];
        for (int o = 0; o < O; ++o) s += exp(x[(size_t)n * O + o] - m);
        for (int o = 0; o < O; ++o) y[(size_t)n * O + o] = exp(x[(size_t)n * O + o] - m) / s;
    }
}

/* Round every value to the nearest bf16-representable number, ties to even (bf16 = the upper 16
 * bits of an IEEE binary32).  Used only for the "mirrored" bf16 mode, where each layer's output is
 * stored in bf16 before the next layer reads it.  NaN/Inf pass through. */
void orc_round_bf16(double *x, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        if (!isfinite(x[i]) || x[i] == 0.0) continue;
        int e;
        const double m = frexp(fabs(x[i]), &e);      /* |x| = m * 2^e, m in [0.5,1) */
        int q = e - 8;                               /* bf16 keeps 8 significant bits */
        if (e - 1 < -126) q = -126 - 7;              /* subnormal range of binary32/bf16 */
        const double scaled = ldexp(fabs(x[i]), -q); /* integer part = significand */
        double r = nearbyint(scaled);                /* default rounding mode: ties to even */
        (void)m;
        double v = ldexp(r, q);
        if (v > 3.3895313892515355e38) v = INFINITY;
        x[i] = x[i] < 0 ? -v : v;
    }
}

/* ---- layer-wise regression of a slim layer (Sec. 3.1, the optimisation goal below Eq. (4) and Lemma 1) ----
 * The slim layer f~(W, b; X) = max(conv(X; W, b), 0) is fitted to the feature map Y of the block it replaces
 * by minimising  L(W, b) = sum_i || Y^i - f~(W, b; X^i) ||_F^2  with gradient descent. */

/* L and dL/dz for the pre-activation z of the slim layer, given its output f = max(z, 0) and the target y:
 *   L = sum (f - y)^2,   dz = 2 (f - y) where f > 0 (there z = f and df/dz = 1), else 0. */
double orc_regression_loss_grad(const double *f, const double *y, size_t count, double *dz)
{
    double loss = 0.0;
    for (size_t i = 0; i < count; ++i) {
        const double d = f[i] - y[i];
        loss += d * d;
        dz[i] = f[i] > 0.0 ? 2.0 * d : 0.0;
    }
    return loss;
}

/* Chain rule through z[n,k,p,q] = b[k] + sum_{c,r,s} w[k,c,r,s] x[n,c,p*sh+r-ph,q*sw+s-pw] (Eq. (7)):
 *   dw[k,c,r,s] = sum_{n,p,q} dz[n,k,p,q] x[n,c,p*sh+r-ph,q*sw+s-pw]   (terms in the zero padding drop out),
 *   db[k]       = sum_{n,p,q} dz[n,k,p,q]. */
void orc_conv2d_bwd_params(const double *x, int N, int C, int H, int W, const double *dz, int K, int R, int S,
                           int sh, int sw, int ph, int pw, double *dw, double *db)
{
    const int P = orc_conv_out_size(H, R, sh, ph), Q = orc_conv_out_size(W, S, sw, pw);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k) {
        double sb = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) sb += dz[(((size_t)n * K + k) * P + p) * Q + q];
        db[k] = sb;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p) {
                            const int ih = p * sh + r - ph;
                            if (ih < 0 || ih >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int iw = q * sw + s - pw;
                                if (iw < 0 || iw >= W) continue;
                                acc += dz[(((size_t)n * K + k) * P + p) * Q + q] * x[(((size_t)n * C + c) * H + ih) * W + iw];
                            }
                        }
                    dw[(((size_t)k * C + c) * R + r) * S + s] = acc;
                }
    }
}
