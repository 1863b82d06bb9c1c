/*
 * deeprebirth.h - C ABI of the MI355X (gfx950) forward-pass library for CNN blocks in the two
 * forms of the DeepRebirth paper: the original form (convolution followed by the non-tensor
 * layers ReLU / LRN / max-pool / concat / BatchNorm) and the slim form (one strided conv + ReLU per
 * streamline block, two tensor branches per inception module, BatchNorm folded into the conv).
 *
 * Conventions common to every entry point
 *   - Tensors: activations are dense, in NCHW or NHWC order (dr_tensor.layout); filters are dense
 *     KCRS (output channel, input channel, filter row, filter column) or KRSC (dr_conv.filter_layout);
 *     biases and per-channel vectors are dense K.  DR_F32 tensors hold
 *     IEEE binary32; DR_BF16 tensors hold bfloat16 (upper half of a binary32) and are computed with
 *     fp32 accumulation and round-to-nearest-even on store.  Biases and BatchNorm vectors are
 *     always fp32.
 *   - Pointers named x, y, w, bias, ws, params[i] are DEVICE pointers owned by the caller; the
 *     library never allocates, frees or retains them (a recorded graph, see dr_capture_begin, is the one
 *     exception: it keeps the addresses it was recorded with).  Descriptor structs are HOST memory, read
 *     during the call only.  x and y must not overlap unless an entry point says otherwise.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every entry point
 *     validates its arguments on the host first, then enqueues its kernels on `stream` and
 *     returns without synchronising.
 *   - Return value: DR_OK or a dr_status error; on error nothing has been enqueued (except
 *     DR_ERR_HIP, which reports a failed launch) and dr_last_error() holds a message for the
 *     calling thread.  No C++ exception crosses this boundary.
 */
#ifndef DEEPREBIRTH_H
#define DEEPREBIRTH_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DR_OK = 0,
    DR_ERR_NULL = 1,        /* a required pointer is NULL */
    DR_ERR_SHAPE = 2,       /* inconsistent dimensions, or the output descriptor is not the layer's output shape */
    DR_ERR_UNSUPPORTED = 3, /* dtype / parameter combination the library has no kernel for */
    DR_ERR_WORKSPACE = 4,   /* workspace missing or too small */
    DR_ERR_HIP = 5          /* the HIP runtime reported an error */
} dr_status;

typedef enum { DR_F32 = 0, DR_BF16 = 1 } dr_dtype;

/* Activation orders: DR_NCHW (channel planes) or DR_NHWC (channels last: the c values of one pixel
 * are contiguous).  fp32 convolutions take NCHW; bf16 convolutions take NHWC, the order in which the
 * contraction index of the matrix cores is contiguous (bf16 NCHW runs in a slow fallback kernel).
 * The other layers take either order for both data types.  Inputs and outputs of one call share
 * the order. */
typedef enum { DR_NCHW = 0, DR_NHWC = 1 } dr_layout;

/* Feature map X^i / Y (Sec. 3.1): batch n of c channels of h x w, in the memory order `layout`. */
typedef struct { int n, c, h, w; int dtype; int layout; } dr_tensor;

/* Filter tensor orders.  DR_KCRS is the order the filters are defined in (output channel, input
 * channel, row, column).  DR_KRSC (input channel innermost) is the order the fast kernels read:
 * dr_pack_filters produces it once, offline, like any other model preparation step. */
typedef enum { DR_KCRS = 0, DR_KRSC = 1 } dr_filter_layout;

/* Convolution layer f_conv(W, b) (Sec. 3.1 Eq. (3), Eq. (7)): k filters over c channels, r x s taps.
 * relu != 0 fuses max(.,0) into the store.  filter_layout says how the w passed with this
 * descriptor is ordered; DR_KRSC requires c to be a multiple of 16 (fp32) or 8 (bf16). */
typedef struct { int k, c, r, s, stride_h, stride_w, pad_h, pad_w, relu, filter_layout; } dr_conv;

/* LRN layer f_LRN (Sec. 3.1 Eq. (3)): across-channel window of local_size channels. */
typedef struct { int local_size; float alpha, beta, k; } dr_lrn;

/* Pooling layer f_pooling(p) (Sec. 3.1 Eq. (3)): kh x kw window. */
typedef struct { int kh, kw, stride_h, stride_w, pad_h, pad_w; } dr_pool;

/* ---- shape rules (host only, no GPU needed) ------------------------------------------------- */

/* Convolution output size along one axis: floor((in + 2 pad - filt) / stride) + 1 (0 if the
 * filter does not fit). */
int dr_conv_out_size(int in, int filt, int stride, int pad);

/* Pooling output size along one axis: ceil((in + 2 pad - win) / stride) + 1, minus one if the
 * last window would start beyond the input and its left padding. */
int dr_pool_out_size(int in, int win, int stride, int pad);

/* ---- single layers ------------------------------------------------------------------------------ */

/* Convolution, Eq. (7): y[n, y_c_offset + j, p, q] = bias[j] + sum_{c,r,s} w[j,c,r,s] *
 * x[n, c, p*stride_h + r - pad_h, q*stride_w + s - pad_w], zero outside the input; then ReLU if
 * cd->relu.  Writes channels [y_c_offset, y_c_offset + cd->k) of y, which has yd->c >= that many
 * channels (other channels untouched): this is how a branch writes its part of a concatenated
 * tensor.  bias may be NULL (zero).  xd->c == cd->c, yd->n == xd->n, yd->h/w == dr_conv_out_size.
 * x, w, y share one dtype; w is ordered as cd->filter_layout says.  x and w must each be smaller
 * than 2 GiB.  Uses no workspace. */
int dr_conv2d_fwd(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                  const dr_tensor* yd, void* y, int y_c_offset, void* stream);

/* The same convolution with scratch memory from the caller.  A layer with fewer output tiles than the
 * device has compute units (one image, or a few: the setting of the paper's own measurements, Sec. 4)
 * would leave most of them idle; with scratch the contraction over (c, r, s) is cut into ranges that
 * run side by side, and a second kernel adds the ranges in a fixed order and applies bias and ReLU
 * (no atomics: results are the same from run to run).  dr_conv2d_workspace_bytes gives the size for
 * (xd, cd): 0 when the layer would not be cut (then ws may be NULL); cd with the stride of a slim
 * layer gives the slim layer's size.  ws: device memory, 256-byte aligned, of at least that size
 * (else DR_ERR_WORKSPACE), used only until the call's work on `stream` has finished.  fp32 NCHW layers
 * are cut; every other layer runs exactly as in dr_conv2d_fwd. */
int dr_conv2d_workspace_bytes(const dr_tensor* xd, const dr_conv* cd, size_t* bytes);
int dr_conv2d_fwd_ws(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                     const dr_tensor* yd, void* y, int y_c_offset, void* ws, size_t ws_bytes, void* stream);

/* dr_conv2d_fwd_ws for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it): the scratch is an array inside the library, DR_STATIC_SCRATCH_BYTES per GPU
 * the library runs on, held until the process ends.  The call allocates and frees nothing and gives the same
 * bits as dr_conv2d_fwd_ws.  A layer whose partial sums need more (dr_conv2d_workspace_bytes says how much) is
 * refused with DR_ERR_WORKSPACE before anything is enqueued; a layer that would not be cut needs none and runs
 * as in dr_conv2d_fwd.  All calls on one GPU share that GPU's array (it keeps the last call's contents; the
 * kernels write every value they later read, so nothing is cleared): calls that overlap in time on one GPU,
 * on different streams or from different threads, race on it -- order them on one stream. */
#define DR_STATIC_SCRATCH_BYTES (8u << 20)
int dr_conv2d_fwd_static(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                         const dr_tensor* yd, void* y, int y_c_offset, void* stream);

/* Reorders a filter tensor from KCRS to KRSC on the device: w_krsc[j][r][s][c] = w_kcrs[j][c][r][s]
 * (cd->k, c, r, s give the shape; dtype DR_F32 or DR_BF16; the two buffers must not overlap).
 * Returns DR_ERR_UNSUPPORTED when cd->c is not a multiple of 16 (fp32) or 8 (bf16): such filters
 * stay in KCRS. */
int dr_pack_filters(const dr_conv* cd, int dtype, const void* w_kcrs, void* w_krsc, void* stream);

/* Slim layer of streamline slimming (Sec. 3.1 "Pooling Layer" / "Non-Pooling Layer"): the
 * convolution cd with its stride multiplied by the absorbed pooling layer's stride, LRN/BatchNorm
 * dropped and ReLU kept (forced on whatever cd->relu says).  yd must carry the output size of the
 * convolution at the product stride.  Otherwise as dr_conv2d_fwd. */
int dr_slim_conv_fwd(const dr_tensor* xd, const void* x, const dr_conv* cd, int pool_stride_h, int pool_stride_w,
                     const void* w, const float* bias, const dr_tensor* yd, void* y, int y_c_offset, void* stream);

/* ReLU (non-tensor layer, Fig. 2; retained by slimming, Sec. 3.1 Example): y = max(x, 0).
 * x == y (in place) is allowed. */
int dr_relu(const dr_tensor* d, const void* x, void* y, void* stream);

/* Across-channel LRN: y[n,c,h,w] = x[n,c,h,w] / (k + alpha/local_size * sum x[n,c',h,w]^2)^beta, c'
 * over the local_size channels centred on c (from c - local_size/2), clipped to the tensor. */
int dr_lrn_fwd(const dr_tensor* d, const void* x, const dr_lrn* p, void* y, void* stream);

/* Max-pooling: maximum over the window's intersection with the input (padding never wins).
 * yd->h/w must equal dr_pool_out_size; yd->n/c == xd->n/c. */
int dr_maxpool_fwd(const dr_tensor* xd, const void* x, const dr_pool* p, const dr_tensor* yd, void* y, void* stream);

/* The non-tensor tail of a streamlined block (Sec. 3.1: conv - ReLU - LRN - pool, or pool - LRN as in the first
 * block of GoogLeNet) in one pass over the tensor, without changing the function: y = maxpool(lrn(x)) resp.
 * y = lrn(maxpool(x)), the intermediate tensor never stored (and never rounded to the storage type).  Same
 * descriptors and shape rules as dr_lrn_fwd and dr_maxpool_fwd.  DR_ERR_UNSUPPORTED unless: channels-last
 * tensors whose channel count is a multiple of 8 (bf16) / 4 (fp32) and at most 512 / 256, 16-byte aligned
 * pointers, a 3x3 pooling window of stride 1 or 2 with padding 0 or 1, local_size 5. */
int dr_lrn_maxpool_fwd(const dr_tensor* xd, const void* x, const dr_lrn* l, const dr_pool* p, const dr_tensor* yd, void* y, void* stream);

/* The original form of a streamlined block (Sec. 3.1, Fig. 3: convolution, ReLU, LRN, max-pooling) in ONE kernel:
 *   y = maxpool(lrn(relu(conv(x; w) + bias)))
 * with the function of the four layers unchanged -- the fusion the paper's Discussion sets against slimming: it
 * saves the passes over memory, not the convolution's arithmetic at the unpooled resolution.  A workgroup holds
 * all filters of a patch of convolution outputs, lays the patch down in LDS in the precision the layer-by-layer
 * form stores it in (bf16), normalises across channels there and stores only the pooled pixels.
 * bf16, DR_NHWC tensors, KRSC filters, cd->k <= 192 and a multiple of 8, cd->c a multiple of 8, LRN window of 5,
 * pooling 3x3 at stride 2 without padding (ceil-mode sizes); anything else: DR_ERR_UNSUPPORTED.  cd->relu is
 * ignored (the ReLU is part of the block).  yd = {n, >= y_c_offset + cd->k, pooled h, pooled w}; channels
 * [y_c_offset, y_c_offset + cd->k) are written.  No workspace. */
int dr_conv_lrn_maxpool_fwd(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                            const dr_lrn* l, const dr_pool* p, const dr_tensor* yd, void* y, int y_c_offset, void* stream);
int dr_maxpool_lrn_fwd(const dr_tensor* xd, const void* x, const dr_pool* p, const dr_lrn* l, const dr_tensor* yd, void* y, void* stream);

/* Concatenation along channels, Eq. (11): y = [x_0; x_1; ...; x_{nb-1}].  xds/xs are host arrays
 * of nb descriptors / device pointers; all inputs share n, h, w and dtype; yd->c = sum of x_i c.
 * nb <= DR_MAX_BRANCHES. */
#define DR_MAX_BRANCHES 8
int dr_concat(int nb, const dr_tensor* xds, const void* const* xs, const dr_tensor* yd, void* y, void* stream);

/* BatchNorm + Scale at inference, Eq. (8) with m = 1 and eps under the root:
 * y = gamma_c (x - mean_c) / sqrt(var_c + eps) + beta_c, then ReLU if relu != 0.  In place allowed.
 * gamma, beta, mean, var: fp32 device vectors of d->c entries. */
int dr_bn_fwd(const dr_tensor* d, const void* x, const float* gamma, const float* beta, const float* mean,
              const float* var, float eps, int relu, void* y, void* stream);

/* Residual merge of a ResNet bottleneck (Sec. 4.2): y = max(a + b, 0).  y may alias a or b. */
int dr_add_relu(const dr_tensor* d, const void* a, const void* b, void* y, void* stream);

/* Lemma 2, Eq. (6) with m = 1: folds BatchNorm + Scale into the preceding convolution.
 * HOST arrays, fp32: eta_j = gamma_j / sqrt(var_j + eps), w_out[j,:] = eta_j w[j,:],
 * b_out[j] = eta_j b[j] + beta_j - eta_j mean_j.  crs = weights per output channel; b may be NULL.
 * w_out may alias w, b_out may alias b.  Runs on the CPU (it is an offline model transform). */
int dr_fold_bn(int k, size_t crs, const float* w, const float* b, const float* gamma, const float* beta,
               const float* mean, const float* var, float eps, float* w_out, float* b_out);

/* Average pooling over a kh x kw window (floor sizes, no padding); the 7x7 pool of GoogLeNet's
 * classifier (Table 4, row loss3).  p->pad_* must be 0. */
int dr_avgpool_fwd(const dr_tensor* xd, const void* x, const dr_pool* p, const dr_tensor* yd, void* y, void* stream);

/* Inner-product layer (a tensor layer, Sec. 1): y[n,o] = bias[o] + sum_i w[o,i] x[n,i], with
 * i running over (c, h, w) of xd in that order.  yd = {n, out, 1, 1}.  w: out x (c*h*w), dtype of x.
 * A DR_NHWC input whose map is larger than 1x1 is refused (DR_ERR_UNSUPPORTED): its memory order
 * is (h, w, c), not the order of i. */
int dr_fc_fwd(const dr_tensor* xd, const void* x, const void* w, const float* bias, const dr_tensor* yd, void* y,
              void* stream);

/* Softmax over the channel axis of an {n, c, 1, 1} tensor; the output y is always fp32. */
int dr_softmax_fwd(const dr_tensor* xd, const void* x, float* y, void* stream);

/* ---- learning a slim layer (Sec. 3.1: the optimisation goal below Eq. (4), Lemma 1) ------------------------------
 * The slim layer f~(W, b; X) = max(conv(X; W, b), 0) (dr_slim_conv_fwd) is fitted to the feature map Y of the block
 * it replaces by gradient descent on L(W, b) = sum || Y - f~(W, b; X) ||_F^2.  One step: the forward pass, then
 * dr_regression_loss_grad, dr_conv2d_bwd_params, and dr_sgd_step on the filters and on the biases.
 * fp32, NCHW tensors, KCRS filters; anything else is DR_ERR_UNSUPPORTED. */

/* L = sum (f - target)^2 and dL/dz for the layer's pre-activation z: dz = 2 (f - target) where f > 0, else 0.
 * f: the layer's output (after its ReLU), target, dz: tensors of descriptor d (dz may alias f).  loss: one
 * device float.  ws: device scratch of at least dr_regression_loss_workspace_bytes(). */
size_t dr_regression_loss_workspace_bytes(void);
int dr_regression_loss_grad(const dr_tensor* d, const void* f, const void* target, void* dz, float* loss, void* ws, size_t ws_bytes,
                            void* stream);

/* Gradient of the convolution's parameters from the gradient dz of its output (chain rule through Eq. (7)):
 *   dw[k,c,r,s] = sum_{n,p,q} dz[n,k,p,q] x[n,c,p*sh+r-ph,q*sw+s-pw],   db[k] = sum_{n,p,q} dz[n,k,p,q].
 * dzd must be the convolution's output descriptor for input xd; dw has the filters' shape (KCRS), db (may be
 * NULL) k floats.  ws: device scratch of at least dr_conv2d_bwd_params_workspace_bytes (partial sums over ranges
 * of images, added in a fixed order: the result does not depend on scheduling). */
int dr_conv2d_bwd_params_workspace_bytes(const dr_tensor* xd, const dr_conv* cd, size_t* bytes);
int dr_conv2d_bwd_params(const dr_tensor* xd, const void* x, const dr_conv* cd, const dr_tensor* dzd, const void* dz, void* dw,
                         float* db, void* ws, size_t ws_bytes, void* stream);

/* One step of gradient descent on count fp32 parameters: w[i] = w[i] - lr * dw[i]. */
int dr_sgd_step(size_t count, float* w, const float* dw, float lr, void* stream);

/* ---- inception module (Sec. 3.2, Fig. 4) ---------------------------------------------------- */

#define DR_MAX_STEPS 4
typedef enum { DR_STEP_CONV = 0, DR_STEP_MAXPOOL = 1 } dr_step_kind;
/* One step of a branch; conv.relu != 0 means a ReLU layer follows the convolution. */
typedef struct { int kind; dr_conv conv; dr_pool pool; } dr_step;
typedef struct { int n_steps; dr_step steps[DR_MAX_STEPS]; } dr_branch;

/* How the module is executed.  0 = the layer-by-layer form the paper times: every ReLU is its own
 * kernel and the branch outputs are gathered by a concat kernel.  Flags remove passes without
 * changing the function computed: */
#define DR_FUSE_RELU   1   /* ReLU in the convolution's store */
#define DR_FUSE_CONCAT 2   /* a branch ending in a convolution writes its channel range of y directly
                              (that convolution then also applies its ReLU in the store) */
#define DR_FUSE_STACK  4   /* Eq. (12): first-step 1x1 convolutions (stride 1, no padding, followed by ReLU)
                              that read the module input run as one convolution with stacked filters, each
                              writing its own destination (needs DR_FUSE_RELU).  Taken for bf16 NHWC and
                              fp32 NCHW tensors when the caller has laid the filters of those convolutions
                              back to back in device memory in branch order (weights[j] of the next one
                              starts where the previous one's k*c elements end; the same for the fp32
                              biases, or all biases NULL), all in one filter_layout, and (bf16) every bank
                              but the last has a multiple of 8 filters; otherwise the convolutions run one
                              by one, with the same result */
#define DR_CONCURRENT_BRANCHES 8 /* branches 1.. run on streams the library owns (per host thread and
                              device, created on first use, default priority), forked from the caller's
                              stream by an event before the module and joined to it by events before the
                              concat: to the caller the module is still one piece of work on `stream`,
                              also when the call returns an error after some branches have been started
                              (they are joined before it returns).  Devices 0..15 of a process.
                              Without it the branches run one after another on the caller's stream.
                              Pays when a module's kernels are long next to the cost of the events
                              (several microseconds per fork / join) and leave compute units idle */
typedef struct { int n_branches; dr_branch branches[DR_MAX_BRANCHES]; int mode; } dr_inception;

/* Bytes of workspace dr_inception_fwd needs for input xd. */
int dr_inception_workspace_bytes(const dr_tensor* xd, const dr_inception* desc, size_t* bytes);

/* Every branch is a chain of steps applied to the module input x; y = concat of the branch
 * outputs in branch order.  The original module has four branches (1x1 | 1x1,3x3 | 1x1,5x5 |
 * pool,1x1), the branch-slimmed one has two.  weights[i] / biases[i]: parameters of the i-th
 * convolution step counted branch by branch, step by step.  ws: device scratch of at least
 * dr_inception_workspace_bytes, 256-byte aligned. */
int dr_inception_fwd(const dr_tensor* xd, const void* x, const dr_inception* desc, const void* const* weights,
                     const float* const* biases, const dr_tensor* yd, void* y, void* ws, size_t ws_bytes,
                     void* stream);

/* ---- whole networks --------------------------------------------------------------------------- */

typedef enum {
    DR_LAYER_CONV = 0, DR_LAYER_RELU, DR_LAYER_LRN, DR_LAYER_MAXPOOL, DR_LAYER_INCEPTION,
    DR_LAYER_BOTTLENECK, DR_LAYER_AVGPOOL, DR_LAYER_FC, DR_LAYER_SOFTMAX,
    DR_LAYER_LRN_MAXPOOL,    /* dr_lrn_maxpool_fwd: uses .lrn and .pool */
    DR_LAYER_MAXPOOL_LRN,    /* dr_maxpool_lrn_fwd: uses .pool and .lrn */
    DR_LAYER_CONV_LRN_MAXPOOL /* dr_conv_lrn_maxpool_fwd: uses .conv, .lrn and .pool; parameters: filters, bias */
} dr_layer_kind;

/* ResNet bottleneck (Sec. 4.2): 1x1 (mid) - 3x3 (mid) - 1x1 (out), each followed by BatchNorm
 * (+ReLU after the first two), shortcut = identity or (project != 0) a 1x1 convolution + BatchNorm;
 * output = ReLU(sum).  folded != 0 is the slim form: no BatchNorm layers, the convolutions carry
 * folded weights (dr_fold_bn), ReLU and the residual sum run in the convolutions' stores. */
typedef struct { int mid, out, project, folded; float eps; int filter_layout; /* of all its convolutions */ } dr_bottleneck;

typedef struct {
    int kind;
    dr_conv conv;            /* DR_LAYER_CONV, DR_LAYER_CONV_LRN_MAXPOOL */
    dr_lrn lrn;              /* DR_LAYER_LRN, DR_LAYER_LRN_MAXPOOL, DR_LAYER_MAXPOOL_LRN */
    dr_pool pool;            /* DR_LAYER_MAXPOOL, DR_LAYER_AVGPOOL, DR_LAYER_LRN_MAXPOOL, DR_LAYER_MAXPOOL_LRN */
    dr_inception inception;  /* DR_LAYER_INCEPTION */
    dr_bottleneck bottleneck;/* DR_LAYER_BOTTLENECK */
    int fc_out;              /* DR_LAYER_FC */
} dr_layer_desc;

typedef struct dr_net dr_net;   /* host-side object: a validated copy of the layer list */

/* Builds a network from n_layers descriptors (copied).  Parameter order expected by dr_net_fwd:
 * forward order; conv: w, bias; inception: per branch, per conv step: w, bias; bottleneck:
 * conv a, [bn a], conv b, [bn b], conv c, [bn c], then projection conv, [bn] if present, where a
 * conv is (w, bias) and a bn is (gamma, beta, mean, var) and the bn entries are absent when
 * folded; fc: w, bias. */
int dr_net_create(const dr_layer_desc* layers, int n_layers, dr_net** out);
void dr_net_destroy(dr_net* net);

/* Number of parameter pointers dr_net_fwd expects. */
int dr_net_num_params(const dr_net* net, int* count);

/* Output descriptor and workspace need of the network for input xd. */
int dr_net_output_desc(const dr_net* net, const dr_tensor* xd, dr_tensor* yd);
int dr_net_workspace_bytes(const dr_net* net, const dr_tensor* xd, size_t* bytes);

/* Runs the layer list on x.  params: host array of dr_net_num_params device pointers.  The output
 * has the dtype of the input except after a softmax layer (fp32).  ws: at least
 * dr_net_workspace_bytes, 256-byte aligned.
 * Layers run one after the other with one exception, which changes no value: a bf16 NHWC
 * convolution on at most 4 input channels (a network's first layer) with at most 64 filters and
 * a 1x1 convolution with at most 64 filters right behind it run as ONE kernel when the first
 * layer's kernel takes the pair; the tensor between them (rounded to bf16 as it would be stored)
 * stays in registers and is never written.  Per-layer timing then books the kernel under the
 * first of the two layers; the second shows only the gap between two event records. */
int dr_net_fwd(dr_net* net, const dr_tensor* xd, const void* x, const void* const* params,
               const dr_tensor* yd, void* y, void* ws, size_t ws_bytes, void* stream);

/* Per-layer timing: when enabled, dr_net_fwd brackets every top-level layer with events on
 * `stream`; dr_net_layer_times synchronises with the last run and writes n_layers durations in
 * milliseconds (used to report the paper's "% Latency" of non-tensor layers, Eq. (1)). */
int dr_net_set_timing(dr_net* net, int enabled);
int dr_net_layer_times(dr_net* net, float* ms_per_layer, int n);

/* The forward pass as a HIP graph.  dr_net_capture records what dr_net_fwd would enqueue for these arguments
 * into a graph (nothing runs) and instantiates it; dr_graph_launch enqueues the whole forward on `stream` with one
 * call.  For callers that run the same forward many times: the launches of a layer-by-layer network are short, and
 * with DR_CONCURRENT_BRANCHES the graph also carries the branches' dependencies without the events between queues
 * that the same mode costs when every kernel is launched by itself.  The graph holds the pointers it was captured
 * with: x, the parameters, y and ws must stay allocated, their contents may change between launches (every launch
 * reads them anew); two launches of one graph must not overlap in time (they share ws).  `stream` of dr_net_capture
 * must be a stream the caller created (not the default stream); per-layer timing and a running kernel trace must
 * be off (DR_ERR_UNSUPPORTED).  Capture and instantiation allocate host and device memory; a launch allocates
 * nothing.  Errors of the layer list are reported as by dr_net_fwd. */
typedef struct dr_graph dr_graph;
/* The general form: between dr_capture_begin and dr_capture_end every dr_* call that is given `stream` is recorded
 * instead of run (several forwards, single layers, ...); dr_capture_end instantiates the recording (out = NULL:
 * discards it).  Nothing else may be enqueued on `stream` in between, and dr_net_set_timing must be off for the
 * networks recorded.  dr_net_capture is dr_capture_begin, dr_net_fwd, dr_capture_end. */
int dr_capture_begin(void* stream);
int dr_capture_end(void* stream, dr_graph** out);
int dr_net_capture(dr_net* net, const dr_tensor* xd, const void* x, const void* const* params,
                   const dr_tensor* yd, void* y, void* ws, size_t ws_bytes, void* stream, dr_graph** out);
int dr_graph_launch(dr_graph* graph, void* stream);
void dr_graph_destroy(dr_graph* graph);

/* ---- measurement ---------------------------------------------------------------------------------- */

/* One traced kernel launch.  label: kernel family ("conv_f32", "conv_bf16", "relu", "lrn", "maxpool",
 * "concat", "bn", "add_relu", "avgpool", "fc", "softmax").  For convolutions k, c, r, s are the
 * filter dimensions and items = N*P*Q (the GEMM n extent); otherwise items = elements written.  bytes:
 * the bytes the launch must move at least: convolutions input + filters + output + residual, each once;
 * the other layers their input(s) and output once each (pooling: whole input + output); 0 for the
 * library's own repacking kernels. */
typedef struct { char label[24]; int k, c, r, s; long long items; float ms; long long bytes; } dr_trace_record;

/* Starts recording one HIP event pair around every kernel launch the library makes (on the stream
 * of that launch) whose label contains label_filter (NULL or "" = all) and, for convolutions, whose
 * k / c / r equal conv_k / conv_c / conv_r (0 = any).  At most `capacity` launches are recorded,
 * later ones run untraced.  Per-process state, not thread safe: meant for benchmarks, which use it
 * to time the dominant kernel inside their timed region (the measure behind the paper's per-layer
 * tables, Table 4).  Creates events (the only entry point besides dr_net_set_timing that does). */
int dr_trace_begin(const char* label_filter, int conv_k, int conv_c, int conv_r, int capacity);

/* Stops recording, waits for the recorded events, writes up to out_capacity records (launch order)
 * and the number written to *count, and releases the events. */
int dr_trace_end(dr_trace_record* out, int out_capacity, int* count);

/* ---- misc ------------------------------------------------------------------------------------------ */

/* Message of the last error raised on the calling thread ("" if none). */
const char* dr_last_error(void);

/* Library version string. */
const char* dr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DEEPREBIRTH_H */
