// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/deeprebirth.h"

namespace dr {

// Records a message for dr_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// Checks the launch status of the kernels just enqueued.
int check_launch(const char* what);
// compute units of the current device (256 when the query fails)
int device_cus();

inline size_t elem_size(int dtype) { return dtype == DR_BF16 ? 2 : 4; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t tensor_elems(const dr_tensor& t) { return (size_t)t.n * t.c * t.h * t.w; }
inline size_t tensor_bytes(const dr_tensor& t) { return tensor_elems(t) * elem_size(t.dtype); }

struct ConvGeom;
// Brackets one kernel launch with an event pair when tracing is on (see dr_trace_begin).
struct TraceScope {
    // bytes: what the launch must move (convolutions: computed from g)
    TraceScope(const char* label, const ConvGeom* g, long long items, hipStream_t st, long long bytes = 0);
    ~TraceScope();
    int slot;
    hipStream_t st;
};

// Geometry of one convolution launch, filled by the host after validation.
struct ConvGeom {
    int N, C, H, W;      // input
    int K, R, S;         // filters
    int sh, sw, ph, pw;  // stride, padding
    int P, Q;            // output spatial size
    int Kg;              // GEMM K = C*R*S
    int Ng;              // GEMM N = N*P*Q
    int y_ctot, y_coff;  // channels of the output tensor, first channel written
    int relu;            // fused max(.,0)
    int res_ctot;        // channels of the residual tensor (0 = no residual add)
    int w_krsc;          // filters are in KRSC order (else KCRS)
    int nhwc;            // activations (x, y, residual) are channels-last
    int c_logical;       // channels of the layer when C counts zero padding added by the caller (0: C itself); for trace records
};

// conv_f32.hip / conv_bf16.hip: y = conv(x, w) + bias [+ residual] [ReLU].
// `residual` (may be NULL) has the output's n, P, Q and res_ctot channels, read at channel j.
// ws (may be NULL): scratch of conv_f32_scratch_bytes(g) bytes, 16-byte aligned, which lets a layer with few
// output tiles cut its contraction over several workgroups (see conv_f32.hip); too small = not used.
size_t conv_f32_scratch_bytes(const ConvGeom& g);
struct ConvSplit;
// split (may be NULL): destinations of a stacked convolution, as for launch_conv_bf16_dma (no residual, no scratch then)
int launch_conv_f32(const ConvGeom& g, const float* x, const float* w, const float* bias, const float* residual,
                    float* y, hipStream_t st, void* ws = nullptr, size_t ws_bytes = 0, const ConvSplit* split = nullptr);
int launch_conv_bf16(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias,
                     const uint16_t* residual, uint16_t* y, hipStream_t st);

// conv_bf16_dma.hip: the main bf16 kernel (NHWC, KRSC filters, C % 8 == 0, 16-byte aligned tensors)
bool conv_bf16_dma_eligible(const ConvGeom& g, const void* x, const void* w);
// Destinations of a stacked convolution (Eq. (12)): the first k filters write channels [c_offset, c_offset + k)
// of tensor y (ctot channels per pixel), the next destination takes the following filters, and so on.
// Every k but the last is a multiple of 8, there is no residual, g.K is the sum of the k.  split = NULL or
// n <= 1: the ordinary single destination (y, g.y_ctot, g.y_coff).
struct ConvDest { void* y; int ctot, c_offset, k; };
struct ConvSplit { int n; ConvDest dst[4]; };
int launch_conv_bf16_dma(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias,
                         const uint16_t* residual, uint16_t* y, hipStream_t st, const ConvSplit* split = nullptr);

// conv_bf16_patch.hip: filters of several taps at stride 1, C % 64 == 0, maps at most 256 pixels wide whose patch of
// TH + R - 1 input rows fits LDS: the tile's input patch is loaded once and every tap multiplies from there
bool conv_bf16_patch_eligible(const ConvGeom& g, const void* x, const void* w, const void* y);
// tm: 32-filter blocks per workgroup (2 or 3); 0 = the launcher's choice
int launch_conv_bf16_patch(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, uint16_t* y, hipStream_t st, int tm = 0);
// conv_bf16_rows.hip: the same idea for up to 64 channels (a multiple of 16) on maps of any size: a tile is a run of
// output rows of the whole batch's row stack, image borders inside it allowed
bool conv_bf16_rows_eligible(const ConvGeom& g, const void* x, const void* w, const void* y);
int launch_conv_bf16_rows(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, uint16_t* y, hipStream_t st);
// ... and for the padded 4-channel copy of a 3-channel input (xp, wp8 as for launch_conv_bf16_stem)
// tail (may be NULL): a 1x1 convolution (stride 1, no padding) on the layer's output, run in the same kernel; g.y_ctot,
// g.y_coff and y then belong to its destination and the layer's own output is never written
struct RowsTail {
    const uint16_t* w2;      // [K2][K] filters
    const float* bias2;      // may be NULL
    int K2, relu2;
};
bool conv_bf16_rows_stem_eligible(const ConvGeom& g, int hp, int wp, const void* xp, const void* y, const RowsTail* tail = nullptr);
int launch_conv_bf16_rows_stem(const ConvGeom& g, const uint16_t* xp, int hp, int wp, const uint16_t* wp8, const float* bias, uint16_t* y,
                               hipStream_t st, const RowsTail* tail = nullptr);

// conv_bf16_dma.hip: convolution, ReLU, LRN (window of 5) and 3x3 stride-2 max-pooling in one kernel (the streamlined
// block's original form, Sec. 3.1); y is the pooled tensor (PP x QQ pixels per image, y_ctot channels, written from y_coff)
bool conv_bf16_block_eligible(const ConvGeom& g, const void* x, const void* w, const dr_pool& p, const dr_lrn& l);
int launch_conv_bf16_block(const ConvGeom& g, const uint16_t* x, const uint16_t* w, const float* bias, const dr_lrn& l, int PP, int QQ,
                           uint16_t* y, int y_ctot, int y_coff, hipStream_t st);

// conv_bf16_dma.hip: inputs of at most 4 channels through a padded 4-channel copy (see the definition)
bool conv_bf16_stem_eligible(const ConvGeom& g);
int launch_conv_bf16_stem(const ConvGeom& real, const uint16_t* xp, int hp, int wp, const uint16_t* wp8, const float* bias,
                          uint16_t* y, hipStream_t st);
// While one of these lives on a host thread, convolutions launched by that thread share the device with
// kernels on other streams (branches of a module side by side): the launcher then keeps its larger
// tiles instead of cutting a small layer into enough workgroups to fill the device by itself.
struct SharedDeviceScope {
    explicit SharedDeviceScope(bool on);
    ~SharedDeviceScope();
    bool on_;
};


// train.hip: regression of a slim layer (fp32, NCHW, KCRS)
size_t regression_loss_workspace_bytes();
int launch_regression_loss_grad(const float* f, const float* y, float* dz, size_t count, float* loss, void* ws, hipStream_t st);
size_t conv_wgrad_workspace_bytes(const ConvGeom& g);
int launch_conv_wgrad_f32(const ConvGeom& g, const float* x, const float* dz, float* dw, float* db, void* ws, hipStream_t st);
int launch_sgd_step(float* w, const float* dw, float lr, size_t count, hipStream_t st);

// pointwise.hip
int launch_pack_filters(int dtype, const void* w_kcrs, void* w_krsc, int K, int C, int RS, hipStream_t st);
int launch_relu(int dtype, const void* x, void* y, size_t count, hipStream_t st);
int launch_lrn(const dr_tensor& d, const void* x, void* y, const dr_lrn& p, hipStream_t st);
int launch_maxpool(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, hipStream_t st);
int launch_avgpool(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, hipStream_t st);
struct ConcatSeg { const void* src; int c; int c_off; };
int launch_concat(const dr_tensor& yd, int nb, const ConcatSeg* segs, void* y, hipStream_t st);
int launch_bn(const dr_tensor& d, const void* x, void* y, const float* gamma, const float* beta, const float* mean,
              const float* var, float eps, int relu, hipStream_t st);
int launch_add_relu(int dtype, const void* a, const void* b, void* y, size_t count, hipStream_t st);

// pointwise_nhwc.hip: the channels-last versions (called by the launchers above)
int launch_lrn_nhwc(const dr_tensor& d, const void* x, void* y, const dr_lrn& p, hipStream_t st);
int launch_pool_nhwc(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, bool avg, hipStream_t st);
// LRN (window of 5 channels) and 3x3 max-pooling (stride 1 or 2) in one pass, in either order; channels-last,
// 16-byte channel groups, at most 64 of them
bool pool_lrn_nhwc_supported(const dr_tensor& xd, const void* x, const void* y, const dr_pool& p, const dr_lrn& l);
int launch_pool_lrn_nhwc(const dr_tensor& xd, const void* x, const dr_tensor& yd, void* y, const dr_pool& p, const dr_lrn& l, bool lrn_first,
                         hipStream_t st);
int launch_concat_nhwc(const dr_tensor& yd, int nb, const ConcatSeg* segs, void* y, hipStream_t st);
int launch_bn_nhwc(const dr_tensor& d, const void* x, void* y, const float* gamma, const float* beta, const float* mean,
                   const float* var, float eps, int relu, hipStream_t st);
// bf16 channel padding to a multiple of 8 (pixels x C -> pixels x Cp; filters KCRS or KRSC -> KRSC with Cp channels)
int launch_pad_channels_bf16(const void* x, void* y, size_t pixels, int C, int Cp, hipStream_t st);
int launch_pad_filters_bf16(const void* w, void* y, int K, int C, int RS, int Cp, int krsc, hipStream_t st);
// the copies launch_conv_bf16_stem takes: xp[N][hp][wp][4] and wp8[K][8][8][4]
int launch_stem_pack_bf16(const void* x, void* xp, int N, int C, int H, int W, int pad_h, int pad_w, int hp, int wp, hipStream_t st);
int launch_stem_filters_bf16(const void* w, void* wp8, int K, int C, int R, int S, int krsc, hipStream_t st);
int launch_fc(int dtype, const void* x, const void* w, const float* bias, void* y, int N, int I, int O, hipStream_t st);
int launch_softmax(int dtype, const void* x, float* y, int N, int O, hipStream_t st);

}  // namespace dr
