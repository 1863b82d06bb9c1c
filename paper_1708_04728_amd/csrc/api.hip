// C ABI of the library: argument validation (host only, before anything is enqueued), shape rules,
// and the orchestration of inception modules, bottlenecks and whole networks out of the kernels.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "dr_internal.h"

namespace dr {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// compute units of the current device (asked once per device; 256 if the runtime will not say)
int device_cus()
{
    constexpr int MAX_DEV = 64;
    static std::atomic<int> cus[MAX_DEV];
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return 256;
    if ((v = cus[dev].load(std::memory_order_relaxed)) > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cus[dev].store(v, std::memory_order_relaxed);
    return v;
}

int check_launch(const char* what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DR_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return DR_OK;
}

// ---- kernel tracing -------------------------------------------------------------------------------
static struct {
    bool active = false;
    char filter[24] = "";
    int k = 0, c = 0, r = 0;
    std::vector<hipEvent_t> ev;            // 2 per slot
    std::vector<dr_trace_record> recs;
    size_t capacity = 0;
} g_trace;

TraceScope::TraceScope(const char* label, const ConvGeom* g, long long items, hipStream_t s, long long bytes) : slot(-1), st(s)
{
    if (!g_trace.active || g_trace.recs.size() >= g_trace.capacity) return;
    if (g_trace.filter[0] && !strstr(label, g_trace.filter)) return;
    if (g && ((g_trace.k && g_trace.k != g->K) || (g_trace.c && g_trace.c != (g->c_logical ? g->c_logical : g->C)) || (g_trace.r && g_trace.r != g->R))) return;
    dr_trace_record rec;
    memset(&rec, 0, sizeof rec);
    snprintf(rec.label, sizeof rec.label, "%s", label);
    if (g) {
        const long long c = g->c_logical ? g->c_logical : g->C, esz = strstr(label, "f32") ? 4 : 2;
        rec.k = g->K; rec.c = (int)c; rec.r = g->R; rec.s = g->S;
        rec.bytes = esz * ((long long)g->N * c * g->H * g->W + (long long)g->K * c * g->R * g->S + (long long)g->Ng * g->K * (g->res_ctot ? 2 : 1));
    }
    if (!g || bytes > 0) rec.bytes = bytes;          // (a caller that knows better: e.g. a block whose output is the pooled tensor)
    rec.items = items;
    slot = (int)g_trace.recs.size();
    g_trace.recs.push_back(rec);
    (void)hipEventRecord(g_trace.ev[2 * slot], st);
}

TraceScope::~TraceScope()
{
    if (slot >= 0) (void)hipEventRecord(g_trace.ev[2 * slot + 1], st);
}

namespace {

#define DR_TRY(expr) do { const int dr_rc_ = (expr); if (dr_rc_ != DR_OK) return dr_rc_; } while (0)

int check_tensor(const char* who, const char* name, const dr_tensor* t)
{
    if (!t) return fail(DR_ERR_NULL, "%s: descriptor %s is NULL", who, name);
    if (t->n < 0 || t->c < 0 || t->h < 0 || t->w < 0)
        return fail(DR_ERR_SHAPE, "%s: %s has a negative dimension (%d,%d,%d,%d)", who, name, t->n, t->c, t->h, t->w);
    if (t->dtype != DR_F32 && t->dtype != DR_BF16) return fail(DR_ERR_UNSUPPORTED, "%s: %s has unknown dtype %d", who, name, t->dtype);
    if (t->layout != DR_NCHW && t->layout != DR_NHWC) return fail(DR_ERR_UNSUPPORTED, "%s: %s has unknown layout %d", who, name, t->layout);
    if ((double)t->n * t->c * t->h * t->w >= 2147483648.0)
        return fail(DR_ERR_UNSUPPORTED, "%s: %s has more than 2^31-1 elements", who, name);
    return DR_OK;
}

int check_conv_desc(const char* who, const dr_conv* c)
{
    if (!c) return fail(DR_ERR_NULL, "%s: convolution descriptor is NULL", who);
    if (c->k < 1 || c->c < 1 || c->r < 1 || c->s < 1 || c->stride_h < 1 || c->stride_w < 1 || c->pad_h < 0 || c->pad_w < 0)
        return fail(DR_ERR_SHAPE, "%s: bad convolution k=%d c=%d r=%d s=%d stride=%d,%d pad=%d,%d", who, c->k, c->c, c->r, c->s,
                    c->stride_h, c->stride_w, c->pad_h, c->pad_w);
    if (c->filter_layout != DR_KCRS && c->filter_layout != DR_KRSC)
        return fail(DR_ERR_UNSUPPORTED, "%s: unknown filter layout %d", who, c->filter_layout);
    if (c->filter_layout == DR_KRSC && c->c % 8 != 0)
        return fail(DR_ERR_UNSUPPORTED, "%s: KRSC filters need a channel count that is a multiple of 8 (got %d)", who, c->c);
    return DR_OK;
}

int check_pool_desc(const char* who, const dr_pool* p)
{
    if (!p) return fail(DR_ERR_NULL, "%s: pooling descriptor is NULL", who);
    if (p->kh < 1 || p->kw < 1 || p->stride_h < 1 || p->stride_w < 1 || p->pad_h < 0 || p->pad_w < 0 || p->pad_h >= p->kh ||
        p->pad_w >= p->kw)
        return fail(DR_ERR_SHAPE, "%s: bad pooling window %dx%d stride %d,%d pad %d,%d", who, p->kh, p->kw, p->stride_h,
                    p->stride_w, p->pad_h, p->pad_w);
    return DR_OK;
}

// Output descriptors (shape rules live here and nowhere else in the library).
dr_tensor conv_out(const dr_tensor& x, const dr_conv& c)
{
    return dr_tensor{x.n, c.k, dr_conv_out_size(x.h, c.r, c.stride_h, c.pad_h), dr_conv_out_size(x.w, c.s, c.stride_w, c.pad_w),
                     x.dtype, x.layout};
}
dr_tensor pool_out(const dr_tensor& x, const dr_pool& p)
{
    return dr_tensor{x.n, x.c, dr_pool_out_size(x.h, p.kh, p.stride_h, p.pad_h), dr_pool_out_size(x.w, p.kw, p.stride_w, p.pad_w),
                     x.dtype, x.layout};
}
dr_tensor avgpool_out(const dr_tensor& x, const dr_pool& p)
{
    return dr_tensor{x.n, x.c, dr_conv_out_size(x.h, p.kh, p.stride_h, 0), dr_conv_out_size(x.w, p.kw, p.stride_w, 0), x.dtype, x.layout};
}
bool same_shape(const dr_tensor& a, const dr_tensor& b)
{
    return a.n == b.n && a.c == b.c && a.h == b.h && a.w == b.w && a.layout == b.layout;
}

// Validated convolution launch (shared by the single-layer entry points and the composite ones).
// Geometry of layer cd on input xd with output descriptor o (the output tensor's fields are set by the caller).
ConvGeom conv_geom(const dr_tensor& xd, const dr_conv& cd, const dr_tensor& o)
{
    ConvGeom g;
    g.N = xd.n; g.C = xd.c; g.H = xd.h; g.W = xd.w;
    g.K = cd.k; g.R = cd.r; g.S = cd.s;
    g.sh = cd.stride_h; g.sw = cd.stride_w; g.ph = cd.pad_h; g.pw = cd.pad_w;
    g.P = o.h; g.Q = o.w;
    g.Kg = cd.c * cd.r * cd.s;
    g.Ng = o.n * o.h * o.w;
    g.y_ctot = o.c; g.y_coff = 0;
    g.relu = cd.relu != 0;
    g.res_ctot = 0;
    g.w_krsc = cd.filter_layout == DR_KRSC;
    g.nhwc = xd.layout == DR_NHWC;
    g.c_logical = 0;
    return g;
}

// Scratch a convolution uses when its caller has some to give (fp32: the partial sums of a contraction
// cut over several workgroups, for layers with too few output tiles to occupy the device); 0 = none.
size_t conv_scratch_bytes(const dr_tensor& xd, const dr_conv& cd)
{
    if (xd.dtype != DR_F32 || xd.layout != DR_NCHW) return 0;
    const dr_tensor o = conv_out(xd, cd);
    if ((double)cd.c * cd.r * cd.s >= 2147483648.0 || (double)o.n * o.h * o.w >= 2147483648.0 || tensor_elems(o) == 0) return 0;
    return conv_f32_scratch_bytes(conv_geom(xd, cd, o));
}

int conv_run(const char* who, const dr_tensor& xd, const void* x, const dr_conv& cd, const void* w, const float* bias,
             const void* residual, int res_ctot, const dr_tensor& yd, void* y, int y_c_offset, hipStream_t st, int c_logical = 0,
             void* scratch = nullptr, size_t scratch_bytes = 0)
{
    if (xd.c != cd.c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd.c, cd.c);
    const dr_tensor o = conv_out(xd, cd);
    if (yd.n != o.n || yd.h != o.h || yd.w != o.w)
        return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%d per channel, the layer produces %dx%dx%d", who, yd.n, yd.h, yd.w, o.n, o.h, o.w);
    if (y_c_offset < 0 || y_c_offset + cd.k > yd.c)
        return fail(DR_ERR_SHAPE, "%s: channels [%d,%d) do not fit an output of %d channels", who, y_c_offset, y_c_offset + cd.k, yd.c);
    if (yd.dtype != xd.dtype || yd.layout != xd.layout) return fail(DR_ERR_UNSUPPORTED, "%s: input and output differ in dtype or layout", who);
    if (xd.dtype == DR_F32 && xd.layout != DR_NCHW) return fail(DR_ERR_UNSUPPORTED, "%s: fp32 convolution takes NCHW tensors", who);
    if (xd.dtype == DR_F32 && cd.filter_layout == DR_KRSC && cd.c % 16 != 0)
        return fail(DR_ERR_UNSUPPORTED, "%s: fp32 KRSC filters need a channel count that is a multiple of 16 (got %d)", who, cd.c);
    if ((double)cd.c * cd.r * cd.s >= 2147483648.0 || (double)o.n * o.h * o.w >= 2147483648.0)
        return fail(DR_ERR_UNSUPPORTED, "%s: problem too large", who);
    if ((size_t)o.n * cd.k * o.h * o.w == 0) return DR_OK;   // nothing to compute: pointers may be NULL
    if (!x || !w || !y) return fail(DR_ERR_NULL, "%s: x, w or y is NULL", who);
    ConvGeom g = conv_geom(xd, cd, o);
    g.y_ctot = yd.c; g.y_coff = y_c_offset;
    g.res_ctot = residual ? res_ctot : 0;
    g.c_logical = c_logical;
    if (xd.dtype == DR_F32)
        return launch_conv_f32(g, (const float*)x, (const float*)w, bias, (const float*)residual, (float*)y, st, scratch, scratch_bytes);
    return launch_conv_bf16(g, (const uint16_t*)x, (const uint16_t*)w, bias, (const uint16_t*)residual, (uint16_t*)y, st);
}

// The streamlined block's original form in one kernel (see dr_conv_lrn_maxpool_fwd).
int conv_block_run(const char* who, const dr_tensor& xd, const void* x, const dr_conv& cd, const void* w, const float* bias, const dr_lrn& l,
                   const dr_pool& p, const dr_tensor& yd, void* y, int y_c_offset, hipStream_t st)
{
    if (xd.c != cd.c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd.c, cd.c);
    const dr_tensor c = conv_out(xd, cd);
    const dr_tensor o = pool_out(c, p);
    if (yd.n != o.n || yd.h != o.h || yd.w != o.w)
        return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%d per channel, the block produces %dx%dx%d", who, yd.n, yd.h, yd.w, o.n, o.h, o.w);
    if (y_c_offset < 0 || y_c_offset + cd.k > yd.c)
        return fail(DR_ERR_SHAPE, "%s: channels [%d,%d) do not fit an output of %d channels", who, y_c_offset, y_c_offset + cd.k, yd.c);
    if (xd.dtype != DR_BF16 || yd.dtype != DR_BF16 || xd.layout != DR_NHWC || yd.layout != DR_NHWC || cd.filter_layout != DR_KRSC)
        return fail(DR_ERR_UNSUPPORTED, "%s: bf16 channels-last tensors and KRSC filters only", who);
    if ((double)cd.c * cd.r * cd.s >= 2147483648.0 || (double)c.n * c.h * c.w >= 2147483648.0) return fail(DR_ERR_UNSUPPORTED, "%s: problem too large", who);
    if (tensor_elems(o) == 0 || cd.k == 0) return DR_OK;
    if (!x || !w || !y) return fail(DR_ERR_NULL, "%s: x, w or y is NULL", who);
    ConvGeom g = conv_geom(xd, cd, c);
    g.relu = 1;
    if (!conv_bf16_block_eligible(g, x, w, p, l) || yd.c % 8 != 0 || y_c_offset % 8 != 0 || ((uintptr_t)y & 15) != 0)
        return fail(DR_ERR_UNSUPPORTED, "%s: needs at most 192 filters (a multiple of 8), channels a multiple of 8, an LRN window of 5, 3x3 pooling at "
                    "stride 2 without padding, 16-byte aligned tensors below 2 GiB", who);
    TraceScope trace("conv_lrn_pool", &g, g.Ng, st, (long long)(tensor_bytes(xd) + (size_t)cd.k * g.Kg * 2 + (size_t)o.n * o.h * o.w * cd.k * 2));
    return launch_conv_bf16_block(g, (const uint16_t*)x, (const uint16_t*)w, bias, l, o.h, o.w, (uint16_t*)y, yd.c, y_c_offset, st);
}

// ---- bump allocator over the caller's workspace (also used in "measure" mode with base = NULL)
struct Arena {
    char* base;
    size_t size, used, peak;
    bool measure;
    Arena(void* b, size_t s, bool m) : base((char*)b), size(s), used(0), peak(0), measure(m) {}
    void* take(size_t bytes)
    {
        const size_t off = used;
        used = align_up(used + bytes, 256);
        if (used > peak) peak = used;
        if (measure) return (void*)(uintptr_t)(256 + off);   // never dereferenced
        return used <= size ? base + off : nullptr;
    }
};

// A bf16 channels-last convolution whose channel count is not a multiple of 8 (the 3-channel network input)
// cannot use the matrix-core kernels, which fetch 16-byte channel groups.  Where a workspace exists
// (dr_net_fwd) the input and the filters are copied with their channels zero-padded to a multiple of 8
// first; the zeros add nothing to the sums.  Returns the scratch the layer needs / runs it.
bool conv_wants_padding(const dr_tensor& xd, const dr_conv& cd)
{
    return xd.dtype == DR_BF16 && xd.layout == DR_NHWC && cd.c % 8 != 0 && cd.c < 8;
}
// A 1x1 convolution right behind such a layer (stride 1, no padding, at most 64 filters over at most 64) can run in the
// same kernel: the layer's output tile stays in registers and is multiplied from there (conv_bf16_rows.hip, TAIL).
bool conv_tail_ok(const dr_conv& cd, const dr_conv& next)
{
    return next.r == 1 && next.s == 1 && next.stride_h == 1 && next.stride_w == 1 && next.pad_h == 0 && next.pad_w == 0 && next.c == cd.k &&
           cd.k <= 64 && cd.k % 8 == 0 && next.k <= 64 && next.k % 8 == 0 && next.k >= 8;
}
// tail != NULL: yd / y are the 1x1 convolution's output; *fused says whether the pair ran (as one kernel) -- when the
// kernel does not take the pair nothing has been run and the caller runs the two layers one after the other.
int padded_conv_run(const char* who, const dr_tensor& xd, const void* x, const dr_conv& cd, const void* w, const float* bias,
                    const dr_tensor& yd, void* y, Arena& ar, hipStream_t st, const dr_conv* tail = nullptr, const void* w2 = nullptr,
                    const float* b2 = nullptr, bool* fused = nullptr)
{
    if (fused) *fused = false;
    if (tail) {
        // (the pair or nothing)
        const dr_tensor o1 = conv_out(xd, cd);
        if (!(cd.c <= 4 && cd.r <= 8 && cd.s <= 8 && cd.stride_w % 2 == 0 && (double)o1.h * o1.w <= 65536.0 && (double)o1.n * o1.h * o1.w < 16777216.0)) return DR_OK;
        const int hp = std::max(xd.h + 2 * cd.pad_h, (o1.h - 1) * cd.stride_h + 8);
        const int wp = (std::max(xd.w + 2 * cd.pad_w, (o1.w - 1) * cd.stride_w + 8) + 7) / 8 * 8;
        const size_t xbytes = (size_t)xd.n * hp * wp * 8;
        if (xbytes >= (1ull << 31) || !x || !w || !w2 || !y || xd.c != cd.c) return DR_OK;
        const dr_tensor o2 = conv_out(o1, *tail);
        if (yd.n != o2.n || yd.h != o2.h || yd.w != o2.w || yd.c != tail->k || yd.dtype != xd.dtype || yd.layout != xd.layout) return DR_OK;
        ConvGeom g;
        g.N = xd.n; g.C = xd.c; g.H = xd.h; g.W = xd.w;
        g.K = cd.k; g.R = cd.r; g.S = cd.s;
        g.sh = cd.stride_h; g.sw = cd.stride_w; g.ph = cd.pad_h; g.pw = cd.pad_w;
        g.P = o1.h; g.Q = o1.w;
        g.Kg = cd.c * cd.r * cd.s;
        g.Ng = o1.n * o1.h * o1.w;
        g.y_ctot = yd.c; g.y_coff = 0;
        g.relu = cd.relu != 0;
        g.res_ctot = 0;
        g.w_krsc = cd.filter_layout == DR_KRSC;
        g.nhwc = 1;
        g.c_logical = 0;
        const RowsTail rt{(const uint16_t*)w2, b2, tail->k, tail->relu != 0};
        // (probe with the addresses the buffers will have: 256-byte aligned workspace pieces)
        Arena probe = ar;
        void* xbuf = probe.take(xbytes);
        void* wbuf = probe.take((size_t)cd.k * 512);
        if (!xbuf || !wbuf || !conv_bf16_rows_stem_eligible(g, hp, wp, xbuf, y, &rt)) return DR_OK;
        ar = probe;
        DR_TRY(launch_stem_pack_bf16(x, xbuf, xd.n, xd.c, xd.h, xd.w, cd.pad_h, cd.pad_w, hp, wp, st));
        DR_TRY(launch_stem_filters_bf16(w, wbuf, cd.k, cd.c, cd.r, cd.s, g.w_krsc, st));
        DR_TRY(launch_conv_bf16_rows_stem(g, (const uint16_t*)xbuf, hp, wp, (const uint16_t*)wbuf, bias, (uint16_t*)y, st, &rt));
        if (fused) *fused = true;
        return DR_OK;
    }
    if (cd.c <= 4 && cd.r <= 8 && cd.s <= 8 && cd.stride_w % 2 == 0 && (double)yd.h * yd.w <= 65536.0 && (double)yd.n * yd.h * yd.w < 16777216.0) {
        // packed form: 4 channels per pixel, padding laid out physically (launch_conv_bf16_stem)
        const int hp = std::max(xd.h + 2 * cd.pad_h, (yd.h - 1) * cd.stride_h + 8);
        const int wp = (std::max(xd.w + 2 * cd.pad_w, (yd.w - 1) * cd.stride_w + 8) + 7) / 8 * 8;
        const size_t xbytes = (size_t)xd.n * hp * wp * 8;
        if (xbytes < (1ull << 31)) {
            void* xbuf = ar.take(xbytes);
            void* wbuf = ar.take((size_t)cd.k * 512);
            if (ar.measure) return DR_OK;
            if (!xbuf || !wbuf) return fail(DR_ERR_WORKSPACE, "%s: workspace too small", who);
            if (!x || !w || !y) return fail(DR_ERR_NULL, "%s: x, w or y is NULL", who);
            if (xd.c != cd.c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd.c, cd.c);
            const dr_tensor o = conv_out(xd, cd);
            if (yd.n != o.n || yd.h != o.h || yd.w != o.w || yd.c != cd.k || yd.dtype != xd.dtype || yd.layout != xd.layout)
                return fail(DR_ERR_SHAPE, "%s: output descriptor does not match the layer", who);
            ConvGeom g;
            g.N = xd.n; g.C = xd.c; g.H = xd.h; g.W = xd.w;
            g.K = cd.k; g.R = cd.r; g.S = cd.s;
            g.sh = cd.stride_h; g.sw = cd.stride_w; g.ph = cd.pad_h; g.pw = cd.pad_w;
            g.P = o.h; g.Q = o.w;
            g.Kg = cd.c * cd.r * cd.s;
            g.Ng = o.n * o.h * o.w;
            g.y_ctot = yd.c; g.y_coff = 0;
            g.relu = cd.relu != 0;
            g.res_ctot = 0;
            g.w_krsc = cd.filter_layout == DR_KRSC;
            g.nhwc = 1;
            g.c_logical = 0;
            DR_TRY(launch_stem_pack_bf16(x, xbuf, xd.n, xd.c, xd.h, xd.w, cd.pad_h, cd.pad_w, hp, wp, st));
            DR_TRY(launch_stem_filters_bf16(w, wbuf, cd.k, cd.c, cd.r, cd.s, g.w_krsc, st));
            if (conv_bf16_rows_stem_eligible(g, hp, wp, xbuf, y))
                return launch_conv_bf16_rows_stem(g, (const uint16_t*)xbuf, hp, wp, (const uint16_t*)wbuf, bias, (uint16_t*)y, st);
            return launch_conv_bf16_stem(g, (const uint16_t*)xbuf, hp, wp, (const uint16_t*)wbuf, bias, (uint16_t*)y, st);
        }
    }
    const int Cp = (cd.c + 7) / 8 * 8;
    dr_tensor xp = xd;
    xp.c = Cp;
    dr_conv cp = cd;
    cp.c = Cp;
    cp.filter_layout = DR_KRSC;
    void* xbuf = ar.take(tensor_bytes(xp));
    void* wbuf = ar.take((size_t)cd.k * cd.r * cd.s * Cp * 2);
    if (ar.measure) return DR_OK;
    if (!xbuf || !wbuf) return fail(DR_ERR_WORKSPACE, "%s: workspace too small", who);
    if (!x || !w) return fail(DR_ERR_NULL, "%s: x or w is NULL", who);
    DR_TRY(launch_pad_channels_bf16(x, xbuf, (size_t)xd.n * xd.h * xd.w, cd.c, Cp, st));
    DR_TRY(launch_pad_filters_bf16(w, wbuf, cd.k, cd.c, cd.r * cd.s, Cp, cd.filter_layout == DR_KRSC, st));
    return conv_run(who, xp, xbuf, cp, wbuf, bias, nullptr, 0, yd, y, 0, st, cd.c);
}

// ---- inception ---------------------------------------------------------------------------------------
struct ParamCursor {
    const void* const* p;
    int i;
    const void* next() { return p ? p[i++] : (++i, nullptr); }
};

int inception_validate(const dr_tensor& xd, const dr_inception& d, dr_tensor* out)
{
    const char* who = "dr_inception_fwd";
    if (d.n_branches < 1 || d.n_branches > DR_MAX_BRANCHES) return fail(DR_ERR_SHAPE, "%s: %d branches", who, d.n_branches);
    if ((d.mode & DR_FUSE_STACK) && !(d.mode & DR_FUSE_RELU)) return fail(DR_ERR_UNSUPPORTED, "%s: DR_FUSE_STACK needs DR_FUSE_RELU", who);
    int ctot = 0, oh = -1, ow = -1;
    for (int b = 0; b < d.n_branches; ++b) {
        const dr_branch& br = d.branches[b];
        if (br.n_steps < 1 || br.n_steps > DR_MAX_STEPS) return fail(DR_ERR_SHAPE, "%s: branch %d has %d steps", who, b, br.n_steps);
        dr_tensor t = xd;
        for (int s = 0; s < br.n_steps; ++s) {
            const dr_step& stp = br.steps[s];
            if (stp.kind == DR_STEP_CONV) {
                DR_TRY(check_conv_desc(who, &stp.conv));
                if (stp.conv.c != t.c) return fail(DR_ERR_SHAPE, "%s: branch %d step %d expects %d channels, gets %d", who, b, s, stp.conv.c, t.c);
                t = conv_out(t, stp.conv);
            } else if (stp.kind == DR_STEP_MAXPOOL) {
                DR_TRY(check_pool_desc(who, &stp.pool));
                t = pool_out(t, stp.pool);
            } else {
                return fail(DR_ERR_UNSUPPORTED, "%s: unknown step kind %d", who, stp.kind);
            }
        }
        if (b == 0) { oh = t.h; ow = t.w; }
        else if (t.h != oh || t.w != ow) return fail(DR_ERR_SHAPE, "%s: branch %d ends at %dx%d, branch 0 at %dx%d", who, b, t.h, t.w, oh, ow);
        ctot += t.c;
    }
    *out = dr_tensor{xd.n, ctot, oh, ow, xd.dtype, xd.layout};
    return DR_OK;
}

// Streams and events for running the branches of a module side by side.  Branch 0 stays on the caller's
// stream; the others run on these streams between a fork event (recorded on the caller's stream before
// the module) and one join event per branch (awaited by the caller's stream before the concat, or before
// whatever the caller enqueues next).  One set per host thread and device, created on first use, default
// priority, never destroyed.  Events are handed out round-robin: a wait refers to the record that
// preceded it, so an event can be recorded again once its wait has been enqueued.
struct BranchStreams {
    bool ready = false;
    hipStream_t s[DR_MAX_BRANCHES - 1];
    hipEvent_t ev[64];
    unsigned next = 0;
    hipEvent_t event() { return ev[next++ & 63]; }
};
BranchStreams* branch_streams()
{
    constexpr int MAX_DEV = 16;                      // devices of one process that can run branches side by side
    static thread_local BranchStreams pools[MAX_DEV];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return nullptr;
    BranchStreams& pool = pools[dev];
    if (!pool.ready) {
        // all or nothing: what a failed attempt had created is released again, and the next call starts afresh
        int ns = 0, ne = 0;
        bool ok = true;
        for (auto& s : pool.s) {
            if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) { ok = false; break; }
            ++ns;
        }
        for (auto& e : pool.ev) {
            if (!ok) break;
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { ok = false; break; }
            ++ne;
        }
        if (!ok) {
            for (int i = 0; i < ne; ++i) (void)hipEventDestroy(pool.ev[i]);
            for (int i = 0; i < ns; ++i) (void)hipStreamDestroy(pool.s[i]);
            (void)hipGetLastError();
            return nullptr;
        }
        pool.ready = true;
    }
    return &pool;
}

// The stacked first steps of a module (see inception_run).  Marks the branches it has served in `stacked`
// and leaves their step-0 outputs in `dst` (workspace buffers; NULL for a one-step branch that wrote y).
// Serves nothing, without error, when the parameters are not laid out for it.
int run_stacked_first_steps(const dr_tensor& xd, const void* x, const dr_inception& d, const ParamCursor& wts, const ParamCursor& bss,
                            const dr_tensor& yd, void* y, Arena& ar, hipStream_t st, bool* stacked, void** dst)
{
    const char* who = "dr_inception_fwd";
    const bool fuse_cat = d.mode & DR_FUSE_CONCAT;
    int pidx = wts.i, c_off = 0, nb = 0, members[DR_MAX_BRANCHES], coffs[DR_MAX_BRANCHES], pidxs[DR_MAX_BRANCHES];
    for (int b = 0; b < d.n_branches; ++b) {
        const dr_branch& br = d.branches[b];
        const dr_conv& c0 = br.steps[0].conv;
        if (br.steps[0].kind == DR_STEP_CONV && c0.r == 1 && c0.s == 1 && c0.stride_h == 1 && c0.stride_w == 1 && c0.pad_h == 0 &&
            c0.pad_w == 0 && c0.relu && nb < 4) {
            members[nb] = b; coffs[nb] = c_off; pidxs[nb] = pidx; ++nb;
        }
        int c = xd.c;
        for (int s = 0; s < br.n_steps; ++s)
            if (br.steps[s].kind == DR_STEP_CONV) { c = br.steps[s].conv.k; ++pidx; }
        c_off += c;
    }
    if (nb < 2) return DR_OK;
    // back to back in memory, in branch order; bf16: every bank but the last a multiple of 8 filters (16-byte stores)
    const bool f32 = xd.dtype == DR_F32;
    const size_t esz = f32 ? 4 : 2;
    const char* w0 = (const char*)wts.p[pidxs[0]];
    const char* b0 = bss.p ? (const char*)bss.p[pidxs[0]] : nullptr;
    if (!w0) return DR_OK;
    size_t woff = 0, boff = 0;
    int ktot = 0;
    for (int i = 0; i < nb; ++i) {
        const dr_conv& c0 = d.branches[members[i]].steps[0].conv;
        const char* bi = bss.p ? (const char*)bss.p[pidxs[i]] : nullptr;
        if ((const char*)wts.p[pidxs[i]] != w0 + woff) return DR_OK;
        if ((b0 == nullptr) != (bi == nullptr) || (b0 && bi != b0 + boff)) return DR_OK;
        if (!f32 && i + 1 < nb && c0.k % 8 != 0) return DR_OK;
        if (c0.filter_layout != d.branches[members[0]].steps[0].conv.filter_layout) return DR_OK;
        woff += (size_t)c0.k * xd.c * esz;
        boff += (size_t)c0.k * 4;
        ktot += c0.k;
    }
    ConvGeom g;
    g.N = xd.n; g.C = xd.c; g.H = xd.h; g.W = xd.w;
    g.K = ktot; g.R = 1; g.S = 1;
    g.sh = g.sw = 1; g.ph = g.pw = 0;
    g.P = xd.h; g.Q = xd.w;
    g.Kg = xd.c;
    g.Ng = xd.n * xd.h * xd.w;
    g.relu = 1;
    g.res_ctot = 0;
    // a 1x1 filter bank is the same array in both orders; fp32 keeps the order the branches name, so that the stacked
    // convolution adds its products in the same order as one convolution per branch
    g.w_krsc = f32 ? d.branches[members[0]].steps[0].conv.filter_layout == DR_KRSC : 1;
    g.nhwc = f32 ? 0 : 1;
    g.c_logical = 0;
    if (g.Ng == 0 || !x) return DR_OK;
    if (f32 ? ((size_t)g.Ng * g.C * 4 >= (1ull << 31) || (size_t)ktot * g.C * 4 >= (1ull << 31)) : !conv_bf16_dma_eligible(g, x, w0))
        return DR_OK;
    ConvSplit sp;
    sp.n = nb;
    for (int i = 0; i < nb; ++i) {
        const dr_branch& br = d.branches[members[i]];
        const bool direct = br.n_steps == 1 && fuse_cat;
        const int k = br.steps[0].conv.k;
        void* buf = direct ? y : ar.take((size_t)g.Ng * k * esz);
        if (!buf) return fail(DR_ERR_WORKSPACE, "%s: workspace too small", who);
        sp.dst[i] = ConvDest{buf, direct ? yd.c : k, direct ? coffs[i] : 0, k};
        dst[members[i]] = direct ? nullptr : buf;
        stacked[members[i]] = true;
    }
    g.y_ctot = sp.dst[0].ctot; g.y_coff = sp.dst[0].c_offset;
    if (f32)
        return launch_conv_f32(g, (const float*)x, (const float*)w0, (const float*)b0, nullptr, (float*)sp.dst[0].y, st, nullptr, 0, &sp);
    TraceScope trace("conv_bf16", &g, g.Ng, st);
    return launch_conv_bf16_dma(g, (const uint16_t*)x, (const uint16_t*)w0, (const float*)b0, nullptr, (uint16_t*)sp.dst[0].y, st, &sp);
}

// Runs (or, with a measuring arena, only plans) one module.  y may be NULL when measuring.
int inception_run(const dr_tensor& xd, const void* x, const dr_inception& d, ParamCursor& wts, ParamCursor& bss,
                  const dr_tensor& yd, void* y, Arena& ar, hipStream_t main_st)
{
    const char* who = "dr_inception_fwd";
    const bool fuse_relu = d.mode & DR_FUSE_RELU, fuse_cat = d.mode & DR_FUSE_CONCAT;
    ConcatSeg segs[DR_MAX_BRANCHES];
    int nseg = 0, c_off = 0;
    // DR_FUSE_STACK (Eq. (12)): first-step 1x1 convolutions on the module input run as one convolution
    // when their filters (and biases) lie back to back in memory in branch order, so that they form the
    // stacked filter bank as they are; each keeps its own destination.  bf16 channels-last and fp32 NCHW.
    void* stacked_dst[DR_MAX_BRANCHES] = {};
    bool stacked[DR_MAX_BRANCHES] = {};
    if ((d.mode & DR_FUSE_STACK) && !ar.measure && wts.p &&
        ((xd.dtype == DR_BF16 && xd.layout == DR_NHWC) || (xd.dtype == DR_F32 && xd.layout == DR_NCHW)))
        DR_TRY(run_stacked_first_steps(xd, x, d, wts, bss, yd, y, ar, main_st, stacked, stacked_dst));
    // A trace of every kernel (no label filter) is there to time each kernel on its own: it runs the
    // branches in turn.
    BranchStreams* bs = nullptr;
    hipEvent_t fork = nullptr;
    const bool full_trace = g_trace.active && !g_trace.filter[0];
    if ((d.mode & DR_CONCURRENT_BRANCHES) && d.n_branches > 1 && !ar.measure && !full_trace) {
        bs = branch_streams();
        if (!bs) return fail(DR_ERR_HIP, "%s: cannot create the branch streams", who);
        fork = bs->event();
        if (hipEventRecord(fork, main_st) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipEventRecord failed", who);
    }
    SharedDeviceScope shared(bs != nullptr);
    // Every side stream that has been made to wait for the fork is joined to the caller's stream again, also when
    // the module fails half-way: the caller's stream (or a capture in progress) is never left with loose ends.
    struct Join {
        BranchStreams* bs;
        hipStream_t main;
        bool pending[DR_MAX_BRANCHES] = {};
        ~Join()
        {
            for (int b = 1; bs && b < DR_MAX_BRANCHES; ++b) {
                if (!pending[b]) continue;
                const hipEvent_t e = bs->event();
                if (hipEventRecord(e, bs->s[b - 1]) == hipSuccess) (void)hipStreamWaitEvent(main, e, 0);
            }
        }
    } join{bs, main_st};
    for (int b = 0; b < d.n_branches; ++b) {
        const dr_branch& br = d.branches[b];
        dr_tensor t = xd;
        const void* cur = x;
        const bool side = bs && b > 0;
        const hipStream_t st = side ? bs->s[b - 1] : main_st;
        if (side && hipStreamWaitEvent(st, fork, 0) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipStreamWaitEvent failed", who);
        join.pending[b] = side;
        for (int s = 0; s < br.n_steps; ++s) {
            const dr_step& stp = br.steps[s];
            const bool last = s == br.n_steps - 1;
            if (stp.kind == DR_STEP_CONV) {
                dr_conv cd = stp.conv;
                const bool relu_after = cd.relu != 0;
                cd.relu = relu_after && fuse_relu;
                const dr_tensor o = conv_out(t, cd);
                const void* w = wts.next();
                const float* bias = (const float*)bss.next();
                const bool direct = last && fuse_cat;   // writes its channel range of y, ReLU in the store
                if (direct) cd.relu = relu_after;
                void* dst = direct ? y : (s == 0 && stacked[b]) ? stacked_dst[b] : ar.take(tensor_bytes(o));
                if (!dst && !ar.measure) return fail(DR_ERR_WORKSPACE, "%s: workspace too small", who);
                const size_t sbytes = conv_scratch_bytes(t, cd);
                void* sc = sbytes ? ar.take(sbytes) : nullptr;
                if (!ar.measure && !(s == 0 && stacked[b])) {
                    if (!w) return fail(DR_ERR_NULL, "%s: missing weights of branch %d step %d", who, b, s);
                    DR_TRY(conv_run(who, t, cur, cd, w, bias, nullptr, 0, direct ? yd : o, dst, direct ? c_off : 0, st, 0, sc, sc ? sbytes : 0));
                    if (relu_after && !cd.relu) DR_TRY(launch_relu(o.dtype, dst, dst, tensor_elems(o), st));
                }
                if (last && !direct) segs[nseg++] = ConcatSeg{dst, o.c, c_off};
                cur = dst;
                t = o;
            } else {
                const dr_tensor o = pool_out(t, stp.pool);
                void* dst = ar.take(tensor_bytes(o));
                if (!dst && !ar.measure) return fail(DR_ERR_WORKSPACE, "%s: workspace too small", who);
                if (!ar.measure) DR_TRY(launch_maxpool(t, cur, o, dst, stp.pool, st));
                if (last) segs[nseg++] = ConcatSeg{dst, o.c, c_off};
                cur = dst;
                t = o;
            }
        }
        c_off += t.c;
        if (side) {
            const hipEvent_t done = bs->event();
            if (hipEventRecord(done, st) != hipSuccess || hipStreamWaitEvent(main_st, done, 0) != hipSuccess)
                return fail(DR_ERR_HIP, "%s: joining branch %d failed", who, b);
            join.pending[b] = false;
        }
    }
    if (nseg && !ar.measure) DR_TRY(launch_concat(yd, nseg, segs, y, main_st));
    return DR_OK;
}


// ---- whole networks ------------------------------------------------------------------------------------
int param_count(const dr_layer_desc& L)
{
    switch (L.kind) {
    case DR_LAYER_CONV: return 2;
    case DR_LAYER_CONV_LRN_MAXPOOL: return 2;
    case DR_LAYER_FC: return 2;
    case DR_LAYER_INCEPTION: {
        int n = 0;
        for (int b = 0; b < L.inception.n_branches; ++b)
            for (int s = 0; s < L.inception.branches[b].n_steps; ++s)
                if (L.inception.branches[b].steps[s].kind == DR_STEP_CONV) n += 2;
        return n;
    }
    case DR_LAYER_BOTTLENECK: return (L.bottleneck.project ? 4 : 3) * (L.bottleneck.folded ? 2 : 6);
    default: return 0;
    }
}

// ResNet bottleneck.  Original form: conv, BatchNorm(+Scale) and ReLU are separate passes and the
// residual sum is its own kernel; folded (slim) form: three or four convolutions with folded
// parameters, ReLU and the residual sum applied in the convolutions' stores.
int bottleneck_run(const dr_tensor& xd, const void* x, const dr_bottleneck& bd, const void* const* prm, const dr_tensor& yd,
                   void* y, Arena& ar, hipStream_t st)
{
    const char* who = "dr_net_fwd(bottleneck)";
    const bool run = !ar.measure;
    const int per = bd.folded ? 2 : 6;   // pointers per conv(+bn) group
    auto conv_of = [&](int k, int c, int r, int pad, int relu) { return dr_conv{k, c, r, r, 1, 1, pad, pad, relu, bd.filter_layout}; };
    const dr_conv ca = conv_of(bd.mid, xd.c, 1, 0, bd.folded), cb = conv_of(bd.mid, bd.mid, 3, 1, bd.folded),
                  cc = conv_of(bd.out, bd.mid, 1, 0, bd.folded), cp = conv_of(bd.out, xd.c, 1, 0, 0);
    const dr_tensor ta = conv_out(xd, ca), tb = conv_out(ta, cb), tc = conv_out(tb, cc);
    if (!bd.project && xd.c != bd.out) return fail(DR_ERR_SHAPE, "%s: identity shortcut needs %d input channels, got %d", who, bd.out, xd.c);
    void* sa = ar.take(tensor_bytes(ta));
    void* sb = ar.take(tensor_bytes(tb));
    void* sp = bd.project ? ar.take(tensor_bytes(tc)) : nullptr;
    void* sc = bd.folded ? nullptr : ar.take(tensor_bytes(tc));
    if (!run) return DR_OK;
    if (!sa || !sb || (bd.project && !sp) || (!bd.folded && !sc)) return fail(DR_ERR_WORKSPACE, "%s: workspace too small", who);
    for (int i = 0; i < (bd.project ? 4 : 3) * per; ++i)
        if (!prm[i] && (i % per) != 1) return fail(DR_ERR_NULL, "%s: parameter %d is NULL", who, i);
    auto P = [&](int group, int j) { return prm[group * per + j]; };
    auto F = [&](int group, int j) { return (const float*)prm[group * per + j]; };
    if (bd.folded) {
        DR_TRY(conv_run(who, xd, x, ca, P(0, 0), F(0, 1), nullptr, 0, ta, sa, 0, st));
        DR_TRY(conv_run(who, ta, sa, cb, P(1, 0), F(1, 1), nullptr, 0, tb, sb, 0, st));
        const void* shortcut = x;
        if (bd.project) {
            DR_TRY(conv_run(who, xd, x, cp, P(3, 0), F(3, 1), nullptr, 0, tc, sp, 0, st));
            shortcut = sp;
        }
        return conv_run(who, tb, sb, cc, P(2, 0), F(2, 1), shortcut, tc.c, yd, y, 0, st);
    }
    auto conv_bn = [&](const dr_tensor& in, const void* src, const dr_conv& c, int grp, const dr_tensor& o, void* dst, bool relu) -> int {
        DR_TRY(conv_run(who, in, src, c, P(grp, 0), F(grp, 1), nullptr, 0, o, dst, 0, st));
        DR_TRY(launch_bn(o, dst, dst, F(grp, 2), F(grp, 3), F(grp, 4), F(grp, 5), bd.eps, 0, st));
        if (relu) DR_TRY(launch_relu(o.dtype, dst, dst, tensor_elems(o), st));
        return DR_OK;
    };
    DR_TRY(conv_bn(xd, x, ca, 0, ta, sa, true));
    DR_TRY(conv_bn(ta, sa, cb, 1, tb, sb, true));
    DR_TRY(conv_bn(tb, sb, cc, 2, tc, sc, false));
    const void* shortcut = x;
    if (bd.project) {
        DR_TRY(conv_bn(xd, x, cp, 3, tc, sp, false));
        shortcut = sp;
    }
    return launch_add_relu(tc.dtype, sc, shortcut, y, tensor_elems(tc), st);
}

}  // namespace
}  // namespace dr

struct dr_net {
    std::vector<dr_layer_desc> layers;
    int n_params = 0;
    bool timing = false;
    std::vector<hipEvent_t> events;
    hipStream_t timed_stream = nullptr;
    bool timed_valid = false;
};

namespace dr {
namespace {

// Output descriptor of one layer for input t (validates the layer against its input).
int layer_out(const dr_layer_desc& L, const dr_tensor& t, dr_tensor* o)
{
    const char* who = "dr_net";
    switch (L.kind) {
    case DR_LAYER_CONV:
        DR_TRY(check_conv_desc(who, &L.conv));
        if (L.conv.c != t.c) return fail(DR_ERR_SHAPE, "%s: convolution expects %d channels, gets %d", who, L.conv.c, t.c);
        *o = conv_out(t, L.conv);
        return DR_OK;
    case DR_LAYER_RELU: *o = t; return DR_OK;
    case DR_LAYER_LRN:
        if (L.lrn.local_size < 1) return fail(DR_ERR_SHAPE, "%s: LRN local_size %d", who, L.lrn.local_size);
        *o = t;
        return DR_OK;
    case DR_LAYER_MAXPOOL: DR_TRY(check_pool_desc(who, &L.pool)); *o = pool_out(t, L.pool); return DR_OK;
    case DR_LAYER_LRN_MAXPOOL:
    case DR_LAYER_MAXPOOL_LRN:
        if (L.lrn.local_size < 1) return fail(DR_ERR_SHAPE, "%s: LRN local_size %d", who, L.lrn.local_size);
        DR_TRY(check_pool_desc(who, &L.pool));
        *o = pool_out(t, L.pool);
        return DR_OK;
    case DR_LAYER_CONV_LRN_MAXPOOL:
        DR_TRY(check_conv_desc(who, &L.conv));
        if (L.conv.c != t.c) return fail(DR_ERR_SHAPE, "%s: convolution expects %d channels, gets %d", who, L.conv.c, t.c);
        if (L.lrn.local_size < 1) return fail(DR_ERR_SHAPE, "%s: LRN local_size %d", who, L.lrn.local_size);
        DR_TRY(check_pool_desc(who, &L.pool));
        *o = pool_out(conv_out(t, L.conv), L.pool);
        return DR_OK;
    case DR_LAYER_AVGPOOL:
        DR_TRY(check_pool_desc(who, &L.pool));
        if (L.pool.pad_h || L.pool.pad_w) return fail(DR_ERR_UNSUPPORTED, "%s: padded average pooling", who);
        *o = avgpool_out(t, L.pool);
        return DR_OK;
    case DR_LAYER_INCEPTION: return inception_validate(t, L.inception, o);
    case DR_LAYER_BOTTLENECK:
        if (L.bottleneck.mid < 1 || L.bottleneck.out < 1) return fail(DR_ERR_SHAPE, "%s: bad bottleneck widths", who);
        if (!L.bottleneck.project && t.c != L.bottleneck.out) return fail(DR_ERR_SHAPE, "%s: identity shortcut needs %d channels, gets %d", who, L.bottleneck.out, t.c);
        *o = dr_tensor{t.n, L.bottleneck.out, t.h, t.w, t.dtype, t.layout};
        return DR_OK;
    case DR_LAYER_FC:
        if (L.fc_out < 1) return fail(DR_ERR_SHAPE, "%s: fc_out %d", who, L.fc_out);
        // the inner product pairs w[o][i] with x[n][i], i running over (c, h, w): memory order only for NCHW or a 1x1 map
        if (t.layout == DR_NHWC && t.h * t.w > 1) return fail(DR_ERR_UNSUPPORTED, "%s: inner product on a channels-last %dx%d map", who, t.h, t.w);
        *o = dr_tensor{t.n, L.fc_out, 1, 1, t.dtype, t.layout};
        return DR_OK;
    case DR_LAYER_SOFTMAX:
        if (t.h != 1 || t.w != 1) return fail(DR_ERR_SHAPE, "%s: softmax needs an {n, c, 1, 1} input", who);
        *o = dr_tensor{t.n, t.c, 1, 1, DR_F32, t.layout};
        return DR_OK;
    default: return fail(DR_ERR_UNSUPPORTED, "%s: unknown layer kind %d", who, L.kind);
    }
}

struct NetPlan {
    std::vector<dr_tensor> outs;   // output descriptor of every layer
    size_t act_bytes = 0;          // largest intermediate activation
    size_t scratch_bytes = 0;      // largest per-layer scratch (inception / bottleneck internals)
};

int net_plan(const dr_net& net, const dr_tensor& xd, NetPlan* plan)
{
    dr_tensor t = xd;
    plan->outs.clear();
    for (size_t i = 0; i < net.layers.size(); ++i) {
        const dr_layer_desc& L = net.layers[i];
        dr_tensor o;
        DR_TRY(layer_out(L, t, &o));
        if (L.kind == DR_LAYER_SOFTMAX && i + 1 != net.layers.size())
            return fail(DR_ERR_UNSUPPORTED, "dr_net: softmax must be the last layer");
        Arena ar(nullptr, 0, true);
        if (L.kind == DR_LAYER_CONV && conv_wants_padding(t, L.conv)) {
            DR_TRY(padded_conv_run("dr_net", t, nullptr, L.conv, nullptr, nullptr, o, nullptr, ar, nullptr));
        } else if (L.kind == DR_LAYER_CONV) {
            ar.take(conv_scratch_bytes(t, L.conv));
        } else if (L.kind == DR_LAYER_INCEPTION) {
            ParamCursor w{nullptr, 0}, b{nullptr, 0};
            DR_TRY(inception_run(t, nullptr, L.inception, w, b, o, nullptr, ar, nullptr));
        } else if (L.kind == DR_LAYER_BOTTLENECK) {
            DR_TRY(bottleneck_run(t, nullptr, L.bottleneck, nullptr, o, nullptr, ar, nullptr));
        }
        if (ar.peak > plan->scratch_bytes) plan->scratch_bytes = ar.peak;
        if (i + 1 != net.layers.size()) {
            const size_t b = align_up(tensor_bytes(o), 256);
            if (b > plan->act_bytes) plan->act_bytes = b;
        }
        plan->outs.push_back(o);
        t = o;
    }
    return DR_OK;
}

}  // namespace
}  // namespace dr

// ---- scratch of dr_conv2d_fwd_static: the library's own, for callers that cannot allocate ---------------------
// One array per GPU the library runs on, held until the process ends.  In host code `scratch` is only the
// symbol's stand-in, not a device address: each device's copy is looked up once, with that device current, and
// the looked-up pointer is what host code uses from then on (kernel arguments).
static __device__ __align__(256) unsigned char scratch[DR_STATIC_SCRATCH_BYTES];

namespace dr {
namespace {
void* static_scratch(const char* who, int* status)
{
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void* ptr[MAX_DEV];                       // device address of `scratch` on each device, NULL until asked
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) {
        *status = fail(DR_ERR_HIP, "%s: no current device (or more than %d devices)", who, MAX_DEV);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            *status = fail(DR_ERR_HIP, "%s: hipGetSymbolAddress(scratch) on device %d: %s", who, dev, hipGetErrorString(e));
            return nullptr;
        }
        ptr[dev] = p;
    }
    *status = DR_OK;
    return ptr[dev];
}
}  // namespace
}  // namespace dr

using namespace dr;

// =====================================================================================================
// C ABI
// =====================================================================================================
extern "C" {

const char* dr_last_error(void) { return g_err; }

int dr_trace_begin(const char* label_filter, int conv_k, int conv_c, int conv_r, int capacity)
{
    const char* who = "dr_trace_begin";
    if (g_trace.active) return fail(DR_ERR_UNSUPPORTED, "%s: a trace is already running", who);
    if (capacity < 1 || capacity > (1 << 20)) return fail(DR_ERR_SHAPE, "%s: capacity %d", who, capacity);
    snprintf(g_trace.filter, sizeof g_trace.filter, "%s", label_filter ? label_filter : "");
    g_trace.k = conv_k; g_trace.c = conv_c; g_trace.r = conv_r;
    g_trace.recs.clear();
    g_trace.recs.reserve(capacity);
    g_trace.ev.resize(2 * (size_t)capacity);
    for (size_t i = 0; i < g_trace.ev.size(); ++i)
        if (hipEventCreate(&g_trace.ev[i]) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(g_trace.ev[j]);
            g_trace.ev.clear();
            return fail(DR_ERR_HIP, "%s: hipEventCreate failed", who);
        }
    g_trace.capacity = capacity;
    g_trace.active = true;
    return DR_OK;
}

int dr_trace_end(dr_trace_record* out, int out_capacity, int* count)
{
    const char* who = "dr_trace_end";
    if (!g_trace.active) return fail(DR_ERR_UNSUPPORTED, "%s: no trace is running", who);
    g_trace.active = false;
    int rc = DR_OK;
    const int n = (int)g_trace.recs.size();
    for (int i = 0; i < n && rc == DR_OK; ++i) {
        if (hipEventSynchronize(g_trace.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&g_trace.recs[i].ms, g_trace.ev[2 * i], g_trace.ev[2 * i + 1]) != hipSuccess)
            rc = fail(DR_ERR_HIP, "%s: reading event %d failed", who, i);
    }
    for (hipEvent_t e : g_trace.ev) (void)hipEventDestroy(e);
    g_trace.ev.clear();
    if (rc == DR_OK) {
        if (!out || !count) rc = fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
        else {
            *count = n < out_capacity ? n : out_capacity;
            for (int i = 0; i < *count; ++i) out[i] = g_trace.recs[i];
        }
    }
    g_trace.recs.clear();
    return rc;
}
const char* dr_version(void) { return "deeprebirth-gfx950 0.1"; }

int dr_conv_out_size(int in, int filt, int stride, int pad)
{
    if (stride < 1 || filt < 1 || pad < 0 || in + 2 * pad < filt) return 0;
    return (in + 2 * pad - filt) / stride + 1;
}

int dr_pool_out_size(int in, int win, int stride, int pad)
{
    if (stride < 1 || win < 1 || pad < 0 || in + 2 * pad < win) return 0;
    int out = (in + 2 * pad - win + stride - 1) / stride + 1;
    if (pad > 0 && (out - 1) * stride >= in + pad) --out;
    return out;
}

int dr_conv2d_fwd(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                  const dr_tensor* yd, void* y, int y_c_offset, void* stream)
{
    const char* who = "dr_conv2d_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_conv_desc(who, cd));
    return conv_run(who, *xd, x, *cd, w, bias, nullptr, 0, *yd, y, y_c_offset, (hipStream_t)stream);
}

int dr_conv2d_workspace_bytes(const dr_tensor* xd, const dr_conv* cd, size_t* bytes)
{
    const char* who = "dr_conv2d_workspace_bytes";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_conv_desc(who, cd));
    if (!bytes) return fail(DR_ERR_NULL, "%s: bytes is NULL", who);
    if (xd->c != cd->c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd->c, cd->c);
    *bytes = conv_scratch_bytes(*xd, *cd);
    return DR_OK;
}

int dr_conv2d_fwd_ws(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                     const dr_tensor* yd, void* y, int y_c_offset, void* ws, size_t ws_bytes, void* stream)
{
    const char* who = "dr_conv2d_fwd_ws";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_conv_desc(who, cd));
    if (xd->c != cd->c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd->c, cd->c);
    const size_t need = conv_scratch_bytes(*xd, *cd);
    if (need && (!ws || ws_bytes < need)) return fail(DR_ERR_WORKSPACE, "%s: needs %zu bytes of workspace, got %zu", who, need, ws ? ws_bytes : (size_t)0);
    if (need && ((uintptr_t)ws & 255) != 0) return fail(DR_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned", who);
    return conv_run(who, *xd, x, *cd, w, bias, nullptr, 0, *yd, y, y_c_offset, (hipStream_t)stream, 0, need ? ws : nullptr, need);
}

int dr_conv2d_fwd_static(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                         const dr_tensor* yd, void* y, int y_c_offset, void* stream)
{
    const char* who = "dr_conv2d_fwd_static";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_conv_desc(who, cd));
    if (xd->c != cd->c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd->c, cd->c);
    const size_t need = conv_scratch_bytes(*xd, *cd);
    if (need > (size_t)DR_STATIC_SCRATCH_BYTES)
        return fail(DR_ERR_WORKSPACE, "%s: the layer's partial sums take %zu bytes, the library's scratch holds %zu (use dr_conv2d_fwd_ws)", who,
                    need, (size_t)DR_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (need) {
        int status = DR_OK;
        ws = static_scratch(who, &status);
        if (!ws) return status;
    }
    // every partial sum the second kernel reads is written by the first in the same call: nothing has to be cleared
    return conv_run(who, *xd, x, *cd, w, bias, nullptr, 0, *yd, y, y_c_offset, (hipStream_t)stream, 0, ws, need);
}

int dr_pack_filters(const dr_conv* cd, int dtype, const void* w_kcrs, void* w_krsc, void* stream)
{
    const char* who = "dr_pack_filters";
    if (!cd) return fail(DR_ERR_NULL, "%s: descriptor is NULL", who);
    if (cd->k < 1 || cd->c < 1 || cd->r < 1 || cd->s < 1) return fail(DR_ERR_SHAPE, "%s: bad filter shape", who);
    if (dtype != DR_F32 && dtype != DR_BF16) return fail(DR_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, dtype);
    if (cd->c % (dtype == DR_F32 ? 16 : 8) != 0)
        return fail(DR_ERR_UNSUPPORTED, "%s: channel count %d is not a multiple of %d", who, cd->c, dtype == DR_F32 ? 16 : 8);
    if (!w_kcrs || !w_krsc) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    if ((double)cd->k * cd->c * cd->r * cd->s >= 2147483648.0) return fail(DR_ERR_UNSUPPORTED, "%s: tensor too large", who);
    return launch_pack_filters(dtype, w_kcrs, w_krsc, cd->k, cd->c, cd->r * cd->s, (hipStream_t)stream);
}

int dr_slim_conv_fwd(const dr_tensor* xd, const void* x, const dr_conv* cd, int pool_stride_h, int pool_stride_w,
                     const void* w, const float* bias, const dr_tensor* yd, void* y, int y_c_offset, void* stream)
{
    const char* who = "dr_slim_conv_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_conv_desc(who, cd));
    if (pool_stride_h < 1 || pool_stride_w < 1) return fail(DR_ERR_SHAPE, "%s: pooling stride %d,%d", who, pool_stride_h, pool_stride_w);
    dr_conv slim = *cd;
    slim.stride_h = cd->stride_h * pool_stride_h;   // stride of the slim layer = product of both strides
    slim.stride_w = cd->stride_w * pool_stride_w;
    slim.relu = 1;                                  // the ReLU is retained
    return conv_run(who, *xd, x, slim, w, bias, nullptr, 0, *yd, y, y_c_offset, (hipStream_t)stream);
}

int dr_relu(const dr_tensor* d, const void* x, void* y, void* stream)
{
    DR_TRY(check_tensor("dr_relu", "d", d));
    if (tensor_elems(*d) == 0) return DR_OK;
    if (!x || !y) return fail(DR_ERR_NULL, "dr_relu: x or y is NULL");
    return launch_relu(d->dtype, x, y, tensor_elems(*d), (hipStream_t)stream);
}

int dr_lrn_fwd(const dr_tensor* d, const void* x, const dr_lrn* p, void* y, void* stream)
{
    const char* who = "dr_lrn_fwd";
    DR_TRY(check_tensor(who, "d", d));
    if (!p) return fail(DR_ERR_NULL, "%s: parameters are NULL", who);
    if (p->local_size < 1) return fail(DR_ERR_SHAPE, "%s: local_size %d", who, p->local_size);
    if (tensor_elems(*d) == 0) return DR_OK;
    if (!x || !y) return fail(DR_ERR_NULL, "%s: x or y is NULL", who);
    if (x == y) return fail(DR_ERR_UNSUPPORTED, "%s: in-place operation is not supported", who);
    return launch_lrn(*d, x, y, *p, (hipStream_t)stream);
}

int dr_maxpool_fwd(const dr_tensor* xd, const void* x, const dr_pool* p, const dr_tensor* yd, void* y, void* stream)
{
    const char* who = "dr_maxpool_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_pool_desc(who, p));
    const dr_tensor o = pool_out(*xd, *p);
    if (!same_shape(o, *yd)) return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%dx%d, the layer produces %dx%dx%dx%d", who, yd->n, yd->c, yd->h, yd->w, o.n, o.c, o.h, o.w);
    if (yd->dtype != xd->dtype) return fail(DR_ERR_UNSUPPORTED, "%s: input and output dtypes differ", who);
    if (tensor_elems(o) == 0) return DR_OK;
    if (!x || !y) return fail(DR_ERR_NULL, "%s: x or y is NULL", who);
    return launch_maxpool(*xd, x, o, y, *p, (hipStream_t)stream);
}

static int lrn_pool_entry(const char* who, const dr_tensor* xd, const void* x, const dr_lrn* l, const dr_pool* p, const dr_tensor* yd, void* y,
                          bool lrn_first, void* stream)
{
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    if (!l) return fail(DR_ERR_NULL, "%s: the LRN descriptor is NULL", who);
    if (l->local_size < 1) return fail(DR_ERR_SHAPE, "%s: LRN local_size %d", who, l->local_size);
    DR_TRY(check_pool_desc(who, p));
    const dr_tensor o = pool_out(*xd, *p);
    if (!same_shape(o, *yd)) return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%dx%d, the layer produces %dx%dx%dx%d", who, yd->n, yd->c, yd->h, yd->w, o.n, o.c, o.h, o.w);
    if (yd->dtype != xd->dtype || yd->layout != xd->layout) return fail(DR_ERR_UNSUPPORTED, "%s: input and output differ in dtype or layout", who);
    if (tensor_elems(o) == 0) return DR_OK;
    if (!x || !y) return fail(DR_ERR_NULL, "%s: x or y is NULL", who);
    if (!pool_lrn_nhwc_supported(*xd, x, y, *p, *l))
        return fail(DR_ERR_UNSUPPORTED, "%s: needs channels-last tensors with 16-byte aligned channel groups (at most 64 of them), a 3x3 "
                    "window of stride 1 or 2 with padding 0 or 1, and an LRN window of 5", who);
    return launch_pool_lrn_nhwc(*xd, x, o, y, *p, *l, lrn_first, (hipStream_t)stream);
}

int dr_lrn_maxpool_fwd(const dr_tensor* xd, const void* x, const dr_lrn* l, const dr_pool* p, const dr_tensor* yd, void* y, void* stream)
{
    return lrn_pool_entry("dr_lrn_maxpool_fwd", xd, x, l, p, yd, y, true, stream);
}

int dr_conv_lrn_maxpool_fwd(const dr_tensor* xd, const void* x, const dr_conv* cd, const void* w, const float* bias,
                            const dr_lrn* l, const dr_pool* p, const dr_tensor* yd, void* y, int y_c_offset, void* stream)
{
    const char* who = "dr_conv_lrn_maxpool_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_conv_desc(who, cd));
    if (!l || !p) return fail(DR_ERR_NULL, "%s: l or p is NULL", who);
    if (l->local_size < 1) return fail(DR_ERR_SHAPE, "%s: LRN local_size %d", who, l->local_size);
    DR_TRY(check_pool_desc(who, p));
    return conv_block_run(who, *xd, x, *cd, w, bias, *l, *p, *yd, y, y_c_offset, (hipStream_t)stream);
}

int dr_maxpool_lrn_fwd(const dr_tensor* xd, const void* x, const dr_pool* p, const dr_lrn* l, const dr_tensor* yd, void* y, void* stream)
{
    return lrn_pool_entry("dr_maxpool_lrn_fwd", xd, x, l, p, yd, y, false, stream);
}

int dr_avgpool_fwd(const dr_tensor* xd, const void* x, const dr_pool* p, const dr_tensor* yd, void* y, void* stream)
{
    const char* who = "dr_avgpool_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    DR_TRY(check_pool_desc(who, p));
    if (p->pad_h || p->pad_w) return fail(DR_ERR_UNSUPPORTED, "%s: padding is not supported", who);
    const dr_tensor o = avgpool_out(*xd, *p);
    if (!same_shape(o, *yd)) return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%dx%d, the layer produces %dx%dx%dx%d", who, yd->n, yd->c, yd->h, yd->w, o.n, o.c, o.h, o.w);
    if (yd->dtype != xd->dtype) return fail(DR_ERR_UNSUPPORTED, "%s: input and output dtypes differ", who);
    if (tensor_elems(o) == 0) return DR_OK;
    if (!x || !y) return fail(DR_ERR_NULL, "%s: x or y is NULL", who);
    return launch_avgpool(*xd, x, o, y, *p, (hipStream_t)stream);
}

int dr_concat(int nb, const dr_tensor* xds, const void* const* xs, const dr_tensor* yd, void* y, void* stream)
{
    const char* who = "dr_concat";
    if (nb < 1 || nb > DR_MAX_BRANCHES) return fail(DR_ERR_SHAPE, "%s: %d inputs (1..%d supported)", who, nb, DR_MAX_BRANCHES);
    if (!xds || !xs) return fail(DR_ERR_NULL, "%s: input arrays are NULL", who);
    DR_TRY(check_tensor(who, "yd", yd));
    if (!y) return fail(DR_ERR_NULL, "%s: y is NULL", who);
    ConcatSeg segs[DR_MAX_BRANCHES];
    int c = 0;
    for (int i = 0; i < nb; ++i) {
        DR_TRY(check_tensor(who, "xds[i]", &xds[i]));
        if (!xs[i]) return fail(DR_ERR_NULL, "%s: xs[%d] is NULL", who, i);
        if (xds[i].n != yd->n || xds[i].h != yd->h || xds[i].w != yd->w || xds[i].dtype != yd->dtype || xds[i].layout != yd->layout)
            return fail(DR_ERR_SHAPE, "%s: input %d does not match the output's n, h, w, dtype or layout", who, i);
        segs[i] = ConcatSeg{xs[i], xds[i].c, c};
        c += xds[i].c;
    }
    if (c != yd->c) return fail(DR_ERR_SHAPE, "%s: inputs have %d channels in total, output has %d", who, c, yd->c);
    return launch_concat(*yd, nb, segs, y, (hipStream_t)stream);
}

int dr_bn_fwd(const dr_tensor* d, const void* x, const float* gamma, const float* beta, const float* mean,
              const float* var, float eps, int relu, void* y, void* stream)
{
    const char* who = "dr_bn_fwd";
    DR_TRY(check_tensor(who, "d", d));
    if (tensor_elems(*d) == 0) return DR_OK;
    if (!x || !y || !gamma || !beta || !mean || !var) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    if (!(eps >= 0.f)) return fail(DR_ERR_SHAPE, "%s: eps must be >= 0", who);
    return launch_bn(*d, x, y, gamma, beta, mean, var, eps, relu, (hipStream_t)stream);
}

int dr_add_relu(const dr_tensor* d, const void* a, const void* b, void* y, void* stream)
{
    DR_TRY(check_tensor("dr_add_relu", "d", d));
    if (tensor_elems(*d) == 0) return DR_OK;
    if (!a || !b || !y) return fail(DR_ERR_NULL, "dr_add_relu: a pointer is NULL");
    return launch_add_relu(d->dtype, a, b, y, tensor_elems(*d), (hipStream_t)stream);
}

int dr_fold_bn(int k, size_t crs, const float* w, const float* b, const float* gamma, const float* beta,
               const float* mean, const float* var, float eps, float* w_out, float* b_out)
{
    const char* who = "dr_fold_bn";
    if (k < 0) return fail(DR_ERR_SHAPE, "%s: k = %d", who, k);
    if (!w || !gamma || !beta || !mean || !var || !w_out || !b_out) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    if (!(eps >= 0.f)) return fail(DR_ERR_SHAPE, "%s: eps must be >= 0", who);
    for (int j = 0; j < k; ++j) {
        // evaluated in double so that the folded fp32 parameters are the correctly rounded ones
        const double eta = (double)gamma[j] / sqrt((double)var[j] + (double)eps);
        for (size_t i = 0; i < crs; ++i) w_out[(size_t)j * crs + i] = (float)(eta * (double)w[(size_t)j * crs + i]);
        b_out[j] = (float)(eta * (b ? (double)b[j] : 0.0) + (double)beta[j] - eta * (double)mean[j]);
    }
    return DR_OK;
}

int dr_fc_fwd(const dr_tensor* xd, const void* x, const void* w, const float* bias, const dr_tensor* yd, void* y,
              void* stream)
{
    const char* who = "dr_fc_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    if (!x || !w || !y) return fail(DR_ERR_NULL, "%s: x, w or y is NULL", who);
    if (yd->n != xd->n || yd->h != 1 || yd->w != 1) return fail(DR_ERR_SHAPE, "%s: output must be {n, out, 1, 1}", who);
    if (yd->dtype != xd->dtype) return fail(DR_ERR_UNSUPPORTED, "%s: input and output dtypes differ", who);
    // i runs over (c, h, w): that is the tensor's memory order only for NCHW, or for any layout when the map is 1x1
    if (xd->layout == DR_NHWC && xd->h * xd->w > 1) return fail(DR_ERR_UNSUPPORTED, "%s: channels-last input with a %dx%d map", who, xd->h, xd->w);
    return launch_fc(xd->dtype, x, w, bias, y, xd->n, xd->c * xd->h * xd->w, yd->c, (hipStream_t)stream);
}

int dr_softmax_fwd(const dr_tensor* xd, const void* x, float* y, void* stream)
{
    const char* who = "dr_softmax_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    if (!x || !y) return fail(DR_ERR_NULL, "%s: x or y is NULL", who);
    if (xd->h != 1 || xd->w != 1) return fail(DR_ERR_SHAPE, "%s: input must be {n, c, 1, 1}", who);
    return launch_softmax(xd->dtype, x, y, xd->n, xd->c, (hipStream_t)stream);
}

size_t dr_regression_loss_workspace_bytes(void) { return regression_loss_workspace_bytes(); }

int dr_regression_loss_grad(const dr_tensor* d, const void* f, const void* target, void* dz, float* loss, void* ws, size_t ws_bytes,
                            void* stream)
{
    const char* who = "dr_regression_loss_grad";
    DR_TRY(check_tensor(who, "d", d));
    if (d->dtype != DR_F32) return fail(DR_ERR_UNSUPPORTED, "%s: fp32 tensors only", who);
    if (!loss) return fail(DR_ERR_NULL, "%s: loss is NULL", who);
    if (!ws || ws_bytes < regression_loss_workspace_bytes()) return fail(DR_ERR_WORKSPACE, "%s: needs %zu bytes of workspace", who, regression_loss_workspace_bytes());
    const size_t count = tensor_elems(*d);
    if (count && (!f || !target || !dz)) return fail(DR_ERR_NULL, "%s: f, target or dz is NULL", who);
    return launch_regression_loss_grad((const float*)f, (const float*)target, (float*)dz, count, loss, ws, (hipStream_t)stream);
}

static int bwd_params_geom(const char* who, const dr_tensor* xd, const dr_conv* cd, ConvGeom* g, dr_tensor* o)
{
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_conv_desc(who, cd));
    if (xd->dtype != DR_F32 || xd->layout != DR_NCHW || cd->filter_layout != DR_KCRS)
        return fail(DR_ERR_UNSUPPORTED, "%s: fp32 NCHW tensors and KCRS filters only", who);
    if (xd->c != cd->c) return fail(DR_ERR_SHAPE, "%s: input has %d channels, filters expect %d", who, xd->c, cd->c);
    *o = conv_out(*xd, *cd);
    if ((double)xd->n * xd->c * xd->h * xd->w * 4 >= 2147483648.0 || (double)o->n * o->c * o->h * o->w * 4 >= 2147483648.0)
        return fail(DR_ERR_UNSUPPORTED, "%s: tensors of 2 GiB or more", who);
    g->N = xd->n; g->C = xd->c; g->H = xd->h; g->W = xd->w;
    g->K = cd->k; g->R = cd->r; g->S = cd->s;
    g->sh = cd->stride_h; g->sw = cd->stride_w; g->ph = cd->pad_h; g->pw = cd->pad_w;
    g->P = o->h; g->Q = o->w;
    g->Kg = cd->c * cd->r * cd->s;
    g->Ng = o->n * o->h * o->w;
    g->y_ctot = cd->k; g->y_coff = 0; g->relu = 0; g->res_ctot = 0; g->w_krsc = 0; g->nhwc = 0; g->c_logical = 0;
    return DR_OK;
}

int dr_conv2d_bwd_params_workspace_bytes(const dr_tensor* xd, const dr_conv* cd, size_t* bytes)
{
    const char* who = "dr_conv2d_bwd_params_workspace_bytes";
    if (!bytes) return fail(DR_ERR_NULL, "%s: bytes is NULL", who);
    ConvGeom g;
    dr_tensor o;
    DR_TRY(bwd_params_geom(who, xd, cd, &g, &o));
    *bytes = conv_wgrad_workspace_bytes(g);
    return DR_OK;
}

int dr_conv2d_bwd_params(const dr_tensor* xd, const void* x, const dr_conv* cd, const dr_tensor* dzd, const void* dz, void* dw,
                         float* db, void* ws, size_t ws_bytes, void* stream)
{
    const char* who = "dr_conv2d_bwd_params";
    ConvGeom g;
    dr_tensor o;
    DR_TRY(bwd_params_geom(who, xd, cd, &g, &o));
    DR_TRY(check_tensor(who, "dzd", dzd));
    if (!same_shape(o, *dzd) || dzd->dtype != DR_F32 || dzd->layout != DR_NCHW)
        return fail(DR_ERR_SHAPE, "%s: dz must be the layer's fp32 NCHW output, %dx%dx%dx%d", who, o.n, o.c, o.h, o.w);
    const size_t need = conv_wgrad_workspace_bytes(g);
    if (need > 0 && (!ws || ws_bytes < need)) return fail(DR_ERR_WORKSPACE, "%s: needs %zu bytes of workspace", who, need);
    if ((size_t)g.K * g.Kg == 0) return DR_OK;
    if (!dw) return fail(DR_ERR_NULL, "%s: dw is NULL", who);
    if (g.Ng > 0 && (!x || !dz)) return fail(DR_ERR_NULL, "%s: x or dz is NULL", who);     // (no terms: the kernels write zeros)
    return launch_conv_wgrad_f32(g, (const float*)x, (const float*)dz, (float*)dw, db, ws, (hipStream_t)stream);
}

int dr_sgd_step(size_t count, float* w, const float* dw, float lr, void* stream)
{
    if (count && (!w || !dw)) return fail(DR_ERR_NULL, "dr_sgd_step: w or dw is NULL");
    return launch_sgd_step(w, dw, lr, count, (hipStream_t)stream);
}

int dr_inception_workspace_bytes(const dr_tensor* xd, const dr_inception* desc, size_t* bytes)
{
    const char* who = "dr_inception_workspace_bytes";
    DR_TRY(check_tensor(who, "xd", xd));
    if (!desc || !bytes) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    dr_tensor yd;
    DR_TRY(inception_validate(*xd, *desc, &yd));
    Arena ar(nullptr, 0, true);
    ParamCursor w{nullptr, 0}, b{nullptr, 0};
    DR_TRY(inception_run(*xd, nullptr, *desc, w, b, yd, nullptr, ar, nullptr));
    *bytes = ar.peak;
    return DR_OK;
}

int dr_inception_fwd(const dr_tensor* xd, const void* x, const dr_inception* desc, const void* const* weights,
                     const float* const* biases, const dr_tensor* yd, void* y, void* ws, size_t ws_bytes, void* stream)
{
    const char* who = "dr_inception_fwd";
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    if (!desc || !x || !y || !weights || !biases) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    dr_tensor o;
    DR_TRY(inception_validate(*xd, *desc, &o));
    if (!same_shape(o, *yd) || yd->dtype != xd->dtype)
        return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%dx%d, the module produces %dx%dx%dx%d", who, yd->n, yd->c, yd->h, yd->w, o.n, o.c, o.h, o.w);
    size_t need = 0;
    DR_TRY(dr_inception_workspace_bytes(xd, desc, &need));
    if (need > 0 && (!ws || ws_bytes < need)) return fail(DR_ERR_WORKSPACE, "%s: needs %zu bytes of workspace, got %zu", who, need, ws ? ws_bytes : (size_t)0);
    if (((uintptr_t)ws & 255) != 0) return fail(DR_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned", who);
    Arena ar(ws, ws_bytes, false);
    ParamCursor w{weights, 0}, b{(const void* const*)biases, 0};
    return inception_run(*xd, x, *desc, w, b, *yd, y, ar, (hipStream_t)stream);
}

}  // extern "C"

extern "C" {

int dr_net_create(const dr_layer_desc* layers, int n_layers, dr_net** out)
{
    const char* who = "dr_net_create";
    if (!layers || !out) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    if (n_layers < 1) return fail(DR_ERR_SHAPE, "%s: %d layers", who, n_layers);
    dr_net* net = new (std::nothrow) dr_net;
    if (!net) return fail(DR_ERR_HIP, "%s: out of host memory", who);
    net->layers.assign(layers, layers + n_layers);
    for (const dr_layer_desc& L : net->layers) {
        if (L.kind < DR_LAYER_CONV || L.kind > DR_LAYER_CONV_LRN_MAXPOOL) {
            delete net;
            return fail(DR_ERR_UNSUPPORTED, "%s: unknown layer kind %d", who, L.kind);
        }
        net->n_params += param_count(L);
    }
    *out = net;
    return DR_OK;
}

void dr_net_destroy(dr_net* net)
{
    if (!net) return;
    for (hipEvent_t e : net->events) (void)hipEventDestroy(e);
    delete net;
}

int dr_net_num_params(const dr_net* net, int* count)
{
    if (!net || !count) return fail(DR_ERR_NULL, "dr_net_num_params: a pointer is NULL");
    *count = net->n_params;
    return DR_OK;
}

int dr_net_output_desc(const dr_net* net, const dr_tensor* xd, dr_tensor* yd)
{
    if (!net || !yd) return fail(DR_ERR_NULL, "dr_net_output_desc: a pointer is NULL");
    DR_TRY(check_tensor("dr_net_output_desc", "xd", xd));
    NetPlan plan;
    DR_TRY(net_plan(*net, *xd, &plan));
    *yd = plan.outs.back();
    return DR_OK;
}

int dr_net_workspace_bytes(const dr_net* net, const dr_tensor* xd, size_t* bytes)
{
    if (!net || !bytes) return fail(DR_ERR_NULL, "dr_net_workspace_bytes: a pointer is NULL");
    DR_TRY(check_tensor("dr_net_workspace_bytes", "xd", xd));
    NetPlan plan;
    DR_TRY(net_plan(*net, *xd, &plan));
    *bytes = 2 * plan.act_bytes + plan.scratch_bytes;
    return DR_OK;
}

int dr_net_set_timing(dr_net* net, int enabled)
{
    if (!net) return fail(DR_ERR_NULL, "dr_net_set_timing: net is NULL");
    net->timing = enabled != 0;
    net->timed_valid = false;
    if (net->timing && net->events.empty()) {
        net->events.resize(net->layers.size() + 1);
        for (hipEvent_t& e : net->events)
            if (hipEventCreate(&e) != hipSuccess) {
                net->events.clear();
                net->timing = false;
                return fail(DR_ERR_HIP, "dr_net_set_timing: hipEventCreate failed");
            }
    }
    return DR_OK;
}

int dr_net_layer_times(dr_net* net, float* ms_per_layer, int n)
{
    const char* who = "dr_net_layer_times";
    if (!net || !ms_per_layer) return fail(DR_ERR_NULL, "%s: a pointer is NULL", who);
    if (n != (int)net->layers.size()) return fail(DR_ERR_SHAPE, "%s: the network has %zu layers", who, net->layers.size());
    if (!net->timing || !net->timed_valid) return fail(DR_ERR_UNSUPPORTED, "%s: no timed run recorded", who);
    if (hipEventSynchronize(net->events.back()) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipEventSynchronize failed", who);
    for (int i = 0; i < n; ++i)
        if (hipEventElapsedTime(&ms_per_layer[i], net->events[i], net->events[i + 1]) != hipSuccess)
            return fail(DR_ERR_HIP, "%s: hipEventElapsedTime failed", who);
    return DR_OK;
}

int dr_net_fwd(dr_net* net, const dr_tensor* xd, const void* x, const void* const* params, const dr_tensor* yd, void* y,
               void* ws, size_t ws_bytes, void* stream)
{
    const char* who = "dr_net_fwd";
    if (!net) return fail(DR_ERR_NULL, "%s: net is NULL", who);
    DR_TRY(check_tensor(who, "xd", xd));
    DR_TRY(check_tensor(who, "yd", yd));
    if (!x || !y || (net->n_params && !params)) return fail(DR_ERR_NULL, "%s: x, y or params is NULL", who);
    NetPlan plan;
    DR_TRY(net_plan(*net, *xd, &plan));
    const dr_tensor& o = plan.outs.back();
    if (!same_shape(o, *yd) || o.dtype != yd->dtype)
        return fail(DR_ERR_SHAPE, "%s: output is %dx%dx%dx%d dtype %d, the network produces %dx%dx%dx%d dtype %d", who, yd->n, yd->c,
                    yd->h, yd->w, yd->dtype, o.n, o.c, o.h, o.w, o.dtype);
    const size_t need = 2 * plan.act_bytes + plan.scratch_bytes;
    if (need > 0 && (!ws || ws_bytes < need)) return fail(DR_ERR_WORKSPACE, "%s: needs %zu bytes of workspace, got %zu", who, need, ws ? ws_bytes : (size_t)0);
    if (((uintptr_t)ws & 255) != 0) return fail(DR_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned", who);
    for (int i = 0; i < net->n_params; ++i)
        if (!params[i]) return fail(DR_ERR_NULL, "%s: params[%d] is NULL", who, i);

    hipStream_t st = (hipStream_t)stream;
    char* buf[2] = {(char*)ws, (char*)ws + plan.act_bytes};
    char* scratch = (char*)ws + 2 * plan.act_bytes;
    const void* cur = x;
    int cur_buf = -1;   // -1: the caller's input (read only)
    dr_tensor t = *xd;
    int pi = 0;
    const size_t nl = net->layers.size();
    net->timed_valid = false;
    if (net->timing && hipEventRecord(net->events[0], st) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipEventRecord failed", who);
    for (size_t i = 0; i < nl; ++i) {
        const dr_layer_desc& L = net->layers[i];
        const dr_tensor& od = plan.outs[i];
        const bool last = i + 1 == nl;
        // ReLU runs in place unless it would overwrite the caller's input or is the last layer
        const bool inplace = L.kind == DR_LAYER_RELU && cur_buf >= 0 && !last;
        const int dst_buf = inplace ? cur_buf : (cur_buf == 0 ? 1 : 0);
        void* dst = last ? y : (void*)buf[dst_buf];
        Arena ar(scratch, plan.scratch_bytes, false);
        void* skip_to = nullptr;                       // set when this layer and the next one ran as one kernel
        switch (L.kind) {
        case DR_LAYER_CONV:
            if (conv_wants_padding(t, L.conv) && i + 1 < nl && net->layers[i + 1].kind == DR_LAYER_CONV && conv_tail_ok(L.conv, net->layers[i + 1].conv)) {
                // this layer and the 1x1 convolution behind it as one kernel, written where the second one's output belongs
                const bool last2 = i + 2 == nl;
                void* dst2 = last2 ? y : (void*)buf[dst_buf];
                bool fused = false;
                DR_TRY(padded_conv_run(who, t, cur, L.conv, params[pi], (const float*)params[pi + 1], plan.outs[i + 1], dst2, ar, st,
                                       &net->layers[i + 1].conv, params[pi + 2], (const float*)params[pi + 3], &fused));
                if (fused) {
                    if (net->timing && hipEventRecord(net->events[i + 1], st) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipEventRecord failed", who);
                    pi += param_count(L);
                    ++i;                               // (the loop's tail accounts for the second layer)
                    skip_to = dst2;
                    break;
                }
            }
            if (conv_wants_padding(t, L.conv))
                DR_TRY(padded_conv_run(who, t, cur, L.conv, params[pi], (const float*)params[pi + 1], od, dst, ar, st));
            else {
                const size_t sbytes = conv_scratch_bytes(t, L.conv);
                void* sc = sbytes ? ar.take(sbytes) : nullptr;
                DR_TRY(conv_run(who, t, cur, L.conv, params[pi], (const float*)params[pi + 1], nullptr, 0, od, dst, 0, st, 0, sc, sc ? sbytes : 0));
            }
            break;
        case DR_LAYER_RELU: DR_TRY(launch_relu(t.dtype, cur, dst, tensor_elems(t), st)); break;
        case DR_LAYER_LRN: DR_TRY(launch_lrn(t, cur, dst, L.lrn, st)); break;
        case DR_LAYER_MAXPOOL: DR_TRY(launch_maxpool(t, cur, od, dst, L.pool, st)); break;
        case DR_LAYER_LRN_MAXPOOL:
        case DR_LAYER_MAXPOOL_LRN:
            if (!pool_lrn_nhwc_supported(t, cur, dst, L.pool, L.lrn))
                return fail(DR_ERR_UNSUPPORTED, "%s: layer %zu: fused LRN / pooling needs channels-last tensors, a 3x3 window of stride 1 or 2, "
                            "an LRN window of 5 and at most 64 16-byte channel groups", who, i);
            DR_TRY(launch_pool_lrn_nhwc(t, cur, od, dst, L.pool, L.lrn, L.kind == DR_LAYER_LRN_MAXPOOL, st));
            break;
        case DR_LAYER_CONV_LRN_MAXPOOL:
            DR_TRY(conv_block_run(who, t, cur, L.conv, params[pi], (const float*)params[pi + 1], L.lrn, L.pool, od, dst, 0, st));
            break;
        case DR_LAYER_AVGPOOL: DR_TRY(launch_avgpool(t, cur, od, dst, L.pool, st)); break;
        case DR_LAYER_INCEPTION: {
            const int np = param_count(L) / 2;
            std::vector<const void*> w(np);
            std::vector<const void*> b(np);
            for (int j = 0; j < np; ++j) { w[j] = params[pi + 2 * j]; b[j] = params[pi + 2 * j + 1]; }
            ParamCursor wc{w.data(), 0}, bc{b.data(), 0};
            DR_TRY(inception_run(t, cur, L.inception, wc, bc, od, dst, ar, st));
            break;
        }
        case DR_LAYER_BOTTLENECK: DR_TRY(bottleneck_run(t, cur, L.bottleneck, params + pi, od, dst, ar, st)); break;
        case DR_LAYER_FC:
            DR_TRY(launch_fc(t.dtype, cur, params[pi], (const float*)params[pi + 1], dst, t.n, t.c * t.h * t.w, od.c, st));
            break;
        case DR_LAYER_SOFTMAX: DR_TRY(launch_softmax(t.dtype, cur, (float*)dst, t.n, t.c, st)); break;
        default: return fail(DR_ERR_UNSUPPORTED, "%s: unknown layer kind %d", who, L.kind);
        }
        if (skip_to) {
            pi += param_count(net->layers[i]);
            cur = skip_to;
            cur_buf = i + 1 == nl ? -1 : dst_buf;
            t = plan.outs[i];
            if (net->timing && hipEventRecord(net->events[i + 1], st) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipEventRecord failed", who);
            continue;
        }
        pi += param_count(L);
        cur = dst;
        cur_buf = last ? -1 : dst_buf;
        t = od;
        if (net->timing && hipEventRecord(net->events[i + 1], st) != hipSuccess) return fail(DR_ERR_HIP, "%s: hipEventRecord failed", who);
    }
    net->timed_valid = net->timing;
    return DR_OK;
}

struct dr_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

int dr_capture_begin(void* stream)
{
    const char* who = "dr_capture_begin";
    if (!stream) return fail(DR_ERR_UNSUPPORTED, "%s: capture needs a stream the caller created, not the default stream", who);
    if (g_trace.active) return fail(DR_ERR_UNSUPPORTED, "%s: a kernel trace is running", who);
    // the streams and events of side-by-side branches are created on first use: not inside a capture
    if (!branch_streams()) return fail(DR_ERR_HIP, "%s: cannot create the branch streams", who);
    if (hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal) != hipSuccess)
        return fail(DR_ERR_HIP, "%s: hipStreamBeginCapture failed", who);
    return DR_OK;
}

int dr_capture_end(void* stream, dr_graph** out)
{
    const char* who = "dr_capture_end";
    if (out) *out = nullptr;
    if (!stream) return fail(DR_ERR_UNSUPPORTED, "%s: no capture on the default stream", who);
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture((hipStream_t)stream, &g);
    if (!out) {                              // the caller gives the recording up
        if (g) (void)hipGraphDestroy(g);
        return e == hipSuccess ? DR_OK : fail(DR_ERR_HIP, "%s: hipStreamEndCapture failed (%s)", who, hipGetErrorString(e));
    }
    if (e != hipSuccess || !g) return fail(DR_ERR_HIP, "%s: hipStreamEndCapture failed (%s)", who, hipGetErrorString(e));
    hipGraphExec_t ex = nullptr;
    if (hipGraphInstantiate(&ex, g, nullptr, nullptr, 0) != hipSuccess || !ex) {
        (void)hipGraphDestroy(g);
        return fail(DR_ERR_HIP, "%s: hipGraphInstantiate failed", who);
    }
    *out = new dr_graph{g, ex};
    return DR_OK;
}

int dr_net_capture(dr_net* net, const dr_tensor* xd, const void* x, const void* const* params, const dr_tensor* yd, void* y,
                   void* ws, size_t ws_bytes, void* stream, dr_graph** out)
{
    const char* who = "dr_net_capture";
    if (!out) return fail(DR_ERR_NULL, "%s: out is NULL", who);
    *out = nullptr;
    if (!net) return fail(DR_ERR_NULL, "%s: net is NULL", who);
    if (net->timing) return fail(DR_ERR_UNSUPPORTED, "%s: per-layer timing is on", who);
    DR_TRY(dr_capture_begin(stream));
    const int rc = dr_net_fwd(net, xd, x, params, yd, y, ws, ws_bytes, stream);
    if (rc != DR_OK) {                       // dr_net_fwd's message stands
        char msg[sizeof g_err];
        snprintf(msg, sizeof msg, "%s", g_err);
        (void)dr_capture_end(stream, nullptr);
        snprintf(g_err, sizeof g_err, "%s", msg);
        return rc;
    }
    return dr_capture_end(stream, out);
}

int dr_graph_launch(dr_graph* graph, void* stream)
{
    if (!graph) return fail(DR_ERR_NULL, "dr_graph_launch: graph is NULL");
    if (hipGraphLaunch(graph->exec, (hipStream_t)stream) != hipSuccess) return fail(DR_ERR_HIP, "dr_graph_launch: hipGraphLaunch failed");
    return DR_OK;
}

void dr_graph_destroy(dr_graph* graph)
{
    if (!graph) return;
    (void)hipGraphExecDestroy(graph->exec);
    (void)hipGraphDestroy(graph->graph);
    delete graph;
}

}  // extern "C"
