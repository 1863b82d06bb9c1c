"""ctypes binding of libdeeprebirth.so: argument marshalling only.

Every function here has the name of the C entry point it calls (without the ``dr_`` prefix) and
does nothing but turn torch tensors into device pointers + descriptors.  PyTorch is used for
device memory and streams only; no layer is ever computed by torch, and there is no CPU fallback:
if the library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdeeprebirth.so")

DR_OK = 0
DR_ERR_NULL, DR_ERR_SHAPE, DR_ERR_UNSUPPORTED, DR_ERR_WORKSPACE, DR_ERR_HIP = 1, 2, 3, 4, 5
DR_F32, DR_BF16 = 0, 1
DR_KCRS, DR_KRSC = 0, 1
DR_NCHW, DR_NHWC = 0, 1
DR_MAX_BRANCHES, DR_MAX_STEPS = 8, 4
DR_STEP_CONV, DR_STEP_MAXPOOL = 0, 1
DR_FUSE_RELU, DR_FUSE_CONCAT, DR_FUSE_STACK, DR_CONCURRENT_BRANCHES = 1, 2, 4, 8
(DR_LAYER_CONV, DR_LAYER_RELU, DR_LAYER_LRN, DR_LAYER_MAXPOOL, DR_LAYER_INCEPTION, DR_LAYER_BOTTLENECK,
 DR_LAYER_AVGPOOL, DR_LAYER_FC, DR_LAYER_SOFTMAX, DR_LAYER_LRN_MAXPOOL, DR_LAYER_MAXPOOL_LRN, DR_LAYER_CONV_LRN_MAXPOOL) = range(12)


class dr_tensor(C.Structure):
    _fields_ = [("n", C.c_int), ("c", C.c_int), ("h", C.c_int), ("w", C.c_int), ("dtype", C.c_int), ("layout", C.c_int)]


class dr_conv(C.Structure):
    _fields_ = [(f, C.c_int) for f in ("k", "c", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w", "relu",
                                       "filter_layout")]


class dr_lrn(C.Structure):
    _fields_ = [("local_size", C.c_int), ("alpha", C.c_float), ("beta", C.c_float), ("k", C.c_float)]


class dr_pool(C.Structure):
    _fields_ = [(f, C.c_int) for f in ("kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w")]


class dr_step(C.Structure):
    _fields_ = [("kind", C.c_int), ("conv", dr_conv), ("pool", dr_pool)]


class dr_branch(C.Structure):
    _fields_ = [("n_steps", C.c_int), ("steps", dr_step * DR_MAX_STEPS)]


class dr_inception(C.Structure):
    _fields_ = [("n_branches", C.c_int), ("branches", dr_branch * DR_MAX_BRANCHES), ("mode", C.c_int)]


class dr_bottleneck(C.Structure):
    _fields_ = [("mid", C.c_int), ("out", C.c_int), ("project", C.c_int), ("folded", C.c_int), ("eps", C.c_float),
                ("filter_layout", C.c_int)]


class dr_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int), ("conv", dr_conv), ("lrn", dr_lrn), ("pool", dr_pool),
                ("inception", dr_inception), ("bottleneck", dr_bottleneck), ("fc_out", C.c_int)]


class dr_trace_record(C.Structure):
    _fields_ = [("label", C.c_char * 24), ("k", C.c_int), ("c", C.c_int), ("r", C.c_int), ("s", C.c_int),
                ("items", C.c_longlong), ("ms", C.c_float), ("bytes", C.c_longlong)]


class DeepRebirthError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("deeprebirth error %d: %s" % (code, msg))
        self.code = code


_lib = None
_P = C.POINTER
_vp, _i, _z, _f = C.c_void_p, C.c_int, C.c_size_t, C.c_float

_SIGNATURES = {
    "dr_conv_out_size": ([_i, _i, _i, _i], _i),
    "dr_pool_out_size": ([_i, _i, _i, _i], _i),
    "dr_conv2d_fwd": ([_P(dr_tensor), _vp, _P(dr_conv), _vp, _vp, _P(dr_tensor), _vp, _i, _vp], _i),
    "dr_conv2d_workspace_bytes": ([_P(dr_tensor), _P(dr_conv), _P(_z)], _i),
    "dr_conv2d_fwd_ws": ([_P(dr_tensor), _vp, _P(dr_conv), _vp, _vp, _P(dr_tensor), _vp, _i, _vp, _z, _vp], _i),
    "dr_conv2d_fwd_static": ([_P(dr_tensor), _vp, _P(dr_conv), _vp, _vp, _P(dr_tensor), _vp, _i, _vp], _i),
    "dr_pack_filters": ([_P(dr_conv), _i, _vp, _vp, _vp], _i),
    "dr_slim_conv_fwd": ([_P(dr_tensor), _vp, _P(dr_conv), _i, _i, _vp, _vp, _P(dr_tensor), _vp, _i, _vp], _i),
    "dr_relu": ([_P(dr_tensor), _vp, _vp, _vp], _i),
    "dr_lrn_fwd": ([_P(dr_tensor), _vp, _P(dr_lrn), _vp, _vp], _i),
    "dr_maxpool_fwd": ([_P(dr_tensor), _vp, _P(dr_pool), _P(dr_tensor), _vp, _vp], _i),
    "dr_avgpool_fwd": ([_P(dr_tensor), _vp, _P(dr_pool), _P(dr_tensor), _vp, _vp], _i),
    "dr_lrn_maxpool_fwd": ([_P(dr_tensor), _vp, _P(dr_lrn), _P(dr_pool), _P(dr_tensor), _vp, _vp], _i),
    "dr_maxpool_lrn_fwd": ([_P(dr_tensor), _vp, _P(dr_pool), _P(dr_lrn), _P(dr_tensor), _vp, _vp], _i),
    "dr_conv_lrn_maxpool_fwd": ([_P(dr_tensor), _vp, _P(dr_conv), _vp, _vp, _P(dr_lrn), _P(dr_pool), _P(dr_tensor), _vp, _i, _vp], _i),
    "dr_concat": ([_i, _P(dr_tensor), _P(_vp), _P(dr_tensor), _vp, _vp], _i),
    "dr_bn_fwd": ([_P(dr_tensor), _vp, _vp, _vp, _vp, _vp, _f, _i, _vp, _vp], _i),
    "dr_add_relu": ([_P(dr_tensor), _vp, _vp, _vp, _vp], _i),
    "dr_fold_bn": ([_i, _z, _vp, _vp, _vp, _vp, _vp, _vp, _f, _vp, _vp], _i),
    "dr_fc_fwd": ([_P(dr_tensor), _vp, _vp, _vp, _P(dr_tensor), _vp, _vp], _i),
    "dr_softmax_fwd": ([_P(dr_tensor), _vp, _vp, _vp], _i),
    "dr_regression_loss_workspace_bytes": ([], _z),
    "dr_regression_loss_grad": ([_P(dr_tensor), _vp, _vp, _vp, _vp, _vp, _z, _vp], _i),
    "dr_conv2d_bwd_params_workspace_bytes": ([_P(dr_tensor), _P(dr_conv), _P(_z)], _i),
    "dr_conv2d_bwd_params": ([_P(dr_tensor), _vp, _P(dr_conv), _P(dr_tensor), _vp, _vp, _vp, _vp, _z, _vp], _i),
    "dr_sgd_step": ([_z, _vp, _vp, _f, _vp], _i),
    "dr_inception_workspace_bytes": ([_P(dr_tensor), _P(dr_inception), _P(_z)], _i),
    "dr_inception_fwd": ([_P(dr_tensor), _vp, _P(dr_inception), _P(_vp), _P(_vp), _P(dr_tensor), _vp, _vp, _z, _vp], _i),
    "dr_net_create": ([_P(dr_layer_desc), _i, _P(_vp)], _i),
    "dr_net_destroy": ([_vp], None),
    "dr_net_num_params": ([_vp, _P(_i)], _i),
    "dr_net_output_desc": ([_vp, _P(dr_tensor), _P(dr_tensor)], _i),
    "dr_net_workspace_bytes": ([_vp, _P(dr_tensor), _P(_z)], _i),
    "dr_net_fwd": ([_vp, _P(dr_tensor), _vp, _P(_vp), _P(dr_tensor), _vp, _vp, _z, _vp], _i),
    "dr_net_capture": ([_vp, _P(dr_tensor), _vp, _P(_vp), _P(dr_tensor), _vp, _vp, _z, _vp, _P(_vp)], _i),
    "dr_capture_begin": ([_vp], _i),
    "dr_capture_end": ([_vp, _P(_vp)], _i),
    "dr_graph_launch": ([_vp, _vp], _i),
    "dr_graph_destroy": ([_vp], None),
    "dr_net_set_timing": ([_vp, _i], _i),
    "dr_net_layer_times": ([_vp, _P(_f), _i], _i),
    "dr_trace_begin": ([C.c_char_p, _i, _i, _i, _i], _i),
    "dr_trace_end": ([_P(dr_trace_record), _i, _P(_i)], _i),
    "dr_last_error": ([], C.c_char_p),
    "dr_version": ([], C.c_char_p),
}


def lib():
    """The loaded library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdeeprebirth.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "or `python paper_1708_04728_amd/build.py`")
        L = C.CDLL(LIB_PATH)
        for name, (args, res) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.argtypes, fn.restype = args, res
        _lib = L
    return _lib


def _check(rc):
    if rc != DR_OK:
        raise DeepRebirthError(rc, lib().dr_last_error().decode())


def last_error():
    return lib().dr_last_error().decode()


# ---------------------------------------------------------------------------------- marshalling
def _dtype_code(t):
    if t.dtype == torch.float32:
        return DR_F32
    if t.dtype == torch.bfloat16:
        return DR_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


class NHWC:
    """Marks a contiguous torch tensor of shape (n, h, w, c) as a channels-last activation."""

    def __init__(self, t):
        if t.dim() != 4:
            raise ValueError("NHWC tensors are 4-d (n, h, w, c)")
        self.t = t

    def __getattr__(self, name):          # data_ptr, dtype, numel, ... of the wrapped tensor
        return getattr(self.t, name)


def desc(t):
    """dr_tensor of a contiguous torch tensor: 4-d (n, c, h, w), 2-d {n, c, 1, 1}, or NHWC(...)."""
    if isinstance(t, NHWC):
        if not t.t.is_contiguous():
            raise ValueError("tensor must be contiguous")
        n, h, w, c = t.t.shape
        return dr_tensor(n, c, h, w, _dtype_code(t.t), DR_NHWC)
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    shape = tuple(t.shape) + (1,) * (4 - t.dim())
    return dr_tensor(shape[0], shape[1], shape[2], shape[3], _dtype_code(t), DR_NCHW)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def conv_desc(k, c, r, s=None, stride=1, pad=0, relu=False, layout=DR_KCRS):
    s = r if s is None else s
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return dr_conv(k, c, r, s, sh, sw, ph, pw, int(relu), layout)


def can_pack(c, dtype="f32"):
    """Filters over c input channels have a KRSC form the fast kernels accept."""
    return c % (8 if dtype in ("bf16", torch.bfloat16) else 16) == 0


def pool_desc(k, stride, pad=0):
    return dr_pool(k, k, stride, stride, pad, pad)


def conv_out_size(n, filt, stride, pad):
    return lib().dr_conv_out_size(n, filt, stride, pad)


def pool_out_size(n, win, stride, pad):
    return lib().dr_pool_out_size(n, win, stride, pad)


# ---------------------------------------------------------------------------------- entry points
def conv2d_fwd(x, cd, w, bias, y, y_c_offset=0, stream=None):
    xd, yd = desc(x), desc(y)
    _check(lib().dr_conv2d_fwd(xd, _ptr(x), cd, _ptr(w), _ptr(bias), yd, _ptr(y), y_c_offset, _stream(stream)))
    return y


def conv2d_workspace_bytes(x, cd):
    n = C.c_size_t(0)
    _check(lib().dr_conv2d_workspace_bytes(desc(x), cd, C.byref(n)))
    return n.value


def conv2d_fwd_ws(x, cd, w, bias, y, ws, y_c_offset=0, stream=None):
    """ws: a device tensor of at least conv2d_workspace_bytes(x, cd) bytes, or None when that is 0."""
    xd, yd = desc(x), desc(y)
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().dr_conv2d_fwd_ws(xd, _ptr(x), cd, _ptr(w), _ptr(bias), yd, _ptr(y), y_c_offset, _ptr(ws), nbytes, _stream(stream)))
    return y


STATIC_SCRATCH_BYTES = 8 << 20      # DR_STATIC_SCRATCH_BYTES


def conv2d_fwd_static(x, cd, w, bias, y, y_c_offset=0, stream=None):
    """dr_conv2d_fwd_ws on the library's own scratch: nothing is allocated by the call."""
    xd, yd = desc(x), desc(y)
    _check(lib().dr_conv2d_fwd_static(xd, _ptr(x), cd, _ptr(w), _ptr(bias), yd, _ptr(y), y_c_offset, _stream(stream)))
    return y


def pack_filters(w, stream=None):
    """KCRS device tensor -> new KRSC device tensor (same dtype, shape (k, r, s, c))."""
    k, c, r, s = w.shape
    out = torch.empty((k, r, s, c), dtype=w.dtype, device=w.device)
    _check(lib().dr_pack_filters(conv_desc(k, c, r, s), _dtype_code(w), _ptr(w), _ptr(out), _stream(stream)))
    return out


def slim_conv_fwd(x, cd, pool_stride, w, bias, y, y_c_offset=0, stream=None):
    xd, yd = desc(x), desc(y)
    ps = (pool_stride, pool_stride) if isinstance(pool_stride, int) else pool_stride
    _check(lib().dr_slim_conv_fwd(xd, _ptr(x), cd, ps[0], ps[1], _ptr(w), _ptr(bias), yd, _ptr(y), y_c_offset,
                                  _stream(stream)))
    return y


def relu(x, y, stream=None):
    _check(lib().dr_relu(desc(x), _ptr(x), _ptr(y), _stream(stream)))
    return y


def lrn_fwd(x, y, local_size=5, alpha=1e-4, beta=0.75, k=1.0, stream=None):
    p = dr_lrn(local_size, alpha, beta, k)
    _check(lib().dr_lrn_fwd(desc(x), _ptr(x), p, _ptr(y), _stream(stream)))
    return y


def maxpool_fwd(x, pd, y, stream=None):
    _check(lib().dr_maxpool_fwd(desc(x), _ptr(x), pd, desc(y), _ptr(y), _stream(stream)))
    return y


def lrn_maxpool_fwd(x, ld, pd, y, stream=None):
    """y = maxpool(lrn(x)) in one pass; ld: dr_lrn, pd: dr_pool."""
    _check(lib().dr_lrn_maxpool_fwd(desc(x), _ptr(x), ld, pd, desc(y), _ptr(y), _stream(stream)))
    return y


def conv_lrn_maxpool_fwd(x, cd, w, bias, ld, pd, y, y_c_offset=0, stream=None):
    """y = maxpool(lrn(relu(conv(x; w) + bias))) in one kernel (the original form of a streamlined block)."""
    _check(lib().dr_conv_lrn_maxpool_fwd(desc(x), _ptr(x), cd, _ptr(w), _ptr(bias), ld, pd, desc(y), _ptr(y), y_c_offset, _stream(stream)))
    return y


def maxpool_lrn_fwd(x, pd, ld, y, stream=None):
    """y = lrn(maxpool(x)) in one pass."""
    _check(lib().dr_maxpool_lrn_fwd(desc(x), _ptr(x), pd, ld, desc(y), _ptr(y), _stream(stream)))
    return y


def avgpool_fwd(x, pd, y, stream=None):
    _check(lib().dr_avgpool_fwd(desc(x), _ptr(x), pd, desc(y), _ptr(y), _stream(stream)))
    return y


def concat(xs, y, stream=None):
    nb = len(xs)
    xds = (dr_tensor * nb)(*[desc(x) for x in xs])
    ptrs = (C.c_void_p * nb)(*[x.data_ptr() for x in xs])
    _check(lib().dr_concat(nb, xds, ptrs, desc(y), _ptr(y), _stream(stream)))
    return y


def bn_fwd(x, gamma, beta, mean, var, eps, relu, y, stream=None):
    _check(lib().dr_bn_fwd(desc(x), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(var), eps, int(relu), _ptr(y),
                           _stream(stream)))
    return y


def add_relu(a, b, y, stream=None):
    _check(lib().dr_add_relu(desc(a), _ptr(a), _ptr(b), _ptr(y), _stream(stream)))
    return y


def fold_bn(w, b, gamma, beta, mean, var, eps):
    """Host transform (numpy fp32 arrays in, numpy fp32 arrays out)."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.float32)
    k = w.shape[0]
    vec = [None if v is None else np.ascontiguousarray(v, dtype=np.float32) for v in (b, gamma, beta, mean, var)]
    w_out, b_out = np.empty_like(w), np.empty(k, dtype=np.float32)
    p = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
    _check(lib().dr_fold_bn(k, w.size // max(k, 1), p(w), p(vec[0]), p(vec[1]), p(vec[2]), p(vec[3]), p(vec[4]), eps,
                            p(w_out), p(b_out)))
    return w_out, b_out


def fc_fwd(x, w, bias, y, stream=None):
    _check(lib().dr_fc_fwd(desc(x), _ptr(x), _ptr(w), _ptr(bias), desc(y), _ptr(y), _stream(stream)))
    return y


def softmax_fwd(x, y, stream=None):
    if y.dtype != torch.float32:
        raise TypeError("softmax output is fp32")
    _check(lib().dr_softmax_fwd(desc(x), _ptr(x), _ptr(y), _stream(stream)))
    return y


def inception_workspace_bytes(x, idesc):
    n = C.c_size_t(0)
    _check(lib().dr_inception_workspace_bytes(desc(x), idesc, C.byref(n)))
    return n.value


def inception_fwd(x, idesc, weights, biases, y, ws, stream=None):
    nw = len(weights)
    wp = (C.c_void_p * nw)(*[0 if w is None else w.data_ptr() for w in weights])
    bp = (C.c_void_p * nw)(*[0 if b is None else b.data_ptr() for b in biases])
    _check(lib().dr_inception_fwd(desc(x), _ptr(x), idesc, wp, bp, desc(y), _ptr(y), _ptr(ws),
                                  0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))
    return y


def regression_loss_grad(f, target, dz, loss, ws, stream=None):
    """dz = dL/dz and loss[0] = L = sum (f - target)^2 for a slim layer's output f (after its ReLU); all device tensors."""
    _check(lib().dr_regression_loss_grad(desc(f), _ptr(f), _ptr(target), _ptr(dz), _ptr(loss), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)))
    return dz


def regression_loss_workspace_bytes():
    return int(lib().dr_regression_loss_workspace_bytes())


def conv2d_bwd_params_workspace_bytes(x, cd):
    n = C.c_size_t(0)
    _check(lib().dr_conv2d_bwd_params_workspace_bytes(desc(x), cd, C.byref(n)))
    return n.value


def conv2d_bwd_params(x, cd, dz, dw, db, ws, stream=None):
    _check(lib().dr_conv2d_bwd_params(desc(x), _ptr(x), cd, desc(dz), _ptr(dz), _ptr(dw), _ptr(db), _ptr(ws),
                                      0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))
    return dw, db


def sgd_step(w, dw, lr, stream=None):
    _check(lib().dr_sgd_step(w.numel(), _ptr(w), _ptr(dw), lr, _stream(stream)))
    return w


def trace_begin(label_filter="", conv_k=0, conv_c=0, conv_r=0, capacity=4096):
    _check(lib().dr_trace_begin(label_filter.encode(), conv_k, conv_c, conv_r, capacity))


def trace_end(capacity=4096):
    """List of (label, k, c, r, s, items, ms, bytes) in launch order."""
    arr = (dr_trace_record * capacity)()
    n = C.c_int(0)
    _check(lib().dr_trace_end(arr, capacity, C.byref(n)))
    return [(a.label.decode(), a.k, a.c, a.r, a.s, a.items, a.ms, a.bytes) for a in arr[:n.value]]


class Graph:
    """Owner of a dr_graph handle (a captured forward pass); keeps the tensors it was captured with alive."""

    def __init__(self, handle, keep):
        self._h, self._keep = handle, keep

    def launch(self, stream=None):
        _check(lib().dr_graph_launch(self._h, _stream(stream)))

    def __del__(self):
        if getattr(self, "_h", None) is not None and _lib is not None:
            _lib.dr_graph_destroy(self._h)
            self._h = None


class capture:
    """with capture(stream) as c: ... dr_* calls given `stream` ...; then c.graph is the recorded Graph.  `keep`:
    tensors the recording uses, kept alive with the graph."""

    def __init__(self, stream, keep=()):
        self.stream, self.keep, self.graph = stream, tuple(keep), None

    def __enter__(self):
        _check(lib().dr_capture_begin(_stream(self.stream)))
        return self

    def __exit__(self, exc_type, exc, tb):
        if exc_type is not None:
            lib().dr_capture_end(_stream(self.stream), None)
            return False
        h = C.c_void_p()
        _check(lib().dr_capture_end(_stream(self.stream), C.byref(h)))
        self.graph = Graph(h, self.keep)
        return False


class Net:
    """Owner of a dr_net handle."""

    def __init__(self, layer_descs):
        arr = (dr_layer_desc * len(layer_descs))(*layer_descs)
        h = C.c_void_p()
        _check(lib().dr_net_create(arr, len(layer_descs), C.byref(h)))
        self._h = h
        self.n_layers = len(layer_descs)
        self.kinds = [int(d.kind) for d in layer_descs]

    def __del__(self):
        if getattr(self, "_h", None) is not None and _lib is not None:
            _lib.dr_net_destroy(self._h)
            self._h = None

    def num_params(self):
        n = C.c_int(0)
        _check(lib().dr_net_num_params(self._h, C.byref(n)))
        return n.value

    def output_desc(self, xd):
        yd = dr_tensor()
        _check(lib().dr_net_output_desc(self._h, xd, C.byref(yd)))
        return yd

    def workspace_bytes(self, xd):
        n = C.c_size_t(0)
        _check(lib().dr_net_workspace_bytes(self._h, xd, C.byref(n)))
        return n.value

    def fwd(self, x, params, y, ws, stream=None):
        pp = (C.c_void_p * max(len(params), 1))(*[p.data_ptr() for p in params])
        _check(lib().dr_net_fwd(self._h, desc(x), _ptr(x), pp, desc(y), _ptr(y), _ptr(ws),
                                0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))
        return y

    def capture(self, x, params, y, ws, stream):
        """The forward for these tensors as a HIP graph (see dr_net_capture).  `stream`: a torch stream other than
        the default one, used for the capture only.  The tensors must outlive the returned Graph."""
        pp = (C.c_void_p * max(len(params), 1))(*[p.data_ptr() for p in params])
        h = C.c_void_p()
        _check(lib().dr_net_capture(self._h, desc(x), _ptr(x), pp, desc(y), _ptr(y), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(), _stream(stream), C.byref(h)))
        return Graph(h, (x, params, y, ws))

    def set_timing(self, enabled):
        _check(lib().dr_net_set_timing(self._h, int(enabled)))

    def layer_times(self):
        arr = (C.c_float * self.n_layers)()
        _check(lib().dr_net_layer_times(self._h, arr, self.n_layers))
        return list(arr)
