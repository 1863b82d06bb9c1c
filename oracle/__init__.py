"""CPU oracle (fp64) for the CNN-block forward pass: TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``oracle.c`` (plain nested loops in fp64) plus the composition of
layers into blocks and networks.  Only tests, the smoke check and the benchmark's CPU-baseline leg
may import this package; the HIP library never does, and this package never imports the library.

All tensors are ``numpy.float64`` in NCHW layout.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile oracle.c with the host C compiler (never hipcc)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_D = ctypes.POINTER(ctypes.c_double)


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_conv_out_size.restype = ctypes.c_int
        _lib.orc_pool_out_size.restype = ctypes.c_int
        for name in ("orc_conv2d", "orc_relu", "orc_lrn", "orc_maxpool", "orc_avgpool", "orc_concat_into",
                     "orc_bn", "orc_fold_bn", "orc_add_relu", "orc_fc", "orc_softmax", "orc_round_bf16", "orc_conv2d_bwd_params"):
            getattr(_lib, name).restype = None
        _lib.orc_regression_loss_grad.restype = ctypes.c_double
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(_D)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


_i = ctypes.c_int
_z = ctypes.c_size_t
_d = ctypes.c_double


def conv_out_size(n, filt, stride, pad):
    return int(_L().orc_conv_out_size(_i(n), _i(filt), _i(stride), _i(pad)))


def pool_out_size(n, win, stride, pad):
    return int(_L().orc_pool_out_size(_i(n), _i(win), _i(stride), _i(pad)))


def conv2d(x, w, b=None, stride=1, pad=0, relu=False):
    x, w, b = _f64(x), _f64(w), _f64(b)
    N, C, H, W = x.shape
    K, Cw, R, S = w.shape
    assert C == Cw, (C, Cw)
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    y = np.empty((N, K, conv_out_size(H, R, sh, ph), conv_out_size(W, S, sw, pw)))
    _L().orc_conv2d(_p(x), _i(N), _i(C), _i(H), _i(W), _p(w), _p(b), _i(K), _i(R), _i(S),
                    _i(sh), _i(sw), _i(ph), _i(pw), _i(int(relu)), _p(y))
    return y


def relu(x):
    x = _f64(x)
    y = np.empty_like(x)
    _L().orc_relu(_p(x), _z(x.size), _p(y))
    return y


def lrn(x, n=5, alpha=1e-4, beta=0.75, k=1.0):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty_like(x)
    _L().orc_lrn(_p(x), _i(N), _i(C), _i(H), _i(W), _i(n), _d(alpha), _d(beta), _d(k), _p(y))
    return y


def maxpool(x, k, stride, pad=0):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, pool_out_size(H, k, stride, pad), pool_out_size(W, k, stride, pad)))
    _L().orc_maxpool(_p(x), _i(N), _i(C), _i(H), _i(W), _i(k), _i(k), _i(stride), _i(stride),
                     _i(pad), _i(pad), _p(y))
    return y


def avgpool(x, k, stride=1):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, conv_out_size(H, k, stride, 0), conv_out_size(W, k, stride, 0)))
    _L().orc_avgpool(_p(x), _i(N), _i(C), _i(H), _i(W), _i(k), _i(stride), _p(y))
    return y


def concat(xs):
    xs = [_f64(x) for x in xs]
    N, _, H, W = xs[0].shape
    Cy = sum(x.shape[1] for x in xs)
    y = np.empty((N, Cy, H, W))
    off = 0
    for x in xs:
        assert x.shape[0] == N and x.shape[2:] == (H, W)
        _L().orc_concat_into(_p(x), _i(N), _i(x.shape[1]), _z(H * W), _p(y), _i(Cy), _i(off))
        off += x.shape[1]
    return y


def bn(x, gamma, beta, mean, var, eps):
    x = _f64(x)
    N, C, H, W = x.shape
    g, b, m, v = _f64(gamma), _f64(beta), _f64(mean), _f64(var)
    y = np.empty_like(x)
    _L().orc_bn(_p(x), _i(N), _i(C), _z(H * W), _p(g), _p(b), _p(m), _p(v), _d(eps), _p(y))
    return y


def fold_bn(w, b, gamma, beta, mean, var, eps):
    w, b = _f64(w), _f64(b)
    g, be, m, v = _f64(gamma), _f64(beta), _f64(mean), _f64(var)
    K = w.shape[0]
    w_out, b_out = np.empty_like(w), np.empty(K)
    _L().orc_fold_bn(_i(K), _z(w.size // K), _p(w), _p(b), _p(g), _p(be), _p(m), _p(v), _d(eps),
                     _p(w_out), _p(b_out))
    return w_out, b_out


def add_relu(a, b):
    a, b = _f64(a), _f64(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    _L().orc_add_relu(_p(a), _p(b), _z(a.size), _p(y))
    return y


def fc(x, w, b=None):
    x, w, b = _f64(x), _f64(w), _f64(b)
    N = x.shape[0]
    x2 = x.reshape(N, -1)
    O, I = w.shape
    assert x2.shape[1] == I
    y = np.empty((N, O))
    _L().orc_fc(_p(x2), _i(N), _i(I), _p(w), _p(b), _i(O), _p(y))
    return y


def softmax(x):
    x = _f64(x)
    N, O = x.shape
    y = np.empty_like(x)
    _L().orc_softmax(_p(x), _i(N), _i(O), _p(y))
    return y


def regression_loss_grad(f, y):
    """Sec. 3.1, the optimisation goal of the slim layer: L = sum (f - y)^2 for the layer's output f (after its
    ReLU) and the target feature map y; returns (L, dL/dz) with z the layer's pre-activation."""
    f, y = _f64(f), _f64(y)
    assert f.shape == y.shape
    dz = np.empty_like(f)
    loss = _L().orc_regression_loss_grad(_p(f), _p(y), _z(f.size), _p(dz))
    return float(loss), dz


def conv2d_bwd_params(x, dz, r, s=None, stride=1, pad=0):
    """Gradient of a convolution's parameters given dL/dz of its output (chain rule through Eq. (7)):
    returns (dw of shape (k, c, r, s), db of shape (k,))."""
    x, dz = _f64(x), _f64(dz)
    s = r if s is None else s
    N, C, H, W = x.shape
    K = dz.shape[1]
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    assert dz.shape == (N, K, conv_out_size(H, r, sh, ph), conv_out_size(W, s, sw, pw)), dz.shape
    dw, db = np.empty((K, C, r, s)), np.empty(K)
    _L().orc_conv2d_bwd_params(_p(x), _i(N), _i(C), _i(H), _i(W), _p(dz), _i(K), _i(r), _i(s), _i(sh), _i(sw), _i(ph), _i(pw),
                               _p(dw), _p(db))
    return dw, db


def regression_step(x, w, b, y, stride, pad, lr):
    """One step of gradient descent on L(w, b) = sum || y - max(conv(x; w, b), 0) ||^2 (Lemma 1: the slim layer is
    learned with SGD on Eq. (5)'s objective): returns (L at (w, b), w - lr dL/dw, b - lr dL/db)."""
    f = conv2d(x, w, b, stride, pad, relu=True)
    loss, dz = regression_loss_grad(f, y)
    dw, db = conv2d_bwd_params(x, dz, w.shape[2], w.shape[3], stride, pad)
    return loss, _f64(w) - lr * dw, _f64(b) - lr * db


def round_bf16(x):
    y = np.array(x, dtype=np.float64, order="C", copy=True)
    _L().orc_round_bf16(_p(y), _z(y.size))
    return y


# ------------------------------------------------------------------------------------------------
# Composition: a layer list (see workloads.py for the vocabulary) applied to an input.
# ------------------------------------------------------------------------------------------------
class _Params:
    def __init__(self, params):
        self.params, self.i = params, 0

    def next(self):
        p = self.params[self.i]
        self.i += 1
        return p


def forward(layers, params, x, mirror_bf16=False, fold=False, trace=None):
    """Run `layers` on `x` with `params` (one dict per parameterised layer, forward order).

    mirror_bf16: round every layer's output to bf16 before the next layer reads it (the storage
                 rule of the bf16 configurations); arithmetic inside a layer stays fp64.
    fold:        slim form of a BatchNorm network (Lemma 2): every conv+BN pair is replaced by one
                 conv with folded weights and bias.  True: the fold is computed here from the
                 conv and BN parameters; "given": `params` already holds the folded conv
                 parameters (one dict per conv, no BN dicts), e.g. after rounding them to bf16.
    trace:       optional list; receives (kind, output) after each top-level layer.
    """
    pit = params if isinstance(params, _Params) else _Params(params)
    rnd = round_bf16 if mirror_bf16 else (lambda a: a)
    y = _f64(x)
    for kind, p in layers:
        if kind == "conv":
            q = pit.next()
            y = rnd(conv2d(y, q["w"], q["b"], p["stride"], p["pad"]))
        elif kind == "relu":
            y = relu(y)
        elif kind == "lrn":
            y = rnd(lrn(y, p["n"], p["alpha"], p["beta"], p["k"]))
        elif kind == "maxpool":
            y = maxpool(y, p["k"], p["stride"], p["pad"])
        elif kind == "inception":
            # Sec. 3.2: every branch reads the module input; outputs are concatenated in branch order
            y = concat([forward(br, pit, y, mirror_bf16) for br in p["branches"]])
        elif kind == "bottleneck":
            y = _bottleneck(y, p, pit, rnd, fold)
        elif kind == "avgpool":
            y = rnd(avgpool(y, p["k"]))
        elif kind == "fc":
            q = pit.next()
            y = rnd(fc(y, q["w"], q["b"]))
        elif kind == "softmax":
            y = softmax(y)   # final probabilities are kept in fp32 by the library: no bf16 rounding
        else:
            raise ValueError(kind)
        if trace is not None:
            trace.append((kind, y))
    return y


def _conv_bn(y, cq, bq, stride, pad, eps, rnd, fold, relu_after):
    """conv -> BN(+Scale) [-> ReLU] of Eq. (2); `fold` = the merged conv of Lemma 2 instead."""
    if fold:
        if bq is None:      # parameters were folded by the caller
            wf, bf = cq["w"], cq["b"]
        else:
            wf, bf = fold_bn(cq["w"], cq["b"], bq["gamma"], bq["beta"], bq["mean"], bq["var"], eps)
        y = conv2d(y, wf, bf, stride, pad)
        return rnd(relu(y) if relu_after else y)
    y = rnd(conv2d(y, cq["w"], cq["b"], stride, pad))
    y = rnd(bn(y, bq["gamma"], bq["beta"], bq["mean"], bq["var"], eps))
    return relu(y) if relu_after else y


def _bottleneck(x, p, pit, rnd, fold):
    """ResNet bottleneck (Sec. 4.2: one branch of three convs, one shortcut branch with one conv on
    the first block): relu(bn(conv1x1(relu(bn(conv3x3(relu(bn(conv1x1 x))))))) + shortcut(x))."""
    eps = p["eps"]
    given = fold == "given"
    nxt = (lambda: (pit.next(), None)) if given else (lambda: (pit.next(), pit.next()))
    (ca, ba), (cb, bb), (cc, bc) = nxt(), nxt(), nxt()
    y = _conv_bn(x, ca, ba, 1, 0, eps, rnd, fold, True)
    y = _conv_bn(y, cb, bb, 1, 1, eps, rnd, fold, True)
    if p["project"]:
        cp, bp = nxt()
        sc = _conv_bn(x, cp, bp, 1, 0, eps, rnd, fold, False)
    else:
        sc = x
    if fold:
        # slim form: the last conv's store adds the shortcut and applies the ReLU (one rounding)
        y = _conv_bn(y, cc, bc, 1, 0, eps, (lambda a: a), fold, False)
        return rnd(add_relu(y, sc))
    y = _conv_bn(y, cc, bc, 1, 0, eps, rnd, fold, False)
    return rnd(add_relu(y, sc))
