"""Seeded synthetic workloads: layer lists and random tensors, nothing else.

This module serves both the CPU oracle and the HIP library with *identical*
inputs.  It holds no arithmetic of the method: it only says which layers a
workload is made of (hyper-parameters, never output shapes or values) and draws
the random input / weight tensors for them.

Layer vocabulary (plain tuples ``(kind, params)``):

  ("conv",      {k, r, s, stride, pad})          convolution + bias (Sec. 3.1, the conv definition in the proof of Lemma 2)
  ("relu",      {})
  ("lrn",       {n, alpha, beta, k})             across-channel LRN (Sec. 3.1 parameter list)
  ("maxpool",   {k, stride, pad})
  ("bn",        {eps})                           BatchNorm+Scale at inference (Lemma 2)
  ("inception", {branches: [[layer, ...], ...]}) parallel chains on one input, concatenated (Sec. 3.2)
  ("bottleneck",{mid, out, project, eps})        ResNet bottleneck (Sec. 4.2)
  ("avgpool",   {k}), ("fc", {out}), ("softmax", {})

Random streams: ``numpy.random.Generator(PCG64(SeedSequence([seed, stream])))``
with stream 0 = input images (drawn image after image, so the first b images of
a larger batch are the same tensors), 1 = parameters of the original form,
2 = parameters of the slim form (fresh weights: slim layers are re-learned in
the paper, Sec. 3.1 Eq. (5), and no training data exists here).
Weights are He-normal (std = sqrt(2 / (C*R*S))), biases N(0, 0.01^2).
"""
from __future__ import annotations

import numpy as np

LRN5 = {"n": 5, "alpha": 1e-4, "beta": 0.75, "k": 1.0}
BN_EPS = 1e-5


def conv(k, r, stride=1, pad=0):
    return ("conv", {"k": k, "r": r, "s": r, "stride": stride, "pad": pad})


def relu():
    return ("relu", {})


def lrn():
    return ("lrn", dict(LRN5))


def maxpool(k, stride, pad=0):
    return ("maxpool", {"k": k, "stride": stride, "pad": pad})


# --------------------------------------------------------------------------
# GoogLeNet-v1 inception widths (from the architecture table of the GoogLeNet
# paper that Sec. 3.2 cites): in, 1x1, 3x3reduce, 3x3, 5x5reduce, 5x5, poolproj
# --------------------------------------------------------------------------
INCEPTION_WIDTHS = {
    "3a": (192, 64, 96, 128, 16, 32, 32),
    "3b": (256, 128, 128, 192, 32, 96, 64),
    "4a": (480, 192, 96, 208, 16, 48, 64),
    "4b": (512, 160, 112, 224, 24, 64, 64),
    "4c": (512, 128, 128, 256, 24, 64, 64),
    "4d": (512, 112, 144, 288, 32, 64, 64),
    "4e": (528, 256, 160, 320, 32, 128, 128),
    "5a": (832, 256, 160, 320, 32, 128, 128),
    "5b": (832, 384, 192, 384, 48, 128, 128),
}


def inception_original(name):
    """Four branches: 1x1 | 1x1->3x3 | 1x1->5x5 | maxpool3x3 s1 p1 -> 1x1; ReLU after every conv."""
    _, c1, c3r, c3, c5r, c5, cp = INCEPTION_WIDTHS[name]
    return ("inception", {"branches": [
        [conv(c1, 1), relu()],
        [conv(c3r, 1), relu(), conv(c3, 3, 1, 1), relu()],
        [conv(c5r, 1), relu(), conv(c5, 5, 1, 2), relu()],
        [maxpool(3, 1, 1), conv(cp, 1), relu()],
    ]})


def inception_slim(name):
    """Branch slimming: the 1x1 branch and the pool branch are absorbed into the 5x5 branch,
    whose output width grows by theirs so that the concatenated width is unchanged."""
    _, c1, c3r, c3, c5r, c5, cp = INCEPTION_WIDTHS[name]
    return ("inception", {"branches": [
        [conv(c3r, 1), relu(), conv(c3, 3, 1, 1), relu()],
        [conv(c5r, 1), relu(), conv(c5 + c1 + cp, 5, 1, 2), relu()],
    ]})


def inception_3a_paper_variant():
    """The paper's own 3a example (Sec. 3.2): pool branch -> 5x5 (32 -> 64), 3x3 reducer 96 -> 48,
    1x1 branch -> 3x3 (128 -> 192; the text prints 196, which cannot give 256 channels)."""
    return ("inception", {"branches": [
        [conv(48, 1), relu(), conv(192, 3, 1, 1), relu()],
        [conv(16, 1), relu(), conv(64, 5, 1, 2), relu()],
    ]})


def bottleneck(mid, out, project):
    return ("bottleneck", {"mid": mid, "out": out, "project": project, "eps": BN_EPS})


# --------------------------------------------------------------------------
# The five configurations
# --------------------------------------------------------------------------
def _googlenet(slim):
    inc = inception_slim if slim else inception_original
    if slim:  # streamline slimming of the stem: pools absorbed into strides, LRN pruned
        stem = [conv(64, 7, 4, 3), relu(), conv(64, 1), relu(), conv(192, 3, 2, 1), relu()]
    else:
        stem = [conv(64, 7, 2, 3), relu(), maxpool(3, 2), lrn(),
                conv(64, 1), relu(), conv(192, 3, 1, 1), relu(), lrn(), maxpool(3, 2)]
    return stem + [inc("3a"), inc("3b"), maxpool(3, 2),
                   inc("4a"), inc("4b"), inc("4c"), inc("4d"), inc("4e"), maxpool(3, 2),
                   inc("5a"), inc("5b"),
                   ("avgpool", {"k": 7}), ("fc", {"out": 1000}), ("softmax", {})]


CONFIGS = {
    1: {"name": "streamline_block", "seed": 0, "dtype": "f32", "batch": 1, "in_shape": (64, 56, 56),
        "input": "uniform01",
        "original": [conv(192, 3, 1, 1), relu(), lrn(), maxpool(3, 2)],
        "slim": [conv(192, 3, 2, 1), relu()]},
    2: {"name": "inception_3a", "seed": 1, "dtype": "f32", "batch": 32, "in_shape": (192, 28, 28),
        "input": "absnormal",
        "original": [inception_original("3a")],
        "slim": [inception_slim("3a")]},
    3: {"name": "alexnet_front", "seed": 2, "dtype": "f32", "batch": 128, "in_shape": (3, 227, 227),
        "input": "normal",
        "original": [conv(96, 11, 4, 0), relu(), lrn(), maxpool(3, 2),
                     conv(256, 5, 1, 2), relu(), lrn(), maxpool(3, 2)],
        "slim": [conv(96, 11, 8, 0), relu(), conv(256, 5, 2, 2), relu()]},
    4: {"name": "resnet50_conv2_x", "seed": 3, "dtype": "bf16", "batch": 128, "in_shape": (64, 56, 56),
        "input": "absnormal",
        "original": [bottleneck(64, 256, True), bottleneck(64, 256, False), bottleneck(64, 256, False)],
        "slim": "fold_bn"},   # same layers, BN folded into the conv (exact, Lemma 2): no fresh weights
    5: {"name": "googlenet_v1", "seed": 4, "dtype": "bf16", "batch": 128, "in_shape": (3, 224, 224),
        "input": "normal",
        "original": _googlenet(False),
        "slim": _googlenet(True)},
}


# --------------------------------------------------------------------------
# Random tensors
# --------------------------------------------------------------------------
def _rng(seed, stream):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream])))


def round_to_bf16(a):
    """Round an fp32 array to the nearest bf16-representable fp32 value (ties to even).
    Storage-format rule only: both sides then consume exactly these values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _cast(a, dtype):
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


def make_input(cfg_id, batch=None):
    """Input images of a configuration as fp32 (bf16-representable if the config is bf16)."""
    cfg = CONFIGS[cfg_id]
    b = cfg["batch"] if batch is None else batch
    rng = _rng(cfg["seed"], 0)
    shape = (b,) + cfg["in_shape"]
    if cfg["input"] == "uniform01":
        x = rng.random(shape)
    elif cfg["input"] == "normal":
        x = rng.standard_normal(shape)
    elif cfg["input"] == "absnormal":
        x = np.abs(rng.standard_normal(shape))
    else:
        raise ValueError(cfg["input"])
    return _cast(x, cfg["dtype"])


def _conv_params(rng, c_in, p, dtype):
    fan_in = c_in * p["r"] * p["s"]
    w = rng.standard_normal((p["k"], c_in, p["r"], p["s"])) * np.sqrt(2.0 / fan_in)
    b = rng.standard_normal(p["k"]) * 0.01
    return {"w": _cast(w, dtype), "b": b.astype(np.float32)}


def _bn_params(rng, c):
    return {"gamma": rng.uniform(0.5, 1.5, c).astype(np.float32),
            "beta": (rng.standard_normal(c) * 0.1).astype(np.float32),
            "mean": (rng.standard_normal(c) * 0.1).astype(np.float32),
            "var": rng.uniform(0.5, 1.5, c).astype(np.float32)}


def _walk(rng, layers, c_in, dtype, out):
    """Append one parameter dict per parameterised layer, in forward order; return channels out."""
    c = c_in
    for kind, p in layers:
        if kind == "conv":
            out.append(_conv_params(rng, c, p, dtype))
            c = p["k"]
        elif kind == "bn":
            out.append(_bn_params(rng, c))
        elif kind == "inception":
            widths = [_walk(rng, br, c, dtype, out) for br in p["branches"]]
            c = sum(widths)
        elif kind == "bottleneck":
            # order: conv a, bn a, conv b, bn b, conv c, bn c, then projection conv + bn if present
            for (k, r, pad, cin) in ((p["mid"], 1, 0, c), (p["mid"], 3, 1, p["mid"]), (p["out"], 1, 0, p["mid"])):
                out.append(_conv_params(rng, cin, conv(k, r, 1, pad)[1], dtype))
                out.append(_bn_params(rng, k))
            if p["project"]:
                out.append(_conv_params(rng, c, conv(p["out"], 1)[1], dtype))
                out.append(_bn_params(rng, p["out"]))
            c = p["out"]
        elif kind == "fc":
            w = rng.standard_normal((p["out"], c)) * np.sqrt(2.0 / c)
            b = rng.standard_normal(p["out"]) * 0.01
            out.append({"w": _cast(w, dtype), "b": b.astype(np.float32)})
            c = p["out"]
        # relu, lrn, maxpool, avgpool (global at the shapes used here), softmax: no parameters
    return c


def make_params(cfg_id, form="original", layers=None):
    """Parameter dicts, one per parameterised layer in forward order (inception: branch by branch).

    ``layers`` overrides the layer list (e.g. a variant module) while keeping the config's seed
    and dtype.  For config 4 the slim form has no parameters of its own (it is the original's,
    folded)."""
    cfg = CONFIGS[cfg_id]
    if layers is None:
        layers = cfg[form]
    if isinstance(layers, str):
        raise ValueError("config %d: the %s form is derived from the original's parameters" % (cfg_id, form))
    rng = _rng(cfg["seed"], 1 if form == "original" else 2)
    out = []
    _walk(rng, layers, cfg["in_shape"][0], cfg["dtype"], out)
    return out
