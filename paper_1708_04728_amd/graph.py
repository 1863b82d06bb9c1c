"""Layer lists (vocabulary of ``workloads.py``) -> library descriptors and device parameters.

Host-side marshalling only; every shape is computed by the library itself."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def torch_dtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(a, dtype="f32", device="cuda", nhwc=False):
    """numpy fp32 array -> device tensor; for bf16 the values must already be bf16-representable,
    so the conversion is exact.  nhwc: an (n, c, h, w) array is stored channels-last and returned
    wrapped in binding.NHWC."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    if nhwc:
        return B.NHWC(t.permute(0, 2, 3, 1).contiguous().to(device))
    return t.to(device)


def to_host(t):
    """Device tensor (plain, or binding.NHWC) -> numpy float64 in (n, c, h, w) order."""
    if isinstance(t, B.NHWC):
        return t.t.float().permute(0, 3, 1, 2).contiguous().cpu().numpy().astype(np.float64)
    return t.float().cpu().numpy().astype(np.float64)


def empty_like_desc(d, device="cuda"):
    """Uninitialised device tensor for a dr_tensor descriptor (binding.NHWC-wrapped if channels-last)."""
    dt = torch.bfloat16 if d.dtype == B.DR_BF16 else torch.float32
    if d.layout == B.DR_NHWC:
        return B.NHWC(torch.empty((d.n, d.h, d.w, d.c), dtype=dt, device=device))
    return torch.empty((d.n, d.c, d.h, d.w), dtype=dt, device=device)


def conv_desc(p, c_in, relu=False, pack=False):
    """pack: False, or the dtype ("f32" / "bf16") whose packing rule decides KRSC vs KCRS."""
    layout = B.DR_KRSC if (pack and B.can_pack(c_in, pack)) else B.DR_KCRS
    return B.conv_desc(p["k"], c_in, p["r"], p["s"], p["stride"], p["pad"], relu, layout)


def inception_desc(p, c_in, mode=0, pack=False):
    """dr_inception from an ("inception", {...}) layer; a conv directly followed by a relu gets
    conv.relu = 1."""
    d = B.dr_inception()
    d.n_branches = len(p["branches"])
    d.mode = mode
    for bi, br in enumerate(p["branches"]):
        c, si, i = c_in, 0, 0
        while i < len(br):
            kind, q = br[i]
            step = d.branches[bi].steps[si]
            if kind == "conv":
                relu = i + 1 < len(br) and br[i + 1][0] == "relu"
                step.kind, step.conv = B.DR_STEP_CONV, conv_desc(q, c, relu, pack)
                c = q["k"]
                i += 2 if relu else 1
            elif kind == "maxpool":
                step.kind, step.pool = B.DR_STEP_MAXPOOL, B.pool_desc(q["k"], q["stride"], q["pad"])
                i += 1
            else:
                raise ValueError("step %s not allowed in an inception branch" % kind)
            si += 1
        d.branches[bi].n_steps = si
    return d


def _out_channels(layers, c_in):
    c = c_in
    for kind, p in layers:
        if kind == "conv":
            c = p["k"]
        elif kind == "inception":
            c = sum(_out_channels(br, c) for br in p["branches"])
        elif kind == "bottleneck":
            c = p["out"]
        elif kind == "fc":
            c = p["out"]
    return c


def net_descs(layers, c_in, inception_mode=0, fuse_relu=False, folded=False, pack=False, fuse_nontensor=False):
    """List of dr_layer_desc for a layer list.

    fuse_nontensor: a maxpool directly followed by an lrn becomes one layer that makes a single pass over the
               tensor (channels-last tensors only); "all": so does an lrn directly followed by a maxpool
               (measured slower than the two layers on their own at stride 2: every input pixel is
               normalised, four per output, and that arithmetic, not memory, bounds it); "block": a
               conv - relu - lrn - maxpool run (3x3 pooling at stride 2, at most 192 filters, bf16) becomes the one
               kernel of dr_conv_lrn_maxpool_fwd, and a maxpool - lrn pair one pass as with True.

    fuse_relu: a conv directly followed by a relu becomes one conv with the ReLU in its store
               (the slim form always runs this way; for the original form it is the "fused"
               variant reported next to the layer-by-layer one)."""
    out, c, i = [], c_in, 0
    while i < len(layers):
        kind, p = layers[i]
        L = B.dr_layer_desc()
        if kind == "conv":
            relu = fuse_relu and i + 1 < len(layers) and layers[i + 1][0] == "relu"
            L.kind, L.conv = B.DR_LAYER_CONV, conv_desc(p, c, relu, pack)
            nxt = [k for k, _ in layers[i + 1:i + 4]]
            if (fuse_nontensor == "block" and nxt == ["relu", "lrn", "maxpool"] and p["k"] <= 192 and p["k"] % 8 == 0 and c % 8 == 0 and
                    pack == "bf16" and layers[i + 2][1]["n"] == 5 and (layers[i + 3][1]["k"], layers[i + 3][1]["stride"], layers[i + 3][1]["pad"]) == (3, 2, 0)):
                # the streamlined block's original form as one kernel (dr_conv_lrn_maxpool_fwd)
                ql, qp = layers[i + 2][1], layers[i + 3][1]
                L.kind = B.DR_LAYER_CONV_LRN_MAXPOOL
                L.lrn, L.pool = B.dr_lrn(ql["n"], ql["alpha"], ql["beta"], ql["k"]), B.pool_desc(qp["k"], qp["stride"], qp["pad"])
                i += 3
                relu = False
            c = p["k"]
            if relu:
                i += 1
        elif kind == "relu":
            L.kind = B.DR_LAYER_RELU
        elif kind == "lrn":
            L.kind, L.lrn = B.DR_LAYER_LRN, B.dr_lrn(p["n"], p["alpha"], p["beta"], p["k"])
            if fuse_nontensor == "all" and i + 1 < len(layers) and layers[i + 1][0] == "maxpool":
                q = layers[i + 1][1]
                L.kind, L.pool = B.DR_LAYER_LRN_MAXPOOL, B.pool_desc(q["k"], q["stride"], q["pad"])
                i += 1
        elif kind == "maxpool":
            L.kind, L.pool = B.DR_LAYER_MAXPOOL, B.pool_desc(p["k"], p["stride"], p["pad"])
            if fuse_nontensor and i + 1 < len(layers) and layers[i + 1][0] == "lrn":
                q = layers[i + 1][1]
                L.kind, L.lrn = B.DR_LAYER_MAXPOOL_LRN, B.dr_lrn(q["n"], q["alpha"], q["beta"], q["k"])
                i += 1
        elif kind == "avgpool":
            L.kind, L.pool = B.DR_LAYER_AVGPOOL, B.pool_desc(p["k"], 1, 0)
        elif kind == "inception":
            L.kind, L.inception = B.DR_LAYER_INCEPTION, inception_desc(p, c, inception_mode, pack)
            c = _out_channels([(kind, p)], c)
        elif kind == "bottleneck":
            L.kind = B.DR_LAYER_BOTTLENECK
            lay = B.DR_KRSC if (pack and B.can_pack(c, pack) and B.can_pack(p["mid"], pack)) else B.DR_KCRS
            L.bottleneck = B.dr_bottleneck(p["mid"], p["out"], int(p["project"]), int(folded), p["eps"], lay)
            c = p["out"]
        elif kind == "fc":
            L.kind, L.fc_out = B.DR_LAYER_FC, p["out"]
            c = p["out"]
        elif kind == "softmax":
            L.kind = B.DR_LAYER_SOFTMAX
        else:
            raise ValueError(kind)
        out.append(L)
        i += 1
    return out


def stack_first_steps(layers, flat):
    """Lays the filters (and biases) of every inception module's first-step 1x1 convolutions back to back
    in one device buffer, in branch order, and returns the parameter list with views into those buffers.
    That is the layout DR_FUSE_STACK looks for (Eq. (12): the stacked filter bank is then simply the
    buffer).  `flat` is the list flat_params returned for `layers` (w, bias per convolution / fc)."""
    out, i = list(flat), 0
    for kind, p in layers:
        if kind in ("conv", "fc"):
            i += 2
        elif kind == "inception":
            first, j = [], i
            for br in p["branches"]:
                convs = [q for k_, q in br if k_ == "conv"]
                if br and br[0][0] == "conv" and br[0][1]["r"] == 1 and br[0][1]["s"] == 1 and br[0][1]["stride"] == 1 and br[0][1]["pad"] == 0:
                    first.append(j)
                j += 2 * len(convs)
            if len(first) > 1:
                wbig = torch.cat([out[f].reshape(out[f].shape[0], -1) for f in first], dim=0).contiguous()
                bbig = torch.cat([out[f + 1] for f in first], dim=0).contiguous()
                k0 = 0
                for f in first:
                    k = out[f].shape[0]
                    out[f] = wbig[k0:k0 + k].view(out[f].shape)
                    out[f + 1] = bbig[k0:k0 + k]
                    k0 += k
            i = j
        elif kind == "bottleneck":
            raise NotImplementedError("stack_first_steps: layer lists with bottlenecks")
    return out


def flat_params(params, dtype="f32", device="cuda", pack=False):
    """Device tensors in the order dr_net_fwd expects: conv/fc -> w, bias; bn -> gamma, beta,
    mean, var (all fp32 except w).  pack: convolution filters whose channel count allows it are
    reordered to KRSC by the library (must match the `pack` given to the descriptor builders)."""
    out = []
    for q in params:
        if "w" in q:
            w = to_device(q["w"], dtype, device)
            if pack and w.dim() == 4 and B.can_pack(w.shape[1], dtype):
                w = B.pack_filters(w)
            out += [w, to_device(q["b"], "f32", device)]
        else:
            out += [to_device(q[k], "f32", device) for k in ("gamma", "beta", "mean", "var")]
    return out
