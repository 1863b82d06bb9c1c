"""The two slimming operations of the paper as transforms on layer lists (structure only).

A layer list uses the vocabulary of ``workloads.py``: ``(kind, params)`` tuples.  Slimming changes
the *structure*; the parameters of the new slim layers come from fine-tuning in the paper
(Sec. 3.3) and are supplied by the caller here.  The one closed-form case, BatchNorm folding
(Lemma 2), is ``binding.fold_bn``.
"""
from __future__ import annotations

import copy


def streamline_slim(layers):
    """Streamline slimming (Sec. 3.1): every run conv -> ReLU -> {LRN, max-pool}* becomes one
    conv + ReLU.  A pooling layer is absorbed by multiplying the conv stride by the pooling stride
    ("Pooling Layer"); LRN / BatchNorm layers are pruned ("Non-Pooling Layer").  Non-tensor layers
    that do not follow a conv+ReLU pair (e.g. the pools between inception stages) are kept."""
    out, i = [], 0
    while i < len(layers):
        kind, p = layers[i]
        if kind == "conv" and i + 1 < len(layers) and layers[i + 1][0] == "relu":
            stride, j = p["stride"], i + 2
            while j < len(layers) and layers[j][0] in ("lrn", "maxpool", "bn"):
                if layers[j][0] == "maxpool":
                    stride *= layers[j][1]["stride"]
                j += 1
            q = dict(p)
            q["stride"] = stride
            out += [("conv", q), ("relu", {})]
            i = j
        else:
            out.append((kind, copy.deepcopy(p)))
            i += 1
    return out


def _is_conv_branch(branch):
    return all(kind in ("conv", "relu") for kind, _ in branch)


def _last_conv(branch):
    return [p for kind, p in branch if kind == "conv"][-1]


def branch_slim(inception):
    """Branch slimming (Sec. 3.2) in the form the benchmark configurations use: the non-tensor (pool) branch and the
    single-1x1 tensor branch are removed, and the branch with the largest filter (which must be at
    least as large as the pooling window) emits their feature maps as well, so the concatenated
    width is unchanged."""
    kind, p = inception
    assert kind == "inception"
    branches = copy.deepcopy(p["branches"])
    absorbed, kept = 0, []
    for br in branches:
        convs = [q for k, q in br if k == "conv"]
        has_pool = any(k == "maxpool" for k, _ in br)
        if has_pool or (len(convs) == 1 and convs[0]["r"] == 1):
            absorbed += convs[-1]["k"]          # width this branch contributed to the concat
            if has_pool:
                pool_k = [q["k"] for k, q in br if k == "maxpool"][0]
        else:
            kept.append(br)
    if not absorbed or not kept:
        return (kind, {"branches": branches})
    target = max(kept, key=lambda br: _last_conv(br)["r"])
    if any(k == "maxpool" for br in p["branches"] for k, _ in br):
        assert _last_conv(target)["r"] >= pool_k, "absorbing branch must cover the pooling window"
    _last_conv(target)["k"] += absorbed
    return (kind, {"branches": kept})


def slim_network(layers):
    """Streamline slimming on the sequential part, branch slimming in every inception module."""
    return [branch_slim(l) if l[0] == "inception" else l for l in streamline_slim(layers)]
